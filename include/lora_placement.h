/* Adapter placement and request routing for a group of servers that each run the LoRA delta of
 * include/lora.h: which adapters a server keeps and which share of an adapter's requests it gets.
 * Host code only (no device memory, no stream); C ABI.
 *
 * What is computed: the paper's placement routine (System Design, "Adapter Placement and Request
 * Routing", Algorithm 1), steps 1 to 5, once per time step:
 *   1. per adapter, the projected demand in tokens/s (lora_place_extrapolate); per rank, the
 *      utilisation it asks for = sum of its adapters' demand / the rank's operating point (tokens/s
 *      one server sustains with adapters of that rank); targetUtil = sum over ranks / servers;
 *   2. per rank, the servers it can have for itself: round(rank utilisation / targetUtil);
 *   3. ranks with a budget, highest rank first, get consecutive servers; their adapters, by descending
 *      demand, fill these servers one after the other up to targetUtil each, an adapter that does not
 *      fit continuing on the next server (its requests are split in that proportion); what remains of
 *      a started adapter after the rank's last server stays there;
 *   4. adapters not placed so far (ranks without budget, adapters without demand, a rank's overflow),
 *      highest rank first, go to a server that is empty or already serves a rank at least as high,
 *      the least utilised of those; if there is none, to the server with the highest maximum rank;
 *   5. the servers are relabelled so that the rank-weighted number of (adapter, server) pairs kept
 *      from the previous assignment is largest.
 * The result is the routing table phi[adapter][server] (each row sums to 1).  Step 6 of the listing
 * (pushing the table to the router and the servers) is the caller's.  The listing leaves the
 * extrapolation, the rounding, the order of ranks, the packing rule, the tie-breaks of step 4 and the
 * measure of step 5 open; the choices above are this library's reading. */
#ifndef LORA_PLACEMENT_H
#define LORA_PLACEMENT_H

#include "lora.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t n_servers;        /* >= 1 */
    int32_t n_adapters;       /* >= 0 */
    const int32_t *ranks;     /* [n_adapters] */
    const double *demand_tps; /* [n_adapters] projected demand, >= 0 */
    int32_t n_ops;            /* operating points given */
    const int32_t *op_ranks;  /* [n_ops] distinct ranks; every rank in `ranks` must appear */
    const double *op_tps;     /* [n_ops] tokens/s of one server at that rank, > 0 */
    const double *prev_phi;   /* [n_adapters][n_servers] previous routing table, or NULL (no step 5) */
} lora_place_problem_t;

/* Step 1, one adapter: demand of the next time step from the recorded tokens/s of earlier steps
 * (history[0..n-1], oldest first, n may be 0) and of the step that just ended: the line through the
 * last two values, not below zero.  Host only. */
lora_status_t lora_place_extrapolate(const double *history, int32_t n, double current, double *demand);

/* Steps 1 to 5.  All outputs are caller-allocated host arrays; any of server_util [n_servers],
 * server_max_rank [n_servers], rank_budget [n_ops] and target_util may be NULL.  phi is
 * [n_adapters][n_servers], row-major.  LORA_ERR_INVALID_ARG for NULL or negative input, a rank
 * without operating point, or a non-positive operating point. */
lora_status_t lora_place_assign(const lora_place_problem_t *problem, double *phi, double *server_util,
                                int32_t *server_max_rank, int32_t *rank_budget, double *target_util);

#ifdef __cplusplus
}
#endif
#endif
