// Host-only sanitizer run of the planner (AddressSanitizer + UndefinedBehaviorSanitizer): random pools and
// batches through lora_segments_plan, lora_segments_plan_multi and the export calls.  The launch entry
// points of the kernels are stubbed: nothing here touches a GPU.  With the argument "threads" (and built
// with ThreadSanitizer instead) four threads plan on pools of their own at once.  Built and run by
// test_host_sanitizers.py.
#include "lora.h"
#include "lora_placement.h"
#include "lora_internal.h"
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <string>
#include <thread>
#include <vector>
namespace lora {
hipError_t launch_shrink(const LaunchCtx &, const uint16_t *, int64_t, int, float *, int, int64_t, const SyncArgs *, hipStream_t) { return hipSuccess; }
hipError_t launch_shrink_wide(const LaunchCtx &, bool, const uint16_t *, int64_t, int, int, float *, uint16_t *, uint16_t *, hipStream_t) { return hipSuccess; }
hipError_t launch_expand(const LaunchCtx &, bool, const float *, int, int64_t, uint16_t *, int64_t, const SyncArgs *, hipStream_t) { return hipSuccess; }
hipError_t launch_shrink_prefill(const LaunchCtx &, int, const uint16_t *, int64_t, uint16_t *, uint16_t *, float *, int, int64_t, float *, const SyncArgs *, hipStream_t) { return hipSuccess; }
hipError_t launch_shrink_mixed(const LaunchCtx &, int, const LaunchCtx &, const uint16_t *, int64_t, int, float *, int, int64_t, const SyncArgs *, hipStream_t) { return hipSuccess; }
hipError_t launch_expand_mixed(const LaunchCtx &, const LaunchCtx &, const float *, int, int64_t, uint16_t *, int64_t, const SyncArgs *, hipStream_t) { return hipSuccess; }
hipError_t launch_apply_fused(const LaunchCtx &, const LaunchCtx &, const uint16_t *, int64_t, int, float *, int, int64_t, uint16_t *, int64_t, const SyncArgs *, hipStream_t) { return hipSuccess; }
hipError_t launch_reduce_slices(const float *, int, int64_t, float *, int64_t, hipStream_t) { return hipSuccess; }
hipError_t launch_pack_adapter(const uint16_t *, const uint16_t *, int, int, int, int, uint16_t *, uint16_t *, hipStream_t) { return hipSuccess; }
hipError_t launch_decode_fused(const LaunchCtx &, const LaunchCtx &, int, const uint16_t *, int64_t, int, int, uint16_t *, int64_t, unsigned, const SyncArgs *, hipStream_t) { return hipSuccess; }
hipError_t probe_xcc(unsigned *, int, hipStream_t) { return hipErrorNoDevice; }
hipError_t launch_linear_lora(const int32_t *, const LinBlock *, int, const uint16_t *, const uint16_t *, const uint16_t *, int64_t, int, int, const uint16_t *, const uint16_t *, uint16_t *, int64_t, hipStream_t) { return hipSuccess; }
hipError_t launch_pack_weight(const uint16_t *, int, int, uint16_t *, hipStream_t) { return hipSuccess; }
hipError_t static_scratch(void **p) { *p = nullptr; return hipErrorNoDevice; }
}
#define LK(x) do{lora_status_t s_=(x); if(s_!=LORA_OK){printf("ERR %s: %s %s\n",#x,lora_status_string(s_),lora_last_error()); return 1;} }while(0)
// One round on objects of its own: a pool, a plan, its exports, now and then a second pool and a plan
// over both.  `knobs`: also flip a process-wide setting (only where a single thread runs).
static int pool_round(std::mt19937 &g, int iter, bool knobs, uintptr_t arena_base){
  {
    const int in = 64 * (1 + g() % 128), out = 128 * (1 + g() % 64), N = 1 + g() % 200;
    std::vector<int32_t> ranks(N); std::vector<float> scales(N);
    for (int a = 0; a < N; ++a) { ranks[a] = (g() % 4 == 0) ? 1 + g() % 256 : (8 << (g() % 6)); scales[a] = 2.f / ranks[a]; }
    lora_pool_desc_t d{in, out, N, ranks.data(), scales.data(), LORA_BF16};
    size_t ab; LK(lora_pool_bytes(&d, &ab));
    lora_pool_t *pool; LK(lora_pool_create(&d, (void *)arena_base, ab, &pool));
    for (int a = 0; a < N; ++a) LK(lora_pool_mark_resident(pool, a));
    const int T = g() % 3 == 0 ? 1 + g() % 4000 : 1 + g() % 600;
    std::vector<int32_t> ta(T);
    const int hot = g() % N;
    for (auto &t : ta) { unsigned r = g() % 10; t = r == 0 ? -1 : (r < 4 ? hot : (int)(g() % N)); }
    if (knobs) { if (iter % 7 == 0) lora_set_whole_k_limit(0); else lora_set_whole_k_limit(1024); }
    lora_segments_t *seg; LK(lora_segments_plan(pool, ta.data(), T, &seg));
    lora_segments_info_t info; LK(lora_segments_info(seg, &info));
    std::vector<int32_t> su(6 * (size_t)info.n_shrink_units), eu(6 * (size_t)info.n_expand_units), perm(info.n_active), ss(info.n_segments + 1), sa(info.n_segments);
    std::vector<int64_t> vo(T);
    LK(lora_segments_export_units(seg, su.data(), eu.data()));
    LK(lora_segments_export(seg, perm.data(), ss.data(), sa.data(), vo.data()));
    // every shrink unit index valid, counts add up
    long rows = 0; for (int i = 0; i < info.n_shrink_units; ++i) rows += (long)su[6*i+2] * su[6*i+4];
    if (rows <= 0 && info.n_active > 0) { printf("no rows\n"); return 1; }
    // re-plan into the same object a few times with other routings
    LK(lora_segments_destroy(seg));
    if (iter % 5 == 0) {
      lora_pool_desc_t d2{in, 128 * (1 + (int)(g() % 16)), N, ranks.data(), scales.data(), LORA_BF16};
      size_t ab2; LK(lora_pool_bytes(&d2, &ab2));
      lora_pool_t *p2; LK(lora_pool_create(&d2, (void *)(arena_base + ((ab + 4095) & ~4095ull)), ab2, &p2));
      for (int a = 0; a < N; ++a) LK(lora_pool_mark_resident(p2, a));
      const lora_pool_t *pl[2] = {pool, p2};
      lora_segments_t *m; LK(lora_segments_plan_multi(pl, 2, ta.data(), T, &m));
      LK(lora_segments_info(m, &info));
      std::vector<int32_t> su2(6 * (size_t)info.n_shrink_units), eu2(6 * (size_t)info.n_expand_units);
      LK(lora_segments_export_units(m, su2.data(), eu2.data()));
      LK(lora_segments_destroy(m)); LK(lora_pool_destroy(p2));
    }
    LK(lora_pool_destroy(pool));
  }
  return 0;
}
int main(int argc, char **argv){
  if (argc > 1 && std::string(argv[1]) == "threads") {
    // the header's rule: objects that have nothing to do with each other may be used from different
    // threads at once (built with -fsanitize=thread)
    std::vector<std::thread> th;
    std::vector<int> rc(4, 0);
    for (int t = 0; t < 4; ++t)
      th.emplace_back([t, &rc]{
        std::mt19937 g(100 + t);
        for (int iter = 0; iter < 60 && !rc[t]; ++iter) rc[t] = pool_round(g, iter, false, (uintptr_t)0x10000000 + ((uintptr_t)t << 32));
      });
    // meanwhile a fifth thread changes the process-wide defaults (atomic variables: allowed beside planners)
    std::atomic<bool> stop{false};
    std::thread knobs([&stop]{
      for (unsigned n = 0; !stop.load(); ++n) {
        lora_set_whole_k_limit(n % 3 ? 1024 : 0); lora_set_merged_launches(n & 1); lora_set_side_stream((n >> 1) & 1);
        lora_set_decode_single_launch((n >> 2) & 1); lora_set_fused_apply((n >> 3) & 1); lora_set_fused_wait_limit(n % 5 ? 0 : 7);
      }
      lora_set_whole_k_limit(1024); lora_set_merged_launches(1); lora_set_side_stream(1); lora_set_decode_single_launch(1);
      lora_set_fused_apply(0); lora_set_fused_wait_limit(0);
    });
    for (auto &x : th) x.join();
    stop.store(true); knobs.join();
    for (int r : rc) if (r) return 1;
    printf("planner thread run ok\n");
    return 0;
  }
  std::mt19937 g(1);
  for (int iter = 0; iter < 300; ++iter)
    if (pool_round(g, iter, true, 0x10000000)) return 1;
  {
    // a segment object that outlives its pool, and a pool handle used after lora_pool_destroy: statuses,
    // not reads of freed memory (this is what the sanitizer is here to see)
    const int32_t ranks[3] = {8, 64, 200}; const float scales[3] = {0.25f, 0.03125f, 0.01f};
    lora_pool_desc_t d{512, 256, 3, ranks, scales, LORA_BF16};
    size_t ab; LK(lora_pool_bytes(&d, &ab));
    lora_pool_t *pool; LK(lora_pool_create(&d, (void *)0x10000000, ab, &pool));
    for (int a = 0; a < 3; ++a) LK(lora_pool_mark_resident(pool, a));
    const int32_t ta[6] = {0, 1, 2, -1, 1, 1};
    lora_plan_options_t opt = LORA_PLAN_OPTIONS_DEFAULT; opt.whole_k_limit = 0;
    lora_segments_t *seg; LK(lora_segments_plan_opts(pool, ta, 6, &opt, &seg));
    LK(lora_pool_destroy(pool));
    lora_status_t st = lora_segments_rebuild(seg, ta, 6, nullptr);
    if (st != LORA_ERR_STALE_SEGMENTS) { printf("rebuild after pool destroy: %s\n", lora_status_string(st)); return 1; }
    st = lora_apply(pool, seg, (void *)0x20000000, 512, (void *)0x30000000, 256, (void *)0x40000000, 1 << 20, nullptr);
    if (st != LORA_ERR_INVALID_ARG) { printf("apply on a destroyed pool: %s\n", lora_status_string(st)); return 1; }
    size_t wsb; st = lora_apply_workspace_bytes(pool, seg, &wsb);
    if (st != LORA_ERR_INVALID_ARG) { printf("workspace size on a destroyed pool: %s\n", lora_status_string(st)); return 1; }
    st = lora_pool_destroy(pool);
    if (st != LORA_ERR_INVALID_ARG) { printf("second destroy: %s\n", lora_status_string(st)); return 1; }
    lora_segments_info_t info; LK(lora_segments_info(seg, &info));   // the object itself is intact
    // a new pool (perhaps at the old address) is not the old one
    lora_pool_t *p2; LK(lora_pool_create(&d, (void *)0x10000000, ab, &p2));
    for (int a = 0; a < 3; ++a) LK(lora_pool_mark_resident(p2, a));
    st = lora_segments_rebuild(seg, ta, 6, nullptr);
    if (st != LORA_ERR_STALE_SEGMENTS) { printf("rebuild on a successor pool: %s\n", lora_status_string(st)); return 1; }
    LK(lora_segments_destroy(seg)); LK(lora_pool_destroy(p2));
  }
  // the placement routine (host only): random demands, with and without a previous table
  for (int iter = 0; iter < 200; ++iter) {
    const int S = 1 + g() % 12, N = g() % 120;
    const int32_t rs[5] = {8, 16, 32, 64, 128};
    const double tps[5] = {5000, 4500, 3800, 2900, 1900};
    std::vector<int32_t> ranks(N); std::vector<double> dem(N);
    for (int a = 0; a < N; ++a) { ranks[a] = rs[g() % 5]; dem[a] = (g() % 5 == 0) ? 0.0 : (double)(g() % 4000); }
    std::vector<double> phi((size_t)N * S), prev((size_t)N * S, 0.0), util(S), target(1);
    std::vector<int32_t> maxr(S), budget(5);
    for (int a = 0; a < N; ++a) prev[(size_t)a * S + g() % S] = 1.0;
    lora_place_problem_t pr{S, N, ranks.data(), dem.data(), 5, rs, tps, iter % 2 ? prev.data() : nullptr};
    LK(lora_place_assign(&pr, phi.data(), util.data(), maxr.data(), budget.data(), target.data()));
    for (int a = 0; a < N; ++a) { double sum = 0; for (int q = 0; q < S; ++q) sum += phi[(size_t)a * S + q]; if (sum < 0.999999 || sum > 1.000001) { printf("phi row %d sums to %g\n", a, sum); return 1; } }
    double dnext; std::vector<double> hist(g() % 6); for (auto &h : hist) h = (double)(g() % 1000);
    LK(lora_place_extrapolate(hist.data(), (int32_t)hist.size(), (double)(g() % 1000), &dnext));
    if (dnext < 0) { printf("negative demand\n"); return 1; }
  }
  printf("planner sanitizer run ok\n");
  return 0;
}
