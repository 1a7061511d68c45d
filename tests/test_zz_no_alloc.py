"""lora_apply_static (the entry point that allocates nothing: its workspace is a static device array
of the library) against lora_apply on the same inputs, through the C ABI: the same launches on another
workspace, so y must be bitwise the same, and within the 5e-3 row bar of the oracle.  Two calls in a
row share the array, the second with a smaller batch, so stale contents of the first would show."""
import numpy as np
import pytest
import torch

from paper_2511_22880_amd import binding as L
from paper_2511_22880_amd import workloads as wl

import gpu_util as G

pytestmark = pytest.mark.gpu


def _free_device_bytes() -> int:
    """hipMemGetInfo: sees every device allocation of the process, torch's or not."""
    import ctypes
    rt = ctypes.CDLL("libamdhip64.so")
    free, total = ctypes.c_size_t(0), ctypes.c_size_t(0)
    assert rt.hipMemGetInfo(ctypes.byref(free), ctypes.byref(total)) == 0
    return int(free.value)


def _both(dp, batch):
    x = G.bits_to_dev(batch.x_bits())
    y0 = batch.y0_bits("small")
    seg = L.lora_segments_build(dp.pool, batch.token_adapter)
    need = L.lora_apply_workspace_bytes(dp.pool, seg)
    assert need <= L.LORA_STATIC_WORKSPACE_BYTES
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    y_ref = G.bits_to_dev(y0)
    L.lora_apply(dp.pool, seg, x, y_ref, ws)
    y_new = G.bits_to_dev(y0)
    torch.cuda.synchronize()
    before = _free_device_bytes()
    L.lora_apply_static(dp.pool, seg, x, y_new)
    torch.cuda.synchronize()
    assert _free_device_bytes() >= before, "the call took device memory"
    L.lora_segments_check(seg)
    L.lora_segments_destroy(seg)
    return G.dev_to_bits(y_new), G.dev_to_bits(y_ref), y0


def test_static_workspace_apply_equals_apply_twice_in_a_row():
    big = wl.cfg1_decode()                                                  # whole-k plan, 256 tokens
    small = wl.cfg1_decode(in_features=2048, out_features=512, n_tokens=40)  # k-slice plan (few units), smaller
    dps = [G.DevicePool(big), G.DevicePool(small)]
    for dp, b in zip(dps, (big, small)):
        print(f"[case] lora_apply_static {b.name} T={b.T} in={b.in_features} out={b.out_features}", flush=True)
        y_new, y_old, y0 = _both(dp, b)
        assert np.array_equal(y_new, y_old), "static-workspace apply differs from lora_apply"
        worst = G.check_parity(y_new, G.oracle_apply(dp, b.x_bits(), y0), y0, b.token_adapter)
        print(f"[ok] {b.name}: bitwise equal to lora_apply, max row rel-L2 {worst:.3e}", flush=True)
    for dp in dps:
        dp.close()


def test_static_workspace_apply_on_a_mixed_batch_then_a_tiny_one():
    mixed = wl.small_mixed(seed=11, in_features=2048, out_features=1024, prefill_lens=(300, 500, 260, 40, 7),
                           decode_tokens=60)   # token-heavy groups beside decode-sized ones
    tiny = wl.cfg0_tiny()
    for b in (mixed, tiny):
        print(f"[case] lora_apply_static {b.name} T={b.T}", flush=True)
        dp = G.DevicePool(b)
        y_new, y_old, y0 = _both(dp, b)
        assert np.array_equal(y_new, y_old)
        rows = np.arange(0, b.T, 3, dtype=np.int32)
        G.check_parity(y_new, G.oracle_apply(dp, b.x_bits(), y0, rows=rows), y0, b.token_adapter, rows=rows)
        dp.close()


def test_static_workspace_apply_refuses_a_batch_beyond_its_array():
    """60,000 tokens of rank 256 need 4 k-slices x 15.4 M floats: far more than the 32 MiB the library holds."""
    ranks = np.array([256], dtype=np.int32)
    scales = np.array([2.0 / 256], dtype=np.float32)
    n = L.lora_pool_bytes(4096, 128, ranks, scales)
    arena = torch.zeros(n, dtype=torch.uint8, device="cuda")
    pool = L.lora_pool_create(4096, 128, ranks, scales, arena)
    L.lora_pool_mark_resident(pool, 0)
    T = 60000
    seg = L.lora_segments_build(pool, np.zeros(T, dtype=np.int32))
    assert L.lora_apply_workspace_bytes(pool, seg) > L.LORA_STATIC_WORKSPACE_BYTES
    x = torch.zeros(T, 4096, dtype=torch.bfloat16, device="cuda")
    y = torch.zeros(T, 128, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(L.LoraError) as e:
        L.lora_apply_static(pool, seg, x, y)
    assert e.value.status_name == "LORA_ERR_WORKSPACE" and "LORA_STATIC_WORKSPACE_BYTES" in e.value.detail
    L.lora_segments_destroy(seg)
    L.lora_pool_destroy(pool)
