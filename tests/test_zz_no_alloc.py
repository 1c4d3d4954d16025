"""xattn_decode_noalloc (the decode call for callers that cannot allocate device memory: partial
results in a fixed device array instead of a workspace from hipMalloc) against xattn_decode, bit for
bit, and against the oracle: two calls in a row, the second with a smaller input, so that whatever
the first call left in the array must not matter."""
import math

import numpy as np
import pytest

import oracle
from workloads import normal_bf16

pytestmark = pytest.mark.gpu

D = 128
SCALE = float(np.float32(1.0 / math.sqrt(D)))


def _run(fn, q, store, lens, Hkv):
    import torch
    B, T, Hq, _ = q.shape
    qd = torch.from_numpy(np.ascontiguousarray(q).view(np.int16)).cuda()
    lens_d = torch.from_numpy(np.ascontiguousarray(lens, dtype=np.int32)).cuda()
    out = torch.full((B, T, Hq, D), 0x7FC0, dtype=torch.int16, device="cuda")
    lse = torch.full((B, T, Hq), float("nan"), dtype=torch.float32, device="cuda")
    fn(qd, store.k_ptrs, store.v_ptrs, lens_d, B, T, Hq, Hkv, D, SCALE, out, lse, torch.cuda.current_stream())
    torch.cuda.synchronize()
    return out.cpu().numpy().view(np.uint16), lse.cpu().numpy()


def test_noalloc_entry_point_equals_the_allocating_one_on_two_calls_in_a_row():
    import paper_2510_14686_amd as xa
    from gpu_util import assert_parity
    for key in (xa.XATTN_CFG_PIECES, xa.XATTN_CFG_MIN_PIECE_TOKENS, xa.XATTN_CFG_PATH, xa.XATTN_CFG_PV_MODE):
        xa.xattn_configure(key, 0)
    Hq, Hkv = 16, 4
    # first call: long sequences that are split over many workgroups; second call: fewer, shorter ones
    for call, (T, lens) in enumerate([(2, [3000, 50, 2, 7000, 900, 2048]), (1, [700, 1, 33])]):
        B = len(lens)
        print("no-alloc call", call, "B", B, "T", T, "lens", lens, flush=True)
        q = normal_bf16(300 + call, 0, B * T * Hq * D).reshape(B, T, Hq, D)
        ks = [normal_bf16(300 + call, 1 + 2 * b, L * Hkv * D).reshape(L, Hkv, D) for b, L in enumerate(lens)]
        vs = [normal_bf16(300 + call, 2 + 2 * b, L * Hkv * D).reshape(L, Hkv, D) for b, L in enumerate(lens)]
        with xa.KVStore(ks, vs, xtensor=(call == 0), seed=9) as store:
            want_out, want_lse = _run(xa.xattn_decode, q, store, lens, Hkv)
            got_out, got_lse = _run(xa.xattn_decode_noalloc, q, store, lens, Hkv)
        np.testing.assert_array_equal(got_out, want_out)
        np.testing.assert_array_equal(got_lse, want_lse)
        ref_out, ref_lse = oracle.attn(q, ks, vs, np.asarray(lens, np.int32), SCALE)
        assert_parity(got_out, got_lse, ref_out, ref_lse, "no-alloc call %d" % call)


def test_noalloc_entry_point_rejects_shapes_beyond_its_array():
    import torch

    import paper_2510_14686_amd as xa
    xa.xattn_configure(xa.XATTN_CFG_PIECES, 0)
    B, T, Hq, Hkv = 2, 16, 64, 16           # 258 slots x 1024 query rows x 520 B of partial results: 137 MB
    assert xa.xattn_workspace_bytes(B, T, Hq, Hkv, D) > xa.binding.XATTN_NOALLOC_SCRATCH_BYTES
    assert xa.xattn_workspace_bytes(256, 1, 40, 8, D) < xa.binding.XATTN_NOALLOC_SCRATCH_BYTES     # the largest benchmark shapes fit
    assert xa.xattn_workspace_bytes(128, 4, 32, 8, D) < xa.binding.XATTN_NOALLOC_SCRATCH_BYTES
    ks = [normal_bf16(310, b, 64 * Hkv * D).reshape(64, Hkv, D) for b in range(B)]
    with xa.KVStore(ks, ks) as store:
        qd = torch.zeros((B, T, Hq, D), dtype=torch.int16, device="cuda")
        lens_d = torch.full((B,), 64, dtype=torch.int32, device="cuda")
        out = torch.full((B, T, Hq, D), 0x7FC0, dtype=torch.int16, device="cuda")
        with pytest.raises(xa.XattnError) as e:
            xa.xattn_decode_noalloc(qd, store.k_ptrs, store.v_ptrs, lens_d, B, T, Hq, Hkv, D, SCALE, out, None,
                                    torch.cuda.current_stream())
        assert e.value.status == xa.binding.XATTN_EUNSUPPORTED
        torch.cuda.synchronize()
        assert bool((out == 0x7FC0).all())                # nothing was enqueued
