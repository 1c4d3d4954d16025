"""Helpers of the GPU parity tests: run the HIP path through the C ABI, run the oracle, compare."""
import numpy as np
import torch

import oracle
import paper_2510_14686_amd as xa
from workloads import bf16_to_f32

# Tolerances of the parity bar: GPU (bf16 inputs, fp32 accumulation, bf16 output) against the fp64
# oracle on identical bf16 bytes.
TOL_MAX_ABS = 1e-2
TOL_REL_L2 = 5e-3
TOL_LSE = 1e-3


def gpu_attn(q, ks, vs, kv_lens, scale, xtensor=False, seed=0, want_lse=True, store=None):
    """q uint16 [B,T,Hq,D]; ks/vs lists of uint16 [L,Hkv,D]. Returns (out uint16 [B,T,Hq,D], lse f32)."""
    B, T, Hq, D = q.shape
    Hkv = ks[0].shape[1]
    own = store is None
    if own:
        store = xa.KVStore(ks, vs, device=0, xtensor=xtensor, seed=seed)
    try:
        qd = torch.from_numpy(np.ascontiguousarray(q).view(np.int16)).cuda()
        lens = torch.from_numpy(np.ascontiguousarray(kv_lens, dtype=np.int32)).cuda()
        out = torch.full((B, T, Hq, D), 0x7FC0, dtype=torch.int16, device="cuda")       # NaN pattern
        lse = torch.full((B, T, Hq), float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
        stream = torch.cuda.current_stream()
        xa.xattn_decode(qd, store.k_ptrs, store.v_ptrs, lens, B, T, Hq, Hkv, D, scale, out, lse, stream)
        torch.cuda.synchronize()
        out_h = out.cpu().numpy().view(np.uint16)
        lse_h = lse.cpu().numpy() if want_lse else None
    finally:
        if own:
            store.close()
    return out_h, lse_h


def errors(out_bits, lse_gpu, ref_out, ref_lse):
    """(max-abs, max over rows of relative L2, whole-tensor relative L2, max-abs of lse)."""
    got = bf16_to_f32(out_bits).astype(np.float64).reshape(ref_out.shape)
    diff = got - ref_out
    max_abs = float(np.max(np.abs(diff))) if diff.size else 0.0
    row_num = np.sqrt(np.sum(diff * diff, axis=-1))
    row_den = np.sqrt(np.sum(ref_out * ref_out, axis=-1))
    rel_rows = float(np.max(row_num / np.maximum(row_den, 1e-30))) if diff.size else 0.0
    rel_all = float(np.sqrt(np.sum(diff * diff)) / max(np.sqrt(np.sum(ref_out * ref_out)), 1e-30))
    lse_err = float(np.max(np.abs(lse_gpu.astype(np.float64) - ref_lse))) if lse_gpu is not None else 0.0
    return max_abs, rel_rows, rel_all, lse_err


def assert_parity(out_bits, lse_gpu, ref_out, ref_lse, what=""):
    assert not np.any(np.isnan(bf16_to_f32(out_bits))), "NaN in GPU output " + what
    if lse_gpu is not None:
        assert not np.any(np.isnan(lse_gpu)), "NaN in GPU lse " + what
    max_abs, rel_rows, rel_all, lse_err = errors(out_bits, lse_gpu, ref_out, ref_lse)
    msg = "%s max_abs=%.3e rel_l2_rows=%.3e rel_l2=%.3e lse=%.3e" % (what, max_abs, rel_rows, rel_all, lse_err)
    assert max_abs <= TOL_MAX_ABS, msg
    assert rel_rows <= TOL_REL_L2, msg
    assert lse_err <= TOL_LSE, msg
    return max_abs, rel_rows, rel_all, lse_err


def check_against_oracle(q, ks, vs, kv_lens, scale, what="", **kw):
    out_bits, lse = gpu_attn(q, ks, vs, kv_lens, scale, **kw)
    ref_out, ref_lse = oracle.attn(q, ks, vs, kv_lens, scale)
    return assert_parity(out_bits, lse, ref_out, ref_lse, what), out_bits, lse
