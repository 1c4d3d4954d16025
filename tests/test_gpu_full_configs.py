"""The four large workloads at full size, in the launch configuration bench.py times (automatic
partition, xTensor placement where the workload says so), against the fp64 oracle.

Every output row of a sample of sequences is compared element by element (the sample always holds
the longest and the shortest sequence); the remaining rows are checked for properties that hold at
any size: finite, and |out| bounded by the largest |V| entry (a convex combination of V rows)."""
import numpy as np
import pytest

import oracle
from workloads import CONFIGS, bf16_to_f32

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,n_check", [("qwen3_8b_decode", 64), ("long_context", 6), ("spec_verify", 24),
                                          ("skewed_xtensor", 64)])
def test_full_size_workload(name, n_check):
    import paper_2510_14686_amd as xa
    from gpu_util import assert_parity, gpu_attn
    xa.xattn_configure(xa.XATTN_CFG_PIECES, 0)
    xa.xattn_configure(xa.XATTN_CFG_MIN_PIECE_TOKENS, 0)
    w = CONFIGS[name]
    lens = w.kv_lens()
    q = w.make_q()
    ks, vs = w.make_kv(lens)
    print("case", name, "tokens", int(lens.sum()), flush=True)
    out_bits, lse = gpu_attn(q, ks, vs, lens, w.scale, xtensor=w.xtensor, seed=w.seed)
    B = w.batch
    sel = sorted(set(np.linspace(0, B - 1, min(n_check, B)).astype(int).tolist()
                     + [int(np.argmax(lens)), int(np.argmin(lens))]))
    ref_out, ref_lse = oracle.attn(q[sel], [ks[b] for b in sel], [vs[b] for b in sel], lens[sel], w.scale)
    print(name, "max_abs=%.2e rel_l2_rows=%.2e rel_l2=%.2e lse=%.2e"
          % assert_parity(out_bits[sel], lse[sel], ref_out, ref_lse, name), flush=True)
    got = bf16_to_f32(out_bits)
    assert np.all(np.isfinite(got)) and np.all(np.isfinite(lse))
    vmax = max(float(np.max(np.abs(bf16_to_f32(v)))) for v in vs)
    assert float(np.max(np.abs(got))) <= vmax * (1 + 2 ** -7)


@pytest.mark.parametrize("name,n_check", [("mla_decode", 6), ("mla_verify", 4)])
def test_full_size_latent_kv_workload(name, n_check):
    """The two latent-KV workloads at full size, as bench.py launches them (automatic partition and
    workgroup shape, xTensor ranges): sampled sequences element by element, every row bounded."""
    import paper_2510_14686_amd as xa
    from gpu_util import assert_parity
    from test_gpu_mla import gpu_mla
    from workloads import MLA_CONFIGS
    for key in (xa.XATTN_CFG_PIECES, xa.XATTN_CFG_MIN_PIECE_TOKENS, xa.XATTN_CFG_PV_MODE, xa.XATTN_CFG_MLA_LAYOUT):
        xa.xattn_configure(key, 0)
    w = MLA_CONFIGS[name]
    lens = w.kv_lens()
    q, cs = w.make_q(), w.make_cache(lens)
    print("case", name, "tokens", int(lens.sum()), flush=True)
    out_bits, lse = gpu_mla(q, cs, lens, w.scale, xtensor=w.xtensor, seed=w.seed)
    B = w.batch
    sel = sorted(set(np.linspace(0, B - 1, n_check).astype(int).tolist() + [int(np.argmax(lens)), int(np.argmin(lens))]))
    ref_out, ref_lse = oracle.mla(q[sel], [cs[b] for b in sel], lens[sel], w.d_latent, w.scale)
    print(name, "max_abs=%.2e rel_l2_rows=%.2e rel_l2=%.2e lse=%.2e"
          % assert_parity(out_bits[sel], lse[sel], ref_out, ref_lse, name), flush=True)
    got = bf16_to_f32(out_bits)
    assert np.all(np.isfinite(got)) and np.all(np.isfinite(lse))
    vmax = max(float(np.max(np.abs(bf16_to_f32(c[:, :w.d_latent])))) for c in cs)
    assert float(np.max(np.abs(got))) <= vmax * (1 + 2 ** -6)
