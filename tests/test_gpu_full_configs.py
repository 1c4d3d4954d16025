"""The four large workloads and the two latent-KV workloads at full size, in the launch configuration
bench.py times (automatic partition, xTensor placement where the workload says so), against the fp64
oracle: every output row of EVERY sequence is compared element by element."""
import numpy as np
import pytest

import oracle
from workloads import CONFIGS

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["qwen3_8b_decode", "long_context", "spec_verify", "skewed_xtensor"])
def test_full_size_workload(name):
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
    ref_out, ref_lse = oracle.attn(q, ks, vs, lens, w.scale)
    print(name, "all %d sequences: max_abs=%.2e rel_l2_rows=%.2e rel_l2=%.2e lse=%.2e"
          % ((w.batch,) + assert_parity(out_bits, lse, ref_out, ref_lse, name)), flush=True)


@pytest.mark.parametrize("name", ["mla_decode", "mla_verify"])
def test_full_size_latent_kv_workload(name):
    """The two latent-KV workloads at full size, as bench.py launches them (automatic partition and
    workgroup shape, xTensor ranges): every sequence element by element."""
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
    ref_out, ref_lse = oracle.mla(q, cs, lens, w.d_latent, w.scale)
    print(name, "all %d sequences: max_abs=%.2e rel_l2_rows=%.2e rel_l2=%.2e lse=%.2e"
          % ((w.batch,) + assert_parity(out_bits, lse, ref_out, ref_lse, name)), flush=True)
