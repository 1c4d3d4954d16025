"""HIP path (through the C ABI) against the fp64 CPU oracle, element by element, on seeded inputs."""
import math

import numpy as np
import pytest

import oracle
import workloads as wl
from workloads import CONFIGS, normal_bf16

pytestmark = pytest.mark.gpu

D = 128
SCALE = float(np.float32(1.0 / math.sqrt(D)))


def _rand_case(seed, lens, T, Hq, Hkv, extra_rows=0):
    B = len(lens)
    q = normal_bf16(seed, 0, B * T * Hq * D).reshape(B, T, Hq, D)
    ks = [normal_bf16(seed, 1 + 2 * b, (L + extra_rows) * Hkv * D).reshape(L + extra_rows, Hkv, D)
          for b, L in enumerate(lens)]
    vs = [normal_bf16(seed, 2 + 2 * b, (L + extra_rows) * Hkv * D).reshape(L + extra_rows, Hkv, D)
          for b, L in enumerate(lens)]
    return q, ks, vs


@pytest.fixture(autouse=True)
def _default_partition():
    import paper_2510_14686_amd as xa
    def reset():
        xa.xattn_configure(xa.XATTN_CFG_PIECES, 0)
        xa.xattn_configure(xa.XATTN_CFG_MIN_PIECE_TOKENS, 0)
        xa.xattn_configure(xa.XATTN_CFG_PATH, 0)
        xa.xattn_configure(xa.XATTN_CFG_PV_MODE, 0)
    reset()
    yield
    reset()


def test_tiny_config():
    """Workload 'tiny' exactly: batch 4, 8/2 heads, KV lengths 17/64/100/256, seed 0."""
    from gpu_util import check_against_oracle
    w = CONFIGS["tiny"]
    ks, vs = w.make_kv()
    check_against_oracle(w.make_q(), ks, vs, w.kv_lens(), w.scale, what="tiny")


PATHS = {"auto": 0, "vector": 1, "matrix": 2}


@pytest.mark.parametrize("path", ["auto", "vector", "matrix"])
@pytest.mark.parametrize("name,batch,div", [("qwen3_8b_decode", 12, 4), ("long_context", 3, 16),
                                            ("spec_verify", 10, 8), ("skewed_xtensor", 40, 4)])
def test_scaled_down_configs(name, batch, div, path):
    """The four large workloads with fewer sequences and shorter lengths, every element checked,
    with the automatic inner loop and with each of the two forced.  Lengths still span many 16-key
    blocks, several pieces and ragged tails."""
    import paper_2510_14686_amd as xa
    from gpu_util import check_against_oracle
    xa.xattn_configure(xa.XATTN_CFG_PATH, PATHS[path])
    w = CONFIGS[name].scaled(name + "_small", batch, div)
    lens = w.kv_lens()
    ks, vs = w.make_kv(lens)
    check_against_oracle(w.make_q(), ks, vs, lens, w.scale, what=w.name, xtensor=w.xtensor, seed=w.seed)


@pytest.mark.parametrize("path", ["auto", "vector", "matrix"])
@pytest.mark.parametrize("T", [1, 2, 3, 4])
@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (4, 4), (5, 1), (7, 1), (16, 2), (12, 2), (6, 2), (32, 16)])
def test_head_and_token_shapes(T, Hq, Hkv, path):
    """GQA groups 1..8, 1..16 KV heads (more than 8 spills into a second workgroup set), 1..4 new
    tokens with the causal mask; rows = group * T runs from 1 to 32 (above 16: two row tiles)."""
    import paper_2510_14686_amd as xa
    from gpu_util import check_against_oracle
    xa.xattn_configure(xa.XATTN_CFG_PATH, PATHS[path])
    lens = [T, T + 1, 15 + T, 16 + T, 17 + T, 63, 64, 65, 200, 333]
    q, ks, vs = _rand_case(100 + T, lens, T, Hq, Hkv)
    check_against_oracle(q, ks, vs, lens, SCALE, what="T=%d Hq=%d Hkv=%d" % (T, Hq, Hkv))


def test_single_key_and_short_sequences():
    from gpu_util import check_against_oracle
    lens = [1, 1, 2, 3, 4, 5, 15, 16, 17]
    q, ks, vs = _rand_case(7, lens, 1, 8, 2)
    (max_abs, _, _, lse_err), out_bits, lse = check_against_oracle(q, ks, vs, lens, SCALE, what="short")
    # kv_len = 1: the output is exactly the V row (bf16 in, bf16 out)
    for b in (0, 1):
        for h in range(8):
            np.testing.assert_array_equal(out_bits[b, 0, h], vs[b][0, h // 4])


def test_rows_past_kv_len_are_not_read():
    """Buffers longer than kv_len hold NaN past the end: a read of them would poison the result."""
    from gpu_util import gpu_attn, assert_parity
    lens = [5, 16, 37, 100]
    q, ks, vs = _rand_case(8, lens, 2, 8, 2, extra_rows=40)
    for b, L in enumerate(lens):
        ks[b][L:] = 0x7FC0
        vs[b][L:] = 0x7FC0
    out_bits, lse = gpu_attn(q, ks, vs, lens, SCALE)
    ref_out, ref_lse = oracle.attn(q, [k[:L] for k, L in zip(ks, lens)], [v[:L] for v, L in zip(vs, lens)],
                                   lens, SCALE)
    assert_parity(out_bits, lse, ref_out, ref_lse, what="padded buffers")


@pytest.mark.parametrize("path", ["vector", "matrix"])
@pytest.mark.parametrize("pieces,min_piece", [(8, 16), (64, 16), (1024, 16), (4096, 16), (1, 0), (37, 48)])
def test_result_does_not_depend_on_the_partition(pieces, min_piece, path):
    """Any cut of the key stream into pieces gives the same result up to fp32 re-association
    (section 4.4.3: splitting a long sequence over compute units is exact)."""
    import paper_2510_14686_amd as xa
    from gpu_util import gpu_attn, assert_parity
    lens = [700, 33, 2, 2049, 16, 512, 90]
    q, ks, vs = _rand_case(9, lens, 2, 8, 2)
    ref_out, ref_lse = oracle.attn(q, ks, vs, lens, SCALE)
    xa.xattn_configure(xa.XATTN_CFG_PIECES, pieces)
    xa.xattn_configure(xa.XATTN_CFG_MIN_PIECE_TOKENS, min_piece)
    xa.xattn_configure(xa.XATTN_CFG_PATH, PATHS[path])
    out_bits, lse = gpu_attn(q, ks, vs, lens, SCALE)
    assert_parity(out_bits, lse, ref_out, ref_lse, what="pieces=%d %s" % (pieces, path))


def test_xtensor_and_plain_allocations_give_identical_bits():
    """The kernel sees only a starting address (section 4.3, Operator Adaptation): the same bytes in
    randomly permuted 2 MiB chunks and in an ordinary allocation give bit-identical results."""
    from gpu_util import gpu_attn
    lens = [3000, 1025, 40, 2048]          # 2048 B per token row: 1024 tokens per chunk
    q, ks, vs = _rand_case(10, lens, 1, 16, 8)
    a_out, a_lse = gpu_attn(q, ks, vs, lens, SCALE, xtensor=False)
    b_out, b_lse = gpu_attn(q, ks, vs, lens, SCALE, xtensor=True, seed=5)
    c_out, c_lse = gpu_attn(q, ks, vs, lens, SCALE, xtensor=True, seed=6)
    np.testing.assert_array_equal(a_out, b_out)
    np.testing.assert_array_equal(a_lse, b_lse)
    np.testing.assert_array_equal(a_out, c_out)


def test_causal_block_equals_sequential_calls_on_gpu():
    """q_len = 4 in one call against four q_len = 1 calls with growing kv_len (section 4.4.1)."""
    from gpu_util import gpu_attn
    lens = [40, 4, 300, 77]
    T = 4
    q, ks, vs = _rand_case(11, lens, T, 8, 2)
    out4, lse4 = gpu_attn(q, ks, vs, lens, SCALE)
    for t in range(T):
        lens_t = [L - T + t + 1 for L in lens]
        out1, lse1 = gpu_attn(np.ascontiguousarray(q[:, t:t + 1]), ks, vs, lens_t, SCALE)
        a = wl.bf16_to_f32(out4[:, t]).astype(np.float64)
        b = wl.bf16_to_f32(out1[:, 0]).astype(np.float64)
        # the two calls split the keys differently, so fp32 sums differ in the last bits and a bf16
        # output may round the other way: at most one bf16 ulp (2^-7 relative), element by element
        assert np.all(np.abs(a - b) <= 2.0 ** -7 * np.maximum(np.abs(a), np.abs(b)) + 1e-30)
        assert np.max(np.abs(lse4[:, t] - lse1[:, 0])) < 1e-4


def test_lse_may_be_null_and_kv_len_below_q_len():
    from gpu_util import gpu_attn
    lens = [2, 50]
    T = 4                                   # sequence 0 has fewer keys than new tokens
    q, ks, vs = _rand_case(12, [4, 50], T, 4, 2)
    out_bits, lse = gpu_attn(q, ks, vs, lens, SCALE)
    # tokens 0 and 1 of sequence 0 see no key: out = 0, lse = -inf; tokens 2, 3 see 1 and 2 keys
    assert np.all(out_bits[0, :2] == 0) and np.all(np.isneginf(lse[0, :2]))
    ref_out, ref_lse = oracle.attn(q[:, 2:], [ks[0][:2], ks[1]], [vs[0][:2], vs[1]], [2, 50], SCALE)
    from gpu_util import assert_parity
    assert_parity(out_bits[:, 2:], lse[:, 2:], ref_out, ref_lse, what="kv_len < q_len tail")
    out2, none = gpu_attn(q, ks, vs, lens, SCALE, want_lse=False)
    assert none is None
    np.testing.assert_array_equal(out2, out_bits)


def test_repeated_calls_and_caller_workspace():
    """Calls of different shapes in a row, first on the library's workspace and then on a caller's
    buffer (handed over dirty): no call depends on what an earlier one left in the workspace."""
    import torch

    import paper_2510_14686_amd as xa
    from gpu_util import check_against_oracle
    cases = [([900, 33, 2049, 500], 1, 8, 2), ([64, 3000], 4, 16, 4), ([900, 33, 2049, 500], 1, 8, 2),
             ([5000], 2, 10, 2)]
    for rounds in range(2):
        for i, (lens, T, Hq, Hkv) in enumerate(cases):
            q, ks, vs = _rand_case(40 + i, lens, T, Hq, Hkv)
            check_against_oracle(q, ks, vs, lens, SCALE, what="repeat %d.%d" % (rounds, i))
    need = max(xa.xattn_workspace_bytes(len(l), T, Hq, Hkv, D) for l, T, Hq, Hkv in cases)
    buf = torch.full((need,), 0x55, dtype=torch.uint8, device="cuda")      # dirty on purpose
    xa.xattn_set_workspace(buf, need)
    try:
        for i, (lens, T, Hq, Hkv) in enumerate(cases):
            q, ks, vs = _rand_case(40 + i, lens, T, Hq, Hkv)
            check_against_oracle(q, ks, vs, lens, SCALE, what="caller workspace %d" % i)
        small = torch.zeros(1 << 12, dtype=torch.uint8, device="cuda")
        xa.xattn_set_workspace(small, 1 << 12)
        with pytest.raises(xa.XattnError) as e:
            q, ks, vs = _rand_case(40, cases[0][0], 1, 8, 2)
            check_against_oracle(q, ks, vs, cases[0][0], SCALE)
        assert e.value.status == xa.binding.XATTN_ENOMEM
    finally:
        torch.cuda.synchronize()
        xa.xattn_set_workspace(None, 0)


def test_sequences_without_keys():
    """kv_len = 0 (a contract violation the library tolerates): out = 0 and lse = -inf for that
    sequence, the others unaffected."""
    from gpu_util import assert_parity, gpu_attn
    lens = [0, 40, 0, 700]
    q, ks, vs = _rand_case(13, [1, 40, 1, 700], 2, 8, 2)
    lens_gpu = [0, 40, 0, 700]
    out_bits, lse = gpu_attn(q, ks, vs, lens_gpu, SCALE)
    assert np.all(out_bits[[0, 2]] == 0) and np.all(np.isneginf(lse[[0, 2]]))
    ref_out, ref_lse = oracle.attn(q[[1, 3]], [ks[1], ks[3]], [vs[1], vs[3]], [40, 700], SCALE)
    assert_parity(out_bits[[1, 3]], lse[[1, 3]], ref_out, ref_lse, what="neighbours of empty sequences")


@pytest.mark.parametrize("path", ["vector", "matrix"])
def test_split_sequences_are_aggregated_identically_every_time(path):
    """Long sequences cut into many segments whose partial results cross compute units: 300 calls in
    a row must give the same bits (the aggregation order is fixed) and match the oracle.  A stale or
    half-written partial read by the aggregation would show up as a differing call."""
    import torch

    import paper_2510_14686_amd as xa
    from gpu_util import assert_parity
    xa.xattn_configure(xa.XATTN_CFG_PATH, PATHS[path])
    xa.xattn_configure(xa.XATTN_CFG_MIN_PIECE_TOKENS, 16)
    lens = [9000, 300, 12000, 64, 7000]
    T, Hq, Hkv = 1, 16, 4
    q, ks, vs = _rand_case(50, lens, T, Hq, Hkv)
    ref_out, ref_lse = oracle.attn(q, ks, vs, lens, SCALE)
    with xa.KVStore(ks, vs) as store:
        qd = torch.from_numpy(q.view(np.int16)).cuda()
        lens_d = torch.tensor(lens, dtype=torch.int32, device="cuda")
        outs = torch.zeros((300, len(lens), T, Hq, D), dtype=torch.int16, device="cuda")
        lses = torch.zeros((300, len(lens), T, Hq), dtype=torch.float32, device="cuda")
        stream = torch.cuda.current_stream()
        for i in range(300):
            xa.xattn_decode(qd, store.k_ptrs, store.v_ptrs, lens_d, len(lens), T, Hq, Hkv, D, SCALE, outs[i], lses[i],
                            stream)
        torch.cuda.synchronize()
        outs_h = outs.cpu().numpy().view(np.uint16)
        lses_h = lses.cpu().numpy()
    assert_parity(outs_h[0], lses_h[0], ref_out, ref_lse, what="first call")
    for i in range(1, 300):
        assert np.array_equal(outs_h[i], outs_h[0]) and np.array_equal(lses_h[i], lses_h[0]), "call %d differs" % i


@pytest.mark.parametrize("pv_mode", [0, 1, 2])
def test_matrix_path_pv_modes(pv_mode):
    """The three ways the matrix path multiplies softmax weights with V all meet the parity bar;
    the default (hi + lo bf16 parts) and fp32 agree with the oracle as closely as bf16 output allows."""
    import paper_2510_14686_amd as xa
    from gpu_util import check_against_oracle
    xa.xattn_configure(xa.XATTN_CFG_PATH, PATHS["matrix"])
    xa.xattn_configure(xa.XATTN_CFG_PV_MODE, pv_mode)
    lens = [700, 33, 4, 2049, 16, 512, 90, 5000]
    q, ks, vs = _rand_case(60, lens, 4, 16, 4)
    (max_abs, rel_rows, rel_all, lse_err), _, _ = check_against_oracle(q, ks, vs, lens, SCALE, what="pv %d" % pv_mode)
    if pv_mode in (0, 1):
        assert rel_all < 1.9e-3        # bf16 rounding of the output alone gives about 1.66e-3
