"""Beam-search selection step (section 4.5.1, "Beam Search Optimization"): the oracle (sort everything)
against pins that do not use it, planted mistakes that the pins must catch, and the product's heap with
early exit (host code in libxattn.so, no GPU needed) against the oracle, bit for bit."""
import inspect
import os

import numpy as np
import pytest

import oracle
import oracle.beam as oracle_beam
from workloads import BEAM_CONFIGS, BeamWorkload

HERE = os.path.dirname(os.path.abspath(__file__))


# ---------------------------------------------------------------- pins of the oracle
def _brute_force(beam_lp, cand_lp, cand_tok):
    """Repeatedly take the best remaining candidate; plain Python, tiny inputs only."""
    R, W, K = cand_lp.shape
    res = []
    for r in range(R):
        cands = [(np.float32(beam_lp[r, w]) + np.float32(cand_lp[r, w, k]), w, k) for w in range(W) for k in range(K)]
        picked = []
        for _ in range(W):
            best = None
            for c in cands:
                if c in picked:
                    continue
                if best is None or c[0] > best[0] or (c[0] == best[0] and (c[1], c[2]) < (best[1], best[2])):
                    best = c
            picked.append(best)
        res.append(picked)
    s = np.array([[c[0] for c in p] for p in res], np.float32)
    par = np.array([[c[1] for c in p] for p in res], np.int32)
    tok = np.array([[cand_tok[r, c[1], c[2]] for c in p] for r, p in enumerate(res)], np.int32)
    return s, par, tok


def _read_example():
    vals = {}
    for line in open(os.path.join(HERE, "golden", "beam_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, *rest = line.split()
        vals[key] = [float(x) for x in rest]
    beam_lp = np.array([vals["beam_lp"]], np.float32)
    cand_lp = np.array([[vals["cand_lp0"], vals["cand_lp1"]]], np.float32)
    cand_tok = np.array([[vals["cand_tok0"], vals["cand_tok1"]]], np.int32)
    want = (np.array([vals["out_lp"]], np.float32), np.array([vals["out_parent"]], np.int32), np.array([vals["out_tok"]], np.int32))
    return beam_lp, cand_lp, cand_tok, want


def _tiny_cases():
    rng = np.random.default_rng(11)
    for W, K in ((1, 1), (1, 5), (3, 1), (2, 3), (4, 4), (5, 2)):
        cand = -np.sort(rng.integers(0, 12, size=(2, W, K)) / 4.0, axis=2).astype(np.float32)    # many ties
        beam = -(rng.integers(0, 8, size=(2, W)) / 4.0).astype(np.float32)
        tok = rng.integers(0, 1000, size=(2, W, K)).astype(np.int32)
        yield beam, cand, tok


def check_oracle(select):
    """Every pin of the oracle; raises AssertionError on the first one that fails."""
    beam_lp, cand_lp, cand_tok, want = _read_example()
    got = select(beam_lp, cand_lp, cand_tok)
    for g, w in zip(got, want):
        assert np.array_equal(g, w), "hand-computed example"
    for beam, cand, tok in _tiny_cases():
        got, want = select(beam, cand, tok), _brute_force(beam, cand, tok)
        for g, w in zip(got, want):
            assert np.array_equal(g, w), "brute force"
    # top_k = 1: the selection is a sort of beam_lp + cand_lp[..., 0]; beam_width = 1: candidate 0 wins
    rng = np.random.default_rng(12)
    beam = -rng.random((3, 6)).astype(np.float32)
    cand = -rng.random((3, 6, 1)).astype(np.float32)
    s, par, tok = select(beam, cand, None)
    tot = beam + cand[..., 0]
    assert np.array_equal(s, -np.sort(-tot, axis=1)) and np.array_equal(tot[np.arange(3)[:, None], par], s) and not tok.any()
    cand = -np.sort(rng.random((2, 1, 9)), axis=2).astype(np.float32)
    s, par, tok = select(np.zeros((2, 1), np.float32), cand, None)
    assert np.array_equal(s[:, 0], cand[:, 0, 0]) and not par.any() and not tok.any()
    # invariants on a larger case: descending output, nothing left out beats the last one kept,
    # -inf candidates (masked items) come last
    w = BeamWorkload("pin", 3, 16, 24, seed=21, vocab=256)
    beam, cand, tok = w.make()
    cand[:, :, 20:] = -np.inf
    s, par, tok_out = select(beam, cand, tok)
    assert (np.diff(s, axis=1) <= 0).all() and np.isfinite(s).all()
    score = beam[:, :, None] + cand
    for r in range(3):
        kept = np.zeros_like(score[r], dtype=bool)
        for i in range(16):
            ks = np.nonzero((tok[r, par[r, i]] == tok_out[r, i]))[0]
            assert len(ks) == 1 and score[r, par[r, i], ks[0]] == s[r, i]
            kept[par[r, i], ks[0]] = True
        assert kept.sum() == 16 and score[r][~kept].max() <= s[r, -1]


def test_oracle_passes_its_pins():
    check_oracle(oracle.beam_select)


MUTANTS = [
    ("order = np.argsort(-flat.astype(np.float64), kind=\"stable\")[:W]", "order = np.argsort(flat.astype(np.float64), kind=\"stable\")[:W]", "ascending sort"),
    ("score = (beam_lp[:, :, None] + cand_lp).astype(np.float32)", "score = (0 * beam_lp[:, :, None] + cand_lp).astype(np.float32)", "sequence log-probability dropped"),
    ("out_p[r] = order // K", "out_p[r] = order % W", "wrong parent index"),
    ("k = order % K", "k = order // K", "wrong candidate index"),
    ("kind=\"stable\")[:W]", "kind=\"stable\")[::-1][:W][::-1]", "worst instead of best"),
    ("order = np.argsort(-flat.astype(np.float64), kind=\"stable\")[:W]", "order = (W * K - 1 - np.argsort(-flat[::-1].astype(np.float64), kind=\"stable\"))[:W]", "ties broken the other way"),
]


@pytest.mark.parametrize("old,new,what", MUTANTS, ids=[m[2] for m in MUTANTS])
def test_pins_catch_planted_mistakes(old, new, what):
    """A mistake planted in a copy of the oracle's source must fail a pin."""
    src = inspect.getsource(oracle_beam)
    assert src.count(old) == 1, "mutation site not found: " + old
    ns = {}
    exec(compile(src.replace(old, new), "mutant_" + what.replace(" ", "_"), "exec"), ns)
    with pytest.raises(AssertionError):
        check_oracle(ns["beam_select"])


# ---------------------------------------------------------------- the product against the oracle
def _assert_same(got, want, what):
    for g, w, name in zip(got[:3], want, ("scores", "parents", "tokens")):
        assert np.array_equal(g, w), "%s: %s differ" % (what, name)


@pytest.mark.parametrize("flags", [0, 1])
def test_product_matches_oracle_on_tie_heavy_inputs(flags):
    import paper_2510_14686_amd as xa
    for beam, cand, tok in _tiny_cases():
        _assert_same(xa.xbeam_select(beam, cand, tok, flags=flags | xa.XBEAM_CHECK_INPUT), oracle.beam_select(beam, cand, tok), "tiny")
    rng = np.random.default_rng(5)
    for W, K in ((4, 16), (16, 4), (33, 7), (128, 128)):
        cand = -np.sort(rng.integers(0, 40, size=(3, W, K)) / 8.0, axis=2).astype(np.float32)
        beam = -np.sort(rng.integers(0, 16, size=(3, W)) / 8.0, axis=1).astype(np.float32)
        _assert_same(xa.xbeam_select(beam, cand, None, flags=flags), oracle.beam_select(beam, cand, None), "W=%d K=%d" % (W, K))


@pytest.mark.parametrize("name", sorted(BEAM_CONFIGS))
def test_product_matches_oracle_on_the_workloads(name):
    import paper_2510_14686_amd as xa
    beam, cand, tok = BEAM_CONFIGS[name].make()
    want = oracle.beam_select(beam, cand, tok)
    got = xa.xbeam_select(beam, cand, tok)
    _assert_same(got, want, name)
    _assert_same(xa.xbeam_select(beam, cand, tok, flags=xa.XBEAM_FULL_SORT), want, name + " full sort")
    W, K = cand.shape[1:]
    assert (got[3] <= W * K).all() and (got[3] >= W).all()
    if W * K >= 1024:
        assert got[3].max() < 0.25 * W * K, "early exit examined %s of %d candidates" % (got[3], W * K)


def test_masked_candidates_and_unsorted_sequences():
    import paper_2510_14686_amd as xa
    w = BeamWorkload("masked", 2, 8, 32, seed=31, vocab=128)
    beam, cand, tok = w.make()
    cand[:, :, 5:] = -np.inf                     # item filter: only 5 valid continuations per sequence
    cand[0, 3, :] = -np.inf                      # a sequence with no valid continuation
    _assert_same(xa.xbeam_select(beam, cand, tok, flags=xa.XBEAM_CHECK_INPUT), oracle.beam_select(beam, cand, tok), "masked")
    beam2 = beam[:, ::-1].copy()                 # the sequences themselves need not be sorted
    _assert_same(xa.xbeam_select(beam2, cand, tok), oracle.beam_select(beam2, cand, tok), "unsorted sequences")


def test_outputs_are_written_in_place_and_arguments_checked():
    import paper_2510_14686_amd as xa
    beam, cand, tok = BEAM_CONFIGS["beam_small"].make()
    R, W, K = cand.shape
    out = (np.full((R, W), 9, np.float32), np.full((R, W), 9, np.int32), np.full((R, W), 9, np.int32), np.zeros(R, np.int64))
    got = xa.xbeam_select(beam, cand, tok, out_lp=out[0], out_parent=out[1], out_tok=out[2], visited=out[3])
    assert all(g is o for g, o in zip(got, out))
    _assert_same(out, oracle.beam_select(beam, cand, tok), "in place")
    bad = cand.copy()
    bad[1, 2, 3] = bad[1, 2, 2] + 1.0
    with pytest.raises(xa.XattnError) as e:
        xa.xbeam_select(beam, bad, tok, flags=xa.XBEAM_CHECK_INPUT)
    assert e.value.status == xa.binding.XATTN_EINVAL and "descending" in str(e.value)
    bad = cand.copy()
    bad[0, 0, 0] = np.nan
    with pytest.raises(xa.XattnError):
        xa.xbeam_select(beam, bad, tok, flags=xa.XBEAM_CHECK_INPUT)
    with pytest.raises(xa.XattnError):
        xa.xbeam_select(beam, cand, tok, flags=64)
    with pytest.raises(TypeError):
        xa.xbeam_select(beam.astype(np.float64), cand, tok)
