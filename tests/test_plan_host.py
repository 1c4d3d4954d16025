"""Properties of the token-stream partition (section 4.4.3, "Layer 3": compute units balanced by token
count, long sequences split, short ones share a unit), checked on the CPU.  The functions under test
are the ones the kernels run (csrc/xattn_plan.h compiled for the host into the host test library);
only the wave-parallel sum and search of the device front end are replaced by plain loops there."""
import numpy as np
import pytest

import host_lib

GQA_COST, MLA_COST = 16, 192


def _cases():
    rng = np.random.RandomState(11)
    yield "tiny", [17, 64, 100, 256]
    yield "single token", [1]
    yield "all empty but one", [0, 0, 5, 0]
    yield "negative and zero lengths", [-3, 0, 40, -1, 0, 700, 0]
    yield "uniform 64", rng.randint(512, 4097, size=64)
    yield "long 16", rng.randint(16384, 32769, size=16)
    yield "lognormal 256", np.clip(np.rint(1024 * np.exp(1.2 * rng.randn(256))), 16, 65536).astype(np.int64)
    yield "one 65536-token sequence", [65536]
    yield "short ones around a long one", [3] * 50 + [65536] + [2] * 50
    yield "batch 4096 of short sequences", 1 + rng.randint(0, 40, size=4096)
    yield "batch 4096 with empties", rng.randint(0, 3, size=4096) * rng.randint(1, 30, size=4096)


CASES = list(_cases())
PARTITIONS = [(256, 64), (1, 16), (8, 16), (37, 48), (1024, 16), (65536, 16)]


def _all_segments(lens, n_pieces, min_piece, cost, skew=0):
    total, used = host_lib.plan(lens, n_pieces, min_piece, cost, skew)
    rows = []
    for p in range(used):
        for b, j0, j1, slot, whole in host_lib.piece_segments(lens, n_pieces, min_piece, cost, p, skew=skew):
            rows.append((p, b, j0, j1, slot, whole))
    return total, used, rows


@pytest.mark.parametrize("cost", [0, GQA_COST, MLA_COST])
@pytest.mark.parametrize("n_pieces,min_piece", PARTITIONS)
@pytest.mark.parametrize("name,lens", CASES, ids=[c[0] for c in CASES])
def test_pieces_tile_the_stream_and_balance(name, lens, n_pieces, min_piece, cost):
    lens = np.asarray(lens, np.int64)
    N = int(sum(L + cost for L in lens if L > 0))
    total, used = host_lib.plan(lens, n_pieces, min_piece, cost)
    assert total == N
    assert used == max(1, min(n_pieces, N // min_piece))
    bounds = host_lib.piece_bounds(lens, n_pieces, min_piece, cost)
    assert bounds[0] == 0 and bounds[-1] == N and len(bounds) == used + 1
    sizes = np.diff(bounds.astype(np.int64))
    if N > 0:
        assert np.all(sizes > 0), "an empty piece"
        assert np.all(bounds[:-1] % 16 == 0), "inner piece bounds are multiples of the 16-key block"
        assert np.all(np.abs(sizes - N / used) <= 16), "pieces differ from N / P by more than one block"
    # piece_of is the inverse of the bounds
    rng = np.random.RandomState(3)
    xs = set(int(x) for x in rng.randint(0, max(N, 1), size=64)) | set(int(b) for b in bounds[:-1]) | \
        set(int(b) - 1 for b in bounds[1:])
    for x in sorted(xs):
        if 0 <= x < N:
            assert host_lib.piece_of(lens, n_pieces, min_piece, cost, x) == int(np.searchsorted(bounds, x, side="right")) - 1


@pytest.mark.parametrize("cost,skew", [(0, 0), (GQA_COST, 0), (MLA_COST, 0), (GQA_COST, 32), (MLA_COST, 200)])
@pytest.mark.parametrize("n_pieces,min_piece", PARTITIONS[:5])
@pytest.mark.parametrize("name,lens", CASES, ids=[c[0] for c in CASES])
def test_every_token_is_in_exactly_one_segment(name, lens, n_pieces, min_piece, cost, skew):
    lens = np.asarray(lens, np.int64)
    B = len(lens)
    total, used, rows = _all_segments(lens, n_pieces, min_piece, cost, skew)
    bounds = host_lib.piece_bounds(lens, n_pieces, min_piece, cost, skew)
    covered = {b: [] for b in range(B)}
    slots = set()
    tokens_of_piece = np.zeros(used, np.int64)
    for p, b, j0, j1, slot, whole in rows:
        assert 0 <= b < B and 0 <= j0 < j1 <= lens[b], "an empty or out-of-range segment"
        assert slot == p + b and 0 <= slot < n_pieces + B
        assert slot not in slots, "two segments share a partial-result slot"
        slots.add(slot)
        assert bool(whole) == (j0 == 0 and j1 == lens[b])
        covered[b].append((j0, j1, p))
        tokens_of_piece[p] += j1 - j0
    for b in range(B):
        L = max(int(lens[b]), 0)
        segs = covered[b]                       # pieces are walked in stream order
        if L == 0:
            assert segs == []
            continue
        assert segs[0][0] == 0 and segs[-1][1] == L
        for (a0, a1, pa), (b0, b1, pb) in zip(segs, segs[1:]):
            assert a1 == b0 and pb == pa + 1, "segments of a sequence are contiguous, in consecutive pieces"
    # a piece never holds more tokens than positions
    assert np.all(tokens_of_piece <= np.diff(bounds.astype(np.int64)))
    assert int(tokens_of_piece.sum()) == int(lens[lens > 0].sum())


@pytest.mark.parametrize("cost,skew", [(GQA_COST, 0), (MLA_COST, 0), (GQA_COST, 32), (MLA_COST, 200)])
@pytest.mark.parametrize("n_pieces,min_piece", PARTITIONS[:5])
@pytest.mark.parametrize("name,lens", CASES, ids=[c[0] for c in CASES])
def test_segment_table_for_the_merge_equals_the_walk(name, lens, n_pieces, min_piece, cost, skew):
    lens = np.asarray(lens, np.int64)
    total, used, rows = _all_segments(lens, n_pieces, min_piece, cost, skew)
    meta = host_lib.meta(lens, n_pieces, min_piece, cost, skew)
    for b in range(len(lens)):
        mine = [r for r in rows if r[1] == b]
        first_slot, n_seg = int(meta[b, 0]), int(meta[b, 1])
        assert n_seg == len(mine)
        if mine:
            assert [r[4] for r in mine] == list(range(first_slot, first_slot + n_seg))
            assert (n_seg == 1) == bool(mine[0][5]), "exactly the unsplit sequences are finished by the decode kernel"


@pytest.mark.parametrize("skew", [1, 32, 200])
@pytest.mark.parametrize("n_pieces,min_piece", [(256, 64), (8, 16), (1024, 16), (65536, 16), (37, 48)])
@pytest.mark.parametrize("name,lens", CASES, ids=[c[0] for c in CASES])
def test_unequal_xcd_parts(name, lens, n_pieces, min_piece, skew):
    """With a skew the stream is cut into eight XCD parts, the even ones longer and the odd ones shorter
    by skew / 1000, each cut into equal pieces; the pieces still tile the stream and piece_of inverts
    the bounds.  Too few or too small pieces switch the skew off."""
    lens = np.asarray(lens, np.int64)
    N = int(sum(L + GQA_COST for L in lens if L > 0))
    total, used = host_lib.plan(lens, n_pieces, min_piece, GQA_COST, skew)
    assert total == N and used == max(1, min(n_pieces, N // min_piece))
    bounds = host_lib.piece_bounds(lens, n_pieces, min_piece, GQA_COST, skew).astype(np.int64)
    assert bounds[0] == 0 and bounds[-1] == N and len(bounds) == used + 1
    sizes = np.diff(bounds)
    if N == 0:
        return
    assert np.all(sizes > 0) and np.all(bounds[:-1] % 16 == 0)
    skewed = used % 8 == 0 and N // used >= 512
    if skewed:
        m = used // 8
        for x in range(8):
            want = N / used * (1 + skew / 1000.0 * (1 if x % 2 == 0 else -1))
            assert np.all(np.abs(sizes[x * m:(x + 1) * m] - want) <= 17), "XCD part %d" % x
            assert abs(bounds[x * m] - N * (x + (skew / 1000.0 if x % 2 else 0)) / 8) <= 9
    else:
        assert np.array_equal(bounds, host_lib.piece_bounds(lens, n_pieces, min_piece, GQA_COST, 0))
    rng = np.random.RandomState(4)
    xs = set(int(x) for x in rng.randint(0, N, size=64)) | set(int(b) for b in bounds[:-1]) | set(int(b) - 1 for b in bounds[1:])
    for x in sorted(xs):
        if 0 <= x < N:
            assert host_lib.piece_of(lens, n_pieces, min_piece, GQA_COST, x, skew) == int(np.searchsorted(bounds, x, side="right")) - 1


def test_stream_positions_up_to_the_32_bit_limit():
    """N just below 2^31 with the largest piece count: the 32-bit products of piece_bound do not wrap;
    beyond 2^31 - 1 the documented limit is reported, not wrapped."""
    lens = np.full(4096, 524287 - GQA_COST, np.int64)            # N = 4096 * 524287 = 2^31 - 4096
    N = 4096 * 524287
    for n_pieces, skew in ((256, 0), (65535, 0), (65536, 0), (256, 200), (65536, 32)):
        total, used = host_lib.plan(lens, n_pieces, 64, GQA_COST, skew)
        assert total == N and used == n_pieces
        bounds = host_lib.piece_bounds(lens, n_pieces, 64, GQA_COST, skew).astype(np.int64)
        assert bounds[0] == 0 and bounds[-1] == N
        sizes = np.diff(bounds)
        assert np.all(sizes > 0) and np.all(np.abs(sizes - N / used) <= 16 + N / used * skew / 1000.0)
        for x in (0, 1, N // 3, N - 1):
            assert host_lib.piece_of(lens, n_pieces, 64, GQA_COST, x, skew) == int(np.searchsorted(bounds, x, side="right")) - 1
    segs = host_lib.piece_segments(lens, 65536, 64, GQA_COST, 65535)
    assert segs[-1][0] == 4095 and segs[-1][2] == lens[-1]
    too_many = np.full(4096, 524288, np.int64)                   # N = 2^31 + ...: outside the limit
    assert host_lib.plan(too_many, 256, 64, GQA_COST) == (-1, -1)
