"""xTensor ranges, the page pool and write_kvcache on the real HIP virtual-memory driver."""
import math

import numpy as np
import pytest

import oracle
import workloads as wl
from workloads import normal_bf16

pytestmark = pytest.mark.gpu

PAGE = 2 << 20
D = 128
SCALE = float(np.float32(1.0 / math.sqrt(D)))


def _pattern(n_bytes, seed):
    return normal_bf16(seed, 77, n_bytes // 2)


def test_map_is_contiguous_to_kernels_and_scattered_physically():
    """Bytes written through the range come back unchanged (contiguous view), the chunk order is a
    seeded permutation, and read through a second mapping in physical order they sit where the
    address identity of section 4.3 says: virtual chunk i is physical chunk order[i]."""
    import paper_2510_14686_amd as xa
    n = 7
    data = _pattern(n * PAGE - 4096, 1)
    base, h = xa.xtensor_map(64 * PAGE, data.nbytes, 123, 0)
    base2, h2 = xa.xtensor_map(64 * PAGE, data.nbytes, 124, 0)
    try:
        assert base % PAGE == 0
        order, order2 = xa.xtensor_chunk_order(h), xa.xtensor_chunk_order(h2)
        assert sorted(order.tolist()) == list(range(n)) and sorted(order2.tolist()) == list(range(n))
        assert not np.array_equal(order, np.arange(n)) and not np.array_equal(order, order2)
        assert np.array_equal(order, xa.xtensor_chunk_order(h))
        xa.xtensor_upload(base, data)
        back = np.empty_like(data)
        xa.xtensor_download(back, base)
        np.testing.assert_array_equal(back, data)
        # unaligned sub-range crossing chunk boundaries
        sub = np.empty(3 * PAGE // 2, dtype=np.uint16)
        xa.xtensor_download(sub, base + PAGE // 2 + 64)
        np.testing.assert_array_equal(sub, data[(PAGE // 2 + 64) // 2:][:sub.size])
        try:
            view = xa.xtensor_physical_view(h)
        except xa.XattnError as e:
            pytest.skip("the driver refuses a second mapping of a physical chunk: %s" % e)
        phys = np.empty(n * PAGE // 2, dtype=np.uint16)
        xa.xtensor_download(phys, view)
        padded = np.zeros(n * PAGE // 2, dtype=np.uint16)
        padded[:data.size] = data
        per = PAGE // 2
        for i in range(n):
            page, off = oracle.page_of(base + i * PAGE + 10, base, PAGE)
            assert (page, off) == (i, 10)
            want = padded[i * per:(i + 1) * per]
            got = phys[order[i] * per:(order[i] + 1) * per]
            valid = min(per, max(0, data.size - i * per))
            np.testing.assert_array_equal(got[:valid], want[:valid])
    finally:
        xa.xtensor_unmap(h)
        xa.xtensor_unmap(h2)
    with pytest.raises(xa.XattnError) as e:
        xa.xtensor_unmap(h)
    assert e.value.status == xa.binding.XATTN_EINVAL


def test_map_argument_errors_and_empty_prefix():
    import paper_2510_14686_amd as xa
    for args in ((0, 0, 1, 0), (PAGE, 2 * PAGE, 1, 0), (PAGE, PAGE, 1, 99)):
        with pytest.raises(xa.XattnError):
            xa.xtensor_map(*args)
    base, h = xa.xtensor_map(4 * PAGE, 0, 5, 0)                # a reservation alone backs nothing
    assert len(xa.xtensor_chunk_order(h)) == 0
    xa.xtensor_unmap(h)
    for _ in range(20):                                        # map/unmap cycles leak neither memory nor addresses
        base, h = xa.xtensor_map(256 * PAGE, 64 * PAGE, 6, 0)
        xa.xtensor_unmap(h)


def test_pool_on_the_hip_driver_reuse_keeps_addresses_and_bytes():
    import paper_2510_14686_amd as xa
    pool = xa.xtensor_pool_create(0, 24, 3)
    try:
        base, rng, reused = xa.xtensor_open(pool, 1, 16 * PAGE, 5 * PAGE)
        data = _pattern(5 * PAGE, 2)
        xa.xtensor_upload(base, data)
        assert xa.xtensor_grow(rng, 9 * PAGE) == 4
        more = _pattern(4 * PAGE, 3)
        xa.xtensor_upload(base + 5 * PAGE, more)
        back = np.empty(9 * PAGE // 2, dtype=np.uint16)
        xa.xtensor_download(back, base)                        # growth left the old pages in place
        np.testing.assert_array_equal(back, np.concatenate([data, more]))
        xa.xtensor_close(rng, True)
        assert xa.xtensor_pool_counts(pool) == (15, 0, 0, 9)
        b2, r2, reused2 = xa.xtensor_open(pool, 2, 16 * PAGE, 9 * PAGE)
        assert reused2 and b2 == base
        xa.xtensor_download(back, b2)                          # same physical pages, still mapped
        np.testing.assert_array_equal(back, np.concatenate([data, more]))
        xa.xtensor_premap_async(r2, 12 * PAGE)
        xa.xtensor_premap_wait(r2)
        tail = _pattern(3 * PAGE, 4)
        xa.xtensor_upload(b2 + 9 * PAGE, tail)
        got = np.empty_like(tail)
        xa.xtensor_download(got, b2 + 9 * PAGE)
        np.testing.assert_array_equal(got, tail)
        xa.xtensor_close(r2, False)
        assert xa.xtensor_pool_counts(pool) == (24, 0, 0, 0)
    finally:
        xa.xtensor_pool_destroy(pool)


@pytest.mark.parametrize("T,Hkv", [(1, 8), (4, 8), (3, 2), (1, 1)])
def test_write_kvcache_matches_oracle_bit_for_bit(T, Hkv):
    import torch

    import paper_2510_14686_amd as xa
    lens = [T, 17, 1024, 1025, 300]
    B = len(lens)
    cap = [L + 5 for L in lens]
    ks = [normal_bf16(70, 1 + 2 * b, cap[b] * Hkv * D).reshape(cap[b], Hkv, D) for b in range(B)]
    vs = [normal_bf16(70, 2 + 2 * b, cap[b] * Hkv * D).reshape(cap[b], Hkv, D) for b in range(B)]
    k_new = normal_bf16(70, 100, B * T * Hkv * D).reshape(B, T, Hkv, D)
    v_new = normal_bf16(70, 101, B * T * Hkv * D).reshape(B, T, Hkv, D)
    with xa.KVStore(ks, vs, xtensor=True, seed=9) as store:
        kn = torch.from_numpy(k_new.view(np.int16)).cuda()
        vn = torch.from_numpy(v_new.view(np.int16)).cuda()
        lens_d = torch.tensor(lens, dtype=torch.int32, device="cuda")
        xa.xattn_write_kvcache(kn, vn, store.k_ptrs, store.v_ptrs, lens_d, B, T, Hkv, D, torch.cuda.current_stream())
        torch.cuda.synchronize()
        oracle.write_kvcache(k_new, v_new, ks, vs, lens)
        for b in range(B):
            got_k, got_v = np.empty_like(ks[b]), np.empty_like(vs[b])
            xa.xtensor_download(got_k, store.k_addr[b])
            xa.xtensor_download(got_v, store.v_addr[b])
            np.testing.assert_array_equal(got_k, ks[b])
            np.testing.assert_array_equal(got_v, vs[b])


def test_decode_loop_append_then_attend_on_growing_ranges():
    """The serving loop of section 4.3 in small: every step pre-maps the pages the next step needs
    while this step runs, appends the new tokens' K/V with write_kvcache at base + kv_len * row, and
    attends over [base, base + kv_len); each step's output is checked against the oracle on the host
    copy of the same bytes.  Sequences start just below a page boundary so that growth happens."""
    import torch

    import paper_2510_14686_amd as xa
    from gpu_util import assert_parity
    B, T, Hq, Hkv, steps = 3, 2, 8, 2, 6
    row = Hkv * D * 2                                          # 512 bytes per token row
    per_page = PAGE // row
    lens = [per_page - 3, 5, 2 * per_page - 1]                 # prefix lengths
    cap = [L + T * steps for L in lens]
    ks = [normal_bf16(80, 1 + 2 * b, cap[b] * Hkv * D).reshape(cap[b], Hkv, D) for b in range(B)]
    vs = [normal_bf16(80, 2 + 2 * b, cap[b] * Hkv * D).reshape(cap[b], Hkv, D) for b in range(B)]
    pool = xa.xtensor_pool_create(0, 32, 5)
    ranges = []
    try:
        k_addr, v_addr = [], []
        for b in range(B):
            for arr, addrs in ((ks[b], k_addr), (vs[b], v_addr)):
                base, rng, _ = xa.xtensor_open(pool, b, 8 * PAGE, lens[b] * row)
                ranges.append((rng, b))
                xa.xtensor_upload(base, arr[:lens[b]])        # the cached prefix
                addrs.append(base)
        kp = torch.tensor(k_addr, dtype=torch.int64, device="cuda")
        vp = torch.tensor(v_addr, dtype=torch.int64, device="cuda")
        stream = torch.cuda.current_stream()
        cur = list(lens)
        grew = 0
        for step in range(steps):
            new_len = [L + T for L in cur]
            for rng, b in ranges:                              # pages for this step's append: mapped ahead
                xa.xtensor_premap_wait(rng)
                grew += xa.xtensor_grow(rng, new_len[b] * row)
            for rng, b in ranges:                              # and the next step's, in the background
                xa.xtensor_premap_async(rng, (new_len[b] + T) * row)
            k_new = np.stack([ks[b][cur[b]:new_len[b]] for b in range(B)])
            v_new = np.stack([vs[b][cur[b]:new_len[b]] for b in range(B)])
            q = normal_bf16(81, step, B * T * Hq * D).reshape(B, T, Hq, D)
            lens_d = torch.tensor(new_len, dtype=torch.int32, device="cuda")
            kn = torch.from_numpy(np.ascontiguousarray(k_new).view(np.int16)).cuda()
            vn = torch.from_numpy(np.ascontiguousarray(v_new).view(np.int16)).cuda()
            qd = torch.from_numpy(q.view(np.int16)).cuda()
            out = torch.zeros((B, T, Hq, D), dtype=torch.int16, device="cuda")
            lse = torch.zeros((B, T, Hq), dtype=torch.float32, device="cuda")
            xa.xattn_write_kvcache(kn, vn, kp, vp, lens_d, B, T, Hkv, D, stream)
            xa.xattn_decode(qd, kp, vp, lens_d, B, T, Hq, Hkv, D, SCALE, out, lse, stream)
            torch.cuda.synchronize()
            ref_out, ref_lse = oracle.attn(q, ks, vs, new_len, SCALE)
            assert_parity(out.cpu().numpy().view(np.uint16), lse.cpu().numpy(), ref_out, ref_lse, "step %d" % step)
            cur = new_len
        assert grew + sum(1 for _ in ranges) >= 2              # at least two sequences crossed a page boundary
        for rng, _ in ranges:
            xa.xtensor_premap_wait(rng)
    finally:
        for rng, _ in ranges:
            xa.xtensor_close(rng, False)
        xa.xtensor_pool_destroy(pool)
