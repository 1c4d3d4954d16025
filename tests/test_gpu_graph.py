"""xattn_decode and write_kvcache recorded into a HIP graph and replayed with other lengths and data
(section 4.2: shapes reach custom operators as device-side arguments, so a recorded launch stays
valid when they change).  Every replay is checked against the oracle and against an eager call, with
eager work and synchronisations between the replays."""
import math

import numpy as np
import pytest

import oracle
from workloads import normal_bf16

pytestmark = pytest.mark.gpu

D = 128
SCALE = float(np.float32(1.0 / math.sqrt(D)))


def test_graph_replay_with_changing_lengths_and_data():
    import torch

    import paper_2510_14686_amd as xa
    from gpu_util import assert_parity
    B, T, Hq, Hkv = 6, 2, 16, 4
    cap = 6000
    rounds = 5
    ks = [normal_bf16(90, 1 + 2 * b, cap * Hkv * D).reshape(cap, Hkv, D) for b in range(B)]
    vs = [normal_bf16(90, 2 + 2 * b, cap * Hkv * D).reshape(cap, Hkv, D) for b in range(B)]
    with xa.KVStore(ks, vs, xtensor=True, seed=3) as store:
        qd = torch.zeros((B, T, Hq, D), dtype=torch.int16, device="cuda")
        kn = torch.zeros((B, T, Hkv, D), dtype=torch.int16, device="cuda")
        vn = torch.zeros((B, T, Hkv, D), dtype=torch.int16, device="cuda")
        lens_d = torch.full((B,), 100, dtype=torch.int32, device="cuda")
        out = torch.zeros((B, T, Hq, D), dtype=torch.int16, device="cuda")
        lse = torch.zeros((B, T, Hq), dtype=torch.float32, device="cuda")
        out_e, lse_e = torch.zeros_like(out), torch.zeros_like(lse)
        side = torch.cuda.Stream()
        # one eager call of the shape sizes the library's workspace; a capture cannot grow it
        with torch.cuda.stream(side):
            xa.xattn_decode(qd, store.k_ptrs, store.v_ptrs, lens_d, B, T, Hq, Hkv, D, SCALE, out, lse, side)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            xa.xattn_write_kvcache(kn, vn, store.k_ptrs, store.v_ptrs, lens_d, B, T, Hkv, D, side)
            xa.xattn_decode(qd, store.k_ptrs, store.v_ptrs, lens_d, B, T, Hq, Hkv, D, SCALE, out, lse, side)
        rng = np.random.RandomState(5)
        for r in range(rounds):
            lens = rng.randint(T, cap - T, size=B)
            lens[r % B] = [T, 17, cap - 1, 1024, 4097][r]           # edge lengths move around
            q = normal_bf16(91, r, B * T * Hq * D).reshape(B, T, Hq, D)
            k_new = normal_bf16(92, r, B * T * Hkv * D).reshape(B, T, Hkv, D)
            v_new = normal_bf16(93, r, B * T * Hkv * D).reshape(B, T, Hkv, D)
            qd.copy_(torch.from_numpy(q.view(np.int16)))
            kn.copy_(torch.from_numpy(k_new.view(np.int16)))
            vn.copy_(torch.from_numpy(v_new.view(np.int16)))
            lens_d.copy_(torch.from_numpy(lens.astype(np.int32)))
            out.fill_(0x7FC0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            oracle.write_kvcache(k_new, v_new, ks, vs, lens)       # the host copy follows the device's appends
            ref_out, ref_lse = oracle.attn(q, ks, vs, lens, SCALE)
            got, got_lse = out.cpu().numpy().view(np.uint16), lse.cpu().numpy()
            assert_parity(got, got_lse, ref_out, ref_lse, "replay %d" % r)
            # the same call issued eagerly gives the same bits
            xa.xattn_decode(qd, store.k_ptrs, store.v_ptrs, lens_d, B, T, Hq, Hkv, D, SCALE, out_e, lse_e,
                            torch.cuda.current_stream())
            torch.cuda.synchronize()
            np.testing.assert_array_equal(out_e.cpu().numpy().view(np.uint16), got)
            np.testing.assert_array_equal(lse_e.cpu().numpy(), got_lse)
            # the appended rows are in the device ranges
            b = r % B
            row = np.empty((T, Hkv, D), dtype=np.uint16)
            xa.xtensor_download(row, store.k_addr[b] + (int(lens[b]) - T) * Hkv * D * 2)
            np.testing.assert_array_equal(row, k_new[b])


def test_capture_refuses_to_grow_the_workspace():
    """A call that would have to enlarge the library's workspace while its stream is being captured
    returns XATTN_ENOMEM and records nothing; the capture itself stays usable."""
    import torch

    import paper_2510_14686_amd as xa
    B, T, Hq, Hkv = 2, 1, 8, 2
    ks = [normal_bf16(94, 1 + 2 * b, 64 * Hkv * D).reshape(64, Hkv, D) for b in range(B)]
    with xa.KVStore(ks, ks) as store:
        qd = torch.zeros((B, T, Hq, D), dtype=torch.int16, device="cuda")
        lens_d = torch.full((B,), 64, dtype=torch.int32, device="cuda")
        out = torch.zeros((B, T, Hq, D), dtype=torch.int16, device="cuda")
        marker = torch.zeros(8, device="cuda")
        # a caller workspace that is too small stands for "the workspace would have to grow":
        # the library may not replace it, captured or not
        small = torch.zeros(4096, dtype=torch.uint8, device="cuda")
        xa.xattn_set_workspace(small, 4096)
        try:
            with pytest.raises(xa.XattnError) as e:
                xa.xattn_decode(qd, store.k_ptrs, store.v_ptrs, lens_d, B, T, Hq, Hkv, D, SCALE, out, None,
                                torch.cuda.current_stream())
            assert e.value.status == xa.binding.XATTN_ENOMEM
        finally:
            xa.xattn_set_workspace(None, 0)
        # library-owned workspace, a shape larger than any call so far (64k pieces x 1024 query rows:
        # tens of GB of partial results, far beyond what any other test leaves behind), under capture
        T2, Hq2, Hkv2 = 16, 64, 16
        ks2 = [normal_bf16(94, 10 + b, 64 * Hkv2 * D).reshape(64, Hkv2, D) for b in range(B)]
        xa.xattn_configure(xa.XATTN_CFG_PIECES, 65536)
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        status = None
        try:
            with xa.KVStore(ks2, ks2) as store2:
                qd2 = torch.zeros((B, T2, Hq2, D), dtype=torch.int16, device="cuda")
                out2 = torch.zeros((B, T2, Hq2, D), dtype=torch.int16, device="cuda")
                torch.cuda.synchronize()
                with torch.cuda.graph(graph, stream=side):
                    marker.add_(1.0)
                    try:
                        xa.xattn_decode(qd2, store2.k_ptrs, store2.v_ptrs, lens_d, B, T2, Hq2, Hkv2, D, SCALE, out2, None, side)
                    except xa.XattnError as err:
                        status = err.status
        finally:
            xa.xattn_configure(xa.XATTN_CFG_PIECES, 0)
        assert status == xa.binding.XATTN_ENOMEM
        graph.replay()
        torch.cuda.synchronize()
        assert float(marker[0]) == 1.0                             # the capture recorded the rest and replays


def test_recorded_graph_stays_valid_after_the_workspace_has_grown():
    """A graph records the address of its stream's workspace.  A later, larger eager call on the same
    stream has to replace that workspace; the buffer the graph uses is retired, not freed, so replaying
    the older graph still writes and reads live memory (compared with the oracle after other work has
    had the chance to reuse freed memory)."""
    import torch

    import paper_2510_14686_amd as xa
    from gpu_util import assert_parity
    xa.xattn_configure(xa.XATTN_CFG_PIECES, 0)
    B, T, Hq, Hkv = 4, 1, 8, 2
    lens = np.array([3000, 2000, 50, 4000], np.int32)          # split over many workgroups: partial results in the workspace
    q = normal_bf16(97, 0, B * T * Hq * D).reshape(B, T, Hq, D)
    ks = [normal_bf16(97, 1 + 2 * b, int(L) * Hkv * D).reshape(int(L), Hkv, D) for b, L in enumerate(lens)]
    vs = [normal_bf16(97, 2 + 2 * b, int(L) * Hkv * D).reshape(int(L), Hkv, D) for b, L in enumerate(lens)]
    ref_out, ref_lse = oracle.attn(q, ks, vs, lens, SCALE)
    side = torch.cuda.Stream()                                  # a fresh stream: its workspace starts empty
    with xa.KVStore(ks, vs) as store:
        qd = torch.from_numpy(q.view(np.int16)).cuda()
        lens_d = torch.from_numpy(lens).cuda()
        out = torch.zeros((B, T, Hq, D), dtype=torch.int16, device="cuda")
        lse = torch.zeros((B, T, Hq), dtype=torch.float32, device="cuda")
        xa.xattn_decode(qd, store.k_ptrs, store.v_ptrs, lens_d, B, T, Hq, Hkv, D, SCALE, out, lse, side)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            xa.xattn_decode(qd, store.k_ptrs, store.v_ptrs, lens_d, B, T, Hq, Hkv, D, SCALE, out, lse, side)
        # a larger shape on the same stream: 16 times the query rows, the workspace must be replaced
        T2, Hq2, Hkv2 = 4, 32, 8
        ks2 = [normal_bf16(98, 1 + b, 2000 * Hkv2 * D).reshape(2000, Hkv2, D) for b in range(B)]
        with xa.KVStore(ks2, ks2) as store2:
            q2 = torch.zeros((B, T2, Hq2, D), dtype=torch.int16, device="cuda")
            lens2 = torch.full((B,), 2000, dtype=torch.int32, device="cuda")
            out2 = torch.zeros((B, T2, Hq2, D), dtype=torch.int16, device="cuda")
            assert xa.xattn_workspace_bytes(B, T2, Hq2, Hkv2, D) > 2 * xa.xattn_workspace_bytes(B, T, Hq, Hkv, D)
            xa.xattn_decode(q2, store2.k_ptrs, store2.v_ptrs, lens2, B, T2, Hq2, Hkv2, D, SCALE, out2, None, side)
            side.synchronize()
        # allocations that would land in memory the library had freed
        junk = [torch.full((1 << 20,), 0x7FC07FC0, dtype=torch.int32, device="cuda") for _ in range(8)]
        torch.cuda.synchronize()
        for r in range(2):
            out.fill_(0x7FC0)
            lse.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert_parity(out.cpu().numpy().view(np.uint16), lse.cpu().numpy(), ref_out, ref_lse, "replay %d after growth" % r)
        del junk


def test_graph_replay_of_latent_kv_decode():
    """xattn_mla_decode recorded once and replayed with other lengths and data: every replay against
    the oracle and bit-identical to an eager call (eager work and synchronisations in between)."""
    import torch

    import paper_2510_14686_amd as xa
    from gpu_util import assert_parity
    B, T, H, DQK, DV = 5, 2, 128, 576, 512
    cap = 3000
    scale = float(np.float32(1.0 / math.sqrt(192.0)))
    cs = [normal_bf16(95, 1 + b, cap * DQK).reshape(cap, DQK) for b in range(B)]
    with xa.KVStore(cs, cs, xtensor=True, seed=4) as store:
        qd = torch.zeros((B, T, H, DQK), dtype=torch.int16, device="cuda")
        lens_d = torch.full((B,), 100, dtype=torch.int32, device="cuda")
        out = torch.zeros((B, T, H, DV), dtype=torch.int16, device="cuda")
        lse = torch.zeros((B, T, H), dtype=torch.float32, device="cuda")
        out_e, lse_e = torch.zeros_like(out), torch.zeros_like(lse)
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):     # sizes the workspace: a capture cannot grow it
            xa.xattn_mla_decode(qd, store.k_ptrs, lens_d, B, T, H, DV, DQK - DV, scale, out, lse, side)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            xa.xattn_mla_decode(qd, store.k_ptrs, lens_d, B, T, H, DV, DQK - DV, scale, out, lse, side)
        rng = np.random.RandomState(6)
        for r in range(4):
            lens = rng.randint(T, cap, size=B)
            lens[r % B] = [T, 33, cap, 1025][r]
            q = normal_bf16(96, r, B * T * H * DQK).reshape(B, T, H, DQK)
            qd.copy_(torch.from_numpy(q.view(np.int16)))
            lens_d.copy_(torch.from_numpy(lens.astype(np.int32)))
            out.fill_(0x7FC0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            ref_out, ref_lse = oracle.mla(q, cs, lens, DV, scale)
            got, got_lse = out.cpu().numpy().view(np.uint16), lse.cpu().numpy()
            assert_parity(got, got_lse, ref_out, ref_lse, "latent-KV replay %d" % r)
            xa.xattn_mla_decode(qd, store.k_ptrs, lens_d, B, T, H, DV, DQK - DV, scale, out_e, lse_e, torch.cuda.current_stream())
            torch.cuda.synchronize()
            np.testing.assert_array_equal(out_e.cpu().numpy().view(np.uint16), got)
            np.testing.assert_array_equal(lse_e.cpu().numpy(), got_lse)
