"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (dense layout, library-owned workspace, default stream).

Configurations 3 and 5 (about 1 GiB) are compared whole against the CPU oracle.  Configuration 4
(16 GiB) is checked three ways: (a) the complete receive regions of a sample of receiver ranks
against the oracle (which gets the send buffer downloaded from the GPU); (b) every 4-byte word of
the receive buffer against the value the payload generator gives for the send offset the
definition names -- the payload is a hash of its own position, so the expected words are
regenerated instead of stored; (c) conservation of the word sum.
"""
import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def tuna():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_02581_amd as t
    t.load()
    return t


def _upload(lay):
    dev = "cuda:0"
    return [torch.from_numpy(a).to(dev) for a in (lay.sendcounts, lay.sdispls, lay.recvcounts, lay.rdispls)]


def _modes(tuna):
    """Three-stage phases, fused rounds, and (for hierarchical calls) the staggered schedule."""
    yield "staged", lambda: None
    yield "fused", lambda: tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 1)
    yield "staggered", lambda: tuna.tuna_set_option(tuna.TUNA_OPT_STAGGERED, 1)


def _reset_modes(tuna):
    tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 2)
    tuna.tuna_set_option(tuna.TUNA_OPT_STAGGERED, 0)


def _whole_oracle_case(tuna, cfg_id, calls):
    c = wl.CONFIGS[cfg_id]
    lay = wl.make_layout(wl.make_counts(cfg_id))
    send_host = wl.float32_bit_patterns(lay.send_bytes, c.seed) if cfg_id == 3 else \
        wl.payload_position_hash(c.seed, lay.send_bytes)
    want = np.zeros(lay.recv_bytes, dtype=np.uint8)
    assert oracle.alltoallv(send_host, lay.sendcounts, lay.sdispls, want, lay.recvcounts, lay.rdispls) == 0
    want_dev = torch.from_numpy(want).to("cuda:0")
    send = torch.from_numpy(send_host).to("cuda:0")
    recv = torch.empty(lay.recv_bytes, dtype=torch.uint8, device="cuda:0")
    sc, sd, rc, rd = _upload(lay)
    try:
        for mode, enable in _modes(tuna):
            enable()
            for label, fn in calls(lay.P):
                recv.zero_()
                print("config %d full size, %s, %s" % (cfg_id, mode, label), flush=True)
                code = fn(send, sc, sd, recv, rc, rd)
                assert code == 0, tuna.tuna_strerror(code)
                torch.cuda.synchronize()
                assert torch.equal(recv, want_dev), "config %d %s %s differs from the oracle" % (cfg_id, mode, label)
            _reset_modes(tuna)
    finally:
        _reset_modes(tuna)
    assert torch.equal(send, torch.from_numpy(send_host).to("cuda:0"))


def test_config3_full_hierarchical(tuna):
    c = wl.CONFIGS[3]

    def calls(P):
        for rg in c.global_radices:
            yield ("r_l=%d r_g=%d" % (c.local_radix, rg),
                   lambda s, sc, sd, r, rc, rd, rg=rg: tuna.tuna_alltoallv_hier(
                       s, sc, sd, r, rc, rd, P, c.ranks_per_node, c.local_radix, rg))
    _whole_oracle_case(tuna, 3, calls)
    st = tuna.tuna_get_stats()
    assert (st.Q, st.N, st.K_local, st.K_global) == (16, 64, 6, 16 * 63)     # the last mode run is the staggered one


def test_config3_caller_workspace_and_phase_times(tuna):
    """A profiled call of this size is made in two passes (all metadata, a second read-back, then the payload
    kernels with exact grids).  Here it runs in a caller-owned workspace of tuna_workspace_bytes bytes,
    with per-kernel timing on: same bytes as the oracle, every stage of every phase timed, and the
    workspace it reports fits the one that was asked for."""
    c = wl.CONFIGS[3]
    P = c.P
    lay = wl.make_layout(wl.make_counts(3))
    send_host = wl.float32_bit_patterns(lay.send_bytes, c.seed)
    want = np.zeros(lay.recv_bytes, dtype=np.uint8)
    assert oracle.alltoallv(send_host, lay.sendcounts, lay.sdispls, want, lay.recvcounts, lay.rdispls) == 0
    want_dev = torch.from_numpy(want).to("cuda:0")
    send = torch.from_numpy(send_host).to("cuda:0")
    recv = torch.empty(lay.recv_bytes, dtype=torch.uint8, device="cuda:0")
    sc, sd, rc, rd = _upload(lay)
    for fused in (0, 1):
        tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, fused)
        code, need = tuna.tuna_workspace_bytes(sc, P, c.ranks_per_node, c.local_radix, 8)
        assert code == 0 and need > 0
        ws = torch.empty(need + 256, dtype=torch.uint8, device="cuda:0")
        base = (ws.data_ptr() + 255) // 256 * 256
        assert tuna.tuna_set_workspace(base, need) == 0
        tuna.tuna_set_option(tuna.TUNA_OPT_PROFILE, 1)
        try:
            recv.zero_()
            print("config 3, caller workspace of %d bytes, fused=%d" % (need, fused), flush=True)
            code = tuna.tuna_alltoallv_hier(send, sc, sd, recv, rc, rd, P, c.ranks_per_node, c.local_radix, 8)
            assert code == 0, tuna.tuna_strerror(code)
            st = tuna.tuna_get_stats()
            torch.cuda.synchronize()
            assert torch.equal(recv, want_dev)
            assert 0 < st.workspace_bytes <= need
            assert st.n_phases == 4 and st.ms_total > 0
            for x in range(st.n_phases):
                ph = st.phase[x]
                # one-kernel phases report one payload kernel: the copy engine's hop as pack time, the
                # destination-tiled hop as unpack time
                assert ph.ms_metadata > 0 and (ph.ms_pack > 0 or (fused and ph.ms_unpack > 0))
                assert (ph.ms_exchange > 0 and ph.ms_unpack > 0) or fused
            # the same exchange as a persistent plan (its staging is sized by the largest phase)
            tuna.tuna_set_option(tuna.TUNA_OPT_PROFILE, 0)
            assert tuna.tuna_set_workspace(None, 0) == 0
            code, plan = tuna.tuna_alltoallv_init(send, sc, sd, recv, rc, rd, P, c.ranks_per_node, c.local_radix, 2)
            assert code == 0, tuna.tuna_strerror(code)
            recv.zero_()
            assert tuna.tuna_start(plan) == 0
            torch.cuda.synchronize()
            assert torch.equal(recv, want_dev), "persistent plan, fused=%d" % fused
            assert tuna.tuna_plan_free(plan) == 0
            # a workspace that is too small is refused before anything moves
            assert tuna.tuna_set_workspace(base, need // 8) == 0
            recv.zero_()
            code = tuna.tuna_alltoallv_hier(send, sc, sd, recv, rc, rd, P, c.ranks_per_node, c.local_radix, 8)
            assert code == tuna.TUNA_ERR_WORKSPACE_TOO_SMALL
            torch.cuda.synchronize()
            assert int(recv.count_nonzero()) == 0
        finally:
            tuna.tuna_set_option(tuna.TUNA_OPT_PROFILE, 0)
            tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 2)
            tuna.tuna_set_workspace(None, 0)
        del ws


def test_config5_full_uniform(tuna):
    c = wl.CONFIGS[5]

    def calls(P):
        for r in c.radices:
            yield ("radix=%d" % r, lambda s, sc, sd, rcv, rc, rd, r=r: tuna.tuna_alltoallv(
                s, sc, sd, rcv, rc, rd, P, r, c.ranks_per_node))
    _whole_oracle_case(tuna, 5, calls)
    st = tuna.tuna_get_stats()
    assert (st.local_radix, st.global_radix, st.K_local, st.K_global) == (32, 64, 31, 32 * 63)


def test_config4_full(tuna):
    c = wl.CONFIGS[4]
    P = c.P
    dev = "cuda:0"
    lay = wl.make_layout(wl.make_counts(4))
    assert lay.payload_bytes > 15.9 * 2**30
    send = wl.payload_position_hash_torch(c.seed, lay.send_bytes, dev)
    recv = torch.empty(lay.recv_bytes, dtype=torch.uint8, device=dev)
    sc, sd, rc, rd = _upload(lay)
    # (a) oracle on sampled receivers, from the send buffer as the GPU holds it
    send_host = send.cpu().numpy()
    assert np.array_equal(send_host[:4096], wl.payload_position_hash(c.seed, 4096))
    rng = np.random.default_rng(4)
    receivers = np.unique(np.concatenate([[0, 1, P // 2, P - 1], rng.integers(0, P, 28)])).astype(np.int32)
    want = np.zeros(lay.recv_bytes, dtype=np.uint8)          # untouched pages are never committed
    assert oracle.alltoallv_receivers(send_host, lay.sendcounts, lay.sdispls, want, lay.recvcounts,
                                      lay.rdispls, receivers) == 0
    del send_host
    regions = [(int(lay.rdispls[j, 0]), int(lay.rdispls[j, P - 1] + lay.recvcounts[j, P - 1])) for j in receivers]
    want_regions = [torch.from_numpy(want[lo:hi].copy()).to(dev) for lo, hi in regions]
    del want
    send_sum = int(send.view(torch.int32).sum(dtype=torch.int64))
    counts_w = (sc.to(torch.int64) // 4)                      # [i, j] words of block i -> j
    sd_w = sd // 4
    # (radix, fused rounds, persistent plan, T in slots of M bytes instead of exact size, rounds per batch)
    cases = [(r, 0, 0, 0, 0) for r in c.radices] + [(2, 1, 0, 0, 0), (4096, 1, 0, 0, 0), (2, 0, 0, 1, 0), (8, 1, 0, 1, 0),
                                                     (2, 0, 1, 0, 0), (8, 1, 1, 0, 0), (4096, 0, 0, 0, 300), (64, 1, 1, 0, 5)]
    for r, fused, persistent, slots, batch in cases:
        recv.zero_()
        print("config 4 full size, radix=%d fused=%d persistent=%d slots-of-M=%d block_count=%d" %
              (r, fused, persistent, slots, batch), flush=True)
        tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, fused)
        tuna.tuna_set_option(tuna.TUNA_OPT_BLOCK_COUNT, batch)
        tuna.tuna_set_option(tuna.TUNA_OPT_DENSE_T, 0 if slots else 1)
        if persistent:
            assert tuna.tuna_release() == 0                # the immediate calls' workspace is not needed here
            code, plan = tuna.tuna_alltoallv_init(send, sc, sd, recv, rc, rd, P, 0, r, r)
            assert code == 0, tuna.tuna_strerror(code)
            code = tuna.tuna_start(plan)
            torch.cuda.synchronize()
            assert tuna.tuna_plan_free(plan) == 0
        else:
            code = tuna.tuna_alltoallv(send, sc, sd, recv, rc, rd, P, r, 0)
        tuna.tuna_set_option(tuna.TUNA_OPT_DENSE_T, 2)
        tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 2)
        tuna.tuna_set_option(tuna.TUNA_OPT_BLOCK_COUNT, 0)
        assert code == 0, tuna.tuna_strerror(code)
        assert tuna.tuna_get_stats().dense_t == (0 if slots else 1)
        torch.cuda.synchronize()
        for (lo, hi), w in zip(regions, want_regions):
            assert torch.equal(recv[lo:hi], w), "radix %d: receiver region [%d, %d) differs from the oracle" % (r, lo, hi)
        # (c) conservation
        assert int(recv.view(torch.int32).sum(dtype=torch.int64)) == send_sum
        # (b) every received word equals the generator's value at the send offset the definition names
        recv_w = recv.view(torch.int32)
        step = 128
        for j0 in range(0, P, step):
            j1 = min(P, j0 + step)
            n = counts_w[:, j0:j1].t().contiguous().view(-1)          # receiver-major: (j, i)
            src0 = sd_w[:, j0:j1].t().contiguous().view(-1)
            total = int(n.sum())
            starts = torch.cumsum(n, 0) - n
            seg = torch.repeat_interleave(torch.arange(n.numel(), device=dev), n, output_size=total)
            src_word = src0[seg] + (torch.arange(total, device=dev) - starts[seg])
            expect = wl.payload_position_hash_words32_torch(c.seed, src_word)
            lo = int(lay.rdispls[j0, 0]) // 4
            got = recv_w[lo:lo + total].to(torch.int64) & 0xFFFFFFFF
            assert torch.equal(got, expect), "radix %d: receivers %d..%d differ" % (r, j0, j1)
            del seg, src_word, expect, got


def test_one_block_of_a_gibibyte(tuna):
    """Maximum block sizes: P = 2 with one block of 1 GiB + 20 bytes (67 million chunks in one
    segment, many wave units per segment) next to a 3-byte block."""
    counts = np.array([[5, (1 << 30) + 20], [3, 0]], dtype=np.int32)
    lay = wl.make_layout(counts, gap=9)
    send = wl.payload_position_hash_torch(321, lay.send_bytes, "cuda:0")
    send_host = send.cpu().numpy()
    want = np.full(lay.recv_bytes, 0x3C, dtype=np.uint8)
    assert oracle.alltoallv(send_host, lay.sendcounts, lay.sdispls, want, lay.recvcounts, lay.rdispls) == 0
    want_dev = torch.from_numpy(want).to("cuda:0")
    sc, sd, rc, rd = _upload(lay)
    recv = torch.empty(lay.recv_bytes, dtype=torch.uint8, device="cuda:0")
    for fused in (0, 1):
        recv.fill_(0x3C)
        tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, fused)
        code = tuna.tuna_alltoallv(send, sc, sd, recv, rc, rd, 2, 2, 0)
        tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 2)
        assert code == 0, tuna.tuna_strerror(code)
        torch.cuda.synchronize()
        assert torch.equal(recv, want_dev)
    assert tuna.tuna_get_stats().max_block_bytes == (1 << 30) + 20


def test_own_blocks_of_64_mebibytes(tuna):
    """P = 64 with about 64 MiB (byte-granular) kept by every rank for itself, 4 GiB on the diagonal,
    small blocks elsewhere: the own blocks are spread over the whole device by the copy engine.  Whole
    result against the oracle, three-stage and one-kernel phases; the own-block copy must not be the
    slow part (it moves 4 GiB: well under 10 ms at HBM speed, seconds if one workgroup per rank did it)."""
    P = 64
    counts = wl.counts_uniform_bytes(P, 64, 2000)
    rng = np.random.default_rng(64)
    for p in range(P):
        counts[p, p] = (64 << 20) + int(rng.integers(-100000, 100000))
    lay = wl.make_layout(counts, gap=5)
    send = wl.payload_position_hash_torch(640, lay.send_bytes, "cuda:0")
    send_host = send.cpu().numpy()
    want = np.full(lay.recv_bytes, 0x3C, dtype=np.uint8)
    assert oracle.alltoallv(send_host, lay.sendcounts, lay.sdispls, want, lay.recvcounts, lay.rdispls) == 0
    want_dev = torch.from_numpy(want).to("cuda:0")
    del want, send_host
    sc, sd, rc, rd = _upload(lay)
    recv = torch.empty(lay.recv_bytes, dtype=torch.uint8, device="cuda:0")
    for fused in (0, 1):
        recv.fill_(0x3C)
        tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, fused)
        tuna.tuna_set_option(tuna.TUNA_OPT_PROFILE, 1)
        try:
            print("own blocks of 64 MiB, fused=%d" % fused, flush=True)
            code = tuna.tuna_alltoallv(send, sc, sd, recv, rc, rd, P, 8, 0)
            st = tuna.tuna_get_stats()
        finally:
            tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 2)
            tuna.tuna_set_option(tuna.TUNA_OPT_PROFILE, 0)
        assert code == 0, tuna.tuna_strerror(code)
        torch.cuda.synchronize()
        assert torch.equal(recv, want_dev)
        diag = int(np.trace(counts.astype(np.int64)))
        print("own-block copy: %.3f ms, %.0f GB/s read + write" % (st.ms_self, 2 * diag / (st.ms_self * 1e-3) / 1e9), flush=True)
        assert st.ms_self < 10.0


def test_byte_granular_two_pass_all_modes(tuna):
    """P = 512, byte-granular sizes 0..2047 (any alignment), 256 MiB of payload, radix 8 (three digit phases):
    large enough for the two-pass form of an immediate call (three stages) and for its pipelined form
    (one-kernel phases), in all four modes (three stages / one-kernel phases x T in slots / in exact size);
    whole receive buffer against the oracle."""
    P = 512
    counts = wl.counts_uniform_bytes(P, 512, 2047)
    lay = wl.make_layout(counts, gap=3)
    assert lay.payload_bytes > 250 << 20
    send_host = wl.payload_position_hash(5120, lay.send_bytes)
    want = np.full(lay.recv_bytes, 0x3C, dtype=np.uint8)
    assert oracle.alltoallv(send_host, lay.sendcounts, lay.sdispls, want, lay.recvcounts, lay.rdispls) == 0
    want_dev = torch.from_numpy(want).to("cuda:0")
    send = torch.from_numpy(send_host).to("cuda:0")
    sc, sd, rc, rd = _upload(lay)
    recv = torch.empty(lay.recv_bytes, dtype=torch.uint8, device="cuda:0")
    for mode in (tuna.TUNA_MODE_STAGED, tuna.TUNA_MODE_FUSED):
        for tl in (tuna.TUNA_T_SLOTS, tuna.TUNA_T_EXACT):
            o = tuna.tuna_opts_init()
            o.mode, o.t_layout = mode, tl
            recv.fill_(0x3C)
            print("byte-granular two-pass: mode %d, T layout %d" % (mode, tl), flush=True)
            code = tuna.tuna_alltoallv_ex(None, send, sc, sd, recv, rc, rd, P, 0, 8, 8, o)
            assert code == 0, tuna.tuna_strerror(code)
            torch.cuda.synchronize()
            assert torch.equal(recv, want_dev), (mode, tl)
            st = tuna.tuna_get_stats()
            assert (st.granularity, st.n_phases, st.dense_t) == (1, 3, tl)


def test_counts_beyond_the_supported_range(tuna):
    """Counts only, no payload: problems whose per-rank chunk prefix would not fit 32 bits, or whose largest
    block leaves no room for rounding in 32-bit arithmetic, are refused with TUNA_ERR_TOO_LARGE by the
    sizing query and by the call itself (before anything moves)."""
    P = 4096
    sc = torch.zeros((P, P), dtype=torch.int32, device="cuda:0")
    sc[7, :] = 16 << 20            # one rank sends 4096 blocks of 16 MiB: 2^32 chunks, and P * (M / 16) = 2^32 too
    rc, nbytes = tuna.tuna_workspace_bytes(sc, P, 0, 2, 2)
    assert rc == tuna.TUNA_ERR_TOO_LARGE, tuna.tuna_strerror(rc)
    sc[7, :] = 1 << 20             # the same shape sixteen times smaller is fine
    rc, nbytes = tuna.tuna_workspace_bytes(sc, P, 0, 2, 2)
    assert rc == 0 and nbytes > 0
    P = 4
    sc = torch.zeros((P, P), dtype=torch.int32, device="cuda:0")
    sc[1, 2] = 2**31 - 100
    rc, nbytes = tuna.tuna_workspace_bytes(sc, P, 0, 2, 2)
    assert rc == tuna.TUNA_ERR_TOO_LARGE
    sd = torch.zeros((P, P), dtype=torch.int64, device="cuda:0")
    buf = torch.zeros(64, dtype=torch.uint8, device="cuda:0")
    rc = tuna.tuna_alltoallv(buf, sc, sd, buf, sc.t().contiguous(), sd, P, 2, 0)
    assert rc == tuna.TUNA_ERR_TOO_LARGE


def test_many_ranks_small_blocks(tuna):
    """P = 8192 (67 million blocks of 0..60 bytes, 4-byte granular): flat with radix 2 (13 digit
    phases) and radix P, and 64 ranks per node x 128 nodes; whole result against the oracle."""
    P = 8192
    counts = wl.counts_uniform_elements(P, 8192, 15, 4)
    lay = wl.make_layout(counts)
    send_host = wl.payload_position_hash(8192, lay.send_bytes)
    want = np.zeros(lay.recv_bytes, dtype=np.uint8)
    assert oracle.alltoallv(send_host, lay.sendcounts, lay.sdispls, want, lay.recvcounts, lay.rdispls) == 0
    want_dev = torch.from_numpy(want).to("cuda:0")
    del want
    send = torch.from_numpy(send_host).to("cuda:0")
    sc, sd, rc, rd = _upload(lay)
    recv = torch.empty(lay.recv_bytes, dtype=torch.uint8, device="cuda:0")
    for radix, rpn in ((2, 0), (P, 0), (8, 64)):
        recv.zero_()
        print("P=8192 radix=%d ranks_per_node=%d" % (radix, rpn), flush=True)
        code = tuna.tuna_alltoallv(send, sc, sd, recv, rc, rd, P, radix, rpn)
        assert code == 0, tuna.tuna_strerror(code)
        torch.cuda.synchronize()
        assert torch.equal(recv, want_dev), (radix, rpn)
    st = tuna.tuna_get_stats()
    assert (st.Q, st.N, st.w_local, st.w_global) == (64, 128, 2, 3)


def test_sixteen_thousand_ranks(tuna):
    """P = 16384 (268 million blocks of 0..28 bytes): table rows, T positions and prefix rows are
    indexed beyond 2^32 entries.  Flat radix 2 (14 digit phases, T in exact size) and radix 128 with
    one-kernel phases; whole result against the oracle."""
    P = 16384
    print("P=16384: counts", flush=True)
    counts = wl.counts_uniform_elements(P, 16384, 7, 4)
    print("P=16384: layout", flush=True)
    lay = wl.make_layout(counts)
    send_host = wl.payload_position_hash(16384, lay.send_bytes)
    want = np.zeros(lay.recv_bytes, dtype=np.uint8)
    print("P=16384: oracle", flush=True)
    assert oracle.alltoallv(send_host, lay.sendcounts, lay.sdispls, want, lay.recvcounts, lay.rdispls) == 0
    want_dev = torch.from_numpy(want).to("cuda:0")
    del want
    send = torch.from_numpy(send_host).to("cuda:0")
    sc, sd, rc, rd = _upload(lay)
    recv = torch.empty(lay.recv_bytes, dtype=torch.uint8, device="cuda:0")
    assert tuna.tuna_release() == 0
    for radix, fused in ((2, 0), (128, 1)):
        recv.zero_()
        print("P=16384 radix=%d fused=%d" % (radix, fused), flush=True)
        tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, fused)
        code = tuna.tuna_alltoallv(send, sc, sd, recv, rc, rd, P, radix, 0)
        tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 2)
        assert code == 0, tuna.tuna_strerror(code)
        torch.cuda.synchronize()
        assert torch.equal(recv, want_dev), (radix, fused)
    st = tuna.tuna_get_stats()
    assert (st.P, st.w_local, st.dense_t) == (P, 2, 1)
    assert tuna.tuna_release() == 0
