"""Contexts and per-call options of the C ABI: options passed with a call leave the process defaults
alone; calls on two contexts share nothing and may be in flight together; calls on one context from two
streams are ordered by the library instead of racing on its workspace.  Every result is compared with the
CPU oracle byte for byte."""
import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
CANARY = 0x5A


@pytest.fixture(scope="module")
def tuna():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_02581_amd as t
    t.load()
    return t


class Prob:
    def __init__(self, counts, seed, gap=3):
        self.lay = lay = wl.make_layout(counts.astype(np.int32), gap=gap)
        dev = "cuda:0"
        host = wl.payload_position_hash(seed, lay.send_bytes)
        self.send = torch.from_numpy(host).to(dev)
        self.meta = [torch.from_numpy(a).to(dev) for a in (lay.sendcounts, lay.sdispls, lay.recvcounts, lay.rdispls)]
        self.recv = torch.full((lay.recv_bytes,), CANARY, dtype=torch.uint8, device=dev)
        self.want = np.full(lay.recv_bytes, CANARY, dtype=np.uint8)
        assert oracle.alltoallv(host, lay.sendcounts, lay.sdispls, self.want, lay.recvcounts, lay.rdispls) == 0

    def call(self, tuna, ctx, Q, rl, rg, opts=None, stream=None):
        sc, sd, rc_, rd = self.meta
        return tuna.tuna_alltoallv_ex(ctx, self.send, sc, sd, self.recv, rc_, rd, self.lay.P, Q, rl, rg, opts, stream)

    def ok(self):
        return np.array_equal(self.recv.cpu().numpy(), self.want)


def test_options_travel_with_the_call(tuna):
    prob = Prob(wl.counts_uniform_bytes(40, 3, 700), 1)
    before = tuna.tuna_opts_init()
    assert before.mode == tuna.TUNA_MODE_AUTO and before.t_layout == tuna.TUNA_T_AUTO
    for mode, want_fused in ((tuna.TUNA_MODE_STAGED, 0), (tuna.TUNA_MODE_FUSED, 1), (tuna.TUNA_MODE_AUTO, 1)):
        for tl in (tuna.TUNA_T_SLOTS, tuna.TUNA_T_EXACT):
            o = tuna.tuna_opts_init()
            o.mode, o.t_layout = mode, tl
            prob.recv.fill_(CANARY)
            assert prob.call(tuna, None, 0, 3, 3, o) == 0
            torch.cuda.synchronize()
            assert prob.ok(), (mode, tl)
            st = tuna.tuna_get_stats()
            assert (st.fused, st.dense_t) == (want_fused, tl)
    after = tuna.tuna_opts_init()
    assert (after.mode, after.t_layout, after.staggered, after.block_count) == (before.mode, before.t_layout, 0, 0)
    # a struct of the wrong size or with a value out of range is refused
    o = tuna.tuna_opts_init()
    o.struct_size = 8
    assert prob.call(tuna, None, 0, 3, 3, o) == tuna.TUNA_ERR_ARG
    o = tuna.tuna_opts_init()
    o.mode = 7
    assert prob.call(tuna, None, 0, 3, 3, o) == tuna.TUNA_ERR_ARG


def test_radix_left_to_the_library(tuna):
    prob = Prob(wl.counts_uniform_bytes(24, 5, 300), 2)
    assert prob.call(tuna, None, 4, tuna.TUNA_RADIX_AUTO, tuna.TUNA_RADIX_AUTO) == 0
    torch.cuda.synchronize()
    assert prob.ok()
    st = tuna.tuna_get_stats()
    assert (st.local_radix, st.global_radix, st.n_phases) == (4, 6, 2)      # the linear schedule in both dimensions
    sc, sd, rc_, rd = prob.meta
    prob.recv.fill_(CANARY)
    assert tuna.tuna_alltoallv(prob.send, sc, sd, prob.recv, rc_, rd, 24, tuna.TUNA_RADIX_AUTO, 0) == 0
    torch.cuda.synchronize()
    assert prob.ok() and tuna.tuna_get_stats().local_radix == 24
    assert tuna.tuna_alltoallv(prob.send, sc, sd, prob.recv, rc_, rd, 24, 1, 0) == tuna.TUNA_ERR_ARG
    assert tuna.tuna_alltoallv(prob.send, sc, sd, prob.recv, rc_, rd, 24, -2, 0) == tuna.TUNA_ERR_ARG


def test_two_contexts_two_streams_in_flight_together(tuna):
    a = Prob(wl.counts_uniform_bytes(96, 7, 4000), 3)
    b = Prob(wl.counts_uniform_elements(64, 8, 500, 4), 4)
    rc, c1 = tuna.tuna_ctx_create()
    assert rc == 0 and c1
    rc, c2 = tuna.tuna_ctx_create()
    assert rc == 0 and c2 and c2 != c1
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    try:
        for it in range(4):
            a.recv.fill_(CANARY); b.recv.fill_(CANARY)
            torch.cuda.synchronize()
            print("two contexts, iteration", it, flush=True)
            assert a.call(tuna, c1, 0, 2, 2, None, s1) == 0
            assert b.call(tuna, c2, 8, 2, 8, None, s2) == 0
            torch.cuda.synchronize()
            assert a.ok() and b.ok(), it
        sa, sb = tuna.tuna_ctx_get_stats(c1), tuna.tuna_ctx_get_stats(c2)
        assert (sa.P, sb.P) == (96, 64) and sa.total_payload_bytes == a.lay.payload_bytes
        assert sb.total_payload_bytes == b.lay.payload_bytes
    finally:
        assert tuna.tuna_ctx_destroy(c1) == 0
        assert tuna.tuna_ctx_destroy(c2) == 0


def test_one_context_two_streams_are_ordered(tuna):
    """Two immediate calls on the default context from two streams, no host synchronisation between them:
    the second waits for the first (they share a workspace) and both results are right."""
    a = Prob(wl.counts_uniform_bytes(128, 9, 6000), 5)
    b = Prob(wl.counts_uniform_bytes(50, 10, 900), 6)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for it in range(4):
        a.recv.fill_(CANARY); b.recv.fill_(CANARY)
        torch.cuda.synchronize()
        assert a.call(tuna, None, 0, 2, 2, None, s1) == 0
        assert b.call(tuna, None, 0, 5, 5, None, s2) == 0
        assert a.call(tuna, None, 0, 128, 128, None, s1) == 0
        torch.cuda.synchronize()
        assert a.ok() and b.ok(), it


def test_large_calls_with_metadata_on_a_second_stream(tuna):
    """Calls of 64 MiB and more with several one-kernel phases compute every phase's metadata on a stream of
    the context's own while the caller's stream moves the payload.  Two such problems back to back on two
    streams of one context, with a small call between them, with no host synchronisation in between; then the
    same call profiled (which keeps to one stream), on a context of its own, and on a caller-owned workspace
    of the size the sizing query names."""
    big = Prob(wl.counts_normal(320, 21, 1024.0, 256.0, 4), 8, gap=0)          # 100 MiB, the tiled hop
    zipf = Prob(wl.counts_zipf(384, 22, 1.2, 16384, 4), 9)                    # 120 MiB, gaps: the copy engine's hop
    small = Prob(wl.counts_uniform_bytes(50, 10, 900), 6)
    assert big.lay.payload_bytes > (64 << 20) and zipf.lay.payload_bytes > (64 << 20)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for it, (r1, r2) in enumerate([(2, 4), (8, 20), (18, 2)]):
        for p in (big, zipf, small):
            p.recv.fill_(CANARY)
        torch.cuda.synchronize()
        print("pipelined calls, iteration", it, flush=True)
        assert big.call(tuna, None, 0, r1, r1, None, s1) == 0
        assert zipf.call(tuna, None, 16, 4, r2, None, s2) == 0
        assert small.call(tuna, None, 0, 5, 5, None, s1) == 0
        assert big.call(tuna, None, 0, r2, r2, None, s2) == 0
        torch.cuda.synchronize()
        assert big.ok() and zipf.ok() and small.ok(), it
        st = tuna.tuna_get_stats()
        assert st.n_phases >= 2 and sum(st.phase[x].payload_bytes for x in range(st.n_phases)) >= big.lay.payload_bytes
    o = tuna.tuna_opts_init()
    o.profile = 1
    big.recv.fill_(CANARY)
    assert big.call(tuna, None, 0, 4, 4, o) == 0
    torch.cuda.synchronize()
    st = tuna.tuna_get_stats()
    assert big.ok() and all(st.phase[x].ms_metadata > 0 and st.phase[x].ms_unpack > 0 for x in range(st.n_phases))
    rc, ctx = tuna.tuna_ctx_create()
    assert rc == 0
    try:
        for r in (3, 7):
            zipf.recv.fill_(CANARY)
            assert zipf.call(tuna, ctx, 16, r, r, None, s1) == 0
            torch.cuda.synchronize()
            assert zipf.ok(), r
    finally:
        assert tuna.tuna_ctx_destroy(ctx) == 0
    rc, need = tuna.tuna_workspace_bytes(big.meta[0], big.lay.P, 0, 4, 4)
    assert rc == 0 and need > 0
    ws = torch.empty(need + 256, dtype=torch.uint8, device="cuda:0")
    base = (ws.data_ptr() + 255) // 256 * 256
    assert tuna.tuna_set_workspace(base, need) == 0
    try:
        big.recv.fill_(CANARY)
        assert big.call(tuna, None, 0, 4, 4) == 0
        torch.cuda.synchronize()
        assert big.ok() and tuna.tuna_get_stats().workspace_bytes <= need
    finally:
        assert tuna.tuna_set_workspace(None, 0) == 0


def test_plan_with_options_and_context(tuna):
    prob = Prob(wl.counts_uniform_bytes(48, 11, 2000), 7)
    rc, ctx = tuna.tuna_ctx_create()
    assert rc == 0
    o = tuna.tuna_opts_init()
    o.mode, o.t_layout = tuna.TUNA_MODE_STAGED, tuna.TUNA_T_SLOTS
    sc, sd, rc_, rd = prob.meta
    code, plan = tuna.tuna_alltoallv_init_ex(ctx, prob.send, sc, sd, prob.recv, rc_, rd, 48, 0, 4, 4, o)
    assert code == 0 and plan
    try:
        for _ in range(2):
            prob.recv.fill_(CANARY)
            assert tuna.tuna_start(plan) == 0
            torch.cuda.synchronize()
            assert prob.ok()
        st = tuna.tuna_ctx_get_stats(ctx)
        assert (st.fused, st.dense_t, st.P) == (0, 0, 48)
    finally:
        assert tuna.tuna_plan_free(plan) == 0
        assert tuna.tuna_ctx_destroy(ctx) == 0
    assert len(tuna.tuna_build_id()) == 16
