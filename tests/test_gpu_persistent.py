"""GPU parity of the persistent form (tuna_alltoallv_init / tuna_start / tuna_plan_free): the plan is
made once from the counts, every start moves whatever the send buffer holds at that time, and a
start can be captured into a HIP graph and replayed.  Every result is compared with the CPU oracle."""
import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")
CANARY = 0x6B


@pytest.fixture(scope="module")
def tuna():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_02581_amd as t
    t.load()
    return t


class Resident:
    def __init__(self, lay):
        dev = "cuda:0"
        self.lay = lay
        self.send = torch.zeros(lay.send_bytes, dtype=torch.uint8, device=dev)
        self.recv = torch.empty(lay.recv_bytes, dtype=torch.uint8, device=dev)
        self.sc = torch.from_numpy(lay.sendcounts).to(dev)
        self.sd = torch.from_numpy(lay.sdispls).to(dev)
        self.rc = torch.from_numpy(lay.recvcounts).to(dev)
        self.rd = torch.from_numpy(lay.rdispls).to(dev)

    def load(self, seed):
        host = wl.payload_position_hash(seed, self.lay.send_bytes)
        self.send.copy_(torch.from_numpy(host))
        want = np.full(self.lay.recv_bytes, CANARY, dtype=np.uint8)
        lay = self.lay
        assert oracle.alltoallv(host, lay.sendcounts, lay.sdispls, want, lay.recvcounts, lay.rdispls) == 0
        return want

    def check(self, want, what):
        torch.cuda.synchronize()
        got = self.recv.cpu().numpy()
        assert np.array_equal(got, want), what


@pytest.mark.parametrize("fused", [0, 1])
@pytest.mark.parametrize("P,Q,rl,rg,cfg", [(16, 0, 2, 2, 1), (96, 0, 4, 4, 2), (96, 0, 96, 96, 2),
                                            (128, 16, 4, 2, 3), (128, 16, 16, 8, 3), (1, 0, 2, 2, 2)])
def test_start_follows_the_send_buffer(tuna, P, Q, rl, rg, cfg, fused):
    lay = wl.make_layout(wl.make_counts(cfg, P), gap=4 if cfg != 2 else 5)
    res = Resident(lay)
    tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, fused)
    try:
        code, plan = tuna.tuna_alltoallv_init(res.send, res.sc, res.sd, res.recv, res.rc, res.rd, P, Q, rl, rg)
    finally:
        tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 2)
    assert code == 0, tuna.tuna_strerror(code)
    try:
        for seed in (11, 12, 13):                      # same counts, new payload every time
            want = res.load(seed)
            res.recv.fill_(CANARY)
            print("persistent P=%d Q=%d rl=%d rg=%d fused=%d seed=%d" % (P, Q, rl, rg, fused, seed), flush=True)
            assert tuna.tuna_start(plan) == 0
            res.check(want, "start %d" % seed)
        st = tuna.tuna_get_stats()
        assert st.fused == fused and st.total_payload_bytes == lay.payload_bytes
        assert sum(st.phase[x].payload_bytes for x in range(st.n_phases)) >= 0
    finally:
        assert tuna.tuna_plan_free(plan) == 0


@pytest.mark.parametrize("fused", [0, 1])
def test_plan_with_large_own_blocks(tuna, fused):
    """The own blocks of a plan are laid out once for the copy engine when blocks can exceed 64 KiB."""
    P = 10
    counts = wl.counts_uniform_bytes(P, 17, 900)
    for p in range(P):
        counts[p, p] = 200000 + 7919 * p
    lay = wl.make_layout(counts, gap=6)
    res = Resident(lay)
    tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, fused)
    try:
        code, plan = tuna.tuna_alltoallv_init(res.send, res.sc, res.sd, res.recv, res.rc, res.rd, P, 0, 3, 3)
    finally:
        tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 2)
    assert code == 0, tuna.tuna_strerror(code)
    try:
        for seed in (21, 22):
            want = res.load(seed)
            res.recv.fill_(CANARY)
            assert tuna.tuna_start(plan) == 0
            res.check(want, "start %d" % seed)
    finally:
        assert tuna.tuna_plan_free(plan) == 0


def test_staggered_plan_and_stats(tuna):
    P, Q = 60, 5
    lay = wl.make_layout(wl.counts_uniform_bytes(P, 3, 900))
    res = Resident(lay)
    tuna.tuna_set_option(tuna.TUNA_OPT_STAGGERED, 1)
    try:
        code, plan = tuna.tuna_alltoallv_init(res.send, res.sc, res.sd, res.recv, res.rc, res.rd, P, Q, 2, 2)
    finally:
        tuna.tuna_set_option(tuna.TUNA_OPT_STAGGERED, 0)
    assert code == 0
    try:
        want = res.load(5)
        res.recv.fill_(CANARY)
        assert tuna.tuna_start(plan) == 0
        res.check(want, "staggered plan")
        st = tuna.tuna_get_stats()
        assert st.K_global == Q * (P // Q - 1) and st.global_radix == P // Q
        # an immediate call in between does not disturb the plan
        res.recv.fill_(CANARY)
        assert tuna.tuna_alltoallv(res.send, res.sc, res.sd, res.recv, res.rc, res.rd, P, 3, 0) == 0
        res.check(want, "immediate call")
        want = res.load(6)
        res.recv.fill_(CANARY)
        assert tuna.tuna_start(plan) == 0
        res.check(want, "plan after an immediate call")
    finally:
        assert tuna.tuna_plan_free(plan) == 0


def test_plan_errors(tuna):
    lay = wl.make_layout(wl.counts_uniform_bytes(8, 1, 64))
    res = Resident(lay)
    bad = res.rc.clone()
    bad[1, 2] += 1
    code, plan = tuna.tuna_alltoallv_init(res.send, res.sc, res.sd, res.recv, bad, res.rd, 8, 0, 2, 2)
    assert code == tuna.TUNA_ERR_COUNT_MISMATCH and not plan
    code, plan = tuna.tuna_alltoallv_init(res.send, res.sc, res.sd, res.recv, res.rc, res.rd, 8, 3, 2, 2)
    assert code == tuna.TUNA_ERR_ARG and not plan
    assert tuna.tuna_start(None) == tuna.TUNA_ERR_ARG
    assert tuna.tuna_plan_free(None) == 0


@pytest.mark.parametrize("fused", [0, 1])
def test_start_captured_in_a_graph(tuna, fused):
    """tuna_start allocates nothing and never synchronises: captured once, replayed with the
    program's own eager work and synchronisations between the replays, every replay checked."""
    P = 64
    lay = wl.make_layout(wl.make_counts(4, P))
    res = Resident(lay)
    tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, fused)
    try:
        code, plan = tuna.tuna_alltoallv_init(res.send, res.sc, res.sd, res.recv, res.rc, res.rd, P, 0, 4, 4)
    finally:
        tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 2)
    assert code == 0
    try:
        want = res.load(1)
        res.recv.fill_(CANARY)
        assert tuna.tuna_start(plan) == 0              # eager first
        res.check(want, "eager")
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            assert tuna.tuna_start(plan) == 0          # on the capture stream
        for seed in (2, 3, 4):
            want = res.load(seed)                      # eager copies and a synchronisation in between
            res.recv.fill_(CANARY)
            torch.cuda.synchronize()
            print("graph replay fused=%d seed=%d" % (fused, seed), flush=True)
            graph.replay()
            res.check(want, "replay %d" % seed)
        del graph
    finally:
        assert tuna.tuna_plan_free(plan) == 0


def test_two_plans_on_two_streams(tuna):
    """Plans own their memory: starts of different plans may overlap on different streams."""
    lay_a = wl.make_layout(wl.make_counts(4, 96))
    lay_b = wl.make_layout(wl.make_counts(3, 64))
    a, b = Resident(lay_a), Resident(lay_b)
    code, plan_a = tuna.tuna_alltoallv_init(a.send, a.sc, a.sd, a.recv, a.rc, a.rd, 96, 0, 4, 4)
    assert code == 0
    code, plan_b = tuna.tuna_alltoallv_init(b.send, b.sc, b.sd, b.recv, b.rc, b.rd, 64, 8, 2, 8)
    assert code == 0
    try:
        want_a, want_b = a.load(1), b.load(2)
        a.recv.fill_(CANARY)
        b.recv.fill_(CANARY)
        torch.cuda.synchronize()
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        for _ in range(3):
            assert tuna.tuna_start(plan_a, stream=s1) == 0
            assert tuna.tuna_start(plan_b, stream=s2) == 0
        s1.synchronize()
        s2.synchronize()
        a.check(want_a, "plan a")
        b.check(want_b, "plan b")
    finally:
        assert tuna.tuna_plan_free(plan_a) == 0
        assert tuna.tuna_plan_free(plan_b) == 0
    assert tuna.tuna_release() == 0          # no plan left: the cached schedules may go


# ---- exact-size T (TUNA_OPT_DENSE_T) ------------------------------------------------------------
def _dense_plan(tuna, res, P, Q, rl, rg, fused=0, staggered=0, dense=1):
    tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, fused)
    tuna.tuna_set_option(tuna.TUNA_OPT_STAGGERED, staggered)
    tuna.tuna_set_option(tuna.TUNA_OPT_DENSE_T, dense)
    try:
        return tuna.tuna_alltoallv_init(res.send, res.sc, res.sd, res.recv, res.rc, res.rd, P, Q, rl, rg)
    finally:
        tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 2)
        tuna.tuna_set_option(tuna.TUNA_OPT_STAGGERED, 0)
        tuna.tuna_set_option(tuna.TUNA_OPT_DENSE_T, 2)             # the library's default


@pytest.mark.parametrize("mode", ["staged", "fused", "staggered"])
@pytest.mark.parametrize("P,Q,rl,rg,cfg", [(16, 0, 2, 2, 1), (97, 0, 2, 2, 2), (97, 0, 3, 3, 2), (96, 0, 10, 10, 4),
                                            (96, 0, 96, 96, 2), (128, 16, 2, 2, 3), (120, 8, 3, 4, 2),
                                            (256, 0, 2, 2, 3), (1, 0, 2, 2, 2), (2, 0, 2, 2, 2)])
def test_exact_size_t_matches_the_oracle(tuna, P, Q, rl, rg, cfg, mode):
    if mode == "staggered" and Q == 0:
        pytest.skip("staggered needs a hierarchy")
    lay = wl.make_layout(wl.make_counts(cfg, P), gap=4 if cfg != 2 else 5)
    res = Resident(lay)
    code, plan = _dense_plan(tuna, res, P, Q, rl, rg, fused=int(mode == "fused"), staggered=int(mode == "staggered"))
    assert code == 0, tuna.tuna_strerror(code)
    try:
        for seed in (21, 22):
            want = res.load(seed)
            res.recv.fill_(CANARY)
            print("exact-size T P=%d Q=%d rl=%d rg=%d %s seed=%d" % (P, Q, rl, rg, mode, seed), flush=True)
            assert tuna.tuna_start(plan) == 0
            res.check(want, "start %d" % seed)
        st = tuna.tuna_get_stats()
        assert st.dense_t == 1 and st.temp_slots_per_rank == 0
    finally:
        assert tuna.tuna_plan_free(plan) == 0


def _t_bounds(counts, Q, rl, rg, one_kernel):
    """(bytes alive in T at one time, bytes that ever pass through T, classes) from tests/t_size.py."""
    import t_size
    cls, nph = t_size.waiting_bytes(counts, Q, rl, rg)
    return t_size.alive_peak(cls, lambda f: one_kernel), t_size.passed_through(cls), len(cls)


@pytest.mark.parametrize("fused", [0, 1])
def test_exact_size_t_holds_what_waits_in_it(tuna, fused):
    """T in exact size holds what waits in it at one time, not what ever passes through it: the blocks that
    wait from phase f to phase y lie together and share memory with blocks whose wait does not overlap
    theirs.  Its size lies between the most bytes alive at one time (counted independently here, blocks
    padded to 16 bytes) and 1.15 times that plus the rounding (a 128-byte line per rank and 256 bytes per
    group of blocks).  With r = 2 and three-stage phases that is about the payload, a third of what passes
    through T; heavy-tailed sizes make the paper's bound of B slots of M bytes many times larger."""
    P = 256
    counts = wl.make_counts(3, P)
    lay = wl.make_layout(counts)
    res = Resident(lay)
    code, plan = _dense_plan(tuna, res, P, 0, 2, 2, fused=fused)
    assert code == 0
    try:
        want = res.load(3)
        res.recv.fill_(CANARY)
        assert tuna.tuna_start(plan) == 0
        res.check(want, "exact-size T")
        st = tuna.tuna_get_stats()
        dense_bytes = st.temp_bytes
    finally:
        assert tuna.tuna_plan_free(plan) == 0
    alive, passed, ncls = _t_bounds(counts, 0, 2, 2, bool(fused))
    rounding = ncls * (P * 128 + 256)
    print("exact-size T: %d bytes; alive at one time %d, passed through %d, payload %d" % (dense_bytes, alive, passed, lay.payload_bytes))
    assert alive <= dense_bytes <= 1.15 * alive + rounding
    assert dense_bytes < 0.6 * passed
    if not fused:
        assert dense_bytes <= 1.1 * lay.payload_bytes + rounding
    code, plan = _dense_plan(tuna, res, P, 0, 2, 2, fused=fused, dense=0)
    assert code == 0
    try:
        assert tuna.tuna_start(plan) == 0
        strided = tuna.tuna_get_stats().temp_bytes
    finally:
        assert tuna.tuna_plan_free(plan) == 0
    M = int(counts.max())
    assert strided == (2 if fused else 1) * P * (P - 9) * (-(-M // 128) * 128)
    assert strided > 4 * dense_bytes


@pytest.mark.parametrize("r", [2, 4, 16])
def test_exact_size_t_is_never_the_larger_layout(tuna, r):
    """Block sizes of the headline workload (normal, 1 KiB +- 256 B), reduced to P = 256: the T the library
    takes by default is never larger than the paper's B slots of M bytes, at any radix, in either mode."""
    P = 256
    counts = wl.make_counts(4, P)
    lay = wl.make_layout(counts)
    res = Resident(lay)
    for fused in (0, 1):
        sizes = {}
        for dense in (2, 0):
            code, plan = _dense_plan(tuna, res, P, 0, r, r, fused=fused, dense=dense)
            assert code == 0
            try:
                assert tuna.tuna_start(plan) == 0
                sizes[dense] = tuna.tuna_get_stats().temp_bytes
            finally:
                assert tuna.tuna_plan_free(plan) == 0
        torch.cuda.synchronize()
        assert sizes[2] <= sizes[0], (r, fused, sizes)
        if not fused:
            assert sizes[2] <= 1.1 * lay.payload_bytes + 64 * (P * 128 + 256)


def test_device_source_tables_match_the_host(tuna):
    for P, Q, rl, rg in [(64, 0, 2, 2), (100, 0, 3, 3), (96, 8, 2, 3), (60, 5, 5, 12)]:
        rc, info = tuna.tuna_plan_info(P, Q, rl, rg)
        assert rc == 0
        for ph in range(info.n_phases):
            rc, hdr, seg = tuna.tuna_plan_phase(P, Q, rl, rg, ph)
            nseg = int(hdr[4])
            rc, host = tuna.tuna_plan_phase_sources(P, Q, rl, rg, ph, nseg)
            assert rc == 0
            rc, dev = tuna.tuna_plan_phase_sources(P, Q, rl, rg, ph, nseg, on_device=True)
            assert rc == 0 and np.array_equal(host, dev)


@pytest.mark.parametrize("P,Q,rl,rg", [(96, 8, 3, 4), (120, 5, 2, 5), (64, 0, 4, 4)])
def test_exact_size_t_bytes_hierarchical(tuna, P, Q, rl, rg):
    """The same bounds with a hierarchy: a block moves once per non-zero digit of its local distance in base
    r_l, then once per non-zero digit of its node distance in base r_g, and waits in T between two moves."""
    counts = wl.make_counts(2, P)
    lay = wl.make_layout(counts)
    res = Resident(lay)
    code, plan = _dense_plan(tuna, res, P, Q, rl, rg)
    assert code == 0
    try:
        want = res.load(9)
        res.recv.fill_(CANARY)
        assert tuna.tuna_start(plan) == 0
        res.check(want, "exact-size T, hierarchical")
        st = tuna.tuna_get_stats()
    finally:
        assert tuna.tuna_plan_free(plan) == 0
    alive, passed, ncls = _t_bounds(counts, Q, rl, rg, False)
    assert alive <= st.temp_bytes <= 1.15 * alive + ncls * (P * 128 + 256)
    assert st.temp_bytes <= passed + ncls * (P * 128 + 256)


def test_t_layout_left_to_the_library(tuna):
    """Option value 2 (the default): blocks of one size keep the paper's slots (they are full),
    blocks of mixed sizes get T in exact size; both match the oracle."""
    P = 64
    assert tuna.tuna_set_option(tuna.TUNA_OPT_DENSE_T, 2) == 0
    for counts, want_exact in ((wl.counts_constant(P, 256), 0), (wl.make_counts(4, P), 1)):
        lay = wl.make_layout(counts)
        res = Resident(lay)
        want = res.load(31)
        res.recv.fill_(CANARY)
        assert tuna.tuna_alltoallv(res.send, res.sc, res.sd, res.recv, res.rc, res.rd, P, 4, 0) == 0
        res.check(want, "automatic T layout")
        assert tuna.tuna_get_stats().dense_t == want_exact
    assert tuna.tuna_set_option(tuna.TUNA_OPT_DENSE_T, 3) == tuna.TUNA_ERR_ARG
