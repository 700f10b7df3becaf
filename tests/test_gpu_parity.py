"""GPU parity: libtuna.so through its C ABI against the CPU oracle, byte for byte over the whole
receive allocation (canary bytes between and around the receive regions included), for every
radix and hierarchy setting.  The result is unique, so the bar is exact equality."""
import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
CANARY = 0xC7


@pytest.fixture(scope="module")
def tuna():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_02581_amd as t
    t.load()
    return t


@pytest.fixture(autouse=True, params=["staged", "fused", "exact", "fused_exact"])
def mode(request, tuna):
    """Every case runs with the three-stage phases (pack, exchange, unpack) and with the fused
    single-kernel phases, each with T in slots of M bytes and with T in exact size."""
    tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 1 if request.param.startswith("fused") else 0)
    tuna.tuna_set_option(tuna.TUNA_OPT_DENSE_T, 1 if request.param.endswith("exact") else 0)
    yield request.param
    tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 2)
    tuna.tuna_set_option(tuna.TUNA_OPT_DENSE_T, 2)                 # the library's default


class Problem:
    """One alltoallv problem resident on the GPU, with the oracle's expected receive buffer."""

    def __init__(self, lay, send_host):
        self.lay = lay
        self.send_host = send_host
        dev = "cuda:0"
        self.send = torch.from_numpy(send_host).to(dev)
        self.sendcounts = torch.from_numpy(lay.sendcounts).to(dev)
        self.sdispls = torch.from_numpy(lay.sdispls).to(dev)
        self.recvcounts = torch.from_numpy(lay.recvcounts).to(dev)
        self.rdispls = torch.from_numpy(lay.rdispls).to(dev)
        self.recv = torch.empty(lay.recv_bytes, dtype=torch.uint8, device=dev)
        want = np.full(lay.recv_bytes, CANARY, dtype=np.uint8)
        assert oracle.alltoallv(send_host, lay.sendcounts, lay.sdispls, want, lay.recvcounts, lay.rdispls) == 0
        self.want = want

    def args(self):
        return (self.send, self.sendcounts, self.sdispls, self.recv, self.recvcounts, self.rdispls, self.lay.P)

    def check(self, what):
        torch.cuda.synchronize()
        got = self.recv.cpu().numpy()
        if not np.array_equal(got, self.want):
            bad = np.flatnonzero(got != self.want)
            raise AssertionError("%s: %d bytes differ, first at offset %d (got %d, want %d)" %
                                 (what, bad.size, bad[0], got[bad[0]], self.want[bad[0]]))
        assert np.array_equal(self.send.cpu().numpy(), self.send_host), what + ": send buffer modified"

    def reset(self):
        self.recv.fill_(CANARY)


def run_flat(tuna, prob, radix, rpn=0):
    prob.reset()
    print("case P=%d radix=%d rpn=%d" % (prob.lay.P, radix, rpn), flush=True)
    rc = tuna.tuna_alltoallv(*prob.args(), radix, rpn)
    assert rc == 0, tuna.tuna_strerror(rc)
    prob.check("P=%d radix=%d rpn=%d" % (prob.lay.P, radix, rpn))


def run_hier(tuna, prob, Q, rl, rg):
    prob.reset()
    print("case P=%d Q=%d rl=%d rg=%d" % (prob.lay.P, Q, rl, rg), flush=True)
    rc = tuna.tuna_alltoallv_hier(*prob.args(), Q, rl, rg)
    assert rc == 0, tuna.tuna_strerror(rc)
    prob.check("P=%d Q=%d rl=%d rg=%d" % (prob.lay.P, Q, rl, rg))


def test_config1_traceable_payload(tuna, mode):
    lay = wl.make_layout(wl.make_counts(1), gap=16)
    prob = Problem(lay, wl.payload_traceable_int32(lay))
    run_flat(tuna, prob, 2)
    st = tuna.tuna_get_stats()
    assert st.fused == (1 if mode.startswith("fused") else 0)
    assert st.dense_t == (1 if mode.endswith("exact") else 0)
    assert (st.P, st.w_local, st.K_local, st.B_local) == (16, 4, 4, 11)
    assert st.total_payload_bytes == lay.payload_bytes and st.max_block_bytes == lay.sendcounts.max()
    assert st.granularity == 4


@pytest.mark.parametrize("P", [1, 2, 3, 5, 8, 13, 16, 31])
def test_small_every_radix(tuna, P):
    """Tiny P, byte-granular sizes, gaps and permuted regions, every radix 2..P."""
    counts = wl.counts_uniform_bytes(P, 77 + P, 300)
    counts[counts % 5 == 0] = 0
    lay = wl.make_layout(counts, gap=7, permute_seed=5)
    prob = Problem(lay, wl.payload_position_hash(P, lay.send_bytes))
    for r in range(2, max(P, 2) + 1):
        run_flat(tuna, prob, r)
    run_flat(tuna, prob, P + 9)       # clamps to P


@pytest.mark.parametrize("align,quantum", [(1, 1), (4, 4), (16, 16), (128, 128)])
def test_granularities(tuna, align, quantum):
    """The copy paths: whole-line, 16-byte, 4-byte and byte granular sizes/displacements."""
    P = 48
    counts = (wl.counts_uniform_bytes(P, 5, 3000) // quantum * quantum).astype(np.int32)
    lay = wl.make_layout(counts, gap=quantum, align=align)
    prob = Problem(lay, wl.payload_position_hash(3, lay.send_bytes))
    for r in (2, 7, 48):
        run_flat(tuna, prob, r)
        assert tuna.tuna_get_stats().granularity == quantum


def test_config2_radix_sweep(tuna):
    c = wl.CONFIGS[2]
    lay = wl.make_layout(wl.make_counts(2))
    prob = Problem(lay, wl.payload_position_hash(c.seed, lay.send_bytes))
    for r in c.radices:
        run_flat(tuna, prob, r)
    st = tuna.tuna_get_stats()
    assert st.granularity == 1 and st.total_payload_bytes == lay.payload_bytes


def test_config3_reduced_hierarchical(tuna):
    """Zipf sizes (many empty and tiny blocks, rare 16 KiB ones), float32 bit patterns, at
    P = 256 = 16 ranks/node x 16 nodes; the full-size case is in test_gpu_full_size.py."""
    P, Q = 256, 16
    counts = wl.make_counts(3, P)
    lay = wl.make_layout(counts)
    prob = Problem(lay, wl.float32_bit_patterns(lay.send_bytes, 33))
    for rg in (2, 8, 16):
        run_hier(tuna, prob, Q, 4, rg)
    run_flat(tuna, prob, 4)


def test_config4_reduced(tuna):
    P = 512
    lay = wl.make_layout(wl.make_counts(4, P))
    prob = Problem(lay, wl.payload_position_hash(44, lay.send_bytes))
    for r in (2, 8, 64, 512):
        run_flat(tuna, prob, r)


def test_config5_reduced_uniform(tuna):
    """All blocks 256 B: the result is a transpose of 256-byte cells."""
    P, Q = 256, 32
    lay = wl.make_layout(wl.counts_constant(P, 256))
    send = wl.payload_position_hash(55, lay.send_bytes)
    prob = Problem(lay, send)
    assert np.array_equal(prob.want.reshape(P, P, 256), send.reshape(P, P, 256).transpose(1, 0, 2))
    for r in (2, 16, 2048):
        run_flat(tuna, prob, r, rpn=Q)
        assert tuna.tuna_get_stats().granularity == 128


@pytest.mark.parametrize("Q,N", [(1, 6), (2, 3), (3, 2), (4, 4), (5, 3), (3, 7), (8, 2), (6, 10)])
def test_hierarchy_shapes(tuna, Q, N):
    P = Q * N
    counts = wl.counts_uniform_bytes(P, 900 + P, 700)
    counts[counts % 3 == 0] = 0
    lay = wl.make_layout(counts, gap=5, permute_seed=9)
    prob = Problem(lay, wl.payload_position_hash(P, lay.send_bytes))
    for rl in sorted({2, 3, max(Q, 2)}):
        for rg in sorted({2, 3, max(N, 2)}):
            run_hier(tuna, prob, Q, rl, rg)


@pytest.mark.parametrize("Q,N", [(2, 3), (4, 4), (5, 3), (16, 8)])
def test_staggered_inter_node_schedule(tuna, Q, N):
    """Algorithm "Staggered TuNA_l^g": one block per inter-node message, straight out of T."""
    P = Q * N
    counts = wl.make_counts(3, P) if P >= 64 else wl.counts_uniform_bytes(P, 31 + P, 900)
    lay = wl.make_layout(counts, gap=3)
    prob = Problem(lay, wl.payload_position_hash(P, lay.send_bytes))
    tuna.tuna_set_option(tuna.TUNA_OPT_STAGGERED, 1)
    try:
        for rl in sorted({2, max(Q, 2)}):
            run_hier(tuna, prob, Q, rl, 2)
            st = tuna.tuna_get_stats()
            assert st.global_radix == N and st.K_global == Q * (N - 1)
            assert st.phase[st.n_phases - 1].rounds == Q * (N - 1)
        run_flat(tuna, prob, 3)
    finally:
        tuna.tuna_set_option(tuna.TUNA_OPT_STAGGERED, 0)


@pytest.mark.parametrize("pattern", ["n1", "n2"])
def test_fft_count_patterns(tuna, pattern):
    """The two closed-form count matrices of the paper's FFT runs: sparse (37.5 % of the ranks
    send nothing, the last 22 % of the blocks are empty) and near uniform."""
    P = 192
    counts = wl.counts_fft_n1(P) if pattern == "n1" else wl.counts_fft_n2(P)
    lay = wl.make_layout(counts)
    prob = Problem(lay, wl.payload_position_hash(70, lay.send_bytes))
    for r in (2, 14, P):
        run_flat(tuna, prob, r)
    run_hier(tuna, prob, 16, 4, 12)


@pytest.mark.parametrize("P,Q,rl,rg", [(16, 0, 2, 2), (30, 0, 3, 3), (64, 0, 64, 64), (24, 4, 2, 3), (60, 5, 5, 2),
                                        (256, 16, 4, 8), (1000, 0, 10, 10)])
def test_device_built_tables_match_the_host_schedule(tuna, P, Q, rl, rg, mode):
    """The kernels read tables that k_build_phase_table built on the GPU; they must equal the
    host-side schedule (which tests/test_host_plan.py replays on the CPU) entry for entry."""
    rc, info = tuna.tuna_plan_info(P, Q, rl, rg)
    assert rc == 0
    for ph in range(info.n_phases):
        rc, hdr, seg = tuna.tuna_plan_phase(P, Q, rl, rg, ph)
        assert rc == 0
        rc, dev = tuna.tuna_plan_phase_device(P, Q, rl, rg, ph, int(hdr[4]))
        assert rc == 0
        assert np.array_equal(dev, seg[:, [0, 3, 4, 5]]), (P, Q, rl, rg, ph, mode)


def test_degenerate_inputs(tuna):
    # all blocks empty
    lay = wl.make_layout(np.zeros((9, 9), dtype=np.int32), gap=4)
    prob = Problem(lay, np.zeros(lay.send_bytes, dtype=np.uint8))
    run_flat(tuna, prob, 3)
    # only self blocks
    counts = np.diag(np.arange(1, 8) * 11).astype(np.int32)
    lay = wl.make_layout(counts, gap=2)
    prob = Problem(lay, wl.payload_position_hash(1, lay.send_bytes))
    run_flat(tuna, prob, 2)
    # one sender, one huge block among empties (1 MiB + 3 bytes), and ranks that send nothing
    counts = np.zeros((6, 6), dtype=np.int32)
    counts[2, 5] = (1 << 20) + 3
    counts[4, 0] = 17
    lay = wl.make_layout(counts, gap=1)
    prob = Problem(lay, wl.payload_position_hash(2, lay.send_bytes))
    for r in (2, 3, 6):
        run_flat(tuna, prob, r)
    run_hier(tuna, prob, 2, 2, 2)


@pytest.mark.parametrize("quantum", [1, 4, 8])
def test_tiny_blocks(tuna, quantum):
    """Blocks of at most 64 bytes (the small-message regime of Section "Performance analysis of TuNA"):
    one-kernel phases move them with one thread per block.  Byte-, 4-byte- and 8-byte-granular sizes from 0
    to 64, many of them empty; flat for several radices, hierarchical, in batches of rounds and with the
    staggered inter-node schedule."""
    P = 45
    counts = (wl.counts_uniform_bytes(P, 91 + quantum, 64) // quantum * quantum).astype(np.int32)
    counts[counts % 3 == 0] = 0
    counts[7, 11] = 64
    lay = wl.make_layout(counts, gap=quantum, align=quantum)
    prob = Problem(lay, wl.payload_position_hash(17, lay.send_bytes))
    for r in (2, 3, 7, 45):
        run_flat(tuna, prob, r)
        assert tuna.tuna_get_stats().max_block_bytes == 64
    run_hier(tuna, prob, 9, 3, 2)
    run_hier(tuna, prob, 5, 5, 9)
    tuna.tuna_set_option(tuna.TUNA_OPT_BLOCK_COUNT, 2)
    try:
        run_flat(tuna, prob, 45)
        run_hier(tuna, prob, 9, 3, 5)
    finally:
        tuna.tuna_set_option(tuna.TUNA_OPT_BLOCK_COUNT, 0)
    tuna.tuna_set_option(tuna.TUNA_OPT_STAGGERED, 1)
    try:
        run_hier(tuna, prob, 9, 2, 5)
    finally:
        tuna.tuna_set_option(tuna.TUNA_OPT_STAGGERED, 0)


def test_large_own_blocks(tuna):
    """Blocks a rank keeps for itself above 64 KiB go through the byte-balanced copy engine (one more
    one-kernel phase of one block per rank) instead of one workgroup per rank: byte-granular sizes of
    about 1 MiB on the diagonal, some ranks with an empty own block, small blocks elsewhere; also
    P = 1 (nothing but the own block) and a hierarchy."""
    P = 12
    counts = wl.counts_uniform_bytes(P, 31, 400)
    rng = np.random.default_rng(3)
    for p in range(P):
        counts[p, p] = 0 if p in (4, 9) else (1 << 20) + int(rng.integers(-5000, 5000))
    lay = wl.make_layout(counts, gap=3, permute_seed=8)
    prob = Problem(lay, wl.payload_position_hash(4, lay.send_bytes))
    for r in (2, 12):
        run_flat(tuna, prob, r)
    run_hier(tuna, prob, 3, 2, 4)
    lay = wl.make_layout(np.array([[300001]], dtype=np.int32), gap=5)
    prob = Problem(lay, wl.payload_position_hash(5, lay.send_bytes))
    run_flat(tuna, prob, 2)


def test_many_empty_segments_span_windows(tuna):
    """More than one LDS window of segments inside a tile: long runs of empty blocks."""
    P = 700
    counts = np.zeros((P, P), dtype=np.int32)
    rng = np.random.default_rng(12)
    idx = rng.integers(0, P, size=(3000, 2))
    counts[idx[:, 0], idx[:, 1]] = rng.integers(1, 5000, size=3000)
    lay = wl.make_layout(counts)
    prob = Problem(lay, wl.payload_position_hash(6, lay.send_bytes))
    for r in (2, 700):
        run_flat(tuna, prob, r)


def test_errors(tuna):
    lay = wl.make_layout(wl.counts_uniform_bytes(8, 1, 64))
    prob = Problem(lay, wl.payload_position_hash(1, lay.send_bytes))
    prob.reset()
    bad = prob.recvcounts.clone()
    bad[2, 3] += 1
    a = list(prob.args())
    a[4] = bad
    assert tuna.tuna_alltoallv(*a, 2, 0) == tuna.TUNA_ERR_COUNT_MISMATCH
    neg = prob.sendcounts.clone()
    neg[1, 1] = -5
    a = list(prob.args())
    a[1] = neg
    assert tuna.tuna_alltoallv(*a, 2, 0) == tuna.TUNA_ERR_NEGATIVE_COUNT
    assert tuna.tuna_alltoallv(*prob.args(), 1, 0) == tuna.TUNA_ERR_ARG
    assert tuna.tuna_alltoallv(*prob.args(), 2, 3) == tuna.TUNA_ERR_ARG       # 3 does not divide 8
    for which in (2, 5):                                                      # sdispls, rdispls
        cnt = prob.sendcounts if which == 2 else prob.recvcounts
        nz = torch.nonzero(cnt)[0]
        a = list(prob.args())
        a[which] = a[which].clone()
        a[which][nz[0], nz[1]] = -16                                          # a non-empty block in front of the buffer
        assert tuna.tuna_alltoallv(*a, 2, 0) == tuna.TUNA_ERR_ARG
    torch.cuda.synchronize()
    assert (prob.recv.cpu().numpy() == CANARY).all()                          # nothing was moved
    run_flat(tuna, prob, 2)                                                    # and the library still works
    for which in (2, 5):                                                      # an empty block may sit anywhere
        cnt = prob.sendcounts if which == 2 else prob.recvcounts
        z = torch.nonzero(cnt == 0)
        if len(z) == 0:
            continue
        a = list(prob.args())
        a[which] = a[which].clone()
        a[which][z[0][0], z[0][1]] = -16
        prob.reset()
        assert tuna.tuna_alltoallv(*a, 2, 0) == tuna.TUNA_OK
        prob.check("empty block at a negative displacement")


def test_stats_phase_bytes(tuna):
    """Per-phase payload bytes reported by the device equal those of the per-rank model."""
    from oracle import tuna_model as tm
    P, r = 12, 3
    counts = wl.counts_uniform_bytes(P, 4, 40)
    lay = wl.make_layout(counts)
    send = wl.payload_position_hash(9, lay.send_bytes)
    prob = Problem(lay, send)
    run_flat(tuna, prob, r)
    st = tuna.tuna_get_stats()
    S = [[bytes(send[lay.sdispls[i, j]:lay.sdispls[i, j] + counts[i, j]]) for j in range(P)] for i in range(P)]
    _, ms = tm.simulate_tuna(S, r)
    assert [st.phase[x].payload_bytes for x in range(st.n_phases)] == [ms["phase_bytes"][x] for x in range(st.n_phases)]
    assert [st.phase[x].rounds for x in range(st.n_phases)] == [2, 2, 1]
    assert all(st.phase[x].staged_bytes >= st.phase[x].payload_bytes for x in range(st.n_phases))


def test_caller_workspace_and_profiling(tuna):
    P = 64
    lay = wl.make_layout(wl.make_counts(4, P))
    prob = Problem(lay, wl.payload_position_hash(8, lay.send_bytes))
    rc, need = tuna.tuna_workspace_bytes(prob.sendcounts, P, 0, 4, 4)
    assert rc == 0 and need > 0
    ws = torch.empty(need + 256, dtype=torch.uint8, device="cuda:0")
    base = (ws.data_ptr() + 255) // 256 * 256
    assert tuna.tuna_set_workspace(base, need) == 0
    try:
        run_flat(tuna, prob, 4)
        assert tuna.tuna_get_stats().workspace_bytes <= need
        assert tuna.tuna_set_workspace(base, 1024) == 0
        prob.reset()
        assert tuna.tuna_alltoallv(*prob.args(), 4, 0) == tuna.TUNA_ERR_WORKSPACE_TOO_SMALL
    finally:
        assert tuna.tuna_set_workspace(None, 0) == 0
    tuna.tuna_set_option(tuna.TUNA_OPT_PROFILE, 1)
    try:
        run_flat(tuna, prob, 4)
        st = tuna.tuna_get_stats()
        # every phase has a payload kernel (the destination-tiled hop reports its time as unpack time)
        assert st.ms_total > 0 and all(st.phase[x].ms_pack > 0 or st.phase[x].ms_unpack > 0 for x in range(st.n_phases))
    finally:
        tuna.tuna_set_option(tuna.TUNA_OPT_PROFILE, 0)


def test_side_stream(tuna):
    P = 96
    lay = wl.make_layout(wl.make_counts(2, P))
    prob = Problem(lay, wl.payload_position_hash(10, lay.send_bytes))
    s = torch.cuda.Stream()
    prob.reset()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        rc = tuna.tuna_alltoallv(*prob.args(), 4, 0, stream=s)
    assert rc == 0
    s.synchronize()
    prob.check("side stream")


def test_plain_copy(tuna):
    n = (1 << 20) + 48
    src = torch.from_numpy(wl.payload_position_hash(21, n)).to("cuda:0")
    dst = torch.zeros(n, dtype=torch.uint8, device="cuda:0")
    assert tuna.tuna_plain_copy(src, dst, n - 16) == 0
    torch.cuda.synchronize()
    assert torch.equal(dst[:n - 16], src[:n - 16]) and int(dst[n - 16:].sum()) == 0
    assert tuna.tuna_plain_copy(src, dst, 24) == tuna.TUNA_ERR_ARG


def test_random_problems(tuna, mode):
    """Seeded random problems: rank counts, hierarchy, radices, size distributions (empty rows and
    columns, tiny and large blocks, every alignment), gaps and region order all vary."""
    rng = np.random.default_rng(20241102 + ["staged", "fused", "exact", "fused_exact"].index(mode))
    for case in range(40):
        Q = int(rng.integers(1, 9))
        N = int(rng.integers(1, 9))
        P = Q * N
        kind = int(rng.integers(0, 4))
        if kind == 0:
            counts = rng.integers(0, 40, size=(P, P))
        elif kind == 1:
            counts = (rng.pareto(1.1, size=(P, P)) * 20).astype(np.int64).clip(0, 70000)
        elif kind == 2:
            counts = rng.integers(0, 3000, size=(P, P)) * (rng.random((P, P)) < 0.3)
        else:
            counts = rng.integers(0, 600, size=(P, P)) // 4 * 4
        counts = counts.astype(np.int32)
        if rng.random() < 0.3:
            counts[rng.integers(0, P)] = 0            # a rank that sends nothing
        if rng.random() < 0.3:
            counts[:, rng.integers(0, P)] = 0         # a rank that receives nothing
        gap = int(rng.integers(0, 20))
        lay = wl.make_layout(counts, gap=gap, permute_seed=int(rng.integers(0, 1 << 30)) if rng.random() < 0.5 else None,
                             align=int(rng.choice([1, 1, 4, 16])))
        prob = Problem(lay, wl.payload_position_hash(case, lay.send_bytes))
        rl = int(rng.integers(2, max(Q, 2) + 2))
        rg = int(rng.integers(2, max(N, 2) + 2))
        run_hier(tuna, prob, Q, rl, rg)
        if rng.random() < 0.5:
            run_flat(tuna, prob, int(rng.integers(2, P + 2)))


def test_phase_bytes_closed_form(tuna, mode):
    """Before digit phase x the block at rank p, index i started at rank s = p + (i mod r^x) bound
    for s - i, so the bytes phase x moves follow from the counts alone:
    b_x = sum over p and over i with digit_x(i) != 0 of sendcounts[s][(s - i) mod P]."""
    P = 384
    counts = wl.make_counts(4, P)
    lay = wl.make_layout(counts)
    prob = Problem(lay, wl.payload_position_hash(12, lay.send_bytes))
    p = np.arange(P)[:, None]
    i = np.arange(P)[None, :]
    c64 = counts.astype(np.int64)
    for r in (2, 5, 20, P):
        run_flat(tuna, prob, r)
        st = tuna.tuna_get_stats()
        for x in range(st.n_phases):
            rx = r ** x
            s = (p + i % rx) % P
            moving = (i // rx) % r != 0
            b_x = int((c64[s, (s - i) % P] * moving).sum())
            assert st.phase[x].payload_bytes == b_x, (r, x)
            assert st.phase[x].blocks == int(moving.sum()) * P


def test_temporary_buffer_too_large_is_an_error_not_a_crash(tuna, mode):
    """T has one M-byte slot per intermediate block: one 512 MiB block among 64 ranks at radix 2
    asks for terabytes.  The call must return TUNA_ERR_NOMEM, move nothing, and leave the library
    usable; the same problem runs at radix P, which needs no T -- and at radix 2 with T in exact
    size: the block (index 27: four non-zero bits) waits in T three times, one wait after the other, so
    with three-stage phases T holds it once, and twice with one-kernel phases, where a phase reads one
    wait's copy while it writes the next one's."""
    P = 64
    counts = np.zeros((P, P), dtype=np.int32)
    counts[3, 40] = 512 << 20
    counts[5, 6] = 100
    lay = wl.make_layout(counts)
    dev = "cuda:0"
    send = wl.payload_position_hash_torch(77, lay.send_bytes, dev)
    recv = torch.zeros(lay.recv_bytes, dtype=torch.uint8, device=dev)
    d = [torch.from_numpy(a).to(dev) for a in (lay.sendcounts, lay.sdispls, lay.recvcounts, lay.rdispls)]
    rc = tuna.tuna_alltoallv(send, d[0], d[1], recv, d[2], d[3], P, 2, 0)
    if mode.endswith("exact"):
        assert rc == 0, tuna.tuna_strerror(rc)
        st = tuna.tuna_get_stats()
        # the 100-byte block (index 63: six hops) adds little; rounding: a 128-byte line per rank and 256
        # bytes for every group of blocks that wait together
        copies = 2 if mode.startswith("fused") else 1
        assert copies * (512 << 20) <= st.temp_bytes <= copies * (512 << 20) + 20 * (256 + P * 128) + 4096
    else:
        assert rc == tuna.TUNA_ERR_NOMEM, tuna.tuna_strerror(rc)
        torch.cuda.synchronize()
        assert int(recv.count_nonzero()) == 0
        rc = tuna.tuna_alltoallv(send, d[0], d[1], recv, d[2], d[3], P, P, 0)
        assert rc == 0, tuna.tuna_strerror(rc)
    torch.cuda.synchronize()
    so, ro, n = int(lay.sdispls[3, 40]), int(lay.rdispls[40, 3]), 512 << 20
    assert torch.equal(recv[ro:ro + n], send[so:so + n])
    so, ro = int(lay.sdispls[5, 6]), int(lay.rdispls[6, 5])
    assert torch.equal(recv[ro:ro + 100], send[so:so + 100])


@pytest.mark.parametrize("P,Q,rl,rg,cfg,k", [(64, 0, 64, 64, 2, 1), (64, 0, 64, 64, 2, 7), (100, 0, 10, 10, 4, 3),
                                              (96, 8, 8, 12, 3, 2), (96, 8, 3, 12, 2, 100), (30, 0, 2, 2, 2, 1),
                                              # several batches per phase and several phases whose waiting blocks share T:
                                              # a batch stores into T while the next batch of the same phase still reads
                                              (24, 2, 2, 3, 4, 1), (81, 0, 3, 3, 4, 1), (125, 0, 5, 5, 3, 2)])
def test_block_count_batches_move_the_same_bytes(tuna, P, Q, rl, rg, cfg, k, mode):
    """Rounds moved in batches of k (block_count; with r = P the scattered linear algorithm): the
    result is the same as with all rounds of a phase at once."""
    lay = wl.make_layout(wl.make_counts(cfg, P), gap=5 if cfg == 2 else 4)
    prob = Problem(lay, wl.payload_position_hash(500 + k, lay.send_bytes))
    assert tuna.tuna_set_option(tuna.TUNA_OPT_BLOCK_COUNT, k) == 0
    try:
        prob.reset()
        print("block_count=%d P=%d Q=%d rl=%d rg=%d %s" % (k, P, Q, rl, rg, mode), flush=True)
        assert tuna.tuna_alltoallv_hier(*prob.args(), Q, rl, rg) == 0
        prob.check("block_count %d" % k)
        if Q:
            tuna.tuna_set_option(tuna.TUNA_OPT_STAGGERED, 1)
            prob.reset()
            assert tuna.tuna_alltoallv_hier(*prob.args(), Q, rl, rg) == 0
            prob.check("staggered, block_count %d" % k)
    finally:
        tuna.tuna_set_option(tuna.TUNA_OPT_STAGGERED, 0)
        tuna.tuna_set_option(tuna.TUNA_OPT_BLOCK_COUNT, 0)
    assert tuna.tuna_set_option(tuna.TUNA_OPT_BLOCK_COUNT, -1) == tuna.TUNA_ERR_ARG
