"""tuna_alltoallv_noalloc -- the entry point for callers that cannot allocate device memory -- through
the C ABI against tuna_alltoallv_hier on the same inputs: byte for byte over the whole receive
allocation (canary bytes included), on two calls in a row, the second with a smaller problem, so that
whatever the first call left in the static scratch array is still there.  The oracle's result is
compared too.  The no-allocation call comes first: in a fresh process it is then the library's very
first call and cannot lean on anything another entry point allocated."""
import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
CANARY = 0xA5


@pytest.fixture(scope="module")
def tuna():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_02581_amd as t
    t.load()
    return t


class Case:
    def __init__(self, counts, seed, gap, Q, rl, rg, permute_seed=None):
        self.lay = lay = wl.make_layout(counts.astype(np.int32), gap=gap, permute_seed=permute_seed)
        self.Q, self.rl, self.rg = Q, rl, rg
        dev = "cuda:0"
        self.send_host = wl.payload_position_hash(seed, lay.send_bytes)
        self.send = torch.from_numpy(self.send_host).to(dev)
        self.meta = [torch.from_numpy(a).to(dev) for a in (lay.sendcounts, lay.sdispls, lay.recvcounts, lay.rdispls)]
        self.want = np.full(lay.recv_bytes, CANARY, dtype=np.uint8)
        assert oracle.alltoallv(self.send_host, lay.sendcounts, lay.sdispls, self.want, lay.recvcounts, lay.rdispls) == 0

    def run(self, fn):
        recv = torch.full((self.lay.recv_bytes,), CANARY, dtype=torch.uint8, device="cuda:0")
        sc, sd, rc_, rd = self.meta
        rc = fn(self.send, sc, sd, recv, rc_, rd, self.lay.P, self.Q, self.rl, self.rg)
        torch.cuda.synchronize()
        return rc, recv.cpu().numpy()


def big_case():
    # byte-granular sizes, gaps and permuted regions, three digit phases with a temporary buffer
    return Case(wl.counts_uniform_bytes(64, 11, 3000), seed=5, gap=7, Q=0, rl=4, rg=4, permute_seed=3)


def small_case():
    # hierarchical, 4 ranks per node x 6 nodes, 4-byte granular
    return Case(wl.counts_uniform_elements(24, 13, 120, 4), seed=6, gap=4, Q=4, rl=2, rg=2)


@pytest.mark.parametrize("fused,dense", [(0, 2), (1, 2), (0, 0), (1, 0)])
def test_two_calls_in_a_row_match_the_allocating_entry_point(tuna, fused, dense):
    tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, fused)
    tuna.tuna_set_option(tuna.TUNA_OPT_DENSE_T, dense)
    try:
        for name, case in (("first, larger", big_case()), ("second, smaller", small_case())):
            print("no-alloc call:", name, "P=%d bytes=%d fused=%d dense=%d" % (case.lay.P, case.lay.payload_bytes, fused, dense),
                  flush=True)
            rc, got = case.run(tuna.tuna_alltoallv_noalloc)
            assert rc == 0, tuna.tuna_strerror(rc)
            rc, ref = case.run(tuna.tuna_alltoallv_hier)
            assert rc == 0, tuna.tuna_strerror(rc)
            assert np.array_equal(got, ref), name + ": differs from tuna_alltoallv_hier"
            assert np.array_equal(got, case.want), name + ": differs from the oracle"
            assert np.array_equal(case.send.cpu().numpy(), case.send_host), name + ": send buffer modified"
    finally:
        tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 2)
        tuna.tuna_set_option(tuna.TUNA_OPT_DENSE_T, 2)


def test_a_problem_beyond_the_static_scratch_is_refused(tuna):
    """32 MiB of payload in three-stage phases needs two staging buffers of that size: more than the
    array holds.  The call says so and moves nothing; a small call right after it works; and the same
    problem with one-kernel hops (no staging) fits and is right."""
    case = Case(wl.make_counts(2), seed=9, gap=0, Q=0, rl=16, rg=16)
    assert 2 * case.lay.payload_bytes > tuna.TUNA_NOALLOC_SCRATCH_BYTES
    tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 0)
    try:
        rc, got = case.run(tuna.tuna_alltoallv_noalloc)
    finally:
        tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 2)
    assert rc == tuna.TUNA_ERR_NOALLOC_LIMIT, tuna.tuna_strerror(rc)
    assert (got == CANARY).all()
    assert "static scratch" in tuna.tuna_strerror(rc)
    small = small_case()
    rc, got = small.run(tuna.tuna_alltoallv_noalloc)
    assert rc == 0 and np.array_equal(got, small.want)
    rc, got = case.run(tuna.tuna_alltoallv_noalloc)
    assert rc == 0, tuna.tuna_strerror(rc)
    assert np.array_equal(got, case.want)


def test_argument_errors(tuna):
    case = small_case()
    sc, sd, rc_, rd = case.meta
    recv = torch.full((case.lay.recv_bytes,), CANARY, dtype=torch.uint8, device="cuda:0")
    P = case.lay.P
    assert tuna.tuna_alltoallv_noalloc(case.send, sc, sd, recv, rc_, rd, P, 5, 2, 2) == tuna.TUNA_ERR_ARG   # 5 does not divide 24
    assert tuna.tuna_alltoallv_noalloc(case.send, sc, sd, recv, rc_, rd, P, 4, 1, 2) == tuna.TUNA_ERR_ARG
    assert tuna.tuna_alltoallv_noalloc(case.send, None, sd, recv, rc_, rd, P, 4, 2, 2) == tuna.TUNA_ERR_ARG
    bad = rc_.clone()
    bad[3] += 4
    assert tuna.tuna_alltoallv_noalloc(case.send, sc, sd, recv, bad, rd, P, 4, 2, 2) == tuna.TUNA_ERR_COUNT_MISMATCH
    torch.cuda.synchronize()
    assert (recv.cpu().numpy() == CANARY).all()
