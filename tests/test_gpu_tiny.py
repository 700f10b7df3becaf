"""Problems of at most 64 ranks and 1 MiB of payload, called with everything left to the library, are done
by one kernel launch (k_tiny_call: validation, rotation, own blocks and every digit phase in one workgroup).
Same bar as everywhere: the whole receive allocation equals the CPU oracle's byte for byte, for every radix
and hierarchy; invalid counts and problems that are not tiny after all fall through to the general path,
which reports the error or does the work."""
import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
CANARY = 0xE1


@pytest.fixture(scope="module")
def tuna():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_02581_amd as t
    t.load()
    assert t.tuna_opts_init().mode == t.TUNA_MODE_AUTO        # the defaults: the one-kernel call is eligible
    return t


class Prob:
    def __init__(self, counts, seed, gap=3, permute_seed=None, traceable=False):
        self.lay = lay = wl.make_layout(counts.astype(np.int32), gap=gap, permute_seed=permute_seed)
        dev = "cuda:0"
        self.host = wl.payload_traceable_int32(lay) if traceable else wl.payload_position_hash(seed, lay.send_bytes)
        self.send = torch.from_numpy(self.host).to(dev) if lay.send_bytes else torch.zeros(16, dtype=torch.uint8, device=dev)
        self.meta = [torch.from_numpy(a).to(dev) for a in (lay.sendcounts, lay.sdispls, lay.recvcounts, lay.rdispls)]
        self.recv = torch.full((max(lay.recv_bytes, 16),), CANARY, dtype=torch.uint8, device=dev)
        self.want = np.full(lay.recv_bytes, CANARY, dtype=np.uint8)
        assert oracle.alltoallv(self.host, lay.sendcounts, lay.sdispls, self.want, lay.recvcounts, lay.rdispls) == 0

    def run(self, tuna, Q, rl, rg, what):
        sc, sd, rc_, rd = self.meta
        self.recv.fill_(CANARY)
        print("tiny case", what, flush=True)
        rc = tuna.tuna_alltoallv_hier(self.send, sc, sd, self.recv, rc_, rd, self.lay.P, Q, rl, rg)
        assert rc == 0, tuna.tuna_strerror(rc)
        torch.cuda.synchronize()
        got = self.recv.cpu().numpy()[:self.lay.recv_bytes]
        bad = np.flatnonzero(got != self.want)
        assert bad.size == 0, "%s: %d bytes differ, first at %d" % (what, bad.size, bad[0])
        assert np.array_equal(self.send.cpu().numpy()[:self.lay.send_bytes], self.host), what + ": send buffer modified"


def test_config1_in_one_launch(tuna):
    prob = Prob(wl.make_counts(1), 1, gap=16, traceable=True)
    for r in (2, 4, 16):
        prob.run(tuna, 0, r, r, "config 1 r=%d" % r)
        st = tuna.tuna_get_stats()
        assert (st.P, st.local_radix, st.fused, st.granularity) == (16, r, 1, 4)
        assert st.total_payload_bytes == prob.lay.payload_bytes and st.max_block_bytes == prob.lay.sendcounts.max()
        assert st.workspace_bytes == 4 << 20                  # the one-kernel call's own small T, nothing else
    assert (st.w_local, st.K_local) == (1, 15)


@pytest.mark.parametrize("P", [1, 2, 3, 7, 16, 33, 64])
def test_every_radix(tuna, P):
    """Byte-granular sizes, gaps, permuted regions, empty blocks; every radix 2..P (T in use for the small ones)."""
    counts = wl.counts_uniform_bytes(P, 400 + P, 200)
    counts[counts % 4 == 0] = 0
    prob = Prob(counts, P, gap=5, permute_seed=9)
    for r in sorted(set(list(range(2, min(P, 9) + 1)) + [max(P, 2), P + 3])):
        prob.run(tuna, 0, r, r, "P=%d r=%d" % (P, r))


@pytest.mark.parametrize("P,Q,rl,rg", [(12, 3, 2, 2), (24, 4, 2, 3), (36, 6, 6, 6), (64, 8, 2, 2), (64, 16, 4, 2), (60, 5, 3, 4)])
def test_hierarchies(tuna, P, Q, rl, rg):
    counts = wl.counts_uniform_elements(P, 500 + P, 40, 4)
    prob = Prob(counts, P + 1, gap=4)
    prob.run(tuna, Q, rl, rg, "P=%d Q=%d rl=%d rg=%d" % (P, Q, rl, rg))
    st = tuna.tuna_get_stats()
    assert (st.Q, st.N, st.fused) == (Q, P // Q, 1)


def test_not_tiny_after_all_and_errors(tuna):
    """More than 1 MiB of payload among few ranks, a T that would not fit the small buffer, and invalid
    counts: the kernel declines and the general path takes over."""
    big = Prob(wl.counts_uniform_bytes(32, 5, 4000), 3)                  # about 2 MiB
    assert big.lay.payload_bytes > 1 << 20
    big.run(tuna, 0, 2, 2, "2 MiB among 32 ranks")
    assert tuna.tuna_get_stats().workspace_bytes != 4 << 20
    counts = np.zeros((64, 64), dtype=np.int32)
    counts[3, 40] = 900 << 10                                            # under 1 MiB, but 64 x 2 x 57 slots of it are not
    counts[5, 6] = 100
    wide = Prob(counts, 4)
    wide.run(tuna, 0, 2, 2, "one 900 KiB block among 64 ranks")
    small = Prob(wl.counts_uniform_bytes(8, 6, 64), 5)
    sc, sd, rc_, rd = small.meta
    bad = rc_.clone()
    bad[0, 3] += 1
    small.recv.fill_(CANARY)
    assert tuna.tuna_alltoallv(small.send, sc, sd, small.recv, bad, rd, 8, 2, 0) == tuna.TUNA_ERR_COUNT_MISMATCH
    neg = sc.clone()
    neg[2, 2] = -4
    assert tuna.tuna_alltoallv(small.send, neg, sd, small.recv, rc_, rd, 8, 2, 0) == tuna.TUNA_ERR_NEGATIVE_COUNT
    torch.cuda.synchronize()
    assert (small.recv.cpu().numpy() == CANARY).all()
    small.run(tuna, 0, 2, 2, "valid again")
