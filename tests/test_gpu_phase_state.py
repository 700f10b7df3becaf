"""The device's block-size matrix after every digit phase against its closed form (Section "Two-phase
communication": block sizes travel ahead of the blocks; Algorithm "TuNA", line 14; Algorithm "Coalesced
TuNA_l^g" for the hierarchy).

Rank p = (n, g) indexes the blocks it holds by their distance pair (j, l) (slot index j Q + l): the block
is bound for rank ((n - j) mod N, (g - l) mod Q).  After local phase x every block has made the hops of
its local digits 0..x, i.e. it has come from the rank that lies (l mod r_l^(x+1)) local places above its
holder; after global phase x (all local digits done) also (j mod r_g^(x+1)) nodes above.  So the size the
holder's matrix must show is that of the block this source sends to that destination:
    size[p][(j, l)] = sendcounts[s][d],   s = ((n + dj) mod N, (g + dl) mod Q),   d = s - (j, l),
with dl = l mod r_l^(x+1) (all of l in the global phases) and dj = j mod r_g^(x+1) (0 in the local phases).
The matrices are read back through tuna_debug_phase_sizes: they are the device's own, written by the
kernels of the metadata exchange that every call runs."""
import numpy as np
import pytest

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


def expected_sizes(counts, Q, rl_pow, rg_pow):
    """Closed form above for all ranks and slot indices; rl_pow = r_l^(x+1) of the last local phase done (or
    a value >= Q when all are done), rg_pow likewise for the global phases (1 = none done)."""
    P = counts.shape[0]
    Q = Q if Q else P
    N = P // Q
    p = np.arange(P)[:, None]
    e = np.arange(P)[None, :]
    n, g = p // Q, p % Q
    j, l = e // Q, e % Q
    sn, sg = (n + j % rg_pow) % N, (g + l % rl_pow) % Q
    dn, dg = (sn - j) % N, (sg - l) % Q
    return counts[sn * Q + sg, dn * Q + dg]


@pytest.mark.parametrize("P,Q,rl,rg", [(24, 0, 2, 2), (24, 0, 5, 5), (24, 0, 24, 24), (200, 0, 2, 2), (200, 0, 7, 7),
                                        (24, 4, 2, 3), (24, 4, 4, 6), (200, 10, 3, 4), (300, 20, 2, 15)])
@pytest.mark.parametrize("fused", [0, 1])
def test_size_matrix_after_every_phase(tuna, P, Q, rl, rg, fused):
    counts = wl.counts_uniform_bytes(P, 1000 + P + rl, 50000)      # distinct sizes: a wrong source shows
    counts[counts % 7 == 0] = 0
    lay = wl.make_layout(counts)
    dev = "cuda:0"
    send = torch.zeros(max(lay.send_bytes, 16), dtype=torch.uint8, device=dev)
    recv = torch.zeros(max(lay.recv_bytes, 16), dtype=torch.uint8, device=dev)
    d = [torch.from_numpy(a).to(dev) for a in (lay.sendcounts, lay.sdispls, lay.recvcounts, lay.rdispls)]
    rc, info = tuna.tuna_plan_info(P, Q, rl, rg)
    assert rc == 0
    tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, fused)
    try:
        rc, sizes = tuna.tuna_debug_phase_sizes(send, d[0], d[1], recv, d[2], d[3], P, Q, rl, rg, info.n_phases)
    finally:
        tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 2)
    assert rc == 0, tuna.tuna_strerror(rc)
    Qe = Q if Q else P
    # the initial rotation (Algorithm "TuNA", lines 4-5): index only, nothing has moved
    assert np.array_equal(sizes[0], expected_sizes(counts, Q, 1, 1)), "initial rotation"
    rl_pow, rg_pow = 1, 1
    for ph in range(info.n_phases):
        if ph < info.w_local:
            rl_pow *= info.local_radix
        else:
            rl_pow = max(rl_pow, Qe)            # all local digits are done
            rg_pow *= info.global_radix
        want = expected_sizes(counts, Q, rl_pow, rg_pow)
        bad = np.argwhere(sizes[ph + 1] != want)
        assert bad.size == 0, "phase %d: %d entries differ, first at rank %d slot %d" % (ph, len(bad), bad[0][0], bad[0][1])
    # after the last phase every block is where it is bound for: the matrix is the receive counts by source distance
    p = np.arange(P)[:, None]
    e = np.arange(P)[None, :]
    N = P // Qe
    src = ((p // Qe + e // Qe) % N) * Qe + (p % Qe + e % Qe) % Qe
    assert np.array_equal(sizes[info.n_phases], lay.recvcounts[p, src])
