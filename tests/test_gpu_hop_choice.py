"""Which kernel a one-kernel phase runs (Algorithm "TuNA", lines 15-20 as one hop): the destination-tiled hop
where the library's rule says it pays -- dense receive regions, data at least word-granular, all rounds of a
phase at once; for a schedule's last phase, whose blocks all go into R, blocks that are mostly interior (mean of
700 bytes or more, at most a quarter of them under 256 bytes); for the phases before it, which store whole
chunks into T, a mean block of 512 bytes or more -- and the copy engine's hop everywhere else.  With profiling
on, a phase's tiled hop is timed as its unpack time and the engine's hop as its pack time, which is how the test
tells them apart; every case is also compared with the CPU oracle byte for byte."""
import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
CANARY = 0x5A
P = 96


@pytest.fixture(scope="module")
def tuna():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_02581_amd as t
    t.load()
    return t


def _normal(seed=11):
    return wl.counts_normal(P, seed, 1024.0, 256.0, 4)


def _mostly_short():
    c = wl.counts_normal(P, 13, 1400.0, 256.0, 4).copy()
    rng = np.random.default_rng(5)
    c[rng.random((P, P)) < 0.4] = 64              # two blocks in five under 256 bytes; the mean stays above 700
    assert c.mean() > 800
    return c


CASES = {
    # name: (counts, layout arguments, options, (tiled expected in the phases before the last, in the last)); None: three stages
    "normal 1 KiB, dense": (_normal, {}, {}, (True, True)),
    "normal 1 KiB, chunk-granular": (lambda: _normal() // 16 * 16, {"align": 16}, {}, (True, True)),
    "gaps between the blocks of R": (_normal, {"gap": 8}, {}, (False, False)),
    "byte-granular sizes": (lambda: _normal() + 1, {}, {}, (False, False)),
    "Zipf sizes (most blocks tiny, mean 800 bytes)": (lambda: wl.counts_zipf(P, 12, 1.2, 16384, 4), {}, {}, (True, False)),
    "mean block of 516 bytes": (lambda: np.full((P, P), 516, dtype=np.int32), {}, {}, (True, False)),
    "mean block of 260 bytes": (lambda: np.full((P, P), 260, dtype=np.int32), {}, {}, (False, False)),
    "two blocks in five short": (_mostly_short, {}, {}, (True, False)),
    "rounds in batches": (_normal, {}, {"block_count": 3}, (False, False)),
    "three-stage phases": (_normal, {}, {"mode": "staged"}, None),
}


@pytest.mark.parametrize("name", sorted(CASES))
@pytest.mark.parametrize("radix", [4, P])
def test_which_hop_runs(tuna, name, radix):
    make, lay_args, opts, tiled = CASES[name]
    counts = np.ascontiguousarray(make(), dtype=np.int32)
    lay = wl.make_layout(counts, **lay_args)
    host = wl.payload_position_hash(21, lay.send_bytes)
    want = np.full(lay.recv_bytes, CANARY, dtype=np.uint8)
    assert oracle.alltoallv(host, lay.sendcounts, lay.sdispls, want, lay.recvcounts, lay.rdispls) == 0
    dev = "cuda:0"
    send = torch.from_numpy(host).to(dev)
    recv = torch.full((lay.recv_bytes,), CANARY, dtype=torch.uint8, device=dev)
    meta = [torch.from_numpy(a).to(dev) for a in (lay.sendcounts, lay.sdispls, lay.recvcounts, lay.rdispls)]
    o = tuna.tuna_opts_init()
    o.profile = 1
    o.t_layout = tuna.TUNA_T_EXACT
    o.mode = tuna.TUNA_MODE_STAGED if opts.get("mode") == "staged" else tuna.TUNA_MODE_FUSED
    o.block_count = opts.get("block_count", 0)
    print("case %s, radix %d" % (name, radix), flush=True)
    rc = tuna.tuna_alltoallv_ex(None, send, meta[0], meta[1], recv, meta[2], meta[3], P, 0, radix, radix, o)
    assert rc == 0, tuna.tuna_strerror(rc)
    torch.cuda.synchronize()
    assert np.array_equal(recv.cpu().numpy(), want), name
    st = tuna.tuna_get_stats()
    assert st.n_phases == (1 if radix == P else 4)
    for x in range(st.n_phases):
        ph = st.phase[x]
        if tiled is None:                                   # pack, exchange and unpack all ran
            assert ph.ms_pack > 0 and ph.ms_exchange > 0 and ph.ms_unpack > 0, (name, x)
        elif tiled[1 if x + 1 == st.n_phases else 0]:
            assert ph.ms_unpack > 0 and ph.ms_pack == 0 and ph.ms_exchange == 0, (name, x)
        else:
            assert ph.ms_pack > 0 and ph.ms_unpack == 0 and ph.ms_exchange == 0, (name, x)
