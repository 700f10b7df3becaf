"""Seeded random problems through every way into the library -- immediate calls with per-call options on the
default context and on a context of their own, persistent plans started twice, the call that allocates
nothing -- over random rank counts (up to 1024, several wave units and windows per rank), hierarchies,
radices, modes, T layouts, the staggered schedule, batches of rounds, size distributions (tiny, heavy-tailed,
sparse, equal, large own blocks), alignments, gaps and region orders.  Every result is compared with the CPU
oracle byte for byte, canary gaps included; the send buffer must come back unchanged."""
import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
CANARY = 0xC3
CASES = 200


@pytest.fixture(scope="module")
def tuna():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_02581_amd as t
    t.load()
    return t


def _divisors(P):
    return [q for q in range(2, P) if P % q == 0]


def _counts(rng, P):
    kind = int(rng.integers(0, 8))
    if P > 300:                                                     # many ranks: keep the payload in the tens of MiB
        kind = int(rng.choice([0, 1, 4, 5]))
    if kind == 0:                                                   # tiny blocks: the small-block kernel
        q = int(rng.choice([1, 4, 8]))
        c = rng.integers(0, 64 // q + 1, size=(P, P)) * q
    elif kind == 1:                                                 # a few bytes, any alignment
        c = rng.integers(0, 40, size=(P, P))
    elif kind == 2:                                                 # heavy tail
        c = (rng.pareto(1.1, size=(P, P)) * 24).astype(np.int64).clip(0, 70000 if P <= 200 else 20000)
    elif kind == 3:                                                 # sparse
        c = rng.integers(0, 4000, size=(P, P)) * (rng.random((P, P)) < 0.25)
    elif kind == 4:                                                 # float payloads
        c = rng.integers(0, 900, size=(P, P)) // 4 * 4
    elif kind == 5:                                                 # one size
        c = np.full((P, P), int(rng.choice([16, 256, 260, 1000] if P <= 300 else [16, 68])))
    elif kind == 6:                                                 # around one unit and one window
        c = rng.integers(3800, 4400, size=(P, P)) if P <= 128 else rng.integers(0, 130, size=(P, P))
    else:                                                           # normal, like the benchmark workload
        c = (rng.normal(1024, 256, size=(P, P)).clip(0) // 4 * 4).astype(np.int64)
    c = c.astype(np.int64)
    if rng.random() < 0.2:
        c[int(rng.integers(0, P))] = 0
    if rng.random() < 0.2:
        c[:, int(rng.integers(0, P))] = 0
    if rng.random() < 0.25:                                         # own blocks beyond the unit engine's threshold
        for p in rng.choice(P, size=min(P, 3), replace=False):
            c[p, p] = int(rng.integers(66000, 300000)) // 4 * 4
    return c.astype(np.int32)


def _case(rng):
    P = int(rng.choice([1, 2, 3, 7, 12, 16, 24, 36, 48, 60, 64, 65, 96, 100, 128, 144, 200, 256, 300, 512, 777, 1024]))
    divs = _divisors(P)
    Q = int(rng.choice(divs)) if divs and rng.random() < 0.5 else 0
    N = P // Q if Q else 1
    size_l, size_g = (Q if Q else P), N
    rl = int(rng.choice([0, 2, 3, 4, max(2, int(size_l ** 0.5)), max(2, size_l), size_l + 3]))
    rg = int(rng.choice([0, 2, 3, max(2, int(size_g ** 0.5)), max(2, size_g)]))
    return P, Q, rl, rg


@pytest.mark.parametrize("seed", [0x2411_0258, 0x0258_1124])
def test_random_problems_through_every_entry_point(tuna, seed):
    rng = np.random.default_rng(seed)
    dev = "cuda:0"
    rc, own_ctx = tuna.tuna_ctx_create()
    assert rc == 0
    seen = {"ex": 0, "ctx": 0, "plan": 0, "noalloc": 0, "noalloc_refused": 0, "flat_api": 0}
    try:
        for case in range(CASES):
            P, Q, rl, rg = _case(rng)
            counts = _counts(rng, P)
            lay = wl.make_layout(counts, gap=int(rng.integers(0, 24)),
                                 permute_seed=int(rng.integers(0, 1 << 30)) if rng.random() < 0.5 else None,
                                 align=int(rng.choice([1, 4, 4, 16, 128])))
            host = wl.payload_position_hash(1000 + case, lay.send_bytes)
            want = np.full(lay.recv_bytes, CANARY, dtype=np.uint8)
            assert oracle.alltoallv(host, lay.sendcounts, lay.sdispls, want, lay.recvcounts, lay.rdispls) == 0
            send = torch.from_numpy(host).to(dev)
            recv = torch.full((lay.recv_bytes,), CANARY, dtype=torch.uint8, device=dev)
            meta = [torch.from_numpy(a).to(dev) for a in (lay.sendcounts, lay.sdispls, lay.recvcounts, lay.rdispls)]
            sc, sd, rcn, rd = meta
            o = tuna.tuna_opts_init()
            o.mode = int(rng.choice([tuna.TUNA_MODE_AUTO, tuna.TUNA_MODE_STAGED, tuna.TUNA_MODE_FUSED]))
            o.t_layout = int(rng.choice([tuna.TUNA_T_AUTO, tuna.TUNA_T_EXACT, tuna.TUNA_T_SLOTS]))
            o.staggered = int(Q > 1 and P // Q > 1 and rng.random() < 0.3)
            o.block_count = int(rng.choice([0, 0, 0, 1, 3, 8]))
            o.profile = int(rng.random() < 0.1)
            how = str(rng.choice(["ex", "ex", "ctx", "plan", "noalloc", "flat_api"]))
            what = "case %d: P=%d Q=%d r_l=%d r_g=%d mode=%d t=%d staggered=%d block_count=%d via %s, %d bytes, M=%d" % (
                case, P, Q, rl, rg, o.mode, o.t_layout, o.staggered, o.block_count, how, lay.payload_bytes, int(counts.max()))
            print(what, flush=True)
            checks = 1
            if how in ("ex", "ctx"):
                code = tuna.tuna_alltoallv_ex(own_ctx if how == "ctx" else None, send, sc, sd, recv, rcn, rd, P, Q, rl, rg, o)
            elif how == "plan":
                code, plan = tuna.tuna_alltoallv_init_ex(None, send, sc, sd, recv, rcn, rd, P, Q, rl, rg, o)
                if code == 0:
                    assert tuna.tuna_start(plan) == 0
                    torch.cuda.synchronize()
                    assert np.array_equal(recv.cpu().numpy(), want), what + " (first start)"
                    recv.fill_(CANARY)
                    assert tuna.tuna_start(plan) == 0
                    torch.cuda.synchronize()
                    assert tuna.tuna_plan_free(plan) == 0
            elif how == "noalloc":
                # the process defaults are the options of this entry point
                tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, {0: 2, 1: 0, 2: 1}[o.mode])
                tuna.tuna_set_option(tuna.TUNA_OPT_DENSE_T, o.t_layout)
                tuna.tuna_set_option(tuna.TUNA_OPT_STAGGERED, o.staggered)
                tuna.tuna_set_option(tuna.TUNA_OPT_BLOCK_COUNT, o.block_count)
                try:
                    code = tuna.tuna_alltoallv_noalloc(send, sc, sd, recv, rcn, rd, P, Q, rl, rg)
                finally:
                    tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 2)
                    tuna.tuna_set_option(tuna.TUNA_OPT_DENSE_T, 2)
                    tuna.tuna_set_option(tuna.TUNA_OPT_STAGGERED, 0)
                    tuna.tuna_set_option(tuna.TUNA_OPT_BLOCK_COUNT, 0)
                if code == tuna.TUNA_ERR_NOALLOC_LIMIT:
                    torch.cuda.synchronize()
                    assert int((recv != CANARY).sum()) == 0, what + ": refused, yet bytes moved"
                    seen["noalloc_refused"] += 1
                    checks = 0
            else:
                radix = rl
                code = tuna.tuna_alltoallv(send, sc, sd, recv, rcn, rd, P, radix, Q)
            if checks and code == tuna.TUNA_ERR_NOMEM and o.t_layout == tuna.TUNA_T_SLOTS and how != "flat_api":
                # the paper's slots were asked for by name: P x slots x M bytes can exceed the device (one large
                # block among many ranks); the call must say so and move nothing
                torch.cuda.synchronize()
                assert P * P * int(counts.max()) > (8 << 30), what
                assert int((recv != CANARY).sum()) == 0, what + ": refused, yet bytes moved"
                seen["slots_too_large"] = seen.get("slots_too_large", 0) + 1
                checks = 0
            if checks:
                assert code == 0, what + ": " + tuna.tuna_strerror(code)
                torch.cuda.synchronize()
                got = recv.cpu().numpy()
                if not np.array_equal(got, want):
                    bad = np.flatnonzero(got != want)
                    raise AssertionError("%s: %d bytes differ, first at offset %d" % (what, bad.size, bad[0]))
                assert np.array_equal(send.cpu().numpy(), host), what + ": send buffer modified"
                seen[how] += 1
            del send, recv, meta
    finally:
        assert tuna.tuna_ctx_destroy(own_ctx) == 0
        # the default context's workspace only grows; a case with T in the paper's slots can leave it at 200 GiB
        assert tuna.tuna_release() == 0
        torch.cuda.empty_cache()
    print(seen, flush=True)
    assert all(seen[k] >= 5 for k in ("ex", "ctx", "plan", "noalloc", "flat_api")), seen


def test_random_large_problems_back_to_back(tuna):
    """Problems of 70 to 260 MiB -- where calls with one-kernel phases compute their metadata on a second stream
    while the payload moves -- over random rank counts, hierarchies, radices, size distributions, alignments,
    modes and T layouts; every problem is run twice in a row on two streams of the default context with
    different radices and no host synchronisation between the calls."""
    rng = np.random.default_rng(0x1124_0258)
    dev = "cuda:0"
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for case in range(30):
        P = int(rng.choice([64, 96, 128, 200, 256, 384, 512]))
        mean = (int(rng.integers(70, 260)) << 20) // (P * P)
        kind = int(rng.integers(0, 5))
        if kind == 0:                                               # normal, word-granular
            c = rng.normal(mean, mean / 4, size=(P, P)).clip(0) // 4 * 4
        elif kind == 1:                                             # uniform, word-granular
            c = rng.integers(0, 2 * mean, size=(P, P)) // 4 * 4
        elif kind == 2:                                             # heavy tail
            c = (rng.pareto(1.2, size=(P, P)) * mean / 5).clip(0, 40 * mean) // 4 * 4
        elif kind == 3:                                             # one block in five empty, chunk-granular
            c = rng.integers(0, 2 * mean, size=(P, P)) * (rng.random((P, P)) < 0.8) // 16 * 16
        else:                                                       # byte-granular
            c = rng.integers(0, 2 * mean, size=(P, P))
        c = c.astype(np.int64)
        if rng.random() < 0.3:
            c[int(rng.integers(0, P))] = 0
        divs = _divisors(P)
        Q = int(rng.choice(divs)) if rng.random() < 0.5 else 0
        size_l, size_g = (Q if Q else P), (P // Q if Q else 1)
        rl = int(rng.choice([2, 3, 4, max(2, int(size_l ** 0.5)), max(2, size_l)]))
        rg = int(rng.choice([2, 3, max(2, int(size_g ** 0.5)), max(2, size_g)]))
        lay = wl.make_layout(c.astype(np.int32), gap=int(rng.choice([0, 0, 8])), align=int(rng.choice([1, 4, 16])))
        host = wl.payload_position_hash(100 + case, lay.send_bytes)
        want = np.full(lay.recv_bytes, CANARY, dtype=np.uint8)
        assert oracle.alltoallv(host, lay.sendcounts, lay.sdispls, want, lay.recvcounts, lay.rdispls) == 0
        send = torch.from_numpy(host).to(dev)
        recv = torch.full((lay.recv_bytes,), CANARY, dtype=torch.uint8, device=dev)
        sc, sd, rcn, rd = [torch.from_numpy(a).to(dev) for a in (lay.sendcounts, lay.sdispls, lay.recvcounts, lay.rdispls)]
        o = tuna.tuna_opts_init()
        o.mode = int(rng.choice([tuna.TUNA_MODE_AUTO, tuna.TUNA_MODE_FUSED, tuna.TUNA_MODE_STAGED], p=[0.5, 0.4, 0.1]))
        o.t_layout = int(rng.choice([tuna.TUNA_T_AUTO, tuna.TUNA_T_EXACT]))
        o.staggered = int(Q > 1 and P // Q > 1 and rng.random() < 0.2)
        what = "large case %d: P=%d Q=%d r_l=%d r_g=%d mode=%d t=%d staggered=%d kind=%d, %d MiB" % (
            case, P, Q, rl, rg, o.mode, o.t_layout, o.staggered, kind, lay.payload_bytes >> 20)
        print(what, flush=True)
        torch.cuda.synchronize()
        for k, (a, b) in enumerate([(rl, rg), (max(2, rl // 2), rg)]):
            code = tuna.tuna_alltoallv_ex(None, send, sc, sd, recv, rcn, rd, P, Q, a, b, o, streams[(case + k) % 2])
            assert code == 0, what + ": " + tuna.tuna_strerror(code)
        torch.cuda.synchronize()
        got = recv.cpu().numpy()
        if not np.array_equal(got, want):
            bad = np.flatnonzero(got != want)
            raise AssertionError("%s: %d bytes differ, first at offset %d" % (what, bad.size, bad[0]))
        assert np.array_equal(send.cpu().numpy(), host), what + ": send buffer modified"
        del send, recv, sc, sd, rcn, rd
    assert tuna.tuna_release() == 0
    torch.cuda.empty_cache()
