"""Host logic of the GPU library, checked without a GPU: the C ABI loads and exports every
symbol the header declares, the schedule (w, K, B, D, T map) agrees with the oracle-side model
and the paper's printed values, and the per-phase segment tables -- which slot every moving
block is read from and stored to -- carry every block to its destination when replayed on the
host with plain Python containers."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2411_02581_amd as tuna
import workloads as wl
from oracle import tuna_model as tm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "tuna.h")).read()
    declared = set(re.findall(r"^(?:int|const char\*)\s+(tuna_\w+)\s*\(", header, flags=re.M))
    assert declared == set(tuna.EXPORTS)
    lib = ctypes.CDLL(tuna.library_path())
    for name in declared:
        assert hasattr(lib, name), name
    assert tuna.tuna_version() >= 100
    assert "transpose" in tuna.tuna_strerror(tuna.TUNA_ERR_COUNT_MISMATCH)


def test_struct_sizes_match_the_header():
    # 16 int32 + 6 int64 + 4 float + 64 phases of (4 int32 + 3 int64 + 4 float)
    assert ctypes.sizeof(tuna.tuna_phase_stats_t) == 56
    assert ctypes.sizeof(tuna.tuna_stats_t) == 64 + 48 + 16 + 64 * 56
    assert ctypes.sizeof(tuna.tuna_plan_info_t) == 48 + 16


def test_plan_matches_printed_values(golden):
    for P, r, w, K in golden("digits_rounds.txt"):
        rc, info = tuna.tuna_plan_info(P, 0, r, r)
        assert rc == 0 and (info.w_local, info.K_local) == (w, K)
    for P, r, B in golden("temp_slots.txt"):
        rc, info = tuna.tuna_plan_info(P, 0, r, r)
        assert rc == 0 and info.B_local == B and info.temp_slots_per_rank == B
    for P, r, o, t in golden("t_map.txt"):
        assert tuna.tuna_t_index(o, r) == t
    for P, N, Q, r, local_steps, coalesced, _ in golden("hier_rounds.txt"):
        rc, info = tuna.tuna_plan_info(P, Q, r, N)
        assert rc == 0 and (info.K_local, info.K_global) == (local_steps, coalesced)


@pytest.mark.parametrize("P", [1, 2, 3, 5, 8, 9, 16, 27, 30, 64, 100])
def test_plan_matches_the_model(P):
    for r in sorted({2, 3, 4, 7, max(P - 1, 2), max(P, 2), P + 5}):
        rc, info = tuna.tuna_plan_info(P, 0, r, r)
        assert rc == 0
        rr = min(r, max(P, 2))
        assert info.local_radix == rr or P < 2
        assert info.w_local == tm.num_digits(P, rr)
        assert info.K_local == tm.num_rounds(P, rr)
        assert info.B_local == (tm.temp_slots(P, rr) if P > 1 else 0)
        assert info.blocks_sent_per_rank == tm.blocks_sent_per_rank(P, rr)
        assert info.n_phases == info.w_local and info.w_global == 0
        for o in range(1, P):
            want = -1 if tm.is_direct(o, rr) else tm.t_index(o, rr)
            assert tuna.tuna_t_index(o, rr) == want


def test_configured_schedules():
    # the schedules of the five benchmark configurations
    rc, i = tuna.tuna_plan_info(4096, 0, 2, 2)
    assert (i.w_local, i.K_local, i.B_local) == (12, 12, 4083)
    rc, i = tuna.tuna_plan_info(4096, 0, 8, 8)
    assert (i.w_local, i.K_local, i.B_local) == (4, 28, 4067)
    rc, i = tuna.tuna_plan_info(4096, 0, 64, 64)
    assert (i.w_local, i.K_local, i.B_local) == (2, 126, 3969)
    rc, i = tuna.tuna_plan_info(4096, 0, 4096, 4096)
    assert (i.w_local, i.K_local, i.B_local) == (1, 4095, 0)
    rc, i = tuna.tuna_plan_info(1024, 16, 4, 8)
    assert (i.Q, i.N, i.w_local, i.K_local, i.w_global, i.K_global) == (16, 64, 2, 6, 2, 14)
    rc, i = tuna.tuna_plan_info(2048, 32, 2048, 2048)
    assert (i.local_radix, i.global_radix, i.K_local, i.K_global) == (32, 64, 31, 63)


def test_argument_errors_without_a_gpu():
    assert tuna.tuna_plan_info(12, 5, 2, 2)[0] == tuna.TUNA_ERR_ARG      # 5 does not divide 12
    assert tuna.tuna_plan_info(0, 0, 2, 2)[0] == tuna.TUNA_ERR_ARG
    assert tuna.tuna_plan_info(8, 0, 1, 2)[0] == tuna.TUNA_ERR_ARG
    assert tuna.tuna_plan_info(1 << 20, 0, 2, 2)[0] == tuna.TUNA_ERR_TOO_LARGE
    assert tuna.tuna_plan_phase(8, 0, 2, 2, 3)[0] == tuna.TUNA_ERR_ARG    # only 3 phases


# ---- replay of the segment tables on the host -------------------------------------------------
def _replay(counts, Q, rl, rg, fused=False):
    """Moves blocks exactly as the tables say: per phase, every rank reads each moving block from
    the send buffer (source slot -1) or its T slot, the partner at distance z*r^x (downwards, as
    in Algorithm "TuNA") stores it to the receive buffer (destination slot -1) or its T slot.
    Alongside, the exact-size form of T is replayed: a block stored into T in phase f as that
    phase's k-th moving block must be what the later phase that forwards it finds under (f, k)."""
    P = counts.shape[0]
    rc, info = tuna.tuna_plan_info(P, Q, rl, rg)
    assert rc == 0
    Q, N = info.Q, info.N                               # ranks_per_node 0, 1 or P means flat
    S = [[bytes([(7 * i + j) & 0xFF]) * int(counts[i, j]) + b"" for j in range(P)] for i in range(P)]
    R = [[None] * P for _ in range(P)]
    T = [dict() for _ in range(P)]
    arena = [dict() for _ in range(P)]
    for p in range(P):
        R[p][p] = S[p][p]
    per_phase_bytes = []
    for ph in range(info.n_phases):
        rc, hdr, seg = tuna.tuna_plan_phase(P, Q, rl, rg, ph)
        assert rc == 0
        dim, x, r, nz, nseg, rx = (int(v) for v in hdr)
        assert rx == r ** x and nseg == seg.shape[0]
        rc, sources = tuna.tuna_plan_phase_sources(P, Q, rl, rg, ph, nseg)
        assert rc == 0
        # message order: z ascending, then e ascending; e = j*Q + l
        keys = [(int(s[3]), int(s[0])) for s in seg]
        assert keys == sorted(keys) and len(set(keys)) == len(keys)
        assert all(int(s[0]) == int(s[1]) * Q + int(s[2]) for s in seg)
        assert set(int(s[3]) for s in seg) == set(range(1, nz + 1))
        moved = []
        nbytes = 0
        reads = [set() for _ in range(P)]
        for p in range(P):
            n, g = divmod(p, Q)
            for k, (e, j, l, z, src_slot, dst_slot) in enumerate(seg.tolist()):
                coord = l if dim == 0 else j
                assert (coord // rx) % r == z
                if src_slot < 0:
                    blk = S[p][((n - j) % N) * Q + (g - l) % Q]
                    assert tuple(sources[k]) == (-1, 0)
                else:
                    blk = T[p].pop(src_slot)          # a slot is read exactly once after a store
                    reads[p].add(src_slot)
                    f, kk = (int(v) for v in sources[k])
                    assert 0 <= f < ph and arena[p].pop((f, kk)) == (e, blk)
                if dim == 0:
                    q = n * Q + (g - z * rx) % Q
                else:
                    q = ((n - z * rx) % N) * Q + g
                moved.append((q, j, l, dst_slot, blk, k))
                nbytes += len(blk)
        for q, j, l, dst_slot, blk, k in moved:       # every rank packed before anyone unpacks
            nq, gq = divmod(q, Q)
            if dst_slot < 0:
                src = ((nq + j) % N) * Q + (gq + l) % Q
                assert R[q][src] is None
                R[q][src] = blk
            else:
                assert 0 <= dst_slot < info.temp_slots_per_rank
                assert dst_slot not in T[q]           # no live block is overwritten
                if fused:                             # one kernel reads and writes: never the same slot
                    assert dst_slot not in reads[q]
                T[q][dst_slot] = blk
                arena[q][(ph, k)] = (j * Q + l, blk)
        per_phase_bytes.append(nbytes)
    assert all(len(t) == 0 for t in T)                # nothing is left behind in T
    assert all(len(t) == 0 for t in arena)
    return R, S, per_phase_bytes


def _want(S):
    P = len(S)
    return [[S[i][j] for i in range(P)] for j in range(P)]


@pytest.mark.parametrize("P", list(range(1, 13)) + [16, 17, 25, 33])
def test_flat_tables_deliver_every_block(P):
    counts = (wl.make_counts(2, P) % 7).astype(np.int32)
    radices = range(2, max(P, 2) + 1) if P <= 12 else [2, 3, 4, 5, P - 1, P]
    for r in radices:
        R, S, _ = _replay(counts, P, r, r)
        assert R == _want(S), (P, r)


@pytest.mark.parametrize("Q,N", [(1, 5), (2, 2), (2, 3), (3, 2), (4, 4), (5, 3), (3, 7), (8, 2), (4, 9)])
def test_hier_tables_deliver_every_block(Q, N):
    P = Q * N
    counts = (wl.make_counts(3, P) % 5).astype(np.int32)
    for rl in sorted({2, 3, max(Q, 2)}):
        for rg in sorted({2, 3, max(N, 2)}):
            R, S, _ = _replay(counts, Q, rl, rg)
            assert R == _want(S), (Q, N, rl, rg)


def test_phase_bytes_follow_the_model():
    """Payload bytes per digit phase of the table replay equal those of the per-rank model."""
    P, r = 12, 3
    counts = (wl.make_counts(2, P) % 9).astype(np.int32)
    R, S, per_phase = _replay(counts, P, r, r)
    _, st = tm.simulate_tuna(S, r)
    assert per_phase == [st["phase_bytes"][x] for x in range(tm.num_digits(P, r))]
    Q, N, rl, rg = 4, 3, 2, 2
    R, S, per_phase = _replay(counts, Q, rl, rg)
    _, st = tm.simulate_tuna_hier(S, Q, rl, rg)
    wlc = tm.num_digits(Q, rl)
    assert per_phase[:wlc] == [st["local_phase_bytes"][x] for x in range(wlc)]
    assert per_phase[wlc:] == [st["global_phase_bytes"][x] for x in range(tm.num_digits(N, rg))]


@pytest.mark.parametrize("Q,N", [(9, 1), (16, 1), (27, 1), (2, 3), (4, 4), (5, 3), (3, 7), (4, 9)])
def test_fused_tables_never_read_and_write_a_slot_in_one_phase(Q, N):
    """With the fused rounds T is laid out twice and the copy is the parity of the hop count:
    within a phase no rank's slot is both read (forwarded block) and written (arriving block)."""
    P = Q * N
    counts = (wl.make_counts(2, P) % 6).astype(np.int32)
    assert tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 1) == 0
    try:
        for rl in sorted({2, 3, max(Q, 2)}):
            for rg in sorted({2, 3, max(N, 2)}):
                rc, fused_info = tuna.tuna_plan_info(P, Q, rl, rg)
                R, S, _ = _replay(counts, Q, rl, rg, fused=True)
                assert R == _want(S), (Q, N, rl, rg)
    finally:
        tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 2)
    rc, plain = tuna.tuna_plan_info(P, Q, 2, 2)
    tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 1)
    rc, fused_info = tuna.tuna_plan_info(P, Q, 2, 2)
    tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 2)
    assert fused_info.temp_slots_per_rank == 2 * plain.temp_slots_per_rank


def test_staggered_option_schedule(golden):
    """Staggered inter-node schedule: Q (N-1) rounds of one block, global radix N; the tables are
    those of the linear global phase, in which every arrival is final."""
    tuna.tuna_set_option(tuna.TUNA_OPT_STAGGERED, 1)
    try:
        for P, N, Q, r, local_steps, coalesced, staggered in golden("hier_rounds.txt"):
            rc, info = tuna.tuna_plan_info(P, Q, r, 2)
            assert rc == 0 and info.global_radix == N and info.K_global == staggered and info.K_local == local_steps
            rc, hdr, seg = tuna.tuna_plan_phase(P, Q, r, 2, info.n_phases - 1)
            assert rc == 0 and hdr[0] == 1 and (seg[:, 5] == -1).all()
        rc, info = tuna.tuna_plan_info(16, 0, 2, 2)      # flat calls are unaffected
        assert info.K_global == 0 and info.K_local == 4
    finally:
        tuna.tuna_set_option(tuna.TUNA_OPT_STAGGERED, 0)


def test_select_model():
    """One HBM has no per-round latency: with the built-in constants (no GPU here) the model's minimiser
    is the linear schedule with one-kernel hops for every payload, the predicted time of configuration 4
    at r = P is what its bytes cost at about 5.3 TB/s plus under a millisecond, three stages cost three
    times the bytes, and emptier slots cost more than exact-size T."""
    big = 16 << 30
    rc, ch = tuna.tuna_select(4096, 0, big, 2412)
    assert rc == 0 and (ch.local_radix, ch.mode, ch.t_layout, ch.calibrated) == (4096, tuna.TUNA_MODE_FUSED, tuna.TUNA_T_EXACT, 0)
    assert 2 * big * 4095 / 4096 / 5.5e12 * 1e3 < ch.predicted_ms < 2 * big / 5.0e12 * 1e3 + 1.0
    rc, ms_staged = tuna.tuna_predict_ms(4096, 0, 4096, 4096, tuna.TUNA_MODE_STAGED, tuna.TUNA_T_EXACT, big, 2412)
    assert rc == 0 and 2.0 < ms_staged / ch.predicted_ms < 3.0
    rc, ms_r2 = tuna.tuna_predict_ms(4096, 0, 2, 2, tuna.TUNA_MODE_FUSED, tuna.TUNA_T_EXACT, big, 2412)
    rc, ms_r2_slots = tuna.tuna_predict_ms(4096, 0, 2, 2, tuna.TUNA_MODE_FUSED, tuna.TUNA_T_SLOTS, big, 2412)
    assert ms_r2 > 4 * ch.predicted_ms and 1.05 < ms_r2_slots / ms_r2 < 1.6
    rc, ms_full_slots = tuna.tuna_predict_ms(2048, 32, 2, 2, tuna.TUNA_MODE_FUSED, tuna.TUNA_T_SLOTS, 1 << 30, 256)
    rc, ms_full_exact = tuna.tuna_predict_ms(2048, 32, 2, 2, tuna.TUNA_MODE_FUSED, tuna.TUNA_T_EXACT, 1 << 30, 256)
    assert ms_full_slots == ms_full_exact                      # full slots are as dense as exact size
    rc, ch = tuna.tuna_select(1024, 16, 1 << 30, 16384)
    assert rc == 0 and (ch.local_radix, ch.global_radix, ch.mode) == (16, 64, tuna.TUNA_MODE_FUSED)
    rc, small = tuna.tuna_select(256, 0, 1 << 10)
    assert rc == 0 and small.local_radix == 256 and small.predicted_ms < 0.2
    rc, auto = tuna.tuna_predict_ms(256, 0, tuna.TUNA_RADIX_AUTO, tuna.TUNA_RADIX_AUTO, tuna.TUNA_MODE_AUTO, tuna.TUNA_T_AUTO, 1 << 10)
    assert rc == 0 and auto == small.predicted_ms
    assert tuna.tuna_select(12, 5, 100)[0] == tuna.TUNA_ERR_ARG
    assert tuna.tuna_predict_ms(12, 0, 1, 2, 0, 0, 100)[0] == tuna.TUNA_ERR_ARG
    rc, odd = tuna.tuna_predict_ms(256, 0, 256, 256, tuna.TUNA_MODE_FUSED, tuna.TUNA_T_EXACT, 32 << 20, 1024, 1)
    rc, even = tuna.tuna_predict_ms(256, 0, 256, 256, tuna.TUNA_MODE_FUSED, tuna.TUNA_T_EXACT, 32 << 20, 1024, 4)
    assert odd > even                                          # byte-granular kernels cost more per byte
    rc, lines = tuna.tuna_predict_ms(256, 0, 256, 256, tuna.TUNA_MODE_FUSED, tuna.TUNA_T_EXACT, 32 << 20, 1024, 128)
    assert even > lines > 0.5 * even                           # whole-line blocks cost less per byte and per block
    assert tuna.tuna_predict_ms(12, 0, 2, 2, 5, 0, 100)[0] == tuna.TUNA_ERR_ARG
    # the constants are readable; blocks of at most 64 bytes are priced by their own constant in one-kernel mode
    rc, cf = tuna.tuna_model_constants(tuna.TUNA_MODE_FUSED)
    rc2, cs = tuna.tuna_model_constants(tuna.TUNA_MODE_STAGED)
    assert rc == 0 and rc2 == 0 and len(cf) == 10 and all(v >= 0 for v in cf + cs) and 0.5 <= cf[9] <= 1 and 0.5 <= cs[9] <= 1
    assert cs[3] > 2 * cf[3] and cs[5] == 0 and cs[6] == 0 and 0 < cf[5] < cf[4] and cf[6] > cf[3]
    assert tuna.tuna_model_constants(tuna.TUNA_MODE_AUTO)[0] == tuna.TUNA_ERR_ARG
    P, payload = 2048, 32 << 20
    rc, tiny_blocks = tuna.tuna_predict_ms(P, 0, P, P, tuna.TUNA_MODE_FUSED, tuna.TUNA_T_EXACT, payload, 16, 4)
    rc, larger_blocks = tuna.tuna_predict_ms(P, 0, P, P, tuna.TUNA_MODE_FUSED, tuna.TUNA_T_EXACT, payload, 80, 4)
    moving, gb = P * (P - 1) / 1e6, payload * (P - 1) / P / 1e9
    assert abs((larger_blocks - tiny_blocks) - ((cf[4] - cf[5]) * moving + (cf[3] - cf[6]) * gb)) < 1e-9


def test_random_schedules_deliver_every_block():
    """Property test over random (Q, N, r_l, r_g): the tables always deliver every block, in both the
    three-stage and the fused layout of T."""
    from hypothesis import given, settings, strategies as st

    @settings(max_examples=40, deadline=None)
    @given(st.integers(1, 7), st.integers(1, 7), st.integers(2, 9), st.integers(2, 9), st.booleans(),
           st.integers(0, 1000))
    def prop(Q, N, rl, rg, fused, seed):
        P = Q * N
        counts = (wl.counts_uniform_bytes(P, seed, 5)).astype(np.int32)
        tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 1 if fused else 0)
        try:
            R, S, _ = _replay(counts, Q, rl, rg, fused=fused)
        finally:
            tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 2)
        assert R == _want(S)
    prop()


def test_compute_entry_points_fail_loudly_without_a_gpu():
    """No CPU fallback: on a machine without a HIP device every compute entry point returns
    TUNA_ERR_HIP (the host-only schedule functions keep working)."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    lib = tuna.load()
    rc = lib.tuna_alltoallv(1, 1, 1, 1, 1, 1, 4, 2, 0, None)           # never dereferenced: no device
    assert rc == tuna.TUNA_ERR_HIP
    import ctypes
    plan = ctypes.c_void_p(None)
    assert lib.tuna_alltoallv_init(1, 1, 1, 1, 1, 1, 4, 0, 2, 2, None, ctypes.byref(plan)) == tuna.TUNA_ERR_HIP
    assert lib.tuna_plain_copy(16, 32, 16, None) == tuna.TUNA_ERR_HIP
    out = ctypes.c_size_t(0)
    assert lib.tuna_workspace_bytes(1, 4, 0, 2, 2, ctypes.byref(out)) == tuna.TUNA_ERR_HIP
    assert tuna.tuna_plan_info(4, 0, 2, 2)[0] == 0


@pytest.mark.parametrize("P,Q,rl,rg", [(16, 0, 2, 2), (27, 0, 3, 3), (30, 0, 4, 4), (24, 4, 2, 2), (60, 5, 3, 4),
                                        (64, 8, 8, 8), (35, 7, 2, 5)])
def test_exact_size_of_t_counts_hops_minus_one(P, Q, rl, rg):
    """Exact-size T is allocated from sum over blocks of chunks * (hops - 1), hops = non-zero digits
    of the distance pair: every slot index must be stored into T in exactly that many phases."""
    rc, info = tuna.tuna_plan_info(P, Q, rl, rg)
    assert rc == 0
    stores = np.zeros(P, dtype=np.int64)
    for ph in range(info.n_phases):
        rc, hdr, seg = tuna.tuna_plan_phase(P, Q, rl, rg, ph)
        assert rc == 0
        for e, j, l, z, src_slot, dst_slot in seg.tolist():
            stores[e] += dst_slot >= 0
    for e in range(P):
        j, l = divmod(e, info.Q)
        hops = tm.nonzero_digits(l, info.local_radix) + tm.nonzero_digits(j, info.global_radix)
        assert stores[e] == max(hops - 1, 0), (e, j, l)
