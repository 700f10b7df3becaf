"""Pins for oracle/tuna_model.py: the closed forms and the per-rank model of the algorithms
are checked against the values the paper prints (tests/golden/), against the bounds it states,
and against the all-to-all definition (the C oracle, itself pinned in test_oracle_pins.py)."""
import numpy as np
import pytest

import oracle
import workloads as wl
from oracle import tuna_model as tm


# ---- closed forms against printed values ------------------------------------------------------
def test_digits_and_rounds_printed_values(golden):
    for P, r, w, K in golden("digits_rounds.txt"):
        assert tm.num_digits(P, r) == w
        assert tm.num_rounds(P, r) == K


def test_temp_slots_printed_values(golden):
    for P, r, B in golden("temp_slots.txt"):
        assert tm.temp_slots(P, r) == B


def test_t_map_printed_values(golden):
    for P, r, o, t in golden("t_map.txt"):
        assert tm.t_index(o, r) == t
    non_direct = [o for o in range(1, 8) if not tm.is_direct(o, 2)]
    assert sorted(tm.t_index(o, 2) for o in non_direct) == [0, 1, 2, 3]


@pytest.mark.parametrize("P", list(range(1, 41)) + [64, 81, 100, 125, 128])
def test_round_and_block_bounds(P):
    """K <= w(r-1); at most r^(w-1) blocks per round; D <= w(r-1)r^(w-1), with equality when
    P = r^w; Bruck (r=2, P=2^k) has K = log2 P; r = P is the linear algorithm with one block per
    round; r > P-2 needs no temporary buffer."""
    for r in range(2, max(P, 2) + 1):
        w = tm.num_digits(P, r)
        rs = tm.rounds(P, r)
        K = len(rs)
        assert r ** w >= P and (w == 0 or r ** (w - 1) < P)
        assert K <= w * (r - 1)
        if P > 1:
            assert K == (w - 1) * (r - 1) + min(r - 1, (P - 1) // r ** (w - 1))
        for x, z in rs:
            n = sum(1 for i in range(P) if tm.digit(i, x, r) == z)
            assert 1 <= n <= r ** (w - 1) if w else True
        D = tm.blocks_sent_per_rank(P, r)
        assert D <= w * (r - 1) * r ** max(w - 1, 0)
        if r ** w == P and w > 0:
            assert D == w * (r - 1) * r ** (w - 1)
        if r == 2 and P & (P - 1) == 0 and P > 1:
            assert K == P.bit_length() - 1
        if r >= P and P > 1:
            assert K == P - 1 and D == P - 1
        if r > P - 2 and P > 1:
            assert tm.temp_slots(P, r) == 0
        # the T map is a bijection of the non-direct indices onto [0, B)
        nd = [o for o in range(1, P) if not tm.is_direct(o, r)]
        assert sorted(tm.t_index(o, r) for o in nd) == list(range(tm.temp_slots(P, r)))


def test_hop_factor_values():
    # fraction of indices with a non-zero digit, summed over digit positions
    assert tm.hop_factor(4096, 2) == 6.0
    assert tm.hop_factor(4096, 8) == 3.5
    assert abs(tm.hop_factor(4096, 64) - 2 * 63 / 64) < 1e-12
    assert abs(tm.hop_factor(4096, 4096) - 4095 / 4096) < 1e-12


# ---- the per-rank model against the definition ------------------------------------------------
def _blocks(P, seed, max_len=7):
    rng = np.random.default_rng(seed)
    S = []
    for p in range(P):
        row = []
        for d in range(P):
            n = int(rng.integers(0, max_len + 1)) if rng.random() > 0.25 else 0
            row.append(bytes([(p * 16 + d) & 0xFF]) + rng.bytes(n - 1) if n else b"")
        S.append(row)
    return S


def _definition(S):
    """recv[j][i] = send[i][j] through the C oracle (blocks laid out densely)."""
    P = len(S)
    counts = np.array([[len(S[i][j]) for j in range(P)] for i in range(P)], dtype=np.int32)
    lay = wl.make_layout(counts)
    send = np.zeros(lay.send_bytes, dtype=np.uint8)
    for i in range(P):
        for j in range(P):
            send[lay.sdispls[i, j]:lay.sdispls[i, j] + counts[i, j]] = np.frombuffer(S[i][j], dtype=np.uint8)
    recv = np.zeros(lay.recv_bytes, dtype=np.uint8)
    assert oracle.alltoallv(send, lay.sendcounts, lay.sdispls, recv, lay.recvcounts, lay.rdispls) == 0
    return [[bytes(recv[lay.rdispls[j, i]:lay.rdispls[j, i] + counts[i, j]]) for i in range(P)]
            for j in range(P)]


@pytest.mark.parametrize("P", list(range(1, 14)) + [16, 17, 27, 33])
def test_flat_model_reaches_the_definition_for_every_radix(P):
    S = _blocks(P, 1000 + P)
    want = _definition(S)
    radices = range(2, max(P, 2) + 1) if P <= 13 else [2, 3, 4, 5, P - 1, P]
    for r in radices:
        for direction in (-1, +1):
            R, st = tm.simulate_tuna(S, r, direction)
            assert R == want, (P, r, direction)
            assert st["K"] == tm.num_rounds(P, r)
            assert all(b == tm.blocks_sent_per_rank(P, r) for b in st["blocks_sent"])
            for rec in st["rounds"]:
                # at most r^x blocks of a round reach their destination
                assert max(rec["finals"]) <= r ** rec["x"]


def test_second_round_of_p8_r2_has_two_finals():
    """Section "Estimating temporary buffer size": 2^1 = 2 blocks arrive in the second round."""
    R, st = tm.simulate_tuna(_blocks(8, 5), 2)
    assert [rec["finals"][0] for rec in st["rounds"]] == [1, 2, 4]
    assert [rec["temps"][0] for rec in st["rounds"]] == [3, 2, 0]


def test_figure1_trace(golden):
    (P, r, sender, receiver), dests, sizes = golden("fig1_trace.txt")
    S = [[bytes([16 * p + d]) * (1 + (3 * p + d) % 4) for d in range(P)] for p in range(P)]
    S[sender][dests[0]] = b"\x12" * sizes[0]
    S[sender][dests[1]] = b"\x10" * sizes[1]
    S[0][3] = b"\x03" * 5
    # the figure's narrative sends towards p + z r^x; Algorithm "TuNA" is its mirror image
    R, st = tm.simulate_tuna(S, r, direction=+1)
    first = st["rounds"][0]
    assert first["distance"] == 1 and first["sendrank"][sender] == receiver
    assert [(sender + i) % P for i in first["send_indices"]] == dests
    assert first["metadata"][sender] == sizes
    # rank 1 got (0->1) as a final block and (0->3) into T in round one ...
    assert first["finals"][1] == 1 and first["temps"][1] == 1
    # ... and forwards (0->3) with rank distance 2 in round two, so it ends at rank 3
    second = st["rounds"][1]
    assert second["distance"] == 2 and second["sendrank"][1] == 3
    assert 5 in second["metadata"][1]
    assert R[3][0] == b"\x03" * 5
    assert R == _definition(S)
    # the mirrored schedule of the printed algorithm moves the same blocks the other way round
    R2, st2 = tm.simulate_tuna(S, r, direction=-1)
    assert R2 == R and st2["rounds"][0]["sendrank"][sender] == (sender - 1) % P
    assert sorted(st2["rounds"][0]["metadata"][sender]) == sorted(sizes)


def test_metadata_follows_the_closed_form():
    """Before digit phase x the block at rank p, index i, started at rank s = p + (i mod r^x) and
    is bound for s - i: its size is sendcounts[s][(s - i) mod P]."""
    for P, r in [(9, 3), (10, 2), (12, 5), (16, 4)]:
        S = _blocks(P, 7 * P + r)
        _, st = tm.simulate_tuna(S, r)
        for rec in st["rounds"]:
            x = rec["x"]
            for p in range(P):
                for i, n in zip(rec["send_indices"], rec["metadata"][p]):
                    s = (p + i % r ** x) % P
                    assert n == len(S[s][(s - i) % P])


# ---- hierarchical ------------------------------------------------------------------------------
def test_figure4_round_counts(golden):
    for P, N, Q, r, local_steps, coalesced, staggered in golden("hier_rounds.txt"):
        S = _blocks(P, 44)
        R, st = tm.simulate_tuna_hier(S, Q, r, N)
        assert len(st["local_rounds"]) == local_steps
        assert len(st["global_rounds"]) == coalesced == N - 1
        assert Q * (N - 1) == staggered
        assert R == _definition(S)
        # after the intra-node phase R holds exactly the blocks from ranks of the own node
        for p in range(P):
            n = p // Q
            for s in range(P):
                have = st["after_local_R"][p][s] is not None
                assert have == (s // Q == n)
                if have:
                    assert st["after_local_R"][p][s] == S[s][p]


def test_staggered_model(golden):
    """Algorithm "Staggered TuNA_l^g": same result, Q (N-1) inter-node rounds of one block each,
    and the same inter-node bytes as the coalesced schedule."""
    for P, N, Q, r, local_steps, coalesced, staggered in golden("hier_rounds.txt"):
        S = _blocks(P, 45)
        R, st = tm.simulate_tuna_hier(S, Q, r, N, staggered=True)
        assert R == _definition(S)
        assert len(st["global_rounds"]) == staggered == Q * (N - 1)
        _, co = tm.simulate_tuna_hier(S, Q, r, N)
        assert st["global_phase_bytes"][0] == sum(co["global_phase_bytes"].values())
    for Q, N in [(2, 2), (3, 4), (4, 3)]:
        S = _blocks(Q * N, 46)
        R, _ = tm.simulate_tuna_hier(S, Q, 2, N, staggered=True)
        assert R == _definition(S)


@pytest.mark.parametrize("Q,N", [(1, 6), (6, 1), (2, 3), (3, 2), (4, 4), (5, 3), (3, 7), (8, 2)])
def test_hier_model_reaches_the_definition(Q, N):
    P = Q * N
    S = _blocks(P, 300 + P)
    want = _definition(S)
    for rl in sorted({2, 3, max(Q, 2)}):
        for rg in sorted({2, 3, max(N, 2)}):
            R, _ = tm.simulate_tuna_hier(S, Q, rl, rg)
            assert R == want, (Q, N, rl, rg)


def test_hier_equals_flat():
    S = _blocks(12, 9)
    flat, _ = tm.simulate_tuna(S, 3)
    hier, _ = tm.simulate_tuna_hier(S, 4, 2, 3)
    assert flat == hier


# ---- planted mistakes in the model's readings must be caught ----------------------------------
def test_ceil_log_reading_of_the_t_map_is_rejected(monkeypatch):
    """dx = ceil(log_r o) as printed gives a negative slot for P=8, r=3, o=4; floor is the reading."""
    def t_ceil(o, r):
        dx, v = 0, 1
        while v < o:
            v *= r
            dx += 1
        return o - 1 - dx * (r - 1) - o // v
    assert t_ceil(4, 3) < 0
    assert tm.t_index(4, 3) == 0


def test_printed_final_test_is_rejected():
    """Reading the receive test as i % r^x == 0 (as printed) sends P=8, r=2, round-two block i=2
    to R but also i=6, which still has to travel: the model with that test loses blocks."""
    P, r, x = 8, 2, 1
    printed = [i for i in range(P) if tm.digit(i, x, r) == 1 and i % r ** x == 0]
    reading = [i for i in range(P) if tm.digit(i, x, r) == 1 and i < r ** (x + 1)]
    assert printed == [2, 6] and reading == [2, 3]
    assert len(reading) == r ** x          # "2^1 = 2 green data blocks in the second round"
    assert tm.nonzero_digits(6, r) == 2    # index 6 has a higher digit left: not final
