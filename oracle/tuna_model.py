"""TEST INFRASTRUCTURE -- not part of the product path.

Slow, per-rank model of the tunable-radix non-uniform all-to-all (Section "Tunable-radix
Non-uniform All-to-all", Algorithm "TuNA") and of its hierarchical coalesced variant
(Section "Hierarchical Tunable Non-uniform All-to-all", Algorithm "Coalesced TuNA_l^g"),
written in the paper's notation: P ranks, radix r, w digits, round (x, z), rotation array I,
send-index list sd, sendrank / recvrank, metadata then data, receive into R or T, T-slot
index t = o - 1 - dx(r-1) - dz.  Every rank is a Python object that only sees its own
buffers and the messages it receives; messages are (metadata, data) pairs.

Use: pins on the round structure (K, B, D, finals per round, the T map, the worked
examples of Figures 1, 2 and 4) and per-phase byte counts that the GPU library's statistics
are compared against.  The pass/fail oracle for payload bytes is the direct transpose in
alltoallv_oracle.c; this model must itself reproduce that transpose, which is one of its pins.

Readings taken where the printed algorithms are garbled:
half-open loop bounds (0 <= x < w, 1 <= z < r, 0 <= i < P) and rounds with z*r^x >= P skipped;
"x-th digit is 1" means "equals z"; a received block with index i is final iff i < r^(x+1)
(it has no higher non-zero digit), which gives the at-most r^x finals per round that
Section "Estimating temporary buffer size" states; dx = floor(log_r o), dz = floor(o / r^dx).
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple


# ----------------------------------------------------------------------------
# closed forms (Section "Tunable Radix"; Section "Estimating temporary buffer size")
# ----------------------------------------------------------------------------
def num_digits(P: int, r: int) -> int:
    """w = ceil(log_r P): the smallest w with r^w >= P, by repeated multiplication."""
    assert P >= 1 and r >= 2
    w, v = 0, 1
    while v < P:
        v *= r
        w += 1
    return w


def digit(i: int, x: int, r: int) -> int:
    """Digit x of i written in base r."""
    return (i // r ** x) % r


def rounds(P: int, r: int) -> List[Tuple[int, int]]:
    """The point-to-point rounds (x, z), in the order of the two loops of Algorithm "TuNA";
    a round whose rank distance z*r^x is not below P would carry no block and is skipped."""
    w = num_digits(P, r)
    return [(x, z) for x in range(w) for z in range(1, r) if z * r ** x < P]


def num_rounds(P: int, r: int) -> int:
    """K, at most w(r-1)."""
    return len(rounds(P, r))


def temp_slots(P: int, r: int) -> int:
    """B = P - (K + 1): one block is the rank's own, K blocks are direct."""
    return P - (num_rounds(P, r) + 1)


def nonzero_digits(i: int, r: int) -> int:
    n = 0
    while i:
        n += 1 if i % r else 0
        i //= r
    return n


def is_direct(o: int, r: int) -> bool:
    """A direct block has exactly one non-zero digit: sent once, never held in T."""
    return o > 0 and nonzero_digits(o, r) == 1


def blocks_sent_per_rank(P: int, r: int) -> int:
    """D for one rank: block i is sent once per non-zero digit of i."""
    return sum(nonzero_digits(i, r) for i in range(P))


def t_index(o: int, r: int) -> int:
    """Slot of block index o in T: o minus the number of lower indices that never use T
    (index 0 and the direct blocks below o)."""
    assert o > 0
    dx, v = 0, 1
    while v * r <= o:
        v *= r
        dx += 1
    dz = o // v
    return o - 1 - dx * (r - 1) - dz


def hop_factor(P: int, r: int) -> float:
    """Average number of hops of a block = sum over digit positions of the fraction of the P
    indices whose digit there is non-zero."""
    return blocks_sent_per_rank(P, r) / P


# ----------------------------------------------------------------------------
# flat TuNA, one object per rank
# ----------------------------------------------------------------------------
class _Rank:
    def __init__(self, p: int, P: int, r: int, S: Sequence[bytes], direction: int):
        self.p, self.P, self.r, self.dir = p, P, r, direction
        self.S = list(S)                                  # S[d] = block for rank d
        self.R: List[Optional[bytes]] = [None] * P        # R[s] = block from rank s
        self.B = temp_slots(P, r)
        self.T: List[Optional[bytes]] = [None] * max(self.B, 0)
        # rotation array: I[(p + i) % P] names the block at distance index i.  Algorithm "TuNA"
        # prints I[i] = (2p - i + P) % P, i.e. distance i <-> block for rank (p - i) % P; the
        # narrative of Figure 1 is its mirror image (direction = +1).
        if direction < 0:
            self.I = [(2 * p - i + P) % P for i in range(P)]
        else:
            self.I = [i for i in range(P)]
        self.R[p] = self.S[p]                             # the rank's own block

    def dest_of_index(self, i: int) -> int:
        return self.I[(self.p + i) % self.P]

    def where(self, i: int, x: int) -> bytes:
        """Block at distance index i at the start of digit phase x: still in S if it never moved
        (all digits below x are zero), otherwise in T."""
        if i % self.r ** x == 0:
            return self.S[self.dest_of_index(i)]
        blk = self.T[t_index(i, self.r)]
        assert blk is not None
        return blk

    def make_message(self, x: int, z: int):
        sd = [i for i in range(self.P) if digit(i, x, self.r) == z]   # ascending i
        blocks = [self.where(i, x) for i in sd]
        metadata = [len(b) for b in blocks]
        data = b"".join(blocks)
        return sd, metadata, data

    def receive(self, x: int, z: int, metadata: List[int], data: bytes) -> Tuple[int, int]:
        sd = [i for i in range(self.P) if digit(i, x, self.r) == z]
        assert len(sd) == len(metadata)
        off = 0
        finals = temps = 0
        for i, n in zip(sd, metadata):
            blk = data[off:off + n]
            off += n
            if i < self.r ** (x + 1):                     # no higher non-zero digit: arrived
                src = (self.p + i) % self.P if self.dir < 0 else (self.p - i) % self.P
                assert self.R[src] is None
                self.R[src] = blk
                finals += 1
            else:
                self.T[t_index(i, self.r)] = blk
                temps += 1
        assert off == len(data)
        return finals, temps


def simulate_tuna(S: Sequence[Sequence[bytes]], r: int, direction: int = -1):
    """Run Algorithm "TuNA" over P = len(S) ranks.  S[p][d] is the block rank p sends to rank d.
    Returns (R, stats): R[p][s] the block rank p received from rank s; stats has, per round, the
    rank distance, the per-rank send indices, metadata, finals and T stores, plus totals."""
    P = len(S)
    r = min(r, max(P, 2))
    ranks = [_Rank(p, P, r, S[p], direction) for p in range(P)]
    stats = {"P": P, "r": r, "w": num_digits(P, r), "rounds": [], "blocks_sent": [0] * P,
             "phase_bytes": {}}
    for (x, z) in rounds(P, r):
        dist = z * r ** x
        msgs = []
        for rk in ranks:                                   # every rank packs before anyone unpacks
            sendrank = (rk.p + direction * dist) % P
            sd, metadata, data = rk.make_message(x, z)
            msgs.append((sendrank, sd, metadata, data))
        rec = {"x": x, "z": z, "distance": dist, "send_indices": msgs[0][1],
               "metadata": [m[2] for m in msgs], "finals": [0] * P, "temps": [0] * P,
               "sendrank": [m[0] for m in msgs]}
        for p, (sendrank, sd, metadata, data) in enumerate(msgs):
            f, t = ranks[sendrank].receive(x, z, metadata, data)
            rec["finals"][sendrank] = f
            rec["temps"][sendrank] = t
            stats["blocks_sent"][p] += len(sd)
            stats["phase_bytes"][x] = stats["phase_bytes"].get(x, 0) + len(data)
        stats["rounds"].append(rec)
    stats["K"] = len(stats["rounds"])
    stats["B"] = ranks[0].B if ranks else 0
    R = [rk.R for rk in ranks]
    return R, stats


# ----------------------------------------------------------------------------
# hierarchical coalesced TuNA_l^g, one object per rank
# ----------------------------------------------------------------------------
class _HRank:
    def __init__(self, p: int, Q: int, N: int, rl: int, rg: int, S: Sequence[bytes]):
        self.p, self.Q, self.N, self.rl, self.rg = p, Q, N, rl, rg
        self.g, self.n = p % Q, p // Q
        self.S = list(S)
        P = Q * N
        self.R: List[Optional[bytes]] = [None] * P
        # rotation array of Algorithm "Coalesced TuNA_l^g": I[i*Q + j] = i*Q + (2g - j + Q) % Q
        self.I = [i * Q + (2 * self.g - j + Q) % Q for i in range(N) for j in range(Q)]
        self.T: Dict[Tuple[int, int], bytes] = {}          # local phase: key (group, local index)
        self.R[p] = self.S[p]
        self.super: Dict[int, List[bytes]] = {}            # node distance j -> Q sub-blocks
        self.Tg: Dict[int, List[bytes]] = {}               # global phase: slot t(j) -> super-block

    # -- intra-node phase: N concurrent Q x Q exchanges, one per group -----------------------
    def local_block(self, grp: int, l: int, x: int) -> bytes:
        if l % self.rl ** x == 0:
            return self.S[self.I[grp * self.Q + (self.g + l) % self.Q]]
        return self.T[(grp, l)]

    def local_indices(self, x: int, z: int):
        return [(grp, l) for grp in range(self.N) for l in range(self.Q)
                if digit(l, x, self.rl) == z]

    def local_message(self, x: int, z: int):
        idx = self.local_indices(x, z)
        blocks = [self.local_block(grp, l, x) for grp, l in idx]
        return [len(b) for b in blocks], b"".join(blocks)

    def local_receive(self, x: int, z: int, metadata, data):
        off = 0
        for (grp, l), n in zip(self.local_indices(x, z), metadata):
            blk = data[off:off + n]
            off += n
            if grp == self.n and l < self.rl ** (x + 1):
                src = self.n * self.Q + (self.g + l) % self.Q
                assert self.R[src] is None
                self.R[src] = blk                          # own node's group: arrived
            else:
                self.T[(grp, l)] = blk                      # forwarded later, or bound for another node
        assert off == len(data)

    # -- rearrangement: per remote node, the Q blocks in source-local-rank order --------------
    def rearrange(self):
        for grp in range(self.N):
            if grp == self.n:
                continue
            sub = []
            for s in range(self.Q):                         # source rank (n, s)
                l = (s - self.g) % self.Q
                sub.append(self.S[grp * self.Q + self.g] if l == 0 else self.T[(grp, l)])
            self.super[(self.n - grp) % self.N] = sub       # keyed by node distance j

    # -- inter-node phase among ranks of equal g; unit = super-block ---------------------------
    def global_block(self, j: int, x: int) -> List[bytes]:
        if j % self.rg ** x == 0:
            return self.super[j]
        return self.Tg[t_index(j, self.rg)]

    def global_message(self, x: int, z: int):
        js = [j for j in range(self.N) if digit(j, x, self.rg) == z]
        subs = [self.global_block(j, x) for j in js]
        metadata = [[len(b) for b in sub] for sub in subs]
        data = b"".join(b"".join(sub) for sub in subs)
        return js, metadata, data

    def global_receive(self, x: int, z: int, js, metadata, data):
        off = 0
        for j, sizes in zip(js, metadata):
            sub = []
            for n in sizes:
                sub.append(data[off:off + n])
                off += n
            if j < self.rg ** (x + 1):
                nsrc = (self.n + j) % self.N
                for s, blk in enumerate(sub):
                    assert self.R[nsrc * self.Q + s] is None
                    self.R[nsrc * self.Q + s] = blk
            else:
                self.Tg[t_index(j, self.rg)] = sub
        assert off == len(data)


def simulate_tuna_hier(S: Sequence[Sequence[bytes]], Q: int, rl: int, rg: int, staggered: bool = False):
    """Coalesced TuNA_l^g over P = len(S) ranks, Q per node.  rg = N gives the paper's inter-node
    schedule (N-1 rounds, Q blocks per message); rg < N runs the same digit rounds over the N
    node-ranks with super-blocks as the unit.  staggered = True runs Algorithm "Staggered
    TuNA_l^g" instead: no rearrangement, Q (N-1) inter-node rounds of one block each, round
    (gi, gr) carrying block gr of the group for node n - gi to the rank of equal g there.
    Returns (R, stats)."""
    P = len(S)
    assert P % Q == 0
    N = P // Q
    rl = min(rl, max(Q, 2))
    rg = min(rg, max(N, 2))
    ranks = [_HRank(p, Q, N, rl, rg, S[p]) for p in range(P)]
    stats = {"local_rounds": rounds(Q, rl), "global_rounds": rounds(N, rg),
             "local_phase_bytes": {}, "global_phase_bytes": {}, "after_local_R": None}
    for (x, z) in stats["local_rounds"]:
        msgs = []
        for rk in ranks:
            sendrank = rk.n * Q + (rk.g - z * rl ** x + Q) % Q
            msgs.append((sendrank,) + rk.local_message(x, z))
        for sendrank, metadata, data in msgs:
            ranks[sendrank].local_receive(x, z, metadata, data)
            stats["local_phase_bytes"][x] = stats["local_phase_bytes"].get(x, 0) + len(data)
    stats["after_local_R"] = [list(rk.R) for rk in ranks]
    if staggered:
        stats["global_rounds"] = []
        stats["global_phase_bytes"] = {0: 0}
        for gi in range(1, N):                              # node distance
            for gr in range(Q):                             # one block per round
                msgs = []
                for rk in ranks:
                    ndst = (rk.n - gi + N) % N
                    l = (gr - rk.g) % Q                     # block from source (n, gr) bound for (ndst, g)
                    blk = rk.S[ndst * Q + rk.g] if l == 0 else rk.T[(ndst, l)]
                    msgs.append((ndst * Q + rk.g, rk.n * Q + gr, blk))
                for dst, src, blk in msgs:
                    assert ranks[dst].R[src] is None
                    ranks[dst].R[src] = blk
                    stats["global_phase_bytes"][0] += len(blk)
                stats["global_rounds"].append((gi, gr))
        return [rk.R for rk in ranks], stats
    for rk in ranks:
        rk.rearrange()
    for (x, z) in stats["global_rounds"]:
        msgs = []
        for rk in ranks:
            ndst = (rk.n - z * rg ** x + N) % N
            msgs.append((ndst * Q + rk.g,) + rk.global_message(x, z))
        for dst, js, metadata, data in msgs:
            ranks[dst].global_receive(x, z, js, metadata, data)
            stats["global_phase_bytes"][x] = stats["global_phase_bytes"].get(x, 0) + len(data)
    return [rk.R for rk in ranks], stats
