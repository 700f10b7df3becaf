"""Independent arithmetic on the temporary buffer T for the tests (plain Python / numpy, no library code):
which phases a block moves in, how many bytes wait in T from one phase to a later one, and how many bytes
are alive in T at one time.

A block with rank distance (node distance j in base r_g, local distance l in base r_l) moves once per
non-zero digit, local digits first (Section "Tunable Radix"; Section "Hierarchical TuNA"); between two
consecutive moves f < y it waits in T (Section "Estimating temporary buffer size": only blocks that will
be forwarded again are kept there)."""
import numpy as np


def move_phases(j, l, rl, rg, w_l):
    out, x = [], 0
    while l:
        if l % rl:
            out.append(x)
        l //= rl
        x += 1
    x = w_l
    while j:
        if j % rg:
            out.append(x)
        j //= rg
        x += 1
    return out


def digits(size, r):
    w, v = 0, 1
    while v < size:
        v *= r
        w += 1
    return w


def waiting_bytes(counts, Q, rl, rg):
    """{(f, y): bytes (blocks padded to 16) that wait in T from phase f to phase y}, number of phases."""
    P = counts.shape[0]
    Q = Q if Q else P
    N = P // Q
    rl, rg = min(max(rl, 2), max(Q, 2)), min(max(rg, 2), max(N, 2))
    w_l, w_g = digits(Q, rl), digits(N, rg)
    padded = (counts.astype(np.int64) + 15) // 16 * 16
    src = np.arange(P)
    cls = {}
    for e in range(1, P):
        j, l = divmod(e, Q)
        dst = ((src // Q - j) % N) * Q + (src % Q - l) % Q
        nbytes = int(padded[src, dst].sum())
        mv = move_phases(j, l, rl, rg, w_l)
        for f, y in zip(mv, mv[1:]):
            cls[(f, y)] = cls.get((f, y), 0) + nbytes
    return cls, w_l + w_g


def alive_peak(cls, one_kernel_phase):
    """Most bytes alive in T at one time.  Class (f, y) is alive from the kernel that stores it -- the
    unpack of phase f (time 2 f + 1), or the one kernel of phase f (time 2 f) -- to the kernel that reads
    it, at time 2 y."""
    peak = 0
    times = sorted({t for (f, y) in cls for t in (2 * f, 2 * f + 1, 2 * y)})
    for t in times:
        alive = sum(b for (f, y), b in cls.items() if 2 * f + (0 if one_kernel_phase(f) else 1) <= t <= 2 * y)
        peak = max(peak, alive)
    return peak


def passed_through(cls):
    return sum(cls.values())
