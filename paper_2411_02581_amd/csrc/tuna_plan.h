// Host-side schedule ("plan") of the tunable-radix all-to-all: digit counts, round lists, the
// T-slot map and the rank-independent per-phase segment tables that the kernels index.
//
// Index space.  Rank p = n*Q + g (node n, local id g).  At every rank the P blocks are indexed
// by a distance pair (j, l): the block is bound for rank ((n - j) mod N, (g - l) mod Q), the
// direction of Algorithm "TuNA" (sendrank = p - z r^x).  Flat TuNA is Q = P, N = 1 (j = 0).
// Local phases resolve the base-r_l digits of l (Algorithm "Coalesced TuNA_l^g", the intra-node
// loop, run for all N groups at once), then global phases resolve the base-r_g digits of j with
// the Q blocks of one j travelling together as a super-block.  Slot index e = j*Q + l.
#pragma once
#include <cstdint>
#include <vector>

#ifdef __HIPCC__
#define TUNA_HD __host__ __device__
#else
#define TUNA_HD
#endif

namespace tuna {

// One moving block of a phase, in message order (z ascending, then e ascending).  The device keeps
// the fields it needs as one array per field (SegDev).
struct SegInfo {
    int32_t e;         // slot index j*Q + l
    int32_t z;         // value of the phase's digit (1..r-1): which message, and the partner distance z*r^x
    int32_t src_slot;  // T slot the sender reads it from, or -1: still in the send buffer S
    int32_t dst_slot;  // T slot the receiver stores it to, or -1: final, goes to the receive buffer R
    int32_t j;         // node distance
    int32_t l;         // local distance
    int32_t src_phase; // phase in which the block last moved (it arrived in T then), or -1: still in S
    int32_t src_seg;   // its position in that phase's message order
    int32_t nxt_phase; // phase in which the block moves next (it waits in T until then), or -1: final
};

struct PhaseHost {
    int dim;           // 0: local (digits of l, size Q); 1: global (digits of j, size N)
    int x;             // digit position
    int r;             // radix
    int64_t rx;        // r^x
    int size;          // Q or N
    int nz;            // valid digit values z = 1..nz (z*rx < size): point-to-point rounds in this phase
    int nseg;          // moving blocks per rank
    std::vector<SegInfo> seg;     // [nseg], only when the plan was made with tables
    std::vector<int32_t> zt;      // [P]: digit value of slot e in this phase, 0 = does not move (with tables)
};

// The scalars every table entry is computed from; passed by value to the device.
struct PlanScalars {
    int P, Q, N, rl, rg;
    int B_l, B_g;
    long long foreign0;   // first T slot of the other nodes' groups
    long long global0;    // first T slot of the global phase
    long long slots1;     // slots of one copy of T
    int fused;
    int w_l;              // number of local phases (they come first in the phase list)
    int nph;              // number of phases
};

struct PhaseScalars {
    int dim, x, r, size, nz, nseg;
    long long rx, rx1;    // r^x, r^(x+1)
};

struct PlanHost {
    int P = 0, Q = 0, N = 0, rl = 0, rg = 0;
    int w_l = 0, w_g = 0, K_l = 0, K_g = 0, B_l = 0, B_g = 0;
    int64_t slots = 0;             // T slots per rank (fused: both copies)
    bool fused = false;
    int64_t blocks_sent = 0;       // per rank, all phases
    PlanScalars sc{};
    std::vector<PhaseHost> phases;
};

// w = ceil(log_r size): smallest w with r^w >= size (Section "Tunable Radix").
TUNA_HD inline int num_digits(long long size, long long r) {
    int w = 0;
    long long v = 1;
    while (v < size) { v *= r; ++w; }
    return w;
}

// K: rounds (x, z) with 0 <= x < w, 1 <= z < r and z*r^x < size.
TUNA_HD inline int num_rounds(long long size, long long r) {
    int K = 0;
    long long rx = 1;
    for (int x = 0, w = num_digits(size, r); x < w; ++x, rx *= r) {
        long long nz = (size - 1) / rx;
        K += (int)(nz < r - 1 ? nz : r - 1);
    }
    return K;
}

TUNA_HD inline bool is_direct(long long o, long long r) {   // exactly one non-zero digit
    if (o <= 0) return false;
    while (o % r == 0) o /= r;
    return o < r;
}

// t = o - 1 - dx (r-1) - dz (Section "Estimating temporary buffer size"); dx = floor(log_r o).
TUNA_HD inline long long t_index(long long o, long long r) {
    if (o <= 0 || is_direct(o, r)) return -1;
    long long dx = 0, v = 1;
    while (v * r <= o) { v *= r; ++dx; }
    const long long dz = o / v;
    return o - 1 - dx * (r - 1) - dz;
}

// Phases in which the block with slot index e moves: bit x of the mask for phase x of the phase
// list (local phases first, then global ones) -- one hop per non-zero digit of its distance pair.
TUNA_HD inline unsigned long long move_mask(const PlanScalars& pl, int e) {
    const int j = e / pl.Q, l = e - j * pl.Q;
    unsigned long long m = 0;
    int x = 0;
    for (int v = l; v; v /= pl.rl, ++x)
        if (v % pl.rl) m |= 1ull << x;
    x = pl.w_l;
    for (int v = j; v; v /= pl.rg, ++x)
        if (v % pl.rg) m |= 1ull << x;
    return m;
}

// Exact-size T keeps the blocks that wait from phase f to phase y (f < y: stored when they arrive in
// phase f, forwarded in phase y) together, as "class" (f, y); classes are numbered row by row.
TUNA_HD inline int class_id(int f, int y, int nph) { return f * nph - f * (f + 1) / 2 + (y - f - 1); }
TUNA_HD inline int class_count(int nph) { return nph * (nph - 1) / 2; }

// Number of coordinates c in [0, size) whose digit x (base r) equals z.
TUNA_HD inline long long count_with_digit(const PhaseScalars& ph, int z) {
    const long long full = ph.size / ph.rx1, rem = ph.size % ph.rx1;
    long long part = rem - (long long)z * ph.rx;
    part = part < 0 ? 0 : (part > ph.rx ? ph.rx : part);
    return full * ph.rx + part;
}

// Number of coordinates whose digit is in 1 .. z-1 (closed form of the sum of count_with_digit).
TUNA_HD inline long long count_below_digit(const PhaseScalars& ph, int z) {
    const long long full = ph.size / ph.rx1, rem = ph.size % ph.rx1;
    const long long a = rem / ph.rx, b = rem % ph.rx;
    long long whole = (z - 1 < a - 1) ? (z - 1) : (a - 1);
    if (whole < 0) whole = 0;
    return (long long)(z - 1) * full * ph.rx + whole * ph.rx + ((a >= 1 && a <= z - 1) ? b : 0);
}

// Hops a block with distance pair (j, l) has made before phase (dim, x): non-zero digits of l
// below x (all of l's digits once the global phases run) plus non-zero digits of j below x.
TUNA_HD inline int hops_before(const PlanScalars& pl, const PhaseScalars& ph, int j, int l) {
    int h = 0;
    long long v = ph.dim == 0 ? l % ph.rx : l;
    for (; v; v /= pl.rl) h += (v % pl.rl) != 0;
    if (ph.dim == 1) for (v = j % ph.rx; v; v /= pl.rg) h += (v % pl.rg) != 0;
    return h;
}

// The table entry of slot index e in a phase: false when the block does not move; else its digit
// value, its position s in message order (z ascending, then e ascending -- Algorithm "TuNA", the
// loop that collects the send indices runs over ascending i), where the sender reads it from and
// where the receiver stores it.  The same function builds the tables on the device and, for the
// host-only schedule queries, on the host.
//   never moved (all lower digits zero)      -> source is the send buffer S
//   final (no higher non-zero digit)         -> destination is the receive buffer R
//   otherwise a T slot: [0, B_l) own-node blocks by the paper's map t over l; then (N-1)(Q-1)
//   slots for blocks of the other nodes' groups that moved locally (they wait for the global
//   phase); then B_g super-slots of Q blocks for the global phase (map t over j).
// Position of slot index e in a phase's message order and its digit value there (0 and -1 when the
// block does not move in that phase).  Only dim, r, size, rx and rx1 of `ph` are used.
TUNA_HD inline int slot_position(const PlanScalars& pl, const PhaseScalars& ph, int e, int* z_out) {
    const int Q = pl.Q;
    const int j = e / Q, l = e - j * Q;
    const int c = ph.dim == 0 ? l : j;
    const int z = (int)((c / ph.rx) % ph.r);
    *z_out = z;
    if (z == 0) return -1;
    const long long rc = (c / ph.rx1) * ph.rx + (c % ph.rx);          // rank of c among those with digit z
    const long long mult = ph.dim == 0 ? pl.N : Q;
    const long long start = count_below_digit(ph, z) * mult;
    return (int)(ph.dim == 0 ? start + (long long)j * count_with_digit(ph, z) + rc : start + rc * Q + l);
}

// The phase in which the block with slot index e moved last before phase `ph`, and its position in
// that phase's message order: the highest non-zero digit below x of the phase's own coordinate,
// else (global phases) the highest non-zero digit of l.  false: it has not moved, it is still in S.
TUNA_HD inline bool previous_move(const PlanScalars& pl, const PhaseScalars& ph, int e, int* phase, int* seg) {
    const int Q = pl.Q;
    const int j = e / Q, l = e - j * Q;
    PhaseScalars q{};
    long long v = (ph.dim == 0 ? l : j) % ph.rx;
    q.dim = ph.dim;
    if (v == 0) {
        if (ph.dim == 0 || l == 0) return false;
        v = l;
        q.dim = 0;
    }
    q.r = q.dim == 0 ? pl.rl : pl.rg;
    q.size = q.dim == 0 ? Q : pl.N;
    q.x = 0; q.rx = 1;
    while (q.rx * q.r <= v) { q.rx *= q.r; ++q.x; }
    q.rx1 = q.rx * q.r;
    int z = 0;
    *seg = slot_position(pl, q, e, &z);
    *phase = q.dim == 0 ? q.x : pl.w_l + q.x;
    return true;
}

TUNA_HD inline bool slot_entry(const PlanScalars& pl, const PhaseScalars& ph, int e, SegInfo* out, int* pos) {
    const int Q = pl.Q;
    const int j = e / Q, l = e - j * Q;
    int z = 0;
    *pos = slot_position(pl, ph, e, &z);
    if (z == 0) return false;
    auto local_slot = [&](int jj, int ll) -> int {
        if (jj == 0) return (int)t_index(ll, pl.rl);
        return (int)(pl.foreign0 + (long long)(jj - 1) * (Q - 1) + (ll - 1));
    };
    auto global_slot = [&](int jj, int ll) -> int { return (int)(pl.global0 + t_index(jj, pl.rg) * Q + ll); };
    SegInfo s{};
    s.e = e; s.j = j; s.l = l; s.z = z;
    if (ph.dim == 0) {
        s.src_slot = (l % ph.rx == 0) ? -1 : local_slot(j, l);
        s.dst_slot = (j == 0 && l < ph.rx1) ? -1 : local_slot(j, l);
    } else {
        if (j % ph.rx == 0) s.src_slot = (l == 0) ? -1 : local_slot(j, l);
        else                s.src_slot = global_slot(j, l);
        s.dst_slot = (j < ph.rx1) ? -1 : global_slot(j, l);
    }
    if (pl.fused) {   // the copy of T is the parity of the hop count
        const int h = hops_before(pl, ph, j, l);
        if (s.src_slot >= 0) s.src_slot += (int)((h & 1) * pl.slots1);
        if (s.dst_slot >= 0) s.dst_slot += (int)(((h + 1) & 1) * pl.slots1);
    }
    s.src_phase = -1; s.src_seg = 0;
    if (s.src_slot >= 0) previous_move(pl, ph, e, &s.src_phase, &s.src_seg);
    s.nxt_phase = -1;
    if (s.dst_slot >= 0) {            // the lowest phase above this one in which the block moves again
        const int cur = ph.dim == 0 ? ph.x : pl.w_l + ph.x;
        const unsigned long long later = move_mask(pl, e) >> (cur + 1);
        int d = 0;
        while (d < 63 && !((later >> d) & 1ull)) ++d;
        s.nxt_phase = cur + 1 + d;
    }
    *out = s;
    return true;
}

inline PhaseScalars phase_scalars(const PhaseHost& ph) {
    PhaseScalars s{};
    s.dim = ph.dim; s.x = ph.x; s.r = ph.r; s.size = ph.size; s.nz = ph.nz; s.nseg = ph.nseg;
    s.rx = ph.rx; s.rx1 = ph.rx * ph.r;
    return s;
}

// fused = true lays T out twice: a phase then reads every block it forwards from one copy and
// stores every block it receives into the other, so that one kernel can do both at once.  The
// copy a block sits in is the parity of the number of hops it has made, which depends on its
// index only -- it is folded into the slot numbers of the tables.
// with_tables = false computes the scalars only (the device builds its own tables).
inline PlanHost make_plan(int P, int Q, int rl, int rg, bool fused = false, bool with_tables = true) {
    PlanHost pl;
    pl.P = P; pl.Q = Q; pl.N = P / Q;
    const int N = pl.N;
    pl.rl = rl < 2 ? 2 : (rl > Q && Q >= 2 ? Q : rl);
    pl.rg = rg < 2 ? 2 : (rg > N && N >= 2 ? N : rg);
    if (Q < 2) pl.rl = 2;
    if (N < 2) pl.rg = 2;
    rl = pl.rl; rg = pl.rg;
    pl.w_l = num_digits(Q, rl);  pl.K_l = num_rounds(Q, rl);
    pl.w_g = num_digits(N, rg);  pl.K_g = num_rounds(N, rg);
    pl.B_l = Q > 1 ? Q - 1 - pl.K_l : 0;      // B = size - (K + 1)
    pl.B_g = N > 1 ? N - 1 - pl.K_g : 0;
    PlanScalars& sc = pl.sc;
    sc.P = P; sc.Q = Q; sc.N = N; sc.rl = rl; sc.rg = rg; sc.B_l = pl.B_l; sc.B_g = pl.B_g;
    sc.foreign0 = pl.B_l;
    sc.global0 = sc.foreign0 + (long long)(N - 1) * (Q - 1);
    sc.slots1 = sc.global0 + (long long)pl.B_g * Q;
    sc.fused = fused ? 1 : 0;
    sc.w_l = pl.w_l;
    sc.nph = pl.w_l + pl.w_g;
    pl.slots = fused ? 2 * sc.slots1 : sc.slots1;
    pl.fused = fused;
    for (int dim = 0; dim < 2; ++dim) {
        const int size = dim == 0 ? Q : N;
        const int r = dim == 0 ? rl : rg;
        const int w = dim == 0 ? pl.w_l : pl.w_g;
        int64_t rx = 1;
        for (int x = 0; x < w; ++x, rx *= r) {
            PhaseHost ph;
            ph.dim = dim; ph.x = x; ph.r = r; ph.rx = rx; ph.size = size;
            const int64_t nzmax = (size - 1) / rx;
            ph.nz = (int)(nzmax < r - 1 ? nzmax : r - 1);
            PhaseScalars ps = phase_scalars(ph);
            ph.nseg = (int)(count_below_digit(ps, ph.nz + 1) * (dim == 0 ? N : Q));
            ps.nseg = ph.nseg;
            if (with_tables) {
                ph.zt.assign(P, 0);
                ph.seg.assign(ph.nseg, SegInfo{});
                for (int e = 0; e < P; ++e) {
                    SegInfo s{};
                    int pos = 0;
                    if (slot_entry(sc, ps, e, &s, &pos)) { ph.zt[e] = s.z; ph.seg[pos] = s; }
                }
            }
            pl.blocks_sent += ph.nseg;
            pl.phases.push_back(std::move(ph));
        }
    }
    return pl;
}

}  // namespace tuna
