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

namespace tuna {

// One moving block of a phase, in message order (z ascending, then e ascending).  32 bytes, read
// by the kernels as two 16-byte halves: {e, z, src_slot, dst_slot} and {j, l, -, -}.
struct SegInfo {
    int32_t e;         // slot index j*Q + l
    int32_t z;         // value of the phase's digit (1..r-1): which message, and the partner distance z*r^x
    int32_t src_slot;  // T slot the sender reads it from, or -1: still in the send buffer S
    int32_t dst_slot;  // T slot the receiver stores it to, or -1: final, goes to the receive buffer R
    int32_t j;         // node distance
    int32_t l;         // local distance
    int32_t pad0, pad1;
};

struct PhaseHost {
    int dim;           // 0: local (digits of l, size Q); 1: global (digits of j, size N)
    int x;             // digit position
    int r;             // radix
    int64_t rx;        // r^x
    int size;          // Q or N
    int nz;            // valid digit values z = 1..nz (z*rx < size): point-to-point rounds in this phase
    int nseg;          // moving blocks per rank
    std::vector<SegInfo> seg;     // [nseg]
    std::vector<int32_t> zt;      // [P]: digit value of slot e in this phase, 0 = does not move
};

struct PlanHost {
    int P = 0, Q = 0, N = 0, rl = 0, rg = 0;
    int w_l = 0, w_g = 0, K_l = 0, K_g = 0, B_l = 0, B_g = 0;
    int64_t slots = 0;             // T slots per rank (fused: both copies)
    bool fused = false;
    int64_t blocks_sent = 0;       // per rank, all phases
    std::vector<PhaseHost> phases;
};

// w = ceil(log_r size): smallest w with r^w >= size (Section "Tunable Radix").
inline int num_digits(int64_t size, int64_t r) {
    int w = 0;
    int64_t v = 1;
    while (v < size) { v *= r; ++w; }
    return w;
}

// K: rounds (x, z) with 0 <= x < w, 1 <= z < r and z*r^x < size.
inline int num_rounds(int64_t size, int64_t r) {
    int K = 0;
    int64_t rx = 1;
    for (int x = 0, w = num_digits(size, r); x < w; ++x, rx *= r) {
        int64_t nz = (size - 1) / rx;
        K += (int)(nz < r - 1 ? nz : r - 1);
    }
    return K;
}

inline bool is_direct(int64_t o, int64_t r) {   // exactly one non-zero digit
    if (o <= 0) return false;
    while (o % r == 0) o /= r;
    return o < r;
}

// t = o - 1 - dx (r-1) - dz (Section "Estimating temporary buffer size"); dx = floor(log_r o).
inline int64_t t_index(int64_t o, int64_t r) {
    if (o <= 0 || is_direct(o, r)) return -1;
    int64_t dx = 0, v = 1;
    while (v * r <= o) { v *= r; ++dx; }
    const int64_t dz = o / v;
    return o - 1 - dx * (r - 1) - dz;
}

// fused = true lays T out twice: a phase then reads every block it forwards from one copy and
// stores every block it receives into the other, so that one kernel can do both at once.  The
// copy a block sits in is the parity of the number of hops it has made, which depends on its
// index only -- it is folded into the slot numbers of the tables.
inline PlanHost make_plan(int P, int Q, int rl, int rg, bool fused = false) {
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
    // T layout per rank: [0, B_l) own-node blocks still travelling (paper's map t over l);
    // then (N-1)(Q-1) slots for blocks of the other nodes' groups that moved locally (they wait
    // for the global phase); then B_g super-slots of Q blocks for the global phase (map t over j).
    const int64_t foreign0 = pl.B_l;
    const int64_t global0 = foreign0 + (int64_t)(N - 1) * (Q - 1);
    const int64_t slots1 = global0 + (int64_t)pl.B_g * Q;
    pl.slots = fused ? 2 * slots1 : slots1;
    pl.fused = fused;
    // hops a block with distance pair (j, l) has made before phase (dim, x): non-zero digits of l
    // below x (all of l's digits once the global phases run) plus non-zero digits of j below x
    auto hops_before = [&](int dim, int64_t rx, int j, int l) -> int {
        int h = 0;
        int64_t v = dim == 0 ? l % rx : l;
        for (; v; v /= rl) h += (v % rl) != 0;
        if (dim == 1) for (v = j % rx; v; v /= rg) h += (v % rg) != 0;
        return h;
    };
    auto local_slot = [&](int j, int l) -> int32_t {
        if (j == 0) return (int32_t)t_index(l, rl);
        return (int32_t)(foreign0 + (int64_t)(j - 1) * (Q - 1) + (l - 1));
    };
    auto global_slot = [&](int j, int l) -> int32_t {
        return (int32_t)(global0 + t_index(j, rg) * Q + l);
    };
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
            ph.zt.assign(P, 0);
            const int64_t rx1 = rx * r;
            // message order: digit value z ascending, then slot index e ascending (Algorithm
            // "TuNA", the loop that collects the send indices runs over ascending i)
            std::vector<int32_t> first(ph.nz + 2, 0);
            for (int j = 0; j < N; ++j)
                for (int l = 0; l < Q; ++l) {
                    const int z = (int)(((dim == 0 ? l : j) / rx) % r);
                    ph.zt[j * Q + l] = z;
                    if (z) ++first[z + 1];
                }
            for (int z = 1; z <= ph.nz; ++z) first[z + 1] += first[z];
            ph.nseg = first[ph.nz + 1];
            ph.seg.assign(ph.nseg, SegInfo{});
            for (int j = 0; j < N; ++j)
                for (int l = 0; l < Q; ++l) {
                    const int z = ph.zt[j * Q + l];
                    if (!z) continue;
                    SegInfo s{};
                    s.e = j * Q + l; s.j = j; s.l = l; s.z = z;
                    if (dim == 0) {
                        s.src_slot = (l % rx == 0) ? -1 : local_slot(j, l);
                        s.dst_slot = (j == 0 && l < rx1) ? -1 : local_slot(j, l);
                    } else {
                        if (j % rx == 0) s.src_slot = (l == 0) ? -1 : local_slot(j, l);
                        else             s.src_slot = global_slot(j, l);
                        s.dst_slot = (j < rx1) ? -1 : global_slot(j, l);
                    }
                    if (fused) {
                        const int h = hops_before(dim, rx, j, l);
                        if (s.src_slot >= 0) s.src_slot += (int32_t)((h & 1) * slots1);
                        if (s.dst_slot >= 0) s.dst_slot += (int32_t)(((h + 1) & 1) * slots1);
                    }
                    ph.seg[first[z]++] = s;
                }
            pl.blocks_sent += ph.nseg;
            pl.phases.push_back(std::move(ph));
        }
    }
    return pl;
}

}  // namespace tuna
