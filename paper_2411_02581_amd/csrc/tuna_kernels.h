// Device kernels of the tunable-radix all-to-all for gfx950 (wave64).
//
// All kernels are pure data movement or 32/64-bit integer index arithmetic; none uses MFMA.
// Staging buffers are addressed in 16-byte "chunks": every block is padded to a whole number of
// chunks in staging, so staging accesses are always aligned dwordx4 and the only unaligned
// accesses are to the caller's send / receive buffers.
#pragma once
#include <hip/hip_runtime.h>
#include <climits>
#include <cstdint>

#include "tuna_plan.h"

namespace tuna {

typedef unsigned int v4u __attribute__((ext_vector_type(4)));   // one 16-byte chunk

// Shape of the copy kernels' work, chosen by measurement on MI355X: workgroups of 64, 128, 512 and
// 1024 threads and 2 or 8 chunks per lane were all slower than 256 threads x 4 chunks.
constexpr int kWave = 64;
constexpr int kCopyThreads = 256;                        // 4 waves, each an independent work unit
constexpr int kChunksPerLane = 4;
constexpr int kUnitChunks = kWave * kChunksPerLane;      // 256 chunks = 4 KiB per wave unit
constexpr int kWideChunksPerLane = 8;
constexpr int kWideUnitChunks = kWave * kWideChunksPerLane;   // 8 KiB: the last phase of a schedule as a word-granular tiled hop
constexpr int kRankAlignChunks = 8;                      // every rank's region of a staging buffer or of a class of exact-size T starts on a 128-byte line
constexpr int kScanThreads = 256;
constexpr int kScanItems = 4;
constexpr int kExchangeRanks = 8;                        // ranks per thread of the elementwise size kernels

enum CopyMode { kPack = 0, kExchange = 1, kUnpack = 2, kFused = 3 };
// per-segment flags in the copy kernel's window: bits 0-3 = bytes of the first chunk that lie
// before the block (fused rounds), then:
constexpr int kFlagFill = 16;    // destination is a T slot: the tail lane fills up the 128-byte line
constexpr int kFlagSrcT = 32;    // source is a T slot: reading past the block's end is always safe

constexpr int kMaxClasses = 64 * 63 / 2;     // class_count(TUNA_MAX_PHASES)

// Device-side status block: the validation pass writes the head, every phase its own entries of the
// three arrays; the head is read back once after validation.
struct Status {
    unsigned int flags;            // bit 0: negative count, bit 1: recvcounts != transpose(sendcounts), (bit 3: receive regions not dense)
                                   // bit 2: negative displacement of a non-empty block
    unsigned int align_bits;       // OR of all counts and displacements, low 7 bits (they decide the granularity)
    int max_count;                 // M
    int tiny_done;                 // k_tiny_call: 1 = the whole call was done by that one kernel, 0 = it declined (nothing moved)
    unsigned long long total_bytes;    // sum of sendcounts
    unsigned long long total_chunks;   // sum of ceil(count / 16)
    unsigned long long send_extent;    // max over non-empty blocks of sdispls + count: bytes of sendbuf that hold blocks
    unsigned long long t_chunks;       // exact-size T: chunks stored into T over all phases
    unsigned long long short_blocks;   // blocks of fewer than kShortBlockBytes bytes, empty ones included
    unsigned long long phase_bytes[64];   // payload bytes moved per phase
    unsigned long long phase_chunks[64];  // staged chunks per phase
    unsigned int phase_units[64][2];      // wave units per phase: [0] receive-side layout, [1] send-side layout
    unsigned int self_units;              // wave units of the ranks' own blocks when the copy engine moves them
    unsigned int reserved2;
    unsigned long long cls_chunks[kMaxClasses];   // exact-size T: chunks of every class (f, y), summed by the validation pass
};

// The per-phase table of moving blocks on the device, one array per field (message order).
struct SegDev {
    const int32_t* e;      // slot index j*Q + l
    const int32_t* z;      // digit value: which message, partner distance z*r^x
    const int32_t* src;    // source T slot or -1 (send buffer)
    const int32_t* dst;    // destination T slot or -1 (receive buffer)
    const int32_t* srcph;  // phase in which the block arrived in T, or -1 (send buffer)
    const int32_t* srcseg; // its position in that phase's message order
    const int32_t* scls;   // exact-size T: class (arrival phase, this phase) the block is read from, or -1
    const int32_t* dcls;   // exact-size T: class (this phase, next move) the block is stored into, or -1
};

// Exact-size T.  A block that arrives in phase f and moves again in phase y waits in T from f to y: the
// blocks of one such class (f, y) lie together, rank after rank, each rank's part back to back in
// message order (padded to 16 bytes per block, to a 128-byte line per rank).  Where a class lies in T
// is decided on the host from the classes' sizes (the validation pass sums them) and lifetimes: classes
// whose lifetimes do not overlap share memory, so T holds what waits in it at one time, not what ever
// passed through it.  All offsets are in 16-byte chunks.
struct ExactT {
    const long long* cbase;  // [classes]: first chunk of each class in T (from the host)
    long long* tbase;        // [classes][P]: first chunk in T of rank p's part of a class
    int* csub;               // [classes][P]: chunks of rank p's part of a class
    int* tpos;               // [phases][P][P]: chunk offset, inside its rank's part of its class, of the block with slot index e that the phase stored
    int* tpre;               // [P][ld]: the same offsets for the phase being run, in message order
    int ld;
    int phase;               // index of the phase being run
    // the T-bound blocks of the phase being run, grouped by class: tord[tcls[3k+1] .. +tcls[3k+2]) are the
    // segment indices of class tcls[3k], in message order
    const int32_t* tord;
    const int32_t* tcls;
    int ncls;                // classes the phase being run stores into
};

// Distance pair of a slot index.
__device__ __forceinline__ void split_slot_index(int e, int Q, int N, int& j, int& l) {
    if (N == 1) { j = 0; l = e; }
    else { j = e / Q; l = e - j * Q; }
}

// One staging layout (send side or receive side) of the current phase.
struct LayoutDev {
    int* pre;                      // [P][ld]: exclusive prefix of chunk counts over the rank's segments; [nseg] = total
    int* tot;                      // [P]: chunks per rank
    long long* rank_base;          // [P+1]: first chunk of each rank in the staging buffer
    int* unit_base;                // [P+1]: first wave unit of each rank
    int4* units;                   // {rank, first segment, first chunk (rank-local), chunks in unit}
    int* n_units;                  // total units
    int ld;                        // row stride of pre (>= P + 1)
    int unit_chunks;               // chunks (or pieces) per wave unit: kUnitChunks, or kWideUnitChunks for the units of k_copy_tiled<4, 8>
};

// One-kernel phases: where every block a rank receives in the phase is read from and written to,
// resolved once per phase by k_resolve_hop, in the receive-side message order of the rank.  The copy
// kernel then needs one round of loads (prefix, source, destination, size) before its payload loads
// instead of three dependent ones (table, displacement or T position, payload).
struct HopDev {
    unsigned long long* src;       // [P][ld]: source address; kHopInT: an offset into T instead
    unsigned long long* dst;       // [P][ld]: destination address; kHopInT: an offset into T; kHopFill: a T slot whose last line is filled up
    int* size;                     // [P][ld]: bytes the destination takes: the exact count into R, whole chunks into T
    int ld;
};
constexpr unsigned long long kHopInT = 1ull << 62;
constexpr unsigned long long kHopFill = 1ull << 63;
constexpr int kHopLanes = 16;      // lanes of a copy wave that fetch their hop entries before the prefix is known

// ------------------------------------------------------------------------------------------
// small helpers
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ int wave_incl_scan(int v) {
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        int u = __shfl_up(v, d, kWave);
        if (lane >= d) v += u;
    }
    return v;
}

// Sender of the message with digit value z that rank (n, g) receives in a phase: the rank at
// distance +z*r^x in the phase's dimension (Algorithm "TuNA": recvrank = p + z r^x).
__device__ __forceinline__ int partner_up(int n, int g, int Q, int N, int dim, int dist) {
    if (dim == 0) { int gg = g + dist; if (gg >= Q) gg -= Q; return n * Q + gg; }
    int nn = n + dist; if (nn >= N) nn -= N; return nn * Q + g;
}

// ------------------------------------------------------------------------------------------
// k_build_phase_table: the rank-independent table of one digit phase, built on the device.  One
// thread per slot index e: its digit value z in this phase (Algorithm "TuNA", lines 8-11: the
// blocks whose x-th base-r digit equals z), its position in message order, the T slot it is read
// from / stored to by the map t = o - 1 - dx (r-1) - dz (Section "Estimating temporary buffer
// size"), or -1 for the send / receive buffer.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_build_phase_table(const PlanScalars pl, const PhaseScalars ph,
                                                           int32_t* __restrict__ seg_e, int32_t* __restrict__ seg_z,
                                                           int32_t* __restrict__ seg_src, int32_t* __restrict__ seg_dst,
                                                           int32_t* __restrict__ seg_srcph, int32_t* __restrict__ seg_srcseg,
                                                           int32_t* __restrict__ seg_scls, int32_t* __restrict__ seg_dcls,
                                                           int32_t* __restrict__ zt) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= pl.P) return;
    SegInfo s;
    int pos = 0;
    if (slot_entry(pl, ph, e, &s, &pos)) {
        zt[e] = s.z;
        seg_e[pos] = s.e; seg_z[pos] = s.z; seg_src[pos] = s.src_slot; seg_dst[pos] = s.dst_slot;
        seg_srcph[pos] = s.src_phase; seg_srcseg[pos] = s.src_seg;
        const int cur = ph.dim == 0 ? ph.x : pl.w_l + ph.x;
        seg_scls[pos] = s.src_phase >= 0 ? class_id(s.src_phase, cur, pl.nph) : -1;
        seg_dcls[pos] = s.nxt_phase >= 0 ? class_id(cur, s.nxt_phase, pl.nph) : -1;
    } else {
        zt[e] = 0;
    }
}

// ------------------------------------------------------------------------------------------
// k_plain_copy: one aligned 16-byte chunk per thread, nothing else.  The practical HBM copy
// ceiling of the device and the known-size reference that hardware byte counters are scaled by.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_plain_copy(const v4u* __restrict__ src, v4u* __restrict__ dst, size_t n) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// ------------------------------------------------------------------------------------------
// k_fill_uniform: the count and displacement matrices of a dense problem whose blocks all have
// `bytes` bytes (the calibration problems of the cost model); one thread per matrix entry.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_fill_uniform(int32_t* __restrict__ sendcounts, int64_t* __restrict__ sdispls,
                                                      int32_t* __restrict__ recvcounts, int64_t* __restrict__ rdispls,
                                                      int P, int bytes) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)P * P) return;
    sendcounts[i] = bytes; recvcounts[i] = bytes;
    sdispls[i] = (int64_t)i * bytes; rdispls[i] = (int64_t)i * bytes;
}

// ------------------------------------------------------------------------------------------
// k_build_hops: hm1[e] = (hops of the block with slot index e) - 1, at least 0.  A block makes one
// hop per non-zero digit of its distance pair (l in base r_l, j in base r_g) and is stored into T
// after every hop but its last -- hm1[e] times.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_build_hops(const PlanScalars pl, int32_t* __restrict__ hm1,
                                                    unsigned long long* __restrict__ mask) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= pl.P) return;
    mask[e] = move_mask(pl, e);
    int j = e / pl.Q, l = e - j * pl.Q, hops = 0;
    for (; l; l /= pl.rl) hops += (l % pl.rl) != 0;
    for (; j; j /= pl.rg) hops += (j % pl.rg) != 0;
    hm1[e] = hops > 1 ? hops - 1 : 0;
}

// ------------------------------------------------------------------------------------------
// k_validate: one pass over the P x P matrices in 64 x 64 tiles.  Finds M (Algorithm "TuNA",
// line 1: the maximum block size over all ranks, here one device reduction instead of an
// allreduce), the totals the workspace is sized from, checks counts >= 0 and
// recvcounts == transpose(sendcounts) through an LDS tile so both matrices are read row-wise
// (a wave reads 64 consecutive entries of one row).  With `hm1` it also sums the exact size of T:
// ceil(count / 16) * hm1[slot index of the block] chunks over all blocks.
// A non-empty block with a negative displacement is flagged too.  Workgroups of (64, 4) threads
// stride over the tiles and write one row of partial results each.
// ------------------------------------------------------------------------------------------
constexpr int kValTile = 64;
constexpr int kValPartial = 8;              // 64-bit words per workgroup in the partial-result array
constexpr int kShortBlockBytes = 256;       // below this a block is mostly edges to the destination-tiled hop
__global__ void __launch_bounds__(256) k_validate(const int32_t* __restrict__ sendcounts,
                                                  const int32_t* __restrict__ recvcounts,
                                                  const int64_t* __restrict__ sdispls,
                                                  const int64_t* __restrict__ rdispls,
                                                  int P, unsigned long long* __restrict__ partial,
                                                  const int32_t* __restrict__ hm1, int Q, int N,
                                                  const unsigned long long* __restrict__ mask, int nph,
                                                  unsigned long long* __restrict__ cls_chunks) {
    __shared__ int tile[kValTile][kValTile + 1];
    __shared__ unsigned long long red[4][7];
    extern __shared__ unsigned long long lcls[];          // class_count(nph) sums of this workgroup (with `mask`)
    const int tx = threadIdx.x, ty = threadIdx.y;
    const int ncls = mask ? class_count(nph) : 0;
    for (int i = ty * kValTile + tx; i < ncls; i += 4 * kValTile) lcls[i] = 0;
    __syncthreads();
    const int tpr = (P + kValTile - 1) / kValTile;       // tiles per row
    const int ntile = tpr * tpr;
    unsigned int flags = 0, abits = 0;
    int mx = 0;
    unsigned long long bytes = 0, chunks = 0, extent = 0, tchunks = 0, shortb = 0;
    for (int t = blockIdx.x; t < ntile; t += gridDim.x) {        // a workgroup strides over tiles
        const int bi = (t / tpr) * kValTile, bj = (t % tpr) * kValTile;
        const int j = bj + tx;
        const int jn = hm1 ? j / Q : 0, jg = hm1 ? j - jn * Q : 0;   // the destination's node and local id
        // four rows per step, their loads issued together from clamped indices: with one row per step the pass
        // was a chain of 32 dependent memory round trips per tile (48 us for 1024 ranks)
        for (int a0 = ty; a0 < kValTile; a0 += 16) {
            int cv[4];
            long long dv[4];
            bool ok[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = bi + a0 + 4 * u;
                ok[u] = i < P && j < P;
                const size_t idx = ok[u] ? (size_t)i * P + j : 0;
                cv[u] = sendcounts[idx];
                dv[u] = sdispls ? sdispls[idx] : 0;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int a = a0 + 4 * u;
                const int i = bi + a;
                int c = 0;
                if (ok[u]) {
                    c = cv[u];
                    if (c < 0) { flags |= 1u; c = 0; }
                    abits |= (unsigned int)c;
                    if (sdispls) {
                        const int64_t d = dv[u];
                        abits |= (unsigned int)d & 127u;
                        if (c > 0) {
                            if (d >= 0) extent = max(extent, (unsigned long long)d + (unsigned long long)c);
                            else flags |= 4u;
                        }
                    }
                    mx = max(mx, c);
                    bytes += (unsigned long long)c;
                    shortb += c < kShortBlockBytes ? 1u : 0u;
                    const unsigned long long ch = (unsigned long long)((c + 15) >> 4);
                    chunks += ch;
                    if (hm1 && c > 0) {
                        const int in = i / Q, ig = i - in * Q;
                        int dn = in - jn; if (dn < 0) dn += N;
                        int dg = ig - jg; if (dg < 0) dg += Q;
                        tchunks += ch * (unsigned long long)hm1[dn * Q + dg];
                        if (mask) {
                            // the block waits in T between every two consecutive phases in which it moves
                            unsigned long long m = mask[dn * Q + dg];
                            int f = __ffsll((long long)m) - 1;
                            m &= m - 1;
                            while (m) {
                                const int y = __ffsll((long long)m) - 1;
                                m &= m - 1;
                                atomicAdd(&lcls[class_id(f, y, nph)], ch);
                                f = y;
                            }
                        }
                    }
                }
                tile[a][tx] = c;
            }
        }
        __syncthreads();
        if (recvcounts) {
            for (int a0 = ty; a0 < kValTile; a0 += 16) {
                int rv[4];
                long long dv[4], dx[4];
                bool in[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int jr = bj + a0 + 4 * u, i = bi + tx;     // recvcounts[jr][i] must equal sendcounts[i][jr]
                    in[u] = i < P && jr < P;
                    const size_t idx = in[u] ? (size_t)jr * P + i : 0;
                    rv[u] = recvcounts[idx];
                    dv[u] = rdispls ? rdispls[idx] : 0;
                    // the last lane of a row reads its successor's displacement itself (below)
                    dx[u] = (rdispls && tx == kValTile - 1 && in[u] && i + 1 < P) ? rdispls[idx + 1] : 0;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int a = a0 + 4 * u;
                    const int i = bi + tx;
                    int rc = 0;
                    long long d = 0;
                    if (in[u]) {
                        rc = rv[u];
                        if (rc < 0) flags |= 1u;
                        else if (rc != tile[tx][a]) flags |= 2u;
                        if (rdispls) {
                            d = dv[u];
                            abits |= (unsigned int)d & 127u;
                            if (rc > 0 && d < 0) flags |= 4u;
                        }
                    }
                    if (rdispls) {
                        // dense receive regions: every block starts where its predecessor in source order ends
                        // (flag 8 when not; the destination-tiled hop needs it).  A wave holds 64
                        // neighbours of one row.
                        long long dn = __shfl_down(d, 1, kWave);
                        if (tx == kValTile - 1) dn = dx[u];
                        if (in[u] && i + 1 < P && dn != d + (long long)max(rc, 0)) flags |= 8u;
                    }
                }
            }
        }
        __syncthreads();
    }
    // wave reduction, workgroup reduction through LDS, then one row of partial results per workgroup
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) {
        flags |= __shfl_xor(flags, d, kWave);
        abits |= __shfl_xor(abits, d, kWave);
        mx = max(mx, __shfl_xor(mx, d, kWave));
        bytes += __shfl_xor(bytes, d, kWave);
        chunks += __shfl_xor(chunks, d, kWave);
        tchunks += __shfl_xor(tchunks, d, kWave);
        shortb += __shfl_xor(shortb, d, kWave);
        extent = max(extent, (unsigned long long)__shfl_xor(extent, d, kWave));
    }
    if (tx == 0) {                                       // one wave per value of ty
        unsigned long long* r = red[ty];
        r[0] = ((unsigned long long)flags << 32) | (abits & 127u);
        r[1] = (unsigned long long)mx; r[2] = bytes; r[3] = chunks; r[4] = extent; r[5] = tchunks; r[6] = shortb;
    }
    __syncthreads();
    if (tx == 0 && ty == 0) {
        unsigned long long fa = 0, m = 0, by = 0, ch = 0, ex = 0, tc = 0, sb = 0;
        for (int w = 0; w < 4; ++w) {
            fa |= red[w][0]; m = max(m, red[w][1]); by += red[w][2]; ch += red[w][3]; ex = max(ex, red[w][4]);
            tc += red[w][5]; sb += red[w][6];
        }
        // one row of partial results per workgroup, folded by k_validate_finish: thousands of atomics
        // on the same few addresses would take longer than reading the matrices
        unsigned long long* o = partial + (size_t)blockIdx.x * kValPartial;
        o[0] = fa; o[1] = m; o[2] = by; o[3] = ch; o[4] = ex; o[5] = tc; o[6] = sb;
    }
    // the class sums: one atomic per class and workgroup that holds any of it (cls_chunks starts at zero)
    for (int i = ty * kValTile + tx; i < ncls; i += 4 * kValTile)
        if (lcls[i]) atomicAdd(&cls_chunks[i], lcls[i]);
}

// k_zero64: n 64-bit words to zero (the class sums before a validation pass).
__global__ void __launch_bounds__(256) k_zero64(unsigned long long* __restrict__ p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// k_validate_finish: folds the workgroups' partial results into the status block (one workgroup).
__global__ void __launch_bounds__(256) k_validate_finish(const unsigned long long* __restrict__ partial, int n,
                                                         Status* __restrict__ st) {
    __shared__ unsigned long long red[4][7];
    unsigned long long fa = 0, m = 0, by = 0, ch = 0, ex = 0, tc = 0, sb = 0;
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
        const unsigned long long* o = partial + (size_t)i * kValPartial;
        fa |= o[0]; m = max(m, o[1]); by += o[2]; ch += o[3]; ex = max(ex, o[4]); tc += o[5]; sb += o[6];
    }
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) {
        fa |= __shfl_xor(fa, d, kWave);
        m = max(m, (unsigned long long)__shfl_xor(m, d, kWave));
        by += __shfl_xor(by, d, kWave);
        ch += __shfl_xor(ch, d, kWave);
        ex = max(ex, (unsigned long long)__shfl_xor(ex, d, kWave));
        tc += __shfl_xor(tc, d, kWave);
        sb += __shfl_xor(sb, d, kWave);
    }
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    if (lane == 0) { red[wv][0] = fa; red[wv][1] = m; red[wv][2] = by; red[wv][3] = ch; red[wv][4] = ex; red[wv][5] = tc; red[wv][6] = sb; }
    __syncthreads();
    if (threadIdx.x == 0) {
        fa = m = by = ch = ex = tc = sb = 0;
        for (int w = 0; w < 4; ++w) {
            fa |= red[w][0]; m = max(m, red[w][1]); by += red[w][2]; ch += red[w][3]; ex = max(ex, red[w][4]);
            tc += red[w][5]; sb += red[w][6];
        }
        st->flags = (unsigned int)(fa >> 32);
        st->align_bits = (unsigned int)(fa & 127u);
        st->max_count = (int)m;
        st->total_bytes = by;
        st->total_chunks = ch;
        st->send_extent = ex;
        st->t_chunks = tc;
        st->short_blocks = sb;
    }
}

// ------------------------------------------------------------------------------------------
// k_rotate_init: the index-only initial rotation (Algorithm "TuNA", lines 4-5; Algorithm
// "Coalesced TuNA_l^g", line 5).  No payload moves: cur[p][j*Q + l] becomes the size of the
// block rank p = (n, g) holds at distance (j, l), i.e. its block for rank ((n-j)%N, (g-l)%Q).
// With `up` the row is rotated the other way, cur[p][j*Q + l] = counts[p][((n+j)%N, (g+l)%Q)]: applied to
// recvcounts that is the size of the block rank p receives from the rank at distance (j, l) -- for a schedule
// of one phase, where every block arrives in its first and only hop, exactly what the metadata exchange of
// that phase leaves in the receiver's size array (Algorithm "TuNA", line 14), without the exchange.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_rotate_init(const int32_t* __restrict__ sendcounts,
                                                     int32_t* __restrict__ cur, int P, int Q, int N, int up) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;      // grid (ceil(P / 256), ceil(P / kExchangeRanks))
    if (e >= P) return;
    const int j = e / Q, l = e - j * Q;
    const int p0 = blockIdx.y * kExchangeRanks;
    int v[kExchangeRanks];
#pragma unroll
    for (int k = 0; k < kExchangeRanks; ++k) {
        const int p = p0 + k;
        v[k] = 0;
        if (p < P) {
            const int n = p / Q, g = p - n * Q;
            int dn = up ? n + j : n - j; if (dn < 0) dn += N; if (dn >= N) dn -= N;
            int dg = up ? g + l : g - l; if (dg < 0) dg += Q; if (dg >= Q) dg -= Q;
            v[k] = sendcounts[(size_t)p * P + dn * Q + dg];
        }
    }
#pragma unroll
    for (int k = 0; k < kExchangeRanks; ++k)
        if (p0 + k < P) cur[(size_t)(p0 + k) * P + e] = v[k];
}

// ------------------------------------------------------------------------------------------
// k_self_copy: the block a rank keeps for itself goes straight from S to R (Section "Estimating
// temporary buffer size": one block is destined for the rank itself).  grid (P, split).
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_self_copy(const unsigned char* __restrict__ S,
                                                   const int32_t* __restrict__ sendcounts,
                                                   const int64_t* __restrict__ sdispls,
                                                   unsigned char* __restrict__ R,
                                                   const int64_t* __restrict__ rdispls, int P) {
    const int p = blockIdx.x;
    const size_t d = (size_t)p * P + p;
    const int n = sendcounts[d];
    const unsigned char* src = S + sdispls[d];
    unsigned char* dst = R + rdispls[d];
    const int nchunk = n >> 4;
    for (int c = blockIdx.y * blockDim.x + threadIdx.x; c < nchunk; c += gridDim.y * blockDim.x) {
        uint4 v;
        __builtin_memcpy(&v, src + ((size_t)c << 4), 16);
        __builtin_memcpy(dst + ((size_t)c << 4), &v, 16);
    }
    if (blockIdx.y == 0) {
        const int tail = n & 15;
        if ((int)threadIdx.x < tail) dst[(nchunk << 4) + threadIdx.x] = src[(nchunk << 4) + threadIdx.x];
    }
}

// ------------------------------------------------------------------------------------------
// k_self_layout: the ranks' own blocks laid out as one more one-kernel phase of a single block per
// rank, source S at sdispls[p][p], destination R at rdispls[p][p], so that the byte-balanced copy
// engine moves them (large own blocks: one workgroup per rank would leave most of the device idle).
// One thread per rank; k_layout_base and k_layout_units then cut the wave units as for any phase.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_self_layout(const unsigned char* __restrict__ S,
                                                     const int32_t* __restrict__ sendcounts,
                                                     const int64_t* __restrict__ sdispls, unsigned char* __restrict__ R,
                                                     const int64_t* __restrict__ rdispls, int P, LayoutDev L, HopDev h) {
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= P) return;
    const size_t d = (size_t)p * P + p;
    const int sz = sendcounts[d];
    const unsigned long long src = (unsigned long long)(S + sdispls[d]);
    const unsigned long long dst = (unsigned long long)(R + rdispls[d]);
    // chunks are cut at the destination's 16-byte boundaries, as in every one-kernel phase
    const int chunks = sz > 0 ? (int)(((unsigned int)(dst & 15ull) + (unsigned int)sz + 15u) >> 4) : 0;
    int* pre = L.pre + (size_t)p * L.ld;
    pre[0] = 0; pre[1] = chunks;
    L.tot[p] = chunks;
    const size_t o = (size_t)p * h.ld;
    h.src[o] = sz > 0 ? src : 0ull; h.dst[o] = sz > 0 ? dst : 0ull; h.size[o] = sz > 0 ? sz : 0;
}

// ------------------------------------------------------------------------------------------
// k_size_exchange: the metadata exchange of one digit phase (Section "Two-phase communication";
// Algorithm "TuNA", line 14): the size of every moving block travels from the sender's size array
// to the receiver's, nxt[q][e] = cur[q + z r^x][e] with z the digit of e; sizes of blocks that stay
// are carried over.  One thread per (rank, slot index): both rows are read and written along e.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_size_exchange(const int32_t* __restrict__ cur, int32_t* __restrict__ nxt,
                                                       const int32_t* __restrict__ zt, int P, int Q, int N, int dim,
                                                       int rx) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= P) return;
    const int dist = zt[e] * rx;                      // 0: the block stays
    const int q0 = blockIdx.y * kExchangeRanks;
    int v[kExchangeRanks];
#pragma unroll
    for (int k = 0; k < kExchangeRanks; ++k) {        // all loads of a thread are in flight together
        const int q = q0 + k;
        v[k] = 0;
        if (q < P) {
            int src = q;
            if (dist) {
                const int qn = q / Q;
                src = partner_up(qn, q - qn * Q, Q, N, dim, dist);
            }
            v[k] = cur[(size_t)src * P + e];
        }
    }
#pragma unroll
    for (int k = 0; k < kExchangeRanks; ++k)
        if (q0 + k < P) nxt[(size_t)(q0 + k) * P + e] = v[k];
}

// ------------------------------------------------------------------------------------------
// k_phase_layout: the size/displacement scans of one digit phase, one workgroup per rank, from the
// sizes the rank holds before the phase (`cur`) and after it (`nxt`, see k_size_exchange):
//  size/displacement scans (the contiguous send buffer of Algorithm "TuNA", line 15, needs each
//  block's offset inside its message): per rank, the moving blocks' sizes in message order are
//  converted to 16-byte chunks and exclusive-scanned (wave shuffles + LDS across the 4 waves,
//  a running carry across batches of 1024 segments) -- once over the sizes the rank receives
//  (receive-side layout) and once over the sizes it sends (send-side layout);
// With `head_displs` (one-kernel phases) the chunks of a block bound for R are cut at the 16-byte
// boundaries of its destination address: a block that starts `a` bytes into a 16-byte line takes
// ceil((a + size) / 16) chunks; head_base is the low 4 bits of the receive buffer address.
// ------------------------------------------------------------------------------------------
struct PhaseLayoutArgs {
    const int32_t* cur;             // [P][P] sizes before the phase
    int32_t* nxt;                   // [P][P] sizes after it
    int inline_exchange;            // 1: this kernel also does the size exchange (few ranks: one launch less)
    const int32_t* zt;              // [P] digit value of slot e in this phase (0: stays)
    SegDev seg;
    int nseg;
    int P, Q, N, dim, rx;
    LayoutDev Ls, Lr;
    int want_send;                  // 0: only the receive-side layout (one-kernel phases)
    int want_tbound;                // 1: also lay out the blocks this phase stores into exact-size T (see ExactT)
    ExactT x;
    unsigned long long* rank_bytes; // [P]: payload bytes every rank moves in this phase
    unsigned long long* phase_bytes;
    unsigned long long* phase_chunks;
    unsigned int* phase_units;      // [2]: wave units of the receive-side and of the send-side layout
    const int64_t* head_displs;
    unsigned int head_base;
};

// Item k of a thread in a batch of kScanThreads * kScanItems segments: every wave owns
// kScanItems * 64 consecutive segments and lane i takes the ones at i, i + 64, ...: one load
// instruction of a wave reads 64 consecutive table entries.
__device__ __forceinline__ int scan_item_index(int k) {
    const int tid = threadIdx.x;
    return (tid / kWave) * (kWave * kScanItems) + k * kWave + (tid & (kWave - 1));
}

// exclusive scan of the batch in that order; run[k] = start of item k, `carry` grows by the batch total
__device__ __forceinline__ void block_scan_batch(const int (&c)[kScanItems], int (&run)[kScanItems], int& carry,
                                                 int* wsum) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    int wtotal = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        const int incl = wave_incl_scan(c[k]);
        run[k] = wtotal + incl - c[k];
        wtotal += __shfl(incl, kWave - 1, kWave);
    }
    __syncthreads();                                  // wsum of the previous batch is consumed
    if (lane == 0) wsum[wv] = wtotal;
    __syncthreads();
    int woff = 0, total = 0;
#pragma unroll
    for (int k = 0; k < kScanThreads / kWave; ++k) {
        const int v = wsum[k];
        if (k < wv) woff += v;
        total += v;
    }
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) run[k] += carry + woff;
    carry += total;
}

// exclusive scan over the P per-rank totals of one layout by one workgroup of kScanThreads: every
// thread sums a contiguous range of ranks, the thread sums are scanned across the workgroup, then
// every thread writes the bases of its range
__device__ __forceinline__ void scan_rank_bases(int P, const LayoutDev& L, unsigned long long* phase_chunks,
                                                long long* wc, int* wt,
                                                const unsigned long long* rank_bytes = nullptr,
                                                unsigned long long* phase_bytes = nullptr,
                                                unsigned int* units_out = nullptr) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const int per = (P + kScanThreads - 1) / kScanThreads;
    const int p0 = min(P, tid * per), p1 = min(P, p0 + per);
    const int ralign = kRankAlignChunks;
    long long sc = 0;
    int st = 0;
    // a rank's region is rounded up to whole 128-byte lines: units, which are cut every 4 KiB from
    // the region's start, then begin and end on line boundaries and their streaming stores are never
    // split into partial-line writes
    for (int p = p0; p < p1; ++p) {
        const int c = L.tot[p];
        sc += (c + ralign - 1) / ralign * ralign;
        st += (c + L.unit_chunks - 1) / L.unit_chunks;
    }
    long long ic = sc;
    int it = st;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        long long uc = __shfl_up(ic, d, kWave);
        int ut = __shfl_up(it, d, kWave);
        if (lane >= d) { ic += uc; it += ut; }
    }
    if (lane == kWave - 1) { wc[wv] = ic; wt[wv] = it; }
    __syncthreads();
    long long oc = 0, totc = 0;
    int ot = 0, tott = 0;
#pragma unroll
    for (int k = 0; k < kScanThreads / kWave; ++k) {
        if (k < wv) { oc += wc[k]; ot += wt[k]; }
        totc += wc[k]; tott += wt[k];
    }
    long long run_c = oc + ic - sc;
    int run_t = ot + it - st;
    for (int p = p0; p < p1; ++p) {
        const int c = L.tot[p];
        L.rank_base[p] = run_c;
        if (L.unit_base) L.unit_base[p] = run_t;
        run_c += (c + ralign - 1) / ralign * ralign;
        run_t += (c + L.unit_chunks - 1) / L.unit_chunks;
    }
    if (tid == 0) {
        L.rank_base[P] = totc;
        if (L.unit_base) { L.unit_base[P] = tott; *L.n_units = tott; }
        if (units_out) *units_out = (unsigned int)tott;
        if (phase_chunks) *phase_chunks = (unsigned long long)totc;
    }
    if (phase_bytes) {                                // payload bytes of the phase = sum of the ranks' sums
        unsigned long long b = 0;
        for (int p = p0; p < p1; ++p) b += rank_bytes[p];
#pragma unroll
        for (int d = kWave / 2; d > 0; d >>= 1) b += __shfl_xor(b, d, kWave);
        __syncthreads();                              // wc is reused
        if (lane == 0) wc[wv] = (long long)b;
        __syncthreads();
        if (tid == 0) {
            unsigned long long t = 0;
#pragma unroll
            for (int k = 0; k < kScanThreads / kWave; ++k) t += (unsigned long long)wc[k];
            *phase_bytes = t;
        }
    }
}

__global__ void __launch_bounds__(kScanThreads) k_phase_layout(const PhaseLayoutArgs a) {
    __shared__ int wsum[kScanThreads / kWave];
    __shared__ unsigned long long wbytes[kScanThreads / kWave];
    const int P = a.P;
    const int p = blockIdx.x;
    const int pn = p / a.Q, pg = p - pn * a.Q;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int32_t* crow = a.cur + (size_t)p * P;
    int32_t* nrow = a.nxt + (size_t)p * P;
    if (a.inline_exchange) {
        // the metadata exchange (see k_size_exchange), here by the receiving rank's own workgroup:
        // blocks that do not move keep their size, the others arrive with the scan's gather below
        for (int e = tid; e < P; e += kScanThreads)
            if (a.zt[e] == 0) nrow[e] = crow[e];
    }
    int* pre_r = a.Lr.pre + (size_t)p * a.Lr.ld;
    int* pre_s = a.Ls.pre + (size_t)p * a.Ls.ld;
    int carry_r = 0, carry_s = 0;
    unsigned long long bytes = 0;
    for (int base = 0; base < a.nseg; base += kScanThreads * kScanItems) {
        int cr[kScanItems], cs[kScanItems];
#pragma unroll
        for (int k = 0; k < kScanItems; ++k) {
            const int s = base + scan_item_index(k);
            int szr = 0, szs = 0, head = 0;
            if (s < a.nseg) {
                const int e = a.seg.e[s];
                if (a.inline_exchange) {
                    const int ps = partner_up(pn, pg, a.Q, a.N, a.dim, a.seg.z[s] * a.rx);
                    szr = a.cur[(size_t)ps * P + e];
                    nrow[e] = szr;
                } else {
                    szr = nrow[e];
                }
                if (a.want_send) szs = crow[e];
                if (a.head_displs && szr > 0 && a.seg.dst[s] < 0) {
                    int j, l;
                    split_slot_index(e, a.Q, a.N, j, l);
                    int sn = pn + j; if (sn >= a.N) sn -= a.N;
                    int sg = pg + l; if (sg >= a.Q) sg -= a.Q;
                    head = (int)(((unsigned int)a.head_displs[(size_t)p * P + sn * a.Q + sg] + a.head_base) & 15u);
                }
            }
            bytes += (unsigned long long)(a.want_send ? szs : szr);
            cr[k] = (head + szr + 15) >> 4;
            cs[k] = (szs + 15) >> 4;
        }
        int run[kScanItems];
        block_scan_batch(cr, run, carry_r, wsum);
#pragma unroll
        for (int k = 0; k < kScanItems; ++k) {
            const int s = base + scan_item_index(k);
            if (s < a.nseg) pre_r[s] = run[k];
        }
        if (a.want_send) {
            block_scan_batch(cs, run, carry_s, wsum);
#pragma unroll
            for (int k = 0; k < kScanItems; ++k) {
                const int s = base + scan_item_index(k);
                if (s < a.nseg) pre_s[s] = run[k];
            }
        }
    }
    if (a.want_tbound) {
        // Exact-size T: the blocks this phase stores, class by class (a class = the blocks that move next in
        // the same later phase); within a class in message order.  Every block's chunk offset inside this
        // rank's part of its class goes to tpre (by segment, for this phase's own stores) and to tpos (by slot
        // index, for the phase that forwards the block); the part's size goes to csub.
        __syncthreads();                                  // the sizes this workgroup exchanged itself are in nrow
        int* pre_t = a.x.tpre + (size_t)p * a.x.ld;
        int* pos_t = a.x.tpos + ((size_t)a.x.phase * P + p) * P;
        for (int cl = 0; cl < a.x.ncls; ++cl) {
            const int cid = a.x.tcls[3 * cl], c0 = a.x.tcls[3 * cl + 1], cn = a.x.tcls[3 * cl + 2];
            int carry_t = 0;
            for (int base = 0; base < cn; base += kScanThreads * kScanItems) {
                int ct[kScanItems], sg[kScanItems], se[kScanItems];
#pragma unroll
                for (int k = 0; k < kScanItems; ++k) {
                    const int i = base + scan_item_index(k);
                    ct[k] = 0; sg[k] = -1; se[k] = 0;
                    if (i < cn) {
                        sg[k] = a.x.tord[c0 + i];
                        se[k] = a.seg.e[sg[k]];
                        ct[k] = (nrow[se[k]] + 15) >> 4;
                    }
                }
                int run[kScanItems];
                block_scan_batch(ct, run, carry_t, wsum);
#pragma unroll
                for (int k = 0; k < kScanItems; ++k)
                    if (sg[k] >= 0) { pre_t[sg[k]] = run[k]; pos_t[se[k]] = run[k]; }
            }
            if (tid == 0) a.x.csub[(size_t)cid * P + p] = carry_t;
        }
    }
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) bytes += __shfl_xor(bytes, d, kWave);
    // one sum per rank, added up by k_layout_base: thousands of atomics on one address would take
    // longer than the scans
    __syncthreads();
    if (lane == 0) wbytes[tid / kWave] = bytes;
    __syncthreads();
    if (tid == 0) {
        unsigned long long t = 0;
#pragma unroll
        for (int k = 0; k < kScanThreads / kWave; ++k) t += wbytes[k];
        a.rank_bytes[p] = t;
    }
    if (tid == 0) {
        pre_r[a.nseg] = carry_r; a.Lr.tot[p] = carry_r;
        if (a.want_send) { pre_s[a.nseg] = carry_s; a.Ls.tot[p] = carry_s; }
    }
}

// ------------------------------------------------------------------------------------------
// k_layout_base: exclusive scan over the P per-rank totals of a layout -> each rank's first chunk
// in its staging buffer and its first wave unit.  One workgroup per layout the host lists (receive
// side, send side), then one per class of exact-size T that the phase stores into: there the scan
// runs over the ranks' parts of the class and gives every rank's first chunk in T.  A separate
// launch rather than a "last workgroup" step inside k_phase_layout: the kernel boundary is the one
// device-wide release the totals need.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kScanThreads) k_layout_base(int P, LayoutDev L0, LayoutDev L1, int n_layouts,
                                                              unsigned long long* __restrict__ phase_chunks,
                                                              int chunks_from, ExactT x,
                                                              const unsigned long long* __restrict__ rank_bytes,
                                                              unsigned long long* __restrict__ phase_bytes,
                                                              unsigned int* __restrict__ phase_units) {
    __shared__ long long wc[kScanThreads / kWave];
    __shared__ int wt[kScanThreads / kWave];
    const int which = blockIdx.x;
    if (which < n_layouts) {
        scan_rank_bases(P, which == 0 ? L0 : L1, which == chunks_from ? phase_chunks : nullptr, wc, wt,
                        rank_bytes, which == chunks_from ? phase_bytes : nullptr,
                        phase_units + which);             // layout 0 is the receive side, 1 the send side
        return;
    }
    // a class of exact-size T: rank p's part starts at the class's first chunk plus the parts of the
    // ranks before it, each rounded up to a 128-byte line
    const int cid = x.tcls[3 * (which - n_layouts)];
    const int* sub = x.csub + (size_t)cid * P;
    long long* base = x.tbase + (size_t)cid * P;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const int per = (P + kScanThreads - 1) / kScanThreads;
    const int p0 = min(P, tid * per), p1 = min(P, p0 + per);
    long long sc = 0;
    for (int p = p0; p < p1; ++p) sc += (sub[p] + kRankAlignChunks - 1) / kRankAlignChunks * kRankAlignChunks;
    long long ic = sc;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const long long uc = __shfl_up(ic, d, kWave);
        if (lane >= d) ic += uc;
    }
    if (lane == kWave - 1) wc[wv] = ic;
    __syncthreads();
    long long oc = 0;
#pragma unroll
    for (int k = 0; k < kScanThreads / kWave; ++k)
        if (k < wv) oc += wc[k];
    long long run = x.cbase[cid] + oc + ic - sc;
    for (int p = p0; p < p1; ++p) {
        base[p] = run;
        run += (sub[p] + kRankAlignChunks - 1) / kRankAlignChunks * kRankAlignChunks;
    }
}

// ------------------------------------------------------------------------------------------
// k_layout_units: cut every rank's staged chunks into wave units of L.unit_chunks and record, per
// unit, the rank and the first segment that overlaps it (binary search in the rank's prefix
// row, which is staged in LDS when it fits: lds_ints = nseg + 1, else 0 and the search reads
// global memory).  grid (P, layouts): one workgroup per rank and layout (y = 0 receive side,
// 1 send side).
// ------------------------------------------------------------------------------------------
constexpr int kUnitsLdsMaxInts = 12288;     // 48 KiB of the workgroup's LDS
__global__ void __launch_bounds__(256) k_layout_units(int nseg, LayoutDev Lr, LayoutDev Ls, int lds_ints) {
    extern __shared__ int s_row[];
    const LayoutDev& L = blockIdx.y == 0 ? Lr : Ls;
    const int p = blockIdx.x;
    const int tot = L.tot[p];
    const int uc = L.unit_chunks;
    const int nu = (tot + uc - 1) / uc;
    if (nu == 0) return;                       // uniform over the workgroup
    const int* pre = L.pre + (size_t)p * L.ld;
    if (lds_ints) {
        for (int i = threadIdx.x; i < lds_ints; i += blockDim.x) s_row[i] = pre[i];
        __syncthreads();
        pre = s_row;
    }
    const int ub = L.unit_base[p];
    for (int t = threadIdx.x; t < nu; t += blockDim.x) {
        const int c0 = t * uc;
        int lo = 0, hi = nseg;                 // largest s in [0, nseg) with pre[s] <= c0
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (pre[mid] <= c0) lo = mid; else hi = mid;
        }
        L.units[ub + t] = make_int4(p, lo, c0, min(uc, tot - c0));
    }
}

// ------------------------------------------------------------------------------------------
// The copy engine.  pack / exchange / unpack are the same byte-balanced variable-length copy
// with a different "other side":
//   pack     staging(send)  <- S at sdispls, or T slot      (Algorithm "TuNA", line 15, sender side)
//   exchange staging(recv)  <- staging(send) of the partner (the point-to-point transfer itself)
//   unpack   staging(recv)  -> R at rdispls, or T slot      (Algorithm "TuNA", lines 16-20)
//   fused    S / T of the sender -> R / other copy of T at the receiver, tiled over the receiver's
//            layout (all three in one hop, no staging)
// Work unit = one wavefront x 256 consecutive 16-byte chunks (4 KiB) of one rank's staging
// region.  The wave is self-contained -- no workgroup barrier anywhere: lane i loads the chunk
// prefix and the table entry of segment s0 + i, the lanes whose segment overlaps the unit
// resolve its other-side address (T slot arithmetic, a position in exact-size T, or one
// displacement load), the 64 entries
// go to the wave's private LDS window, and every lane finds the segment of each of its 4 chunks
// by a binary search over that window.  Lanes of a wave touch consecutive chunks on the staging
// side (aligned, non-temporal dwordx4) and consecutive bytes of a block on the other side.
// One-shot grid: 4 units per workgroup; the host launches an upper bound of units and waves
// beyond the device-side unit count exit at once.  A launch for a batch of rounds may instead use
// one grid row per rank, as wide as the units a rank can have in the batch.
// ------------------------------------------------------------------------------------------
struct CopyArgs {
    // tiled (staging) side
    v4u* stage;                         // staging buffer being tiled (unused when fused)
    LayoutDev L;                        // its layout
    SegDev seg;
    int nseg;
    // other side: caller buffer + T (pack, unpack, fused source)
    const int32_t* counts;              // recvcounts: exact sizes of the blocks that are final (unpack, fused)
    unsigned char* user;                // S (pack) or R (unpack)
    const int64_t* displs;              // sdispls (pack), rdispls (unpack); unused when fused (k_resolve_hop read them)
    unsigned long long user_limit;      // pack: address one past the last byte of S that holds a block
    unsigned char* T;                   // temporary buffer: slot s of rank p at ((p*slots + s) * slot_bytes)
    long long slots;
    long long slot_bytes;
    // other side: send staging (exchange)
    const v4u* stage_src;
    LayoutDev Ls;
    // fused: every block's source and destination, resolved by k_resolve_hop
    HopDev hop;
    // exact-size T (DENSE kernels): the blocks that wait in T lie back to back, class by class, instead of in slots
    ExactT x;
    // a launch may cover only the rounds of one batch: the segments [seg_lo, seg_hi) of every rank
    int seg_lo, seg_hi;
    // 1: such a launch has a grid of (units a rank can have in the batch / 4, P) -- row y covers the units
    // of rank y that overlap the batch; 0: one-dimensional grid over all units
    int batch_rows;
    int P, Q, N, dim, rx;
};

template <int GRAN>
__device__ __forceinline__ v4u load_block_chunk(const unsigned char* src, int nb) {
    v4u v = {0u, 0u, 0u, 0u};
    if (GRAN >= 16 || nb >= 16) {
        __builtin_memcpy(&v, src, 16);
    } else if (GRAN == 4) {
        const uint32_t* s4 = reinterpret_cast<const uint32_t*>(src);
        if (nb > 0) v.x = s4[0];
        if (nb > 4) v.y = s4[1];
        if (nb > 8) v.z = s4[2];
    } else {
        uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
        for (int b = 0; b < 15; ++b)
            if (b < nb) w[b >> 2] |= (uint32_t)src[b] << (8 * (b & 3));
        v.x = w[0]; v.y = w[1]; v.z = w[2]; v.w = w[3];
    }
    return v;
}

template <int GRAN>
__device__ __forceinline__ void store_block_chunk(unsigned char* dst, v4u v, int nb) {
    if (GRAN >= 16 || nb >= 16) {
        __builtin_memcpy(dst, &v, 16);
    } else if (GRAN == 4) {
        uint32_t* d4 = reinterpret_cast<uint32_t*>(dst);
        if (nb > 0) d4[0] = v.x;
        if (nb > 4) d4[1] = v.y;
        if (nb > 8) d4[2] = v.z;
    } else {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int b = 0; b < 15; ++b)
            if (b < nb) dst[b] = (unsigned char)(w[b >> 2] >> (8 * (b & 3)));
    }
}

// Address of the block a table entry describes, on the caller-buffer / T side of rank (n, g).
// far_is_source = false: the block's destination rank ((n - j) % N, (g - l) % Q) indexes displs
// (send side); true: its source rank ((n + j) % N, (g + l) % Q) (receive side).
__device__ __forceinline__ unsigned long long block_address(int slot, bool far_is_source, int p, int n, int g,
                                                            int j, int l, int P, int Q, int N,
                                                            unsigned char* user, const int64_t* displs,
                                                            unsigned char* T, long long slots, long long slot_bytes,
                                                            const int32_t* counts = nullptr, int* count = nullptr) {
    if (slot >= 0) return (unsigned long long)(T + ((long long)p * slots + slot) * slot_bytes);
    int pn, pg;
    if (!far_is_source) {
        pn = n - j; if (pn < 0) pn += N;
        pg = g - l; if (pg < 0) pg += Q;
    } else {
        pn = n + j; if (pn >= N) pn -= N;
        pg = g + l; if (pg >= Q) pg -= Q;
    }
    const size_t idx = (size_t)p * P + pn * Q + pg;
    if (counts) *count = counts[idx];          // the caller's count for the same pair (exact size into R)
    return (unsigned long long)(user + displs[idx]);
}

// Exact-size T: where rank p stores segment s of the phase being run, and where rank p holds the
// block with slot index e that phase `ph` stored.
__device__ __forceinline__ unsigned long long exact_t_dst(unsigned char* T, const ExactT& x, int P, int p, int s, int dcls) {
    return (unsigned long long)(T + ((x.tbase[(size_t)dcls * P + p] + (long long)x.tpre[(size_t)p * x.ld + s]) << 4));
}
__device__ __forceinline__ unsigned long long exact_t_src(unsigned char* T, const ExactT& x, int P, int ph, int p, int e,
                                                          int scls) {
    return (unsigned long long)(T + ((x.tbase[(size_t)scls * P + p] + (long long)x.tpos[((size_t)ph * P + p) * P + e]) << 4));
}

// ------------------------------------------------------------------------------------------
// k_resolve_hop: for a one-kernel phase, the source and the destination of every block every rank
// receives (Algorithm "TuNA", lines 15-20 collapsed into one hop: the block goes from where its sender
// holds it -- S at sdispls[sender][destination], or the sender's T -- straight to where its receiver
// keeps it -- R at rdispls[receiver][source], or the receiver's T), in the receiver's message order.
// One thread per (segment, receiving rank).  TP = 1: a workgroup takes 256 segments of one rank, grid
// (ceil(nseg / 256), P).  TP = 16: a workgroup takes 16 segments of each of 16 ranks, grid (ceil(nseg / 16),
// ceil(P / 16)), for phases of many rounds: there neighbouring segments have neighbouring senders, the
// never-moved blocks are looked up in a column of sdispls, and a tile of 16 x 16 touches 31 of its lines
// where 256 segments of one rank touch 256.  Addresses in T are stored as offsets (kHopInT) because a
// persistent plan resolves them before its T is allocated.
// ------------------------------------------------------------------------------------------
struct ResolveArgs {
    const int32_t* nxt;                 // [P][P] block sizes after the phase's size exchange (the receiver's view)
    SegDev seg;
    int nseg;
    int P, Q, N, dim, rx;
    const unsigned char* S;
    const int64_t* sdispls;
    unsigned char* R;
    const int64_t* rdispls;
    long long slots;                    // T in slots: slot s of rank p at offset (p * slots + s) * slot_bytes
    long long slot_bytes;
    ExactT x;                           // T in exact size
    HopDev hop;
    int exact_sizes;                    // 1: every size is the block's byte count (k_hop_small copies exactly that), also into T
};

constexpr int kResolveTile = 16;

template <bool DENSE, int TP>
__global__ void __launch_bounds__(256) k_resolve_hop(const ResolveArgs a) {
    static_assert(TP == 1 || TP == kResolveTile, "one rank or a tile of ranks per workgroup");
    const int s = TP == 1 ? blockIdx.x * 256 + threadIdx.x : blockIdx.x * (256 / TP) + (threadIdx.x % (256 / TP));
    const int p = TP == 1 ? blockIdx.y : blockIdx.y * TP + threadIdx.x / (256 / TP);
    if (s >= a.nseg || p >= a.P) return;
    const int n = p / a.Q, g = p - n * a.Q;
    const int e = a.seg.e[s];
    const int sz = a.nxt[(size_t)p * a.P + e];
    const size_t o = (size_t)p * a.hop.ld + s;
    int j, l;
    split_slot_index(e, a.Q, a.N, j, l);
    const int ssrc = a.seg.src[s], sdst = a.seg.dst[s];
    if (sz <= 0) {
        // an empty block owns no chunk and is never copied; a final one still records where it would lie in
        // R, so that the destination-tiled hop sees the blocks around it as one contiguous run
        unsigned long long d0 = 0;
        if (sdst < 0) {
            int sn = n + j; if (sn >= a.N) sn -= a.N;
            int sg = g + l; if (sg >= a.Q) sg -= a.Q;
            d0 = (unsigned long long)(a.R + a.rdispls[(size_t)p * a.P + sn * a.Q + sg]);
        }
        a.hop.src[o] = 0; a.hop.dst[o] = d0; a.hop.size[o] = 0;
        return;
    }
    // the sender: the rank at distance z r^x upwards in the phase's dimension
    const int q = partner_up(n, g, a.Q, a.N, a.dim, a.seg.z[s] * a.rx);
    unsigned long long src, dst;
    if (ssrc < 0) {                      // never moved: in the sender's S, addressed by its destination rank
        const int qn = q / a.Q, qg = q - qn * a.Q;
        int dn = qn - j; if (dn < 0) dn += a.N;
        int dg = qg - l; if (dg < 0) dg += a.Q;
        src = (unsigned long long)(a.S + a.sdispls[(size_t)q * a.P + dn * a.Q + dg]);
    } else if (DENSE) {
        const size_t row = (size_t)a.seg.srcph[s] * a.P + q;
        src = (((unsigned long long)(a.x.tbase[(size_t)a.seg.scls[s] * a.P + q] + (long long)a.x.tpos[row * a.P + e])) << 4) | kHopInT;
    } else {
        src = (unsigned long long)(((long long)q * a.slots + ssrc) * a.slot_bytes) | kHopInT;
    }
    int size = sz;
    if (sdst < 0) {                      // final: into R at the slot of its source rank, exactly `sz` bytes
        int sn = n + j; if (sn >= a.N) sn -= a.N;
        int sg = g + l; if (sg >= a.Q) sg -= a.Q;
        dst = (unsigned long long)(a.R + a.rdispls[(size_t)p * a.P + sn * a.Q + sg]);
    } else {
        if (!a.exact_sizes) size = ((sz + 15) >> 4) << 4;    // T takes whole chunks
        if (DENSE)
            dst = (((unsigned long long)(a.x.tbase[(size_t)a.seg.dcls[s] * a.P + p] + (long long)a.x.tpre[(size_t)p * a.x.ld + s])) << 4) | kHopInT;
        else
            dst = (unsigned long long)(((long long)p * a.slots + sdst) * a.slot_bytes) | kHopInT | kHopFill;
    }
    a.hop.src[o] = src; a.hop.dst[o] = dst; a.hop.size[o] = size;
}

// ------------------------------------------------------------------------------------------
// k_hop_small: a one-kernel phase whose blocks all fit into 64 bytes (Section "Performance analysis of
// TuNA": the small-message regime, S of a few bytes).  The byte-balanced engine above cuts work into
// 4 KiB units and searches a window of block boundaries per unit; with blocks of a few bytes that
// search is most of the work.  Here one thread moves one block: it reads the block's resolved source,
// destination and size (k_resolve_hop) and copies its at most 16 words (or 64 bytes).  Neighbouring
// threads hold neighbouring blocks of one receiver, whose destinations are neighbours in R or T, so a
// wave's stores fall into a few lines.  grid (ceil(segments / 256), P); a batch of rounds covers the
// segments [seg_lo, seg_hi).
// ------------------------------------------------------------------------------------------
constexpr int kSmallBlockBytes = 64;
template <int GRAN>
__global__ void __launch_bounds__(256) k_hop_small(HopDev hop, unsigned char* T, int seg_lo, int seg_hi) {
    const int s = seg_lo + blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= seg_hi) return;
    const size_t o = (size_t)blockIdx.y * hop.ld + s;
    const int size = hop.size[o];
    if (size <= 0) return;
    const unsigned long long hs = hop.src[o], hd = hop.dst[o];
    const unsigned long long tb = (unsigned long long)T;
    const unsigned char* src = reinterpret_cast<const unsigned char*>((hs & ~(kHopInT | kHopFill)) + ((hs & kHopInT) ? tb : 0ull));
    unsigned char* dst = reinterpret_cast<unsigned char*>((hd & ~(kHopInT | kHopFill)) + ((hd & kHopInT) ? tb : 0ull));
    if (GRAN >= 4) {
        // all loads first, then all stores; `size` is the block's exact byte count (ResolveArgs.exact_sizes)
        const uint32_t* s4 = reinterpret_cast<const uint32_t*>(src);
        uint32_t* d4 = reinterpret_cast<uint32_t*>(dst);
        const int n = min(size, kSmallBlockBytes) >> 2;
        uint32_t w[kSmallBlockBytes / 4];
#pragma unroll
        for (int i = 0; i < kSmallBlockBytes / 4; ++i) w[i] = i < n ? s4[i] : 0u;
#pragma unroll
        for (int i = 0; i < kSmallBlockBytes / 4; ++i)
            if (i < n) d4[i] = w[i];
    } else {
        const int n = min(size, kSmallBlockBytes);
        for (int i = 0; i < n; ++i) dst[i] = src[i];
    }
}

// Compiled for 8 waves per SIMD (a workgroup is one wave per SIMD).  The host lowers the number of
// resident workgroups per launch where fewer are faster by asking for unused dynamic LDS.  Unpack
// keeps its payload in registers across the address resolution; left alone the compiler then takes
// 84 registers (5 waves), held to 8 waves it needs 64 and spills nothing (byte-granular calls excepted).
// The one-kernel variant needs 62 to 72 registers by itself.  Where it fits into 64 without spilling
// (4-byte granular, exact-size T) it is held to 8 waves too: scheduled for occupancy, gathers of many
// short pieces run 6 % faster (measured at r = P on 16 GiB); the variants that would spill are left alone.
template <int MODE, int GRAN, bool DENSE>
__global__ void __launch_bounds__(kCopyThreads) __attribute__((amdgpu_waves_per_eu(((MODE == kUnpack && GRAN >= 4) || (MODE == kFused && GRAN == 4 && DENSE)) ? 8 : 1, 8)))
k_copy(const CopyArgs a) {
    __shared__ int s_pre[kCopyThreads / kWave][kWave];
    __shared__ int s_size[kCopyThreads / kWave][kWave];
    __shared__ unsigned long long s_addr[kCopyThreads / kWave][kWave];
    __shared__ unsigned long long s_addr2[MODE == kFused ? kCopyThreads / kWave : 1][kWave];
    __shared__ int s_flag[kCopyThreads / kWave][kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    int unit = blockIdx.x * (kCopyThreads / kWave) + wv;
    if (a.batch_rows) {
        // the batch's chunks [lo, hi) of rank blockIdx.y lie in its units lo / 256 .. (hi - 1) / 256
        const int* brow = a.L.pre + (size_t)blockIdx.y * a.L.ld;
        const int lo = brow[a.seg_lo], hi = brow[a.seg_hi];
        const int u = lo / kUnitChunks + unit;
        if (hi <= lo || (long long)u * kUnitChunks >= hi) return;
        unit = a.L.unit_base[blockIdx.y] + u;
    } else if (unit >= *a.L.n_units) {
        return;                                  // no barrier below: a wave may leave alone
    }
    const int4 ud = a.L.units[unit];
    const int p = __builtin_amdgcn_readfirstlane(ud.x);
    int sw = __builtin_amdgcn_readfirstlane(ud.y);
    const int c0 = __builtin_amdgcn_readfirstlane(ud.z);
    const int cend = c0 + __builtin_amdgcn_readfirstlane(ud.w);
    const int n = p / a.Q, g = p - n * a.Q;
    const int* prow = a.L.pre + (size_t)p * a.L.ld;
    v4u* stage = MODE == kFused ? nullptr : a.stage + a.L.rank_base[p];
    int* wpre = s_pre[wv];
    int* wsize = s_size[wv];
    unsigned long long* waddr = s_addr[wv];
    unsigned long long* waddr2 = s_addr2[MODE == kFused ? wv : 0];
    int* wflag = s_flag[wv];

    // batch of rounds: the rank's chunks [blo, bhi) belong to this launch
    int blo = 0, bhi = INT_MAX;
    if (a.seg_hi - a.seg_lo < a.nseg) {
        blo = prow[a.seg_lo];
        bhi = prow[a.seg_hi];
        if (c0 >= bhi || cend <= blo) return;
    }
    int c[kChunksPerLane];
    bool pend[kChunksPerLane];
#pragma unroll
    for (int k = 0; k < kChunksPerLane; ++k) {
        c[k] = c0 + k * kWave + lane;
        pend[k] = c[k] < cend && c[k] >= blo && c[k] < bhi;
    }
    for (;;) {
        // ---- window: segments sw .. sw+63, one per lane --------------------------------------
        const int s = sw + lane;
        int pre_i, pre_w;                            // pre_w is wave-uniform: the first prefix of the next window
        // table fields this mode needs, fetched together with the prefix
        int se = 0, sz_ = 0, ssrc = -1, sdst = -1, sph = -1, scl = -1;
        unsigned long long addr = 0, addr2 = 0;
        int size = 0, flag = 0;
        if (MODE == kFused) {
            // One-kernel phases: source, destination and size of every block were resolved by k_resolve_hop.
            // Every lane loads from an index clamped into range instead of under a branch, so that the
            // loads sit in one basic block and go out back to back.
            const int s_tab = min(s, a.nseg - 1);
            const size_t hi_ = (size_t)p * a.hop.ld + s_tab;
            const int pre_raw = prow[min(s, a.nseg)];
            const int pre_w_raw = prow[min(sw + kWave, a.nseg)];
            // A unit of 256 chunks seldom overlaps more than a few blocks: the first kHopLanes lanes fetch
            // their entries at once, together with the prefix (the condition depends on no loaded value);
            // the others only when the prefix shows that the unit reaches that far (many tiny blocks).
            const bool early = lane < kHopLanes;
            unsigned long long hs_ = 0, hd_ = 0;
            if (early) { hs_ = a.hop.src[hi_]; hd_ = a.hop.dst[hi_]; size = a.hop.size[hi_]; }
            pre_i = s <= a.nseg ? pre_raw : INT_MAX;
            pre_w = sw + kWave <= a.nseg ? pre_w_raw : INT_MAX;
            const int reach = __popcll(__ballot(pre_i < cend));
            if (reach > kHopLanes) {
                if (!early && lane < reach) { hs_ = a.hop.src[hi_]; hd_ = a.hop.dst[hi_]; size = a.hop.size[hi_]; }
            }
            const unsigned long long tb = (unsigned long long)a.T;
            addr = (hs_ & ~(kHopInT | kHopFill)) + ((hs_ & kHopInT) ? tb : 0ull);
            addr2 = (hd_ & ~(kHopInT | kHopFill)) + ((hd_ & kHopInT) ? tb : 0ull);
            // chunks are cut at the destination's 16-byte boundaries: `head` bytes of the first chunk lie
            // before the block (0 in T, where blocks start on chunk or line boundaries)
            flag = (int)(addr2 & 15ull) | ((hs_ & kHopInT) ? kFlagSrcT : 0) | ((hd_ & kHopFill) ? kFlagFill : 0);
        } else {
            pre_i = s <= a.nseg ? prow[s] : INT_MAX;
            pre_w = sw + kWave <= a.nseg ? prow[sw + kWave] : INT_MAX;
        }
        int pre_n = __shfl_down(pre_i, 1, kWave);
        if (lane == kWave - 1) pre_n = pre_w;
        if (MODE != kFused && s < a.nseg) {
            if (MODE != kExchange) se = a.seg.e[s];
            if (MODE == kExchange) sz_ = a.seg.z[s];
            if (MODE == kPack) {
                ssrc = a.seg.src[s];
                if (DENSE) { sph = a.seg.srcph[s]; scl = a.seg.scls[s]; }
            }
            if (MODE == kUnpack) {
                sdst = a.seg.dst[s];
                if (DENSE) scl = a.seg.dcls[s];
            }
        }
        const int wend = pre_w;                      // chunks below wend resolve in this window
        // unpack reads its own staging region: the payload loads of this window need only its bounds and
        // go out before the addresses are resolved, so the two latencies overlap
        bool act[kChunksPerLane];
        v4u v[kChunksPerLane];
#pragma unroll
        for (int k = 0; k < kChunksPerLane; ++k) {
            act[k] = pend[k] && c[k] < wend;
            if (MODE == kUnpack && act[k]) v[k] = __builtin_nontemporal_load(stage + c[k]);
        }
        const bool need = MODE != kFused && s < a.nseg && pre_i < cend && pre_n > pre_i && pre_n > c0;
        if (need) {
            if (MODE == kExchange) {
                const int ps = partner_up(n, g, a.Q, a.N, a.dim, sz_ * a.rx);
                addr = (unsigned long long)(a.stage_src + a.Ls.rank_base[ps] + a.Ls.pre[(size_t)ps * a.Ls.ld + s]);
                size = (pre_n - pre_i) << 4;
            } else {
                // `size` = bytes of the block the destination may receive.  Staging and T slots are
                // padded to whole chunks (lines), so they take whole chunks; a store into R must end
                // exactly with the block.  A load may always run up to 15 bytes past a block's end in
                // T or staging; in S only while it stays inside the part of S that holds blocks.
                size = (pre_n - pre_i) << 4;
                int bj, bl;
                split_slot_index(se, a.Q, a.N, bj, bl);
                if (MODE == kPack) {
                    if (DENSE && ssrc >= 0)
                        addr = exact_t_src(a.T, a.x, a.P, sph, p, se, scl);
                    else
                        addr = block_address(ssrc, false, p, n, g, bj, bl, a.P, a.Q, a.N, a.user, a.displs, a.T,
                                             a.slots, a.slot_bytes);
                    if (ssrc >= 0) flag |= kFlagSrcT;
                }
                if (MODE == kUnpack) {
                    // a final block's size is the receiver's own recvcounts entry (validated equal to
                    // the sender's count), read next to its displacement
                    if (DENSE && sdst >= 0)           // exact-size T: blocks lie back to back, nothing to fill
                        addr = exact_t_dst(a.T, a.x, a.P, p, s, scl);
                    else
                        addr = block_address(sdst, true, p, n, g, bj, bl, a.P, a.Q, a.N, a.user, a.displs, a.T,
                                             a.slots, a.slot_bytes, a.counts, &size);
                    if (!DENSE && sdst >= 0) flag |= kFlagFill; // T-bound: the tail lane completes the 128-byte line
                }
            }
        }
        wpre[lane] = pre_i;
        wsize[lane] = size;
        wflag[lane] = flag;
        waddr[lane] = addr;
        if (MODE == kFused) waddr2[lane] = addr2;
        // the window is private to this wave; its LDS writes are ordered before the reads below
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // entries that can hold a chunk of this unit: the leading lanes with pre_i < cend
        const int nlive = __popcll(__ballot(pre_i < cend));
        int steps = 0;
        while ((1 << steps) < nlive) ++steps;

        unsigned long long oa[kChunksPerLane], oa2[kChunksPerLane];
        int nb[kChunksPerLane], fill[kChunksPerLane];
        // The four searches of a lane advance together, without branches: every step is four independent
        // LDS reads and one wait instead of a dependent chain per chunk.  Lanes without a chunk search
        // for whatever c[k] holds; their result is masked out below.
        int lo[kChunksPerLane], hi[kChunksPerLane];  // wpre[lo] <= c < wpre[hi] (hi == nlive: sentinel)
#pragma unroll
        for (int k = 0; k < kChunksPerLane; ++k) { lo[k] = 0; hi[k] = nlive; }
        for (int it = 0; it < steps; ++it) {
#pragma unroll
            for (int k = 0; k < kChunksPerLane; ++k) {
                const int mid = (lo[k] + hi[k]) >> 1;
                const bool up = wpre[mid] <= c[k];
                const bool move = mid > lo[k];
                lo[k] = (move && up) ? mid : lo[k];
                hi[k] = (move && !up) ? mid : hi[k];
            }
        }
#pragma unroll
        for (int k = 0; k < kChunksPerLane; ++k) {
            const int lim = wsize[lo[k]];
            const int fl = wflag[lo[k]];
            int off = (c[k] - wpre[lo[k]]) << 4;     // first byte of the chunk, relative to the block
            int end = off + 16;
            if (MODE == kFused) {                     // chunk grid anchored at the destination line
                const int h = fl & 15;
                end = off + 16 - h;
                off = max(off - h, 0);
            }
            const unsigned long long src = waddr[lo[k]] + (unsigned long long)(long long)off;
            oa[k] = act[k] ? src : 0ull;
            if (MODE == kFused) oa2[k] = act[k] ? waddr2[lo[k]] + (unsigned long long)(long long)off : 0ull;
            else oa2[k] = 0;
            nb[k] = act[k] ? min(end, lim) - off : 0;
            // last chunk of a T-bound block in a slot: number of further chunks up to the 128-byte line end
            fill[k] = (!DENSE && act[k] && (fl & kFlagFill) && (end >= lim)) ? ((128 - (end & 127)) & 127) >> 4 : 0;
            pend[k] = pend[k] && !act[k];
            // Rare: a whole-chunk load from S is safe only inside the part of S that holds blocks.  The
            // last few bytes of S are loaded exactly and stored at once; the chunk then takes no part in
            // the batched loads and stores below (and none of its state stays live across them).
            if ((MODE == kPack || MODE == kFused) && act[k] && !(fl & kFlagSrcT) && src + 16 > a.user_limit) {
                const int ns = (int)min((unsigned long long)nb[k], a.user_limit - src);
                const v4u t = load_block_chunk<GRAN>(reinterpret_cast<const unsigned char*>(src), min(ns, 15));
                if (MODE == kPack) {
                    __builtin_nontemporal_store(t, stage + c[k]);
                } else {
                    unsigned char* dst = reinterpret_cast<unsigned char*>(oa2[k]);
                    store_block_chunk<GRAN>(dst, t, min(ns, 15));
                    for (int f = 1; f <= fill[k]; ++f) *reinterpret_cast<v4u*>(dst + 16 * f) = t;
                }
                act[k] = false;
                fill[k] = 0;
            }
        }
        // ---- whole-chunk loads, all in flight before the first store --------------------------
#pragma unroll
        for (int k = 0; k < kChunksPerLane; ++k) {
            if (MODE != kUnpack && act[k]) {
                if (MODE == kExchange) v[k] = *reinterpret_cast<const v4u*>(oa[k]);   // neighbours share its edge lines
                // blocks that are whole 128-byte lines share no line with a neighbour: streaming loads
                // (measured on 256-byte blocks: pack +7 to +19 %, one-kernel phases +3 to +6 %; with blocks
                // that share their edge lines they lose up to 15 %)
                else if (GRAN == 128) v[k] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(oa[k]));
                else __builtin_memcpy(&v[k], reinterpret_cast<const unsigned char*>(oa[k]), 16);
            }
        }
        // ---- stores: whole chunks into staging and T, exact bytes into R -------------------------
#pragma unroll
        for (int k = 0; k < kChunksPerLane; ++k) {
            if (act[k]) {
                if (MODE == kUnpack || MODE == kFused) {
                    unsigned char* dst = reinterpret_cast<unsigned char*>(MODE == kFused ? oa2[k] : oa[k]);
                    // with exact-size T whole chunks stream into R and into T (measured: +3 to +9 %);
                    // slots of M bytes are written through the cache, where the fill completes their lines,
                    // and telling the two apart per chunk costs more registers than it gains.  Byte-granular
                    // calls keep plain stores: the address may have any alignment.
                    if (DENSE && GRAN >= 4 && nb[k] >= 16) {
                        typedef v4u v4u_word_aligned __attribute__((aligned(4)));
                        __builtin_nontemporal_store(v[k], reinterpret_cast<v4u_word_aligned*>(dst));
                    } else {
                        store_block_chunk<GRAN>(dst, v[k], nb[k]);
                    }
                } else {
                    __builtin_nontemporal_store(v[k], stage + c[k]);
                }
            }
        }
        // ---- line fill: after the last chunk of a T-bound block the rest of its 128-byte line is
        // written too (content is don't-care), so that T only ever sees whole-line writes.  One
        // store instruction per block tail: lanes 0..f-1 write the f missing chunks.
        if (!DENSE && (MODE == kUnpack || MODE == kFused)) {
#pragma unroll
            for (int k = 0; k < kChunksPerLane; ++k) {
                const unsigned long long dsta = MODE == kFused ? oa2[k] : oa[k];
                unsigned long long m = __ballot(act[k] && fill[k] > 0);
                while (m) {
                    const int leader = __ffsll((long long)m) - 1;
                    m &= m - 1;
                    const unsigned int lo32 = __builtin_amdgcn_readlane((unsigned int)dsta, leader);
                    const unsigned int hi32 = __builtin_amdgcn_readlane((unsigned int)(dsta >> 32), leader);
                    const int f = __builtin_amdgcn_readlane(fill[k], leader);
                    if (lane < f) {
                        const v4u zero = {0u, 0u, 0u, 0u};
                        unsigned char* base = reinterpret_cast<unsigned char*>(((unsigned long long)hi32 << 32) | lo32);
                        *reinterpret_cast<v4u*>(base + 16 * (lane + 1)) = zero;
                    }
                }
            }
        }
        if (wend >= cend) break;
        sw += kWave;
        __builtin_amdgcn_wave_barrier();
    }
}

// ------------------------------------------------------------------------------------------
// The destination-tiled hop.  What a rank receives in a one-kernel phase lands in a few long contiguous
// runs: the final blocks in R (Algorithm "TuNA", lines 16-18) when the receive regions are dense -- every
// rank's blocks back to back in source order, the usual layout --, the others in exact-size T, where
// the blocks of a class lie back to back.  The copy engine cuts such a phase into 16-byte chunks per
// block; a block that does not start on a 16-byte boundary shares a chunk with its predecessor, the
// chunk count drifts against the addresses, and a wave's 64-lane store never covers whole 128-byte
// lines: measured, streaming stores that begin and end inside lines cost 13 % of the hop's rate
// (blocks of whole lines, destination 4 or 16 bytes off a line: 4.9 and 4.7 TB/s against 5.6 to 5.8
// aligned).  Here the unit of work is the destination itself: a run is cut into its 16-byte pieces
// from the 128-byte line it starts in to the line it ends in, every piece belongs to exactly one lane,
// a piece that holds the end of one block and the start of the next is assembled by that lane from
// both, and every wave store covers eight whole lines.
//
// k_tiled_layout (one workgroup per rank, the scan machinery of k_phase_layout): from the resolved
// destinations and sizes (k_resolve_hop) the number of pieces every segment owns.  Segment s with
// destination a, size n, end E = a + n continues a run when its predecessor in message order ends at a
// (empty blocks lie where they would lie, so they continue runs too); it then owns the pieces from
// ceil(a / 16) to ceil(E / 16) -- the piece that holds its first bytes, if shared, belongs to a
// predecessor.  A segment that starts a run owns the pieces from the start of a's 128-byte line, and
// in front of them come the dead pieces that complete the previous run's last line, so that every run
// starts at a multiple of 8 pieces.  The prefix row has the same form as a chunk prefix row:
// k_layout_base and k_layout_units cut it into wave units of 256 pieces.
// ------------------------------------------------------------------------------------------
struct TiledLayoutArgs {
    HopDev hop;
    int nseg, P;
    LayoutDev Lr;
    unsigned long long* rank_bytes;     // [P]: payload bytes every rank receives in the phase; nullptr: already known
};

// pieces segment s owns, and the dead pieces in front of them
__device__ __forceinline__ int tiled_pieces(unsigned long long a, int n, bool has_prev, unsigned long long e_prev,
                                            int* dead) {
    const unsigned long long e = a + (unsigned long long)n;
    const bool new_run = !has_prev || e_prev != a;
    const unsigned long long last = (e + 15) >> 4;
    const unsigned long long first = new_run ? (a >> 7) << 3 : (a + 15) >> 4;
    *dead = (new_run && has_prev) ? (int)((((e_prev + 127) >> 7) << 3) - ((e_prev + 15) >> 4)) : 0;
    return last > first ? (int)(last - first) : 0;
}

__global__ void __launch_bounds__(kScanThreads) k_tiled_layout(const TiledLayoutArgs a) {
    __shared__ int wsum[kScanThreads / kWave];
    __shared__ unsigned long long wbytes[kScanThreads / kWave];
    const int p = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const size_t o = (size_t)p * a.hop.ld;
    int* pre_r = a.Lr.pre + (size_t)p * a.Lr.ld;
    int carry = 0;
    unsigned long long bytes = 0;
    for (int base = 0; base < a.nseg; base += kScanThreads * kScanItems) {
        int cr[kScanItems];
#pragma unroll
        for (int k = 0; k < kScanItems; ++k) {
            const int s = base + scan_item_index(k);
            cr[k] = 0;
            if (s < a.nseg) {
                // a destination in T is an offset with the in-T bit set; T starts on a 256-byte boundary, so the
                // raw values align and follow each other exactly like the addresses they stand for
                const unsigned long long d = a.hop.dst[o + s];
                const int n = a.hop.size[o + s];
                unsigned long long e_prev = 0;
                if (s > 0) e_prev = a.hop.dst[o + s - 1] + (unsigned long long)a.hop.size[o + s - 1];
                int dead;
                const int own = tiled_pieces(d, n, s > 0, e_prev, &dead);
                cr[k] = dead + own;
                bytes += (unsigned long long)n;
            }
        }
        int run[kScanItems];
        block_scan_batch(cr, run, carry, wsum);
#pragma unroll
        for (int k = 0; k < kScanItems; ++k) {
            const int s = base + scan_item_index(k);
            if (s < a.nseg) pre_r[s] = run[k];
        }
    }
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) bytes += __shfl_xor(bytes, d, kWave);
    __syncthreads();
    if (lane == 0) wbytes[tid / kWave] = bytes;
    __syncthreads();
    if (tid == 0) {
        unsigned long long t = 0;
#pragma unroll
        for (int k = 0; k < kScanThreads / kWave; ++k) t += wbytes[k];
        if (a.rank_bytes) a.rank_bytes[p] = t;
        pre_r[a.nseg] = carry; a.Lr.tot[p] = carry;
    }
}

// ------------------------------------------------------------------------------------------
// k_copy_tiled: the payload kernel of the destination-tiled hop.  Work unit = one wavefront x
// 64 CPL consecutive pieces of one rank (k_tiled_layout; CPL = 4, or 8 for a word-granular last phase: what
// a wave spends on its edge pieces does not grow with the unit, measured 4.6 % per start at r = P on the
// 16 GiB workload, while phases without edge pieces lose 2 % with the larger unit); no workgroup barrier.  Lane i of a window loads
// the prefix and the resolved source, destination and size of segment s0 + i and derives the address of
// the segment's first own piece; every lane finds the segment of each of its CPL pieces by the same
// branch-free search as the copy engine.  A piece that lies inside its block is one 16-byte load at
// the source's own alignment and one aligned streaming store.  A piece at a block's edge is put together
// word by word (GRAN = 4: every size and address is a multiple of 4) from its block and the one behind it
// in the run (a walk over the window's entries, and over the hop arrays behind the window, when more blocks
// than that meet in one piece) and stored whole
// when all four words belong to blocks, else word by word (the ends of a run: bytes outside every block
// are never written).  With GRAN = 16 every piece is inside a block or outside all of them.  Blocks bound
// for T take whole chunks; a load never leaves the part of S that holds blocks.
// ------------------------------------------------------------------------------------------
struct TiledCopyArgs {
    LayoutDev L;
    HopDev hop;
    int nseg;
    unsigned char* T;
    unsigned long long user_limit;      // address one past the last byte of S that holds a block
};

template <int GRAN, int CPL>
__global__ void __launch_bounds__(kCopyThreads) k_copy_tiled(const TiledCopyArgs a) {
    __shared__ int s_pre[kCopyThreads / kWave][kWave];
    __shared__ int s_size[kCopyThreads / kWave][kWave];
    __shared__ int s_off0[kCopyThreads / kWave][kWave];
    __shared__ int s_lim[kCopyThreads / kWave][kWave];
    __shared__ unsigned long long s_src[kCopyThreads / kWave][kWave];
    __shared__ unsigned long long s_dst[kCopyThreads / kWave][kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int unit = blockIdx.x * (kCopyThreads / kWave) + wv;
    if (unit >= *a.L.n_units) return;                // no barrier below: a wave may leave alone
    const int4 ud = a.L.units[unit];
    const int p = __builtin_amdgcn_readfirstlane(ud.x);
    int sw = __builtin_amdgcn_readfirstlane(ud.y);
    const int c0 = __builtin_amdgcn_readfirstlane(ud.z);
    const int cend = c0 + __builtin_amdgcn_readfirstlane(ud.w);
    const int* prow = a.L.pre + (size_t)p * a.L.ld;
    const size_t ho = (size_t)p * a.hop.ld;
    int* wpre = s_pre[wv];
    int* wsize = s_size[wv];
    int* woff0 = s_off0[wv];
    int* wlim = s_lim[wv];
    unsigned long long* wsrc = s_src[wv];
    unsigned long long* wdst = s_dst[wv];
    const unsigned long long tb = (unsigned long long)a.T;
    int c[CPL];
    bool pend[CPL];
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        c[k] = c0 + k * kWave + lane;
        pend[k] = c[k] < cend;
    }
    for (;;) {
        // ---- window: segments sw .. sw+63, one per lane; loads from clamped indices.  A unit of 256 pieces seldom
        // overlaps more than a few blocks: the first kHopLanes lanes fetch their entries together with the
        // prefix, the others only when the prefix shows that the unit reaches that far (two entries more than
        // it reaches: the last piece of the unit may hold the first words of the blocks behind it).
        const int s = sw + lane;
        const int s_tab = min(s, a.nseg - 1);
        const int pre_raw = prow[min(s, a.nseg)];
        const int pre_w_raw = prow[min(sw + kWave, a.nseg)];
        const bool early = lane < kHopLanes;
        unsigned long long hs_ = 0, hd_ = 0;
        int size = 0;
        if (early) { hs_ = a.hop.src[ho + s_tab]; hd_ = a.hop.dst[ho + s_tab]; size = a.hop.size[ho + s_tab]; }
        // the end of the block in front of the window, for its first segment
        unsigned long long e_front = 0;
        if (lane == 0 && sw > 0) e_front = a.hop.dst[ho + sw - 1] + (unsigned long long)a.hop.size[ho + sw - 1];
        const int pre_i = s <= a.nseg ? pre_raw : INT_MAX;
        const int pre_w = sw + kWave <= a.nseg ? pre_w_raw : INT_MAX;
        const int nload = min(kWave, max(kHopLanes, __popcll(__ballot(pre_i < cend)) + 2));
        if (nload > kHopLanes) {
            if (!early && lane < nload) { hs_ = a.hop.src[ho + s_tab]; hd_ = a.hop.dst[ho + s_tab]; size = a.hop.size[ho + s_tab]; }
        }
        unsigned long long e_prev = __shfl_up(hd_ + (unsigned long long)size, 1, kWave);
        if (lane == 0) e_prev = e_front;
        // Offset of piece 0 of the segment's row from the block's first byte: a segment that starts a run owns
        // the pieces from its 128-byte line's start, behind the dead pieces that complete the previous run's
        // line; one that continues a run owns them from the first piece that begins inside the block.  Dead
        // pieces and the pieces in front of the block come out with negative offsets and hold none of its bytes.
        int dead;
        (void)tiled_pieces(hd_, size, s_tab > 0, e_prev, &dead);
        const bool new_run = s_tab == 0 || e_prev != hd_;
        const int off0 = (new_run ? -(int)((unsigned int)hd_ & 127u) : (int)((0u - (unsigned int)hd_) & 15u)) - (dead << 4);
        const unsigned long long src_addr = (hs_ & ~(kHopInT | kHopFill)) + ((hs_ & kHopInT) ? tb : 0ull);
        // A block bound for T takes whole chunks: its last piece is loaded whole and may run up to 15 bytes past
        // the block's end.  In T that is padding; in S it is the next block, except at the very end of S: `lim` =
        // the bytes that may be loaded from the block's start on.
        int lim = size;
        if (!(hs_ & kHopInT)) lim = (int)min((unsigned long long)size, a.user_limit > src_addr ? a.user_limit - src_addr : 0ull);
        wpre[lane] = pre_i;
        wsize[lane] = size;
        woff0[lane] = off0;
        wlim[lane] = lim;
        wsrc[lane] = src_addr;
        wdst[lane] = (hd_ & ~(kHopInT | kHopFill)) + ((hd_ & kHopInT) ? tb : 0ull);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int wend = pre_w;                      // pieces below wend resolve in this window
        const int nlive = __popcll(__ballot(pre_i < cend));
        int steps = 0;
        while ((1 << steps) < nlive) ++steps;
        bool act[CPL];
        int lo[CPL], hi[CPL];
#pragma unroll
        for (int k = 0; k < CPL; ++k) { act[k] = pend[k] && c[k] < wend; lo[k] = 0; hi[k] = nlive; }
        for (int it = 0; it < steps; ++it) {
#pragma unroll
            for (int k = 0; k < CPL; ++k) {
                const int mid = (lo[k] + hi[k]) >> 1;
                const bool up = wpre[mid] <= c[k];
                const bool move = mid > lo[k];
                lo[k] = (move && up) ? mid : lo[k];
                hi[k] = (move && !up) ? mid : hi[k];
            }
        }
        // every piece as a byte offset from its block's start: 32-bit arithmetic from here on
        int off[CPL];
        bool whole[CPL], edge[CPL];
        v4u v[CPL];
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            const int idx = lo[k];
            off[k] = woff0[idx] + ((c[k] - wpre[idx]) << 4);
            whole[k] = act[k] && off[k] >= 0 && off[k] + 16 <= wlim[idx];
            edge[k] = act[k] && !whole[k] && off[k] > -16;
            pend[k] = pend[k] && !act[k];
        }
        // ---- loads of the pieces inside their blocks, issued together ----------------------------------------
#pragma unroll
        for (int k = 0; k < CPL; ++k)
            if (whole[k]) __builtin_memcpy(&v[k], reinterpret_cast<const unsigned char*>(wsrc[lo[k]] + (unsigned long long)(long long)off[k]), 16);
        // ---- pieces at block edges: a word lies in the piece's block, in the block behind it, or in none.  The
        // loads go out at once and travel with the ones above; nothing loaded is looked at before the stores.
        // A unit holds a handful of block edges, seldom two in one lane: every lane takes its first edge piece,
        // then its second ..., so that the code below runs once or twice per wave, not once per piece index.
        unsigned int emask = 0;                      // bit 4 k + q: word q of piece k was loaded
        unsigned int raremask = 0;
        if (GRAN < 16) {
            static_assert(CPL <= 8, "emask holds four bits per piece");
            unsigned int todo = 0;
#pragma unroll
            for (int k = 0; k < CPL; ++k) todo |= edge[k] ? 1u << k : 0u;
            while (__ballot(todo != 0)) {
                bool on = todo != 0;
                const int ks = on ? __ffs((int)todo) - 1 : 0;
                todo &= todo - 1;
                int offk = off[0], t = lo[0];
#pragma unroll
                for (int k = 1; k < CPL; ++k) { offk = ks == k ? off[k] : offk; t = ks == k ? lo[k] : t; }
                const int n = wsize[t];
                const int nlim = wlim[t];                    // < n only for the last block of S when it is bound for T
                const bool has_next = sw + t + 1 < a.nseg;
                const bool next_here = has_next && t + 1 < nload;
                const int tn = min(t + 1, kWave - 1);
                const int nn = wsize[tn];
                const bool follows = next_here && wdst[tn] == wdst[t] + (unsigned long long)n;
                const int over = offk + 16 - n;              // bytes of the piece behind this block's end
                // the walk over several blocks is needed when the block behind is not in the window, is empty,
                // or ends inside this piece too
                if (on && over > 0 && has_next && (!next_here || (follows && nn < over && sw + t + 2 < a.nseg))) {
                    raremask |= 1u << ks;
                    on = false;
                }
                const unsigned long long sa = wsrc[t] + (unsigned long long)(long long)offk;
                const unsigned long long sb = wsrc[tn] + (unsigned long long)(long long)(offk - n);
                uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int o = offk + 4 * q, o2 = o - n;
                    const bool mine = o >= 0 && o < n;
                    const bool theirs = follows && o2 >= 0 && o2 < nn;
                    if (on && (mine || theirs)) {
                        if (mine ? o < nlim : o2 < wlim[tn]) w[q] = *reinterpret_cast<const uint32_t*>((mine ? sa : sb) + 4u * q);
                        emask |= 1u << (4 * ks + q);
                    }
                }
#pragma unroll
                for (int kk = 0; kk < CPL; ++kk)
                    if (on && kk == ks) { v[kk][0] = w[0]; v[kk][1] = w[1]; v[kk][2] = w[2]; v[kk][3] = w[3]; }
            }
            // rare: the blocks of a piece reach past the entries the window holds, or several blocks end inside
            // one piece (a row of tiny or empty blocks): a walk over the entries in the window, and over the hop
            // arrays in global memory behind it
#pragma unroll
            for (int k = 0; k < CPL; ++k) {
                if (!(raremask & (1u << k))) continue;
                int t = sw + lo[k];
                unsigned long long ta = wdst[lo[k]], te = ta + (unsigned long long)wsize[lo[k]], ts = wsrc[lo[k]];
                long long tl = wlim[lo[k]];                         // bytes of the block that may be loaded
                const unsigned long long d = ta + (unsigned long long)(long long)off[k];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const unsigned long long b = d + 4u * q;
                    bool in_run = true;
                    while (b >= te) {                // the word lies behind this block: the next one, if it follows directly
                        ++t;
                        if (t >= a.nseg) { in_run = false; break; }
                        const int wi = t - sw;
                        unsigned long long na, nsa;
                        int nsz;
                        long long nl;
                        if (wi < nload) {            // the window holds the entry
                            na = wdst[wi]; nsa = wsrc[wi]; nsz = wsize[wi]; nl = wlim[wi];
                        } else {
                            const unsigned long long nraw = a.hop.dst[ho + t], nsrc = a.hop.src[ho + t];
                            na = (nraw & ~(kHopInT | kHopFill)) + ((nraw & kHopInT) ? tb : 0ull);
                            nsa = (nsrc & ~(kHopInT | kHopFill)) + ((nsrc & kHopInT) ? tb : 0ull);
                            nsz = a.hop.size[ho + t];
                            nl = nsz;
                            if (!(nsrc & kHopInT)) nl = (long long)min((unsigned long long)nsz, a.user_limit > nsa ? a.user_limit - nsa : 0ull);
                        }
                        if (na != te) { in_run = false; break; }
                        ta = na; te = na + (unsigned long long)nsz; ts = nsa; tl = nl;
                    }
                    if (!in_run) break;              // nothing behind the run's end belongs to a block
                    if (b >= ta) {
                        const unsigned long long o = b - ta;
                        v[k][q] = (long long)o < tl ? *reinterpret_cast<const uint32_t*>(ts + o) : 0u;
                        emask |= 1u << (4 * k + q);
                    }
                }
            }
        }
        // ---- stores: whole pieces and edge pieces with all four words as aligned streaming stores (eight whole
        // lines per wave store), the others word by word (the ends of a run) -----------------------------------
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            if (whole[k] || edge[k]) {
                unsigned char* d = reinterpret_cast<unsigned char*>(wdst[lo[k]] + (unsigned long long)(long long)off[k]);
                const unsigned int em = (emask >> (4 * k)) & 0xfu;
                if (whole[k] || em == 0xfu) {
                    __builtin_nontemporal_store(v[k], reinterpret_cast<v4u*>(d));
                } else {
                    uint32_t* d4 = reinterpret_cast<uint32_t*>(d);
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (em & (1u << q)) d4[q] = v[k][q];
                }
            }
        }
        if (wend >= cend) break;
        sw += kWave;
        __builtin_amdgcn_wave_barrier();
    }
}

// ------------------------------------------------------------------------------------------
// k_tiny_call: a whole call in one kernel, for problems so small that launches, not bytes, are
// what a call costs (Section "Performance analysis of TuNA": with tiny messages the number of rounds
// decides; here the number of kernel launches does).  One workgroup of 1024 threads does what the
// other kernels do between them, in the same order: the validation pass (counts >= 0, recvcounts ==
// transpose(sendcounts), M, total), the index-only initial rotation (Algorithm "TuNA", lines 4-5), the
// ranks' own blocks, then every digit phase: the metadata exchange (line 14: block sizes travel to the
// receiver's size array) and the hop of every moving block from where its sender holds it (S, or its
// slot of T) to where its receiver keeps it (R at the slot of its source rank, or its slot of T; lines
// 15-20).  T is the paper's B slots of M bytes per rank, laid out twice: a phase reads one copy and
// writes the other (the copy is the parity of a block's hop count, folded into the slot tables of the
// schedule), so no slot is read and written in one phase.  Sixteen lanes move one block at a time;
// workgroup barriers separate the phases.
// What a phase needs besides the payload is read from global memory once, at the start, all loads in
// flight together, and kept in LDS: both size matrices, the low 32 bits of both displacement
// matrices and the tables of every phase.  A phase then costs one round trip to memory -- the
// payload's -- instead of four dependent ones (tables, sizes, displacements, payload).
// The kernel declines -- writes tiny_done = 0 and moves nothing -- when the counts are invalid, when
// the problem is not tiny after all (payload above kTinyMaxPayload, T above its capacity) or when a
// displacement of a non-empty block does not fit into 32 bits; the host then takes the general path,
// which reports the error or does the work.
// Dynamic LDS: tiny_lds_bytes(P, total table entries).
// ------------------------------------------------------------------------------------------
constexpr int kTinyMaxRanks = 64;
constexpr int kTinyMaxPhases = 8;
constexpr int kTinyThreads = 1024;
constexpr unsigned long long kTinyMaxPayload = 1ull << 20;      // bytes
struct TinyPhase {
    const int32_t* e;
    const int32_t* z;
    const int32_t* src;
    const int32_t* dst;
    int nseg, dim, rx;
};
struct TinyArgs {
    const unsigned char* S;
    const int32_t* sendcounts;
    const int64_t* sdispls;
    unsigned char* R;
    const int32_t* recvcounts;
    const int64_t* rdispls;
    int P, Q, N, nph;
    TinyPhase ph[kTinyMaxPhases];
    unsigned char* T;               // capacity t_capacity bytes
    long long slots;                // T slots per rank (both copies)
    unsigned long long t_capacity;
    Status* st;                     // the first 64 bytes are written; in pinned host memory, so that the host reads
                                    // them after the stream's synchronisation without a copy of its own
};

// four P x P arrays of 4 bytes (two size matrices, two displacement matrices) and four ints per table entry
inline size_t tiny_lds_bytes(int P, int table_entries) {
    return ((size_t)4 * P * P + (size_t)4 * table_entries) * 4;
}

// one wave copies `n` bytes; dword granular when everything is 4-byte aligned, else byte by byte
__device__ __forceinline__ void tiny_copy(unsigned char* dst, const unsigned char* src, int n, int lane) {
    if ((((unsigned long long)dst | (unsigned long long)src | (unsigned long long)n) & 3ull) == 0) {
        const uint32_t* s4 = reinterpret_cast<const uint32_t*>(src);
        uint32_t* d4 = reinterpret_cast<uint32_t*>(dst);
        for (int i = lane; i < (n >> 2); i += kWave) d4[i] = s4[i];
    } else {
        for (int i = lane; i < n; i += kWave) dst[i] = src[i];
    }
}

__global__ void __launch_bounds__(kTinyThreads) k_tiny_call(const TinyArgs a) {
    extern __shared__ __align__(16) int tiny_lds[];
    __shared__ unsigned long long red[kTinyThreads / kWave][4];
    __shared__ int verdict;
    const int P = a.P, Q = a.Q, N = a.N, P2 = P * P;
    int* cur = tiny_lds;                                            // [P][P] sizes by slot index (the rotation's result)
    int* nxt = cur + P2;
    unsigned int* sd32 = reinterpret_cast<unsigned int*>(nxt + P2); // [P][P] sdispls, low 32 bits
    unsigned int* rd32 = sd32 + P2;                                 // [P][P] rdispls, low 32 bits
    int* tab = reinterpret_cast<int*>(rd32 + P2);                   // per phase: e[nseg], z[nseg], src[nseg], dst[nseg]
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    constexpr int kWaves = kTinyThreads / kWave;
    // ---- the tables of every phase: requested first, so that they travel together with the matrices ------
    {
        int off = 0;
        for (int x = 0; x < a.nph; ++x) {
            const TinyPhase& ph = a.ph[x];
            for (int k = tid; k < 4 * ph.nseg; k += kTinyThreads) {
                const int f = k / ph.nseg, s_ = k - f * ph.nseg;
                const int32_t* srcp = f == 0 ? ph.e : (f == 1 ? ph.z : (f == 2 ? ph.src : ph.dst));
                tab[off + k] = srcp[s_];
            }
            off += 4 * ph.nseg;
        }
    }
    // ---- validation, and the initial rotation (index only) on the way ---------------------------------------
    unsigned int flags = 0, abits = 0;
    int mx = 0;
    unsigned long long bytes = 0, chunks = 0, extent = 0;
    for (int k = tid; k < P2; k += kTinyThreads) {
        const int i = k / P, j = k - i * P;
        int c = a.sendcounts[k];
        const int rc = a.recvcounts[(size_t)j * P + i];
        const int64_t sd = a.sdispls[k], rd = a.rdispls[(size_t)j * P + i];
        if (c < 0) { flags |= 1u; c = 0; }
        if (rc < 0) flags |= 1u;
        else if (rc != c) flags |= 2u;
        abits |= (unsigned int)c | ((unsigned int)sd & 127u) | ((unsigned int)rd & 127u);
        if (c > 0) {
            if (sd < 0 || rd < 0) flags |= 4u;
            else extent = max(extent, (unsigned long long)sd + (unsigned long long)c);
            if (((unsigned long long)sd | (unsigned long long)rd) >> 32) flags |= 8u;      // not an error: beyond this kernel
        }
        mx = max(mx, c);
        bytes += (unsigned long long)c;
        chunks += (unsigned long long)((c + 15) >> 4);
        // rank i = (n, g) holds its block for rank j = (jn, jg) at the slot index of their distance
        const int n = i / Q, g = i - n * Q, jn = j / Q, jg = j - jn * Q;
        int dj = n - jn; if (dj < 0) dj += N;
        int dl = g - jg; if (dl < 0) dl += Q;
        cur[i * P + dj * Q + dl] = c;
        sd32[k] = (unsigned int)sd;
        rd32[j * P + i] = (unsigned int)rd;
    }
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) {
        flags |= __shfl_xor(flags, d, kWave);
        abits |= __shfl_xor(abits, d, kWave);
        mx = max(mx, __shfl_xor(mx, d, kWave));
        bytes += __shfl_xor(bytes, d, kWave);
        chunks += __shfl_xor(chunks, d, kWave);
        extent = max(extent, (unsigned long long)__shfl_xor(extent, d, kWave));
    }
    if (lane == 0) {
        red[wv][0] = ((unsigned long long)flags << 40) | ((unsigned long long)(abits & 127u) << 32) | (unsigned int)mx;
        red[wv][1] = bytes; red[wv][2] = chunks; red[wv][3] = extent;
    }
    __syncthreads();
    long long slot_bytes = 0;
    if (tid == 0) {
        unsigned int fl = 0, ab = 0;
        int m = 0;
        unsigned long long by = 0, ch = 0, ex = 0;
        for (int w = 0; w < kWaves; ++w) {
            fl |= (unsigned int)(red[w][0] >> 40); ab |= (unsigned int)(red[w][0] >> 32) & 127u;
            m = max(m, (int)(unsigned int)(red[w][0] & 0xffffffffull));
            by += red[w][1]; ch += red[w][2]; ex = max(ex, red[w][3]);
        }
        slot_bytes = ((long long)m + 15) / 16 * 16;
        const unsigned long long t_need = (unsigned long long)P * (unsigned long long)a.slots * (unsigned long long)slot_bytes;
        const bool ok = fl == 0 && by <= kTinyMaxPayload && t_need <= a.t_capacity;
        a.st->flags = fl & 7u; a.st->align_bits = ab; a.st->max_count = m; a.st->total_bytes = by; a.st->total_chunks = ch;
        a.st->send_extent = ex; a.st->t_chunks = 0; a.st->tiny_done = ok ? 1 : 0;
        verdict = ok ? m : -1;
    }
    __syncthreads();
    if (verdict < 0) return;                             // uniform: declined, nothing has moved
    slot_bytes = ((long long)verdict + 15) / 16 * 16;
    // ---- the ranks' own blocks ---------------------------------------------------------------------------------
    for (int p = wv; p < P; p += kWaves) {
        const int n = cur[p * P];                        // slot index 0: the block a rank keeps
        if (n > 0) tiny_copy(a.R + rd32[p * P + p], a.S + sd32[p * P + p], n, lane);
    }
    // ---- digit phases ----------------------------------------------------------------------------------------
    int* c0 = cur;
    int* c1 = nxt;
    int off = 0;
    for (int x = 0; x < a.nph; ++x) {
        const int nseg = a.ph[x].nseg, dim = a.ph[x].dim, rx = a.ph[x].rx;
        const int* te = tab + off;
        const int* tz = te + nseg;
        const int* ts = tz + nseg;
        const int* td = ts + nseg;
        off += 4 * nseg;
        // metadata exchange: sizes that do not move are carried over, the others arrive from the sender
        for (int k = tid; k < P2; k += kTinyThreads) c1[k] = c0[k];
        __syncthreads();
        for (int k = tid; k < P * nseg; k += kTinyThreads) {
            const int q = k / nseg, s = k - q * nseg;
            const int e = te[s];
            const int qn = q / Q, qg = q - qn * Q;
            const int sender = partner_up(qn, qg, Q, N, dim, tz[s] * rx);
            c1[q * P + e] = c0[sender * P + e];
        }
        __syncthreads();
        // the hops.  Sixteen lanes move one block; the 64 groups of the workgroup take the blocks 64 apart, two
        // per step, so that the whole workgroup has loads in flight at once (with one thread per block and the
        // copies done wave by wave, a phase of 128 blocks kept two waves busy and fourteen idle).  Every lane of
        // a group resolves the block itself: source, destination and size come from LDS.
        const int nb = P * nseg;
        const int grp = tid >> 4, sub = tid & 15;
        auto resolve = [&](int k, unsigned long long& src, unsigned long long& dst) -> int {
            if (k >= nb) return 0;
            const int q = k / nseg, s = k - q * nseg;
            const int e = te[s];
            const int size = c1[q * P + e];
            if (size <= 0) return 0;
            const int qn = q / Q, qg = q - qn * Q;
            const int sender = partner_up(qn, qg, Q, N, dim, tz[s] * rx);
            const int j = e / Q, l = e - j * Q;
            const int ssrc = ts[s], sdst = td[s];
            if (ssrc < 0) {
                const int sn = sender / Q, sg = sender - sn * Q;
                int dn = sn - j; if (dn < 0) dn += N;
                int dg = sg - l; if (dg < 0) dg += Q;
                src = (unsigned long long)(a.S + sd32[sender * P + dn * Q + dg]);
            } else {
                src = (unsigned long long)(a.T + ((long long)sender * a.slots + ssrc) * slot_bytes);
            }
            if (sdst < 0) {
                int on = qn + j; if (on >= N) on -= N;
                int og = qg + l; if (og >= Q) og -= Q;
                dst = (unsigned long long)(a.R + rd32[q * P + on * Q + og]);
            } else {
                dst = (unsigned long long)(a.T + ((long long)q * a.slots + sdst) * slot_bytes);
            }
            return size;
        };
        for (int b0 = 0; b0 < nb; b0 += 2 * (kTinyThreads / 16)) {
            unsigned long long sa = 0, da = 0, sb = 0, db = 0;
            const int na = resolve(b0 + grp, sa, da);
            const int nbb = resolve(b0 + kTinyThreads / 16 + grp, sb, db);
            const bool wa = ((sa | da | (unsigned long long)na) & 3ull) == 0;
            const bool wb = ((sb | db | (unsigned long long)nbb) & 3ull) == 0;
            const uint32_t* a4 = reinterpret_cast<const uint32_t*>(sa);
            const uint32_t* b4 = reinterpret_cast<const uint32_t*>(sb);
            uint32_t* ad4 = reinterpret_cast<uint32_t*>(da);
            uint32_t* bd4 = reinterpret_cast<uint32_t*>(db);
            const int nwa = wa ? na >> 2 : 0, nwb = wb ? nbb >> 2 : 0;
            for (int i = sub; i < max(nwa, nwb); i += 32) {     // four independent words per step
                const uint32_t a0 = i < nwa ? a4[i] : 0u;
                const uint32_t a1 = i + 16 < nwa ? a4[i + 16] : 0u;
                const uint32_t c0_ = i < nwb ? b4[i] : 0u;
                const uint32_t c1_ = i + 16 < nwb ? b4[i + 16] : 0u;
                if (i < nwa) ad4[i] = a0;
                if (i + 16 < nwa) ad4[i + 16] = a1;
                if (i < nwb) bd4[i] = c0_;
                if (i + 16 < nwb) bd4[i + 16] = c1_;
            }
            if (!wa) {
                const unsigned char* sp = reinterpret_cast<const unsigned char*>(sa);
                unsigned char* dp = reinterpret_cast<unsigned char*>(da);
                for (int i = sub; i < na; i += 16) dp[i] = sp[i];
            }
            if (!wb) {
                const unsigned char* sp = reinterpret_cast<const unsigned char*>(sb);
                unsigned char* dp = reinterpret_cast<unsigned char*>(db);
                for (int i = sub; i < nbb; i += 16) dp[i] = sp[i];
            }
        }
        __syncthreads();                                  // the blocks stored into T are read in a later phase
        int* t = c0; c0 = c1; c1 = t;
    }
}

}  // namespace tuna
