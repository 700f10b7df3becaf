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

constexpr int kWave = 64;
constexpr int kCopyThreads = 256;                        // 4 waves
constexpr int kChunksPerThread = 4;
constexpr int kTileChunks = kCopyThreads * kChunksPerThread;   // 1024 chunks = 16 KiB per tile
constexpr int kWindow = 256;                             // segments resolved per LDS window
constexpr int kScanThreads = 256;
constexpr int kScanItems = 4;

enum CopyMode { kPack = 0, kExchange = 1, kUnpack = 2, kFused = 3 };

// Device-side status block, cleared at the start of a call and read back once after validation.
struct Status {
    unsigned int flags;            // bit 0: negative count, bit 1: recvcounts != transpose(sendcounts)
    unsigned int align_bits;       // OR of all counts and displacements (low bits decide the granularity)
    int max_count;                 // M
    int pad;
    unsigned long long total_bytes;    // sum of sendcounts
    unsigned long long total_chunks;   // sum of ceil(count / 16)
    unsigned long long max_rank_chunks;// unused (reserved)
    unsigned long long phase_bytes[64];   // payload bytes moved per phase
    unsigned long long phase_chunks[64];  // staged chunks per phase
};

// One staging layout (send side or receive side) of the current phase.
struct LayoutDev {
    int* pre;                      // [P][ld]: exclusive prefix of chunk counts over the rank's segments; [nseg] = total
    int* tot;                      // [P]: chunks per rank
    long long* rank_base;          // [P+1]: first chunk of each rank in the staging buffer
    int* tile_base;                // [P+1]: first tile of each rank
    int4* tiles;                   // {rank, first segment, first chunk (rank-local), chunks in tile}
    int* n_tiles;                  // total tiles
    int ld;                        // row stride of pre (>= P + 1)
};

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
// k_clear: zero a small word array (instead of a memset node, so a caller may capture the stream)
// ------------------------------------------------------------------------------------------
__global__ void k_clear(unsigned int* w, int n) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) w[i] = 0u;
}

// ------------------------------------------------------------------------------------------
// k_validate: one pass over the P x P matrices in 32 x 32 tiles.  Finds M (Algorithm "TuNA",
// line 1: the maximum block size over all ranks, here one device reduction instead of an
// allreduce), the totals the workspace is sized from, checks counts >= 0 and
// recvcounts == transpose(sendcounts) through an LDS tile so both matrices are read row-wise.
// grid (ceil(P/32), ceil(P/32)), block (32, 8).
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_validate(const int32_t* __restrict__ sendcounts,
                                                  const int32_t* __restrict__ recvcounts,
                                                  const int64_t* __restrict__ sdispls,
                                                  const int64_t* __restrict__ rdispls,
                                                  int P, Status* __restrict__ st) {
    __shared__ int tile[32][33];
    const int bi = blockIdx.y * 32, bj = blockIdx.x * 32;
    const int tx = threadIdx.x, ty = threadIdx.y;
    unsigned int flags = 0, abits = 0;
    int mx = 0;
    unsigned long long bytes = 0, chunks = 0;
    for (int a = ty; a < 32; a += 8) {
        const int i = bi + a, j = bj + tx;
        int c = 0;
        if (i < P && j < P) {
            c = sendcounts[(size_t)i * P + j];
            if (c < 0) { flags |= 1u; c = 0; }
            abits |= (unsigned int)c;
            if (sdispls) abits |= (unsigned int)sdispls[(size_t)i * P + j] & 15u;
            mx = max(mx, c);
            bytes += (unsigned long long)c;
            chunks += (unsigned long long)((c + 15) >> 4);
        }
        tile[a][tx] = c;
    }
    __syncthreads();
    if (recvcounts) {
        for (int a = ty; a < 32; a += 8) {
            const int j = bj + a, i = bi + tx;      // recvcounts[j][i] must equal sendcounts[i][j]
            if (i < P && j < P) {
                int rc = recvcounts[(size_t)j * P + i];
                if (rc < 0) flags |= 1u;
                else if (rc != tile[tx][a]) flags |= 2u;
                if (rdispls) abits |= (unsigned int)rdispls[(size_t)j * P + i] & 15u;
            }
        }
    }
    // wave reduction, then one atomic per wave
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) {
        flags |= __shfl_xor(flags, d, kWave);
        abits |= __shfl_xor(abits, d, kWave);
        mx = max(mx, __shfl_xor(mx, d, kWave));
        bytes += __shfl_xor(bytes, d, kWave);
        chunks += __shfl_xor(chunks, d, kWave);
    }
    if (((ty * 32 + tx) & (kWave - 1)) == 0) {
        if (flags) atomicOr(&st->flags, flags);
        if (abits & 15u) atomicOr(&st->align_bits, abits & 15u);
        if (mx) atomicMax(&st->max_count, mx);
        if (bytes) atomicAdd(&st->total_bytes, bytes);
        if (chunks) atomicAdd(&st->total_chunks, chunks);
    }
}

// ------------------------------------------------------------------------------------------
// k_rotate_init: the index-only initial rotation (Algorithm "TuNA", lines 4-5; Algorithm
// "Coalesced TuNA_l^g", line 5).  No payload moves: cur[p][j*Q + l] becomes the size of the
// block rank p = (n, g) holds at distance (j, l), i.e. its block for rank ((n-j)%N, (g-l)%Q).
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_rotate_init(const int32_t* __restrict__ sendcounts,
                                                     int32_t* __restrict__ cur, int P, int Q, int N) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)P * P) return;
    const int p = (int)(idx / P), e = (int)(idx - (size_t)p * P);
    const int n = p / Q, g = p - n * Q;
    const int j = e / Q, l = e - j * Q;
    int dn = n - j; if (dn < 0) dn += N;
    int dg = g - l; if (dg < 0) dg += Q;
    cur[idx] = sendcounts[(size_t)p * P + dn * Q + dg];
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
// k_meta_exchange: the metadata phase of a digit phase (Section "Two-phase communication";
// Algorithm "TuNA", line 14).  Every moving block's size travels from the sender's size array to
// the receiver's: nxt[q][e] = cur[q + z r^x][e] where z = digit of e, and sizes of blocks that
// stay are carried over.  One thread per (rank, slot).
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_meta_exchange(const int32_t* __restrict__ cur,
                                                       int32_t* __restrict__ nxt,
                                                       const int32_t* __restrict__ zt,
                                                       int P, int Q, int N, int dim, int rx) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)P * P) return;
    const int q = (int)(idx / P), e = (int)(idx - (size_t)q * P);
    const int z = zt[e];
    int v;
    if (z == 0) {
        v = cur[idx];
    } else {
        const int n = q / Q, g = q - n * Q;
        const int s = partner_up(n, g, Q, N, dim, z * rx);
        v = cur[(size_t)s * P + e];
    }
    nxt[idx] = v;
}

// ------------------------------------------------------------------------------------------
// k_layout_scan: size/displacement scan of one rank's moving blocks (the contiguous send buffer
// of Algorithm "TuNA", line 15, needs each block's offset inside its message).  One workgroup
// per rank: gathers the sizes in message order, converts to 16-byte chunks, exclusive scan with
// wave shuffles + LDS across the 4 waves, a running carry across batches of 1024 segments.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kScanThreads) k_layout_scan(const int32_t* __restrict__ sizes,
                                                              const SegInfo* __restrict__ seg, int nseg,
                                                              int P, LayoutDev L,
                                                              unsigned long long* __restrict__ phase_bytes) {
    __shared__ int wsum[kScanThreads / kWave];
    __shared__ int carry_s;
    const int p = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const int32_t* row = sizes + (size_t)p * P;
    int* pre = L.pre + (size_t)p * L.ld;
    int carry = 0;
    unsigned long long bytes = 0;
    for (int base = 0; base < nseg; base += kScanThreads * kScanItems) {
        int c[kScanItems];
        int sum = 0;
#pragma unroll
        for (int k = 0; k < kScanItems; ++k) {
            const int s = base + tid * kScanItems + k;
            int sz = 0;
            if (s < nseg) sz = row[seg[s].e];
            bytes += (unsigned long long)sz;
            c[k] = (sz + 15) >> 4;
            sum += c[k];
        }
        const int incl = wave_incl_scan(sum);
        if (lane == kWave - 1) wsum[wv] = incl;
        __syncthreads();
        int woff = 0, total = 0;
#pragma unroll
        for (int k = 0; k < kScanThreads / kWave; ++k) {
            const int v = wsum[k];
            if (k < wv) woff += v;
            total += v;
        }
        int run = carry + woff + incl - sum;
#pragma unroll
        for (int k = 0; k < kScanItems; ++k) {
            const int s = base + tid * kScanItems + k;
            if (s < nseg) pre[s] = run;
            run += c[k];
        }
        carry += total;
        __syncthreads();
    }
    // per-rank totals and payload bytes of the phase
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) bytes += __shfl_xor(bytes, d, kWave);
    if (lane == 0 && bytes && phase_bytes) atomicAdd(phase_bytes, bytes);
    if (tid == 0) { pre[nseg] = carry; L.tot[p] = carry; }
    (void)carry_s;
}

// ------------------------------------------------------------------------------------------
// k_layout_base: exclusive scan over the P per-rank totals -> each rank's first chunk in the
// staging buffer and its first tile.  Single workgroup of 1024 threads, carry across batches.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(1024) k_layout_base(int P, LayoutDev L,
                                                      unsigned long long* __restrict__ phase_chunks) {
    __shared__ long long wc[16];
    __shared__ int wt[16];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    long long carry_c = 0;
    int carry_t = 0;
    for (int base = 0; base < P; base += 1024) {
        const int p = base + tid;
        const int c = p < P ? L.tot[p] : 0;
        const int t = (c + kTileChunks - 1) / kTileChunks;
        long long ic = c;
        int it = t;
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
        for (int k = 0; k < 16; ++k) {
            if (k < wv) { oc += wc[k]; ot += wt[k]; }
            totc += wc[k]; tott += wt[k];
        }
        if (p < P) {
            L.rank_base[p] = carry_c + oc + ic - c;
            L.tile_base[p] = carry_t + ot + it - t;
        }
        carry_c += totc;
        carry_t += tott;
        __syncthreads();
    }
    if (tid == 0) {
        L.rank_base[P] = carry_c;
        L.tile_base[P] = carry_t;
        *L.n_tiles = carry_t;
        if (phase_chunks) *phase_chunks = (unsigned long long)carry_c;
    }
}

// ------------------------------------------------------------------------------------------
// k_layout_tiles: cut every rank's staged chunks into tiles of kTileChunks and record, per tile,
// the rank and the first segment that overlaps it (binary search in the rank's prefix row).
// One workgroup per rank.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_layout_tiles(int nseg, LayoutDev L) {
    const int p = blockIdx.x;
    const int tot = L.tot[p];
    const int nt = (tot + kTileChunks - 1) / kTileChunks;
    const int* pre = L.pre + (size_t)p * L.ld;
    const int tb = L.tile_base[p];
    for (int t = threadIdx.x; t < nt; t += blockDim.x) {
        const int c0 = t * kTileChunks;
        int lo = 0, hi = nseg;                 // largest s in [0, nseg) with pre[s] <= c0
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (pre[mid] <= c0) lo = mid; else hi = mid;
        }
        L.tiles[tb + t] = make_int4(p, lo, c0, min(kTileChunks, tot - c0));
    }
}

// ------------------------------------------------------------------------------------------
// The copy engine.  pack / exchange / unpack are the same tiled, byte-balanced variable-length
// copy with a different "other side":
//   pack     staging(send)  <- S at sdispls, or T slot      (Algorithm "TuNA", line 15, sender side)
//   exchange staging(recv)  <- staging(send) of the partner (the point-to-point transfer itself)
//   unpack   staging(recv)  -> R at rdispls, or T slot      (Algorithm "TuNA", lines 16-20)
// A tile is 1024 consecutive chunks of one rank's staging region; its workgroup loads the chunk
// prefix of the overlapping segments into LDS (a window of kWindow segments at a time), resolves
// every segment's other-side address once, and each lane finds the segment of each of its 4
// chunks by binary search in LDS.  Lanes of a wave touch consecutive 16-byte chunks on the
// staging side (aligned dwordx4) and consecutive bytes of a block on the other side.
// Persistent grid: workgroups stride over the tile list, whose length lives in device memory.
// ------------------------------------------------------------------------------------------
struct CopyArgs {
    // tiled (staging) side
    uint4* stage;                       // staging buffer being tiled
    LayoutDev L;                        // its layout
    const SegInfo* seg;
    int nseg;
    // other side: caller buffer + T (pack, unpack)
    const int32_t* sizes;               // [P][P] block sizes at the tiled side's ranks (cur for pack, nxt for unpack)
    unsigned char* user;                // S (pack) or R (unpack)
    const int64_t* displs;              // sdispls (pack) or rdispls (unpack)
    unsigned char* T;                   // temporary buffer: slot s of rank p at ((p*slots + s) * slot_bytes)
    long long slots;
    long long slot_bytes;
    // other side: send staging (exchange)
    const uint4* stage_src;
    LayoutDev Ls;
    int P, Q, N, dim, rx;
};

template <int GRAN>
__device__ __forceinline__ uint4 load_block_chunk(const unsigned char* src, int nb) {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (GRAN == 16 || nb >= 16) {
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
        v = make_uint4(w[0], w[1], w[2], w[3]);
    }
    return v;
}

template <int GRAN>
__device__ __forceinline__ void store_block_chunk(unsigned char* dst, uint4 v, int nb) {
    if (GRAN == 16 || nb >= 16) {
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

template <int MODE, int GRAN>
__global__ void __launch_bounds__(kCopyThreads) k_tile_copy(const CopyArgs a) {
    __shared__ int lpre[kWindow + 1];
    __shared__ unsigned long long laddr[kWindow];
    __shared__ int lsize[kWindow];
    const int tid = threadIdx.x;
    const int ntiles = *a.L.n_tiles;
    for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int4 td = a.L.tiles[tile];
        const int p = td.x, c0 = td.z, cend = td.z + td.w;
        int sw = td.y;
        const int n = p / a.Q, g = p - n * a.Q;
        const int* prow = a.L.pre + (size_t)p * a.L.ld;
        uint4* stage = a.stage + a.L.rank_base[p];
        int c[kChunksPerThread];
        bool pend[kChunksPerThread];
#pragma unroll
        for (int k = 0; k < kChunksPerThread; ++k) {
            c[k] = c0 + k * kCopyThreads + tid;
            pend[k] = c[k] < cend;
        }
        for (;;) {
            __syncthreads();                         // LDS of the previous window / tile is free
            for (int t = tid; t <= kWindow; t += kCopyThreads) {
                const int s = sw + t;
                lpre[t] = s <= a.nseg ? prow[s] : INT_MAX;
            }
            __syncthreads();
            const int wend = lpre[kWindow];          // chunks below wend are resolved by this window
            for (int t = tid; t < kWindow; t += kCopyThreads) {
                const int s = sw + t;
                if (s < a.nseg && lpre[t] < cend && lpre[t + 1] > lpre[t]) {
                    const SegInfo si = a.seg[s];
                    unsigned long long addr;
                    int size;
                    if (MODE == kExchange) {
                        const int ps = partner_up(n, g, a.Q, a.N, a.dim, si.z * a.rx);
                        addr = (unsigned long long)(a.stage_src + a.Ls.rank_base[ps] +
                                                    a.Ls.pre[(size_t)ps * a.Ls.ld + s]);
                        size = (lpre[t + 1] - lpre[t]) << 4;
                    } else {
                        size = a.sizes[(size_t)p * a.P + si.e];
                        const int slot = MODE == kPack ? si.src_slot : si.dst_slot;
                        if (slot >= 0) {
                            addr = (unsigned long long)(a.T + ((long long)p * a.slots + slot) * a.slot_bytes);
                        } else {
                            int pn, pg;            // the rank at the far end of this block's route
                            if (MODE == kPack) {   // its destination: ((n - j) % N, (g - l) % Q)
                                pn = n - si.j; if (pn < 0) pn += a.N;
                                pg = g - si.l; if (pg < 0) pg += a.Q;
                            } else {               // its source: ((n + j) % N, (g + l) % Q)
                                pn = n + si.j; if (pn >= a.N) pn -= a.N;
                                pg = g + si.l; if (pg >= a.Q) pg -= a.Q;
                            }
                            addr = (unsigned long long)(a.user + a.displs[(size_t)p * a.P + pn * a.Q + pg]);
                        }
                    }
                    laddr[t] = addr;
                    lsize[t] = size;
                }
            }
            __syncthreads();
            bool act[kChunksPerThread];
            unsigned long long oa[kChunksPerThread];
            int nb[kChunksPerThread];
            uint4 v[kChunksPerThread];
#pragma unroll
            for (int k = 0; k < kChunksPerThread; ++k) {
                act[k] = pend[k] && c[k] < wend;
                oa[k] = 0; nb[k] = 0;
                if (act[k]) {
                    int lo = 0, hi = kWindow;        // lpre[lo] <= c < lpre[hi]
#pragma unroll
                    for (int it = 0; it < 8; ++it) {
                        const int mid = (lo + hi) >> 1;
                        if (lpre[mid] <= c[k]) lo = mid; else hi = mid;
                    }
                    const int off = (c[k] - lpre[lo]) << 4;
                    oa[k] = laddr[lo] + (unsigned long long)off;
                    nb[k] = min(16, lsize[lo] - off);
                }
            }
#pragma unroll
            for (int k = 0; k < kChunksPerThread; ++k) {
                if (act[k]) {
                    if (MODE == kUnpack) v[k] = stage[c[k]];
                    else if (MODE == kExchange) v[k] = *reinterpret_cast<const uint4*>(oa[k]);
                    else v[k] = load_block_chunk<GRAN>(reinterpret_cast<const unsigned char*>(oa[k]), nb[k]);
                }
            }
#pragma unroll
            for (int k = 0; k < kChunksPerThread; ++k) {
                if (act[k]) {
                    if (MODE == kUnpack) store_block_chunk<GRAN>(reinterpret_cast<unsigned char*>(oa[k]), v[k], nb[k]);
                    else stage[c[k]] = v[k];
                    pend[k] = false;
                }
            }
            if (wend >= cend) break;
            sw += kWindow;
        }
    }
}

}  // namespace tuna
