// C ABI of the tunable-radix non-uniform all-to-all for MI355X: argument checks, the cached
// schedule, workspace management and the per-phase launch sequence.  All payload movement and
// all per-block arithmetic happen in the kernels of tuna_kernels.h; the host only loops over
// the ceil(log_r) digit phases.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <map>
#include <tuple>
#include <vector>

#include "../../include/tuna.h"
#include "tuna_kernels.h"
#include "tuna_plan.h"

namespace tuna {
namespace {

constexpr int kVersion = 100;
constexpr size_t kAlign = 256;

struct DevicePlan {
    PlanHost host;
    std::vector<SegDev> d_seg;
    std::vector<int32_t*> d_seg_mem;
    std::vector<int32_t*> d_zt;
};

enum Category { kCatPrepare = 0, kCatSelf, kCatMeta, kCatPack, kCatExchange, kCatUnpack };

struct Mark { hipEvent_t ev; int cat; int phase; };

struct Ctx {
    bool ready = false;
    int device = -1;
    int num_cus = 256;
    Status* d_status = nullptr;       // device status block (one-time small allocation)
    Status* h_status = nullptr;       // pinned host mirror
    void* meta = nullptr;  size_t meta_bytes = 0;   // library-owned, grow-only
    void* data = nullptr;  size_t data_bytes = 0;
    void* user_ws = nullptr; size_t user_ws_bytes = 0;
    std::map<std::tuple<int, int, int, int, int>, DevicePlan> plans;
    tuna_stats_t stats;
    bool have_stats = false;
    int opt_profile = 0, opt_fused = 0, opt_staggered = 0;
    std::vector<hipEvent_t> ev_pool;
    std::vector<Mark> marks;
    hipEvent_t ev_end = nullptr;
    bool end_recorded = false;
    int last_hip_error = 0;
};

Ctx g;

#define HIPCHK(expr)                                                       \
    do {                                                                   \
        hipError_t _e = (expr);                                            \
        if (_e != hipSuccess) { g.last_hip_error = (int)_e; g.stats.last_hip_error = (int)_e; return TUNA_ERR_HIP; } \
    } while (0)

inline size_t align_up(size_t v, size_t a = kAlign) { return (v + a - 1) / a * a; }

int ensure_ctx() {
    if (g.ready) return TUNA_OK;
    int ndev = 0;
    HIPCHK(hipGetDeviceCount(&ndev));
    if (ndev < 1) { g.last_hip_error = (int)hipErrorNoDevice; return TUNA_ERR_HIP; }
    HIPCHK(hipGetDevice(&g.device));
    hipDeviceProp_t prop;
    HIPCHK(hipGetDeviceProperties(&prop, g.device));
    g.num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    HIPCHK(hipMalloc((void**)&g.d_status, align_up(sizeof(Status))));
    HIPCHK(hipHostMalloc((void**)&g.h_status, sizeof(Status), hipHostMallocDefault));
    HIPCHK(hipEventCreate(&g.ev_end));
    std::memset(&g.stats, 0, sizeof(g.stats));
    g.ready = true;
    return TUNA_OK;
}

// Bump allocator over one device range.
struct Carver {
    char* base; size_t cap; size_t off = 0; bool ok = true;
    Carver(void* b, size_t c) : base((char*)b), cap(c) {}
    template <class T> T* take(size_t count) {
        const size_t bytes = align_up(count * sizeof(T));
        T* p = (T*)(base + off);
        off += bytes;
        if (off > cap) ok = false;
        return p;
    }
};

struct MetaBuffers {
    int32_t *cur, *nxt;
    LayoutDev Ls, Lr;
};

size_t meta_bytes_for(int P) {
    const size_t P2 = (size_t)P * P, ld = (size_t)P + 1;
    size_t b = 0;
    b += 2 * align_up(P2 * 4);
    b += 2 * (align_up(P * ld * 4) + align_up(P * 4) + align_up((P + 1) * 8) + align_up((P + 1) * 4) + align_up(4));
    return b;
}

void carve_layout(Carver& cv, int P, LayoutDev& L) {
    L.ld = P + 1;
    L.pre = cv.take<int>((size_t)P * L.ld);
    L.tot = cv.take<int>(P);
    L.rank_base = cv.take<long long>(P + 1);
    L.unit_base = cv.take<int>(P + 1);
    L.n_units = cv.take<int>(1);
    L.units = nullptr;
}

MetaBuffers carve_meta(Carver& cv, int P) {
    MetaBuffers m;
    m.cur = cv.take<int32_t>((size_t)P * P);
    m.nxt = cv.take<int32_t>((size_t)P * P);
    carve_layout(cv, P, m.Ls);
    carve_layout(cv, P, m.Lr);
    return m;
}

struct DataSizes {
    size_t unit_cap;        // wave units per layout (upper bound)
    size_t stage_chunks;    // chunks per staging buffer
    long long slots;        // T slots per rank
    long long slot_bytes;   // M rounded up to 16
    size_t t_bytes;
    size_t total;
};

DataSizes data_sizes_for(const PlanHost& pl, long long M, unsigned long long total_chunks, bool fused,
                         bool staggered = false) {
    DataSizes d{};
    const bool any_phase = !pl.phases.empty() && total_chunks > 0;
    d.stage_chunks = any_phase ? (size_t)total_chunks : 0;
    // fused rounds cut chunks at destination lines: up to one more chunk per moving block
    const size_t head_chunks = (fused || staggered) ? (size_t)pl.P * pl.P : 0;
    d.unit_cap = any_phase ? (size_t)((total_chunks + head_chunks) / kUnitChunks) + pl.P + 1 : 0;
    d.slots = pl.slots;
    d.slot_bytes = (M + 127) / 128 * 128;     // whole 128-byte lines per slot
    d.t_bytes = any_phase ? (size_t)pl.P * (size_t)d.slots * (size_t)d.slot_bytes : 0;
    // pl.slots already counts both copies of T when the plan is a fused one
    d.total = 2 * align_up(d.unit_cap * sizeof(int4)) + (fused ? 0 : 2 * align_up(d.stage_chunks * 16)) +
              align_up(d.t_bytes);
    return d;
}

int get_plan(int P, int Q, int rl, int rg, bool fused, DevicePlan** out) {
    PlanHost probe;   // clamp radices the same way make_plan does
    const int N = P / Q;
    int crl = rl < 2 ? 2 : rl, crg = rg < 2 ? 2 : rg;
    if (Q >= 2 && crl > Q) crl = Q;
    if (N >= 2 && crg > N) crg = N;
    if (Q < 2) crl = 2;
    if (N < 2) crg = 2;
    auto key = std::make_tuple(P, Q, crl, crg, fused ? 1 : 0);
    auto it = g.plans.find(key);
    if (it == g.plans.end()) {
        DevicePlan dp;
        dp.host = make_plan(P, Q, crl, crg, fused);
        if ((int)dp.host.phases.size() > TUNA_MAX_PHASES) return TUNA_ERR_TOO_LARGE;
        for (auto& ph : dp.host.phases) {
            // field-major copy of the table: e[], z[], src[], dst[]
            const size_t ns = ph.seg.size(), stride = align_up(ns * 4) / 4;
            std::vector<int32_t> soa(4 * stride, 0);
            for (size_t k = 0; k < ns; ++k) {
                soa[k] = ph.seg[k].e; soa[stride + k] = ph.seg[k].z;
                soa[2 * stride + k] = ph.seg[k].src_slot; soa[3 * stride + k] = ph.seg[k].dst_slot;
            }
            int32_t* dm = nullptr;
            int32_t* dz = nullptr;
            HIPCHK(hipMalloc((void**)&dm, 4 * stride * 4 + kAlign));
            HIPCHK(hipMalloc((void**)&dz, align_up((size_t)P * 4)));
            HIPCHK(hipMemcpy(dm, soa.data(), soa.size() * 4, hipMemcpyHostToDevice));
            HIPCHK(hipMemcpy(dz, ph.zt.data(), (size_t)P * 4, hipMemcpyHostToDevice));
            dp.d_seg.push_back(SegDev{dm, dm + stride, dm + 2 * stride, dm + 3 * stride});
            dp.d_seg_mem.push_back(dm);
            dp.d_zt.push_back(dz);
            // the device copies are all the kernels need; drop the host tables
            std::vector<SegInfo>().swap(ph.seg);
            std::vector<int32_t>().swap(ph.zt);
        }
        it = g.plans.emplace(key, std::move(dp)).first;
    }
    *out = &it->second;
    (void)probe;
    return TUNA_OK;
}

int grow(void** buf, size_t* have, size_t need) {
    if (need <= *have) return TUNA_OK;
    if (*buf) {
        HIPCHK(hipDeviceSynchronize());
        HIPCHK(hipFree(*buf));
        *buf = nullptr; *have = 0;
    }
    hipError_t e = hipMalloc(buf, need);
    if (e != hipSuccess) { (void)hipGetLastError(); g.last_hip_error = (int)e; *buf = nullptr; return TUNA_ERR_NOMEM; }
    *have = need;
    return TUNA_OK;
}

void mark(hipStream_t s, int cat, int phase) {
    if (!g.opt_profile) return;
    const size_t k = g.marks.size();
    if (k >= g.ev_pool.size()) {
        hipEvent_t ev;
        if (hipEventCreate(&ev) != hipSuccess) return;
        g.ev_pool.push_back(ev);
    }
    if (hipEventRecord(g.ev_pool[k], s) != hipSuccess) return;
    g.marks.push_back(Mark{g.ev_pool[k], cat, phase});
}

// One-shot grid over an upper bound of wave units (4 per workgroup); waves past the device-side
// unit count exit immediately.
template <int MODE>
int launch_copy(int gran, size_t unit_cap, const CopyArgs& a, hipStream_t s) {
    const size_t waves = kCopyThreads / kWave;
    const dim3 grid((unsigned)((unit_cap + waves - 1) / waves)), block(kCopyThreads);
    if (grid.x == 0) return TUNA_OK;
    if (MODE == kExchange) {
        hipLaunchKernelGGL((k_copy<MODE, 16>), grid, block, 0, s, a);
    } else if (gran == 16) {
        hipLaunchKernelGGL((k_copy<MODE, 16>), grid, block, 0, s, a);
    } else if (gran == 4) {
        hipLaunchKernelGGL((k_copy<MODE, 4>), grid, block, 0, s, a);
    } else {
        hipLaunchKernelGGL((k_copy<MODE, 1>), grid, block, 0, s, a);
    }
    HIPCHK(hipGetLastError());
    return TUNA_OK;
}

// Metadata of one digit phase: sizes exchanged, both staging layouts scanned, wave units cut.
int phase_metadata(const PhaseLayoutArgs& a, hipStream_t s) {
    hipLaunchKernelGGL(k_phase_layout, dim3(a.P), dim3(kScanThreads), 0, s, a);
    HIPCHK(hipGetLastError());
    hipLaunchKernelGGL(k_layout_base, dim3(a.want_send ? 2 : 1), dim3(kScanThreads), 0, s, a.P, a.Lr, a.Ls,
                       a.phase_chunks, a.want_send ? 1 : 0);
    HIPCHK(hipGetLastError());
    hipLaunchKernelGGL(k_layout_units, dim3(a.P, a.want_send ? 2 : 1), dim3(256), 0, s, a.nseg, a.Lr, a.Ls);
    HIPCHK(hipGetLastError());
    return TUNA_OK;
}

int resolve_hierarchy(int P, int ranks_per_node, int* Q) {
    if (P < 1 || P > TUNA_MAX_RANKS) return P < 1 ? TUNA_ERR_ARG : TUNA_ERR_TOO_LARGE;
    if (ranks_per_node < 0) return TUNA_ERR_ARG;
    if (ranks_per_node == 0 || ranks_per_node == 1 || ranks_per_node == P) { *Q = P; return TUNA_OK; }
    if (ranks_per_node > P || P % ranks_per_node != 0) return TUNA_ERR_ARG;
    *Q = ranks_per_node;
    return TUNA_OK;
}

// Validation + sizing pass shared by tuna_alltoallv* and tuna_workspace_bytes: fills *g.h_status.
int run_validate(const int32_t* sendcounts, const int32_t* recvcounts, const int64_t* sdispls,
                 const int64_t* rdispls, int P, hipStream_t s) {
    const int nwords = (int)(sizeof(Status) / 4);
    hipLaunchKernelGGL(k_clear, dim3((nwords + 255) / 256), dim3(256), 0, s, (unsigned int*)g.d_status, nwords);
    HIPCHK(hipGetLastError());
    const size_t t = (size_t)((P + 31) / 32);
    const unsigned vgrid = (unsigned)(t * t < (size_t)g.num_cus * 8 ? t * t : (size_t)g.num_cus * 8);
    hipLaunchKernelGGL(k_validate, dim3(vgrid), dim3(32, 8), 0, s, sendcounts, recvcounts, sdispls, rdispls, P,
                       g.d_status);
    HIPCHK(hipGetLastError());
    HIPCHK(hipMemcpyAsync(g.h_status, g.d_status, 64, hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));
    return TUNA_OK;
}

int run(const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls, void* recvbuf,
        const int32_t* recvcounts, const int64_t* rdispls, int P, int ranks_per_node, int rl, int rg,
        void* stream) {
    int Q = 0;
    int rc = resolve_hierarchy(P, ranks_per_node, &Q);
    if (rc != TUNA_OK) return rc;
    if (rl < 2 || rg < 2) return TUNA_ERR_ARG;
    if (!sendcounts || !recvcounts || !sdispls || !rdispls) return TUNA_ERR_ARG;
    rc = ensure_ctx();
    if (rc != TUNA_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    const int N = P / Q;

    DevicePlan* dp = nullptr;
    const bool fused = g.opt_fused != 0;
    // staggered inter-node schedule: one block per message, N - 1 node distances, straight from T
    const bool staggered = g.opt_staggered != 0 && N > 1;
    if (staggered) rg = N;
    rc = get_plan(P, Q, rl, rg, fused, &dp);
    if (rc != TUNA_OK) return rc;
    const PlanHost& pl = dp->host;

    g.marks.clear();
    g.end_recorded = false;
    g.have_stats = false;
    tuna_stats_t& st = g.stats;
    std::memset(&st, 0, sizeof(st));
    st.P = P; st.Q = Q; st.N = N; st.local_radix = pl.rl; st.global_radix = pl.rg;
    st.w_local = pl.w_l; st.w_global = pl.w_g; st.K_local = pl.K_l; st.K_global = pl.K_g;
    st.B_local = pl.B_l; st.B_global = pl.B_g; st.n_phases = (int)pl.phases.size();
    if (staggered) st.K_global = Q * (N - 1);
    st.temp_slots_per_rank = pl.slots;
    st.fused = fused ? 1 : 0;
    mark(s, -1, -1);

    // ---- prepare: validation, M, totals (one read-back) ---------------------------------------
    rc = run_validate(sendcounts, recvcounts, sdispls, rdispls, P, s);
    if (rc != TUNA_OK) return rc;
    const Status hs = *g.h_status;
    if (hs.flags & 1u) return TUNA_ERR_NEGATIVE_COUNT;
    if (hs.flags & 2u) return TUNA_ERR_COUNT_MISMATCH;
    st.max_block_bytes = hs.max_count;
    st.total_payload_bytes = (int64_t)hs.total_bytes;
    if (hs.total_bytes == 0) { g.have_stats = true; return TUNA_OK; }
    if (!sendbuf || !recvbuf) return TUNA_ERR_ARG;
    // chunk prefixes are 32-bit per rank
    if ((unsigned long long)P * (unsigned long long)((hs.max_count + 15) / 16) >= (1ull << 31)) return TUNA_ERR_TOO_LARGE;
    const unsigned int abits = hs.align_bits | (unsigned int)((uintptr_t)sendbuf & 15u) |
                               (unsigned int)((uintptr_t)recvbuf & 15u);
    const int gran = (abits & 15u) == 0 ? 16 : ((abits & 3u) == 0 ? 4 : 1);
    st.granularity = gran;

    // ---- workspace ---------------------------------------------------------------------------
    const size_t mbytes = meta_bytes_for(P);
    const DataSizes ds = data_sizes_for(pl, hs.max_count, hs.total_chunks, fused, staggered);
    void *mbase, *dbase;
    if (g.user_ws) {
        if (mbytes + ds.total > g.user_ws_bytes) return TUNA_ERR_WORKSPACE_TOO_SMALL;
        mbase = g.user_ws;
        dbase = (char*)g.user_ws + mbytes;
    } else {
        rc = grow(&g.meta, &g.meta_bytes, mbytes);
        if (rc != TUNA_OK) return rc;
        rc = grow(&g.data, &g.data_bytes, ds.total);
        if (rc != TUNA_OK) return rc;
        mbase = g.meta;
        dbase = g.data;
    }
    Carver cm(mbase, mbytes);
    MetaBuffers mb = carve_meta(cm, P);
    Carver cd(dbase, ds.total);
    mb.Ls.units = cd.take<int4>(ds.unit_cap);
    mb.Lr.units = cd.take<int4>(ds.unit_cap);
    v4u* stage_s = cd.take<v4u>(fused ? 0 : ds.stage_chunks);
    v4u* stage_r = cd.take<v4u>(fused ? 0 : ds.stage_chunks);
    unsigned char* T = cd.take<unsigned char>(ds.t_bytes);
    if (!cm.ok || !cd.ok) return TUNA_ERR_WORKSPACE_TOO_SMALL;
    st.temp_bytes = (int64_t)ds.t_bytes;
    st.staging_bytes = fused ? 0 : (int64_t)(2 * ds.stage_chunks * 16);
    st.workspace_bytes = (int64_t)(mbytes + ds.total);

    // ---- initial rotation (index only) and the own block ----------------------------------------
    const size_t P2 = (size_t)P * P;
    const unsigned gP2 = (unsigned)((P2 + 255) / 256);
    hipLaunchKernelGGL(k_rotate_init, dim3(gP2), dim3(256), 0, s, sendcounts, mb.cur, P, Q, N);
    HIPCHK(hipGetLastError());
    mark(s, kCatPrepare, -1);
    {
        const int split = hs.max_count > (1 << 16) ? 16 : 1;
        hipLaunchKernelGGL(k_self_copy, dim3(P, split), dim3(256), 0, s, (const unsigned char*)sendbuf, sendcounts,
                           sdispls, (unsigned char*)recvbuf, rdispls, P);
        HIPCHK(hipGetLastError());
    }
    mark(s, kCatSelf, -1);

    // ---- digit phases -----------------------------------------------------------------------------
    int32_t* cur = mb.cur;
    int32_t* nxt = mb.nxt;
    for (size_t i = 0; i < pl.phases.size(); ++i) {
        const PhaseHost& ph = pl.phases[i];
        tuna_phase_stats_t& ps = st.phase[i];
        ps.dim = ph.dim; ps.x = ph.x; ps.radix = ph.r; ps.rounds = ph.nz;
        const bool one_kernel = fused || (staggered && ph.dim == 1);
        if (staggered && ph.dim == 1) ps.rounds = Q * (N - 1);
        ps.blocks = (int64_t)ph.nseg * P;
        const SegDev seg = dp->d_seg[i];
        // metadata exchange and the send-side and receive-side layouts
        {
            PhaseLayoutArgs m{};
            m.cur = cur; m.nxt = nxt; m.zt = dp->d_zt[i]; m.seg = seg; m.nseg = ph.nseg;
            m.P = P; m.Q = Q; m.N = N; m.dim = ph.dim; m.rx = (int)ph.rx;
            m.Ls = mb.Ls; m.Lr = mb.Lr; m.want_send = one_kernel ? 0 : 1;
            m.phase_bytes = &g.d_status->phase_bytes[i]; m.phase_chunks = &g.d_status->phase_chunks[i];
            m.head_displs = one_kernel ? rdispls : nullptr;
            m.head_base = (unsigned int)((uintptr_t)recvbuf & 15u);
            rc = phase_metadata(m, s);
            if (rc != TUNA_OK) return rc;
        }
        mark(s, kCatMeta, (int)i);

        CopyArgs a{};
        a.seg = seg; a.nseg = ph.nseg;
        a.T = T; a.slots = ds.slots; a.slot_bytes = ds.slot_bytes;
        a.P = P; a.Q = Q; a.N = N; a.dim = ph.dim; a.rx = (int)ph.rx;
        a.user_limit = (unsigned long long)(uintptr_t)sendbuf + hs.send_extent;
        if (one_kernel) {
            // one hop in one kernel: S / T of the sender -> R / the other copy of T at the receiver
            a.stage = nullptr; a.L = mb.Lr; a.sizes = nxt;
            a.user = (unsigned char*)sendbuf; a.displs = sdispls;
            a.user2 = (unsigned char*)recvbuf; a.displs2 = rdispls; a.T2 = T;
            rc = launch_copy<kFused>(gran, ds.unit_cap, a, s);
            if (rc != TUNA_OK) return rc;
            mark(s, kCatPack, (int)i);
            std::swap(cur, nxt);
            continue;
        }
        // pack: S / T -> send staging
        a.stage = stage_s; a.L = mb.Ls; a.sizes = cur;
        a.user = (unsigned char*)sendbuf; a.displs = sdispls;
        rc = launch_copy<kPack>(gran, ds.unit_cap, a, s);
        if (rc != TUNA_OK) return rc;
        mark(s, kCatPack, (int)i);
        // exchange: send staging of the partner -> receive staging
        a.stage = stage_r; a.L = mb.Lr; a.stage_src = stage_s; a.Ls = mb.Ls;
        rc = launch_copy<kExchange>(gran, ds.unit_cap, a, s);
        if (rc != TUNA_OK) return rc;
        mark(s, kCatExchange, (int)i);
        // unpack: receive staging -> R / T
        a.sizes = nxt; a.user = (unsigned char*)recvbuf; a.displs = rdispls;
        rc = launch_copy<kUnpack>(gran, ds.unit_cap, a, s);
        if (rc != TUNA_OK) return rc;
        mark(s, kCatUnpack, (int)i);
        std::swap(cur, nxt);
    }
    HIPCHK(hipEventRecord(g.ev_end, s));
    g.end_recorded = true;
    g.have_stats = true;
    return TUNA_OK;
}

}  // namespace
}  // namespace tuna

using namespace tuna;

extern "C" {

int tuna_alltoallv(const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls, void* recvbuf,
                   const int32_t* recvcounts, const int64_t* rdispls, int P, int radix, int ranks_per_node,
                   void* stream) {
    if (radix < 2) return TUNA_ERR_ARG;
    return run(sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P, ranks_per_node, radix, radix, stream);
}

int tuna_alltoallv_hier(const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls, void* recvbuf,
                        const int32_t* recvcounts, const int64_t* rdispls, int P, int ranks_per_node,
                        int local_radix, int global_radix, void* stream) {
    if (local_radix < 2 || global_radix < 2) return TUNA_ERR_ARG;
    return run(sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P, ranks_per_node, local_radix,
               global_radix, stream);
}

int tuna_workspace_bytes(const int32_t* sendcounts, int P, int ranks_per_node, int local_radix, int global_radix,
                         size_t* bytes) {
    if (!bytes || !sendcounts || local_radix < 2 || global_radix < 2) return TUNA_ERR_ARG;
    int Q = 0;
    int rc = resolve_hierarchy(P, ranks_per_node, &Q);
    if (rc != TUNA_OK) return rc;
    rc = ensure_ctx();
    if (rc != TUNA_OK) return rc;
    rc = run_validate(sendcounts, nullptr, nullptr, nullptr, P, nullptr);
    if (rc != TUNA_OK) return rc;
    if (g.h_status->flags & 1u) return TUNA_ERR_NEGATIVE_COUNT;
    // the schedule's slot count does not need the device tables
    const int N = P / Q;
    int rl = local_radix, rg = global_radix;
    const bool staggered = g.opt_staggered != 0 && N > 1;
    if (staggered) rg = N;
    if (Q >= 2 && rl > Q) rl = Q;
    if (N >= 2 && rg > N) rg = N;
    PlanHost pl;
    pl.P = P; pl.Q = Q; pl.N = N;
    const int Kl = Q > 1 ? num_rounds(Q, rl) : 0, Kg = N > 1 ? num_rounds(N, rg) : 0;
    const int Bl = Q > 1 ? Q - 1 - Kl : 0, Bg = N > 1 ? N - 1 - Kg : 0;
    pl.slots = ((int64_t)Bl + (int64_t)(N - 1) * (Q - 1) + (int64_t)Bg * Q) * (g.opt_fused ? 2 : 1);
    if (P > 1) pl.phases.resize(1);
    const DataSizes ds = data_sizes_for(pl, g.h_status->max_count, g.h_status->total_chunks, g.opt_fused != 0, staggered);
    *bytes = meta_bytes_for(P) + ds.total;
    return TUNA_OK;
}

int tuna_plain_copy(const void* src, void* dst, size_t bytes, void* stream) {
    if (!src || !dst || (bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return TUNA_ERR_ARG;
    int rc = ensure_ctx();
    if (rc != TUNA_OK) return rc;
    const size_t n = bytes / 16;
    if (n == 0) return TUNA_OK;
    if ((n + 255) / 256 > 0x7fffffffull) return TUNA_ERR_TOO_LARGE;
    hipLaunchKernelGGL(k_plain_copy, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                       (const v4u*)src, (v4u*)dst, n);
    HIPCHK(hipGetLastError());
    return TUNA_OK;
}

int tuna_set_workspace(void* workspace, size_t bytes) {
    if (workspace && ((uintptr_t)workspace & (kAlign - 1))) return TUNA_ERR_ARG;
    g.user_ws = workspace;
    g.user_ws_bytes = workspace ? bytes : 0;
    return TUNA_OK;
}

int tuna_release(void) {
    if (!g.ready) return TUNA_OK;
    HIPCHK(hipDeviceSynchronize());
    if (g.meta) { HIPCHK(hipFree(g.meta)); g.meta = nullptr; g.meta_bytes = 0; }
    if (g.data) { HIPCHK(hipFree(g.data)); g.data = nullptr; g.data_bytes = 0; }
    for (auto& kv : g.plans) {
        for (auto* p : kv.second.d_seg_mem) (void)hipFree(p);
        for (auto* p : kv.second.d_zt) (void)hipFree(p);
    }
    g.plans.clear();
    return TUNA_OK;
}

int tuna_set_option(int option, int value) {
    if (option == TUNA_OPT_PROFILE) { g.opt_profile = value ? 1 : 0; return TUNA_OK; }
    if (option == TUNA_OPT_FUSED) { g.opt_fused = value ? 1 : 0; return TUNA_OK; }
    if (option == TUNA_OPT_STAGGERED) { g.opt_staggered = value ? 1 : 0; return TUNA_OK; }
    return TUNA_ERR_ARG;
}

int tuna_get_stats(tuna_stats_t* out) {
    if (!out) return TUNA_ERR_ARG;
    if (!g.have_stats) { std::memset(out, 0, sizeof(*out)); out->last_hip_error = g.last_hip_error; return TUNA_OK; }
    tuna_stats_t& st = g.stats;
    if (g.end_recorded) {
        HIPCHK(hipEventSynchronize(g.ev_end));
        HIPCHK(hipMemcpy(g.h_status, g.d_status, sizeof(Status), hipMemcpyDeviceToHost));
        for (int i = 0; i < st.n_phases; ++i) {
            st.phase[i].payload_bytes = (int64_t)g.h_status->phase_bytes[i];
            st.phase[i].staged_bytes = (int64_t)g.h_status->phase_chunks[i] * 16;
        }
        if (g.marks.size() > 1) {
            st.ms_prepare = st.ms_self = 0.f;
            for (int i = 0; i < st.n_phases; ++i)
                st.phase[i].ms_metadata = st.phase[i].ms_pack = st.phase[i].ms_exchange = st.phase[i].ms_unpack = 0.f;
            for (size_t k = 1; k < g.marks.size(); ++k) {
                float ms = 0.f;
                HIPCHK(hipEventElapsedTime(&ms, g.marks[k - 1].ev, g.marks[k].ev));
                const Mark& m = g.marks[k];
                if (m.cat == kCatPrepare) st.ms_prepare += ms;
                else if (m.cat == kCatSelf) st.ms_self += ms;
                else if (m.phase >= 0 && m.phase < TUNA_MAX_PHASES) {
                    tuna_phase_stats_t& ps = st.phase[m.phase];
                    if (m.cat == kCatMeta) ps.ms_metadata += ms;
                    else if (m.cat == kCatPack) ps.ms_pack += ms;
                    else if (m.cat == kCatExchange) ps.ms_exchange += ms;
                    else if (m.cat == kCatUnpack) ps.ms_unpack += ms;
                }
            }
            float tot = 0.f;
            HIPCHK(hipEventElapsedTime(&tot, g.marks.front().ev, g.marks.back().ev));
            st.ms_total = tot;
        }
    }
    *out = st;
    return TUNA_OK;
}

int tuna_plan_info(int P, int ranks_per_node, int local_radix, int global_radix, tuna_plan_info_t* out) {
    if (!out || local_radix < 2 || global_radix < 2) return TUNA_ERR_ARG;
    int Q = 0;
    int rc = resolve_hierarchy(P, ranks_per_node, &Q);
    if (rc != TUNA_OK) return rc;
    if (g.opt_staggered && P / Q > 1) global_radix = P / Q;
    const PlanHost pl = make_plan(P, Q, local_radix, global_radix, g.opt_fused != 0);
    out->P = P; out->Q = Q; out->N = pl.N;
    out->local_radix = pl.rl; out->global_radix = pl.rg;
    out->w_local = pl.w_l; out->w_global = pl.w_g;
    out->K_local = pl.K_l; out->K_global = (g.opt_staggered && pl.N > 1) ? Q * (pl.N - 1) : pl.K_g;
    out->B_local = pl.B_l; out->B_global = pl.B_g;
    out->n_phases = (int)pl.phases.size();
    out->temp_slots_per_rank = pl.slots;
    out->blocks_sent_per_rank = pl.blocks_sent;
    return TUNA_OK;
}

int tuna_plan_phase(int P, int ranks_per_node, int local_radix, int global_radix, int phase, int32_t* header,
                    int32_t* seg, int seg_capacity) {
    if (!header || local_radix < 2 || global_radix < 2 || phase < 0) return TUNA_ERR_ARG;
    int Q = 0;
    int rc = resolve_hierarchy(P, ranks_per_node, &Q);
    if (rc != TUNA_OK) return rc;
    const PlanHost pl = make_plan(P, Q, local_radix, global_radix, g.opt_fused != 0);
    if (phase >= (int)pl.phases.size()) return TUNA_ERR_ARG;
    const PhaseHost& ph = pl.phases[phase];
    header[0] = ph.dim; header[1] = ph.x; header[2] = ph.r; header[3] = ph.nz; header[4] = ph.nseg;
    header[5] = (int32_t)ph.rx;
    if (seg) {
        const int n = seg_capacity < ph.nseg ? seg_capacity : ph.nseg;
        for (int k = 0; k < n; ++k) {
            const SegInfo& si = ph.seg[k];
            int32_t* o = seg + (size_t)k * 6;
            o[0] = si.e; o[1] = si.j; o[2] = si.l; o[3] = si.z; o[4] = si.src_slot; o[5] = si.dst_slot;
        }
    }
    return TUNA_OK;
}

int tuna_select_radix(int P, int ranks_per_node, int64_t payload_bytes, int* local_radix, int* global_radix,
                      double* predicted_ms) {
    if (!local_radix || !global_radix || payload_bytes < 0) return TUNA_ERR_ARG;
    int Q = 0;
    int rc = resolve_hierarchy(P, ranks_per_node, &Q);
    if (rc != TUNA_OK) return rc;
    const int N = P / Q;
    // measured on MI355X at P = 4096 (see profiles/): copy stages ~5.2e12 B/s, metadata kernels of
    // a phase ~60 us + 20 ps per matrix entry, validation + rotation ~0.3 ms at P = 4096
    const double bw = 5.2e12, c = g.opt_fused ? 2.0 : 6.0;
    const double t_phase = 60e-6 + 2.0e-11 * (double)P * P, t_call = 50e-6 + 1.5e-11 * (double)P * P;
    auto hops = [](int size, int r) {           // H(r) over one dimension
        long long nz = 0;
        for (int i = 0; i < size; ++i)
            for (int v = i; v; v /= r) nz += (v % r) != 0;
        return (double)nz / size;
    };
    auto best = [&](int size, int* radix) -> double {
        if (size < 2) { *radix = 2; return 0.0; }
        std::vector<int> cand;
        for (long long r = 2; r < size; r *= 2) cand.push_back((int)r);
        int sq = 2;
        while ((long long)sq * sq < size) ++sq;
        cand.push_back(sq);
        cand.push_back(size);
        double bt = -1.0;
        for (int r : cand) {
            const double t = num_digits(size, r) * t_phase + c * hops(size, r) * (double)payload_bytes / bw;
            if (bt < 0 || t < bt) { bt = t; *radix = r; }
        }
        return bt;
    };
    const double tl = best(Q, local_radix), tg = best(N, global_radix);
    if (predicted_ms) *predicted_ms = (t_call + tl + tg) * 1e3;
    return TUNA_OK;
}

int tuna_t_index(int o, int radix) {
    if (radix < 2) return -1;
    return (int)t_index(o, radix);
}

const char* tuna_strerror(int code) {
    switch (code) {
        case TUNA_OK: return "ok";
        case TUNA_ERR_ARG: return "invalid argument";
        case TUNA_ERR_COUNT_MISMATCH: return "recvcounts is not the transpose of sendcounts";
        case TUNA_ERR_NEGATIVE_COUNT: return "negative count";
        case TUNA_ERR_NOMEM: return "out of device memory";
        case TUNA_ERR_WORKSPACE_TOO_SMALL: return "caller-supplied workspace too small";
        case TUNA_ERR_HIP: return "HIP runtime error";
        case TUNA_ERR_TOO_LARGE: return "problem exceeds the supported range";
        default: return "unknown error";
    }
}

int tuna_version(void) { return kVersion; }

}  // extern "C"
