// C ABI of the tunable-radix non-uniform all-to-all for MI355X: argument checks, the cached
// schedule, workspace management and the per-phase launch sequence.  All payload movement and
// all per-block arithmetic happen in the kernels of tuna_kernels.h; the host only loops over
// the ceil(log_r) digit phases.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <map>
#include <tuple>
#include <vector>

#include "../../include/tuna.h"
#include "tuna_kernels.h"
#include "tuna_plan.h"

// Scratch memory of tuna_alltoallv_noalloc: everything the kernels of a call need beyond the caller's
// six arrays (status block, schedule tables, size matrices, scans, work lists, staging buffers, T).
// One array per GPU, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels receive the address that call returned for the current device.
static __device__ __align__(256) unsigned char scratch[TUNA_NOALLOC_SCRATCH_BYTES];

namespace tuna {
namespace {

constexpr int kVersion = 101;
constexpr size_t kAlign = 256;
// A one-kernel phase cuts chunks at the destination's 16-byte lines, so its last load of a block
// that lies in T may run up to 15 bytes past the block: T is allocated with this much room behind it.
constexpr size_t kTailSlack = 256;

struct DevicePlan {
    PlanHost host;
    std::vector<SegDev> d_seg;
    std::vector<int32_t*> d_seg_mem;
    hipStream_t built_on = nullptr;      // stream the table kernels were enqueued on
    bool complete = false;               // known to have finished (a later call synchronised)
    std::vector<int32_t*> d_zt;
    int32_t* d_hm1 = nullptr;            // [P]: hops - 1 of every slot index (how often the block is stored into T)
    unsigned long long* d_mask = nullptr; // [P]: phases in which the block with a slot index moves (move_mask)
    // exact-size T: per phase the T-bound segments grouped by class (see ExactT), on the device and,
    // for the launch shapes, the classes on the host
    std::vector<int32_t*> d_tord, d_tcls;
    std::vector<std::vector<int32_t>> tcls;   // per phase: {class id, first entry of tord, entries} per class
    bool borrowed = false;               // the device memory belongs to someone else (static scratch)
};

// The T-bound segments of every phase grouped by the class they are stored into, in message order
// within a class: tord[phase] lists segment indices, tcls[phase] holds {class id, start, count} triples.
void build_class_tables(const PlanHost& pl, std::vector<std::vector<int32_t>>& tord, std::vector<std::vector<int32_t>>& tcls) {
    const size_t nph = pl.phases.size();
    tord.assign(nph, {}); tcls.assign(nph, {});
    for (size_t i = 0; i < nph; ++i) {
        PhaseScalars ps = phase_scalars(pl.phases[i]);
        std::vector<std::vector<int32_t>> by_next(nph);       // segment indices by the phase of the next move
        for (int e = 0; e < pl.P; ++e) {
            SegInfo si{};
            int pos = 0;
            if (slot_entry(pl.sc, ps, e, &si, &pos) && si.nxt_phase >= 0 && si.nxt_phase < (int)nph)
                by_next[si.nxt_phase].push_back(pos);
        }
        for (size_t y = i + 1; y < nph; ++y) {
            if (by_next[y].empty()) continue;
            std::sort(by_next[y].begin(), by_next[y].end());
            tcls[i].push_back(class_id((int)i, (int)y, (int)nph));
            tcls[i].push_back((int32_t)tord[i].size());
            tcls[i].push_back((int32_t)by_next[y].size());
            tord[i].insert(tord[i].end(), by_next[y].begin(), by_next[y].end());
        }
    }
}

// Where a call's validation pass and per-phase totals are written and read back: the library's own
// small allocations, or a part of the static scratch of the entry point that allocates nothing.
struct StatusBufs {
    Status* d_status = nullptr;              // device status block
    Status* h_status = nullptr;              // host mirror (pinned for the library's own)
    Status* h_status_dev = nullptr;          // the device's address of the pinned mirror (nullptr: not mapped)
    unsigned long long* d_vpart = nullptr;   // partial results of the validation pass, one row per workgroup
    int num_cus = 256;
};

enum Category { kCatPrepare = 0, kCatSelf, kCatMeta, kCatPack, kCatExchange, kCatUnpack };

struct Mark { hipEvent_t ev; int cat; int phase; };

// Options of one call or plan (tuna_opts_t, or the process-wide defaults that tuna_set_option edits).
struct Options {
    int profile = 0;
    int mode = TUNA_MODE_AUTO;
    int staggered = 0;
    int t_layout = TUNA_T_AUTO;
    int block_count = 0;
};

// Process-wide state: the device, the cached schedules (read-only once built), the default options.
struct Shared {
    bool ready = false;
    int device = -1;
    int num_cus = 256;
    std::map<std::tuple<int, int, int, int, int>, DevicePlan> plans;
    int live_plans = 0;                 // persistent plans not yet freed (they point into `plans`)
    int live_contexts = 0;              // contexts made by tuna_ctx_create and not yet destroyed
    int last_hip_error = 0;
    Options defaults;
};

Shared sh;

// Everything one immediate call writes besides the caller's receive buffer: the workspace, the status
// block, the statistics and the profiling events.  Calls that share a context share these; calls on
// different contexts share nothing and may overlap in time.
struct Ctx {
    bool ready = false;
    StatusBufs sb;                    // status block, its pinned host mirror, validation partials (one-time small allocations)
    void* meta = nullptr;  size_t meta_bytes = 0;   // library-owned, grow-only
    void* data = nullptr;  size_t data_bytes = 0;
    void* user_ws = nullptr; size_t user_ws_bytes = 0;
    tuna_stats_t stats;
    bool have_stats = false;
    bool profile = false;               // the call being issued records events
    std::vector<hipEvent_t> ev_pool;
    std::vector<Mark> marks;
    hipEvent_t ev_end = nullptr;
    bool end_recorded = false;
    hipStream_t last_stream = nullptr;  // stream of the last immediate call (its end is ev_end when end_recorded)
    unsigned char* tiny_t = nullptr;    // T of the one-kernel call for tiny problems (kTinyTBytes, allocated at its first use)
    const void* tiny_declined = nullptr; // sendcounts of the last problem that kernel declined: it is not asked again for it
    const void* stats_plan = nullptr;   // the statistics on file belong to this persistent plan (payload bytes known)
    // pipelined calls (run_pipelined): the stream the metadata kernels run on, the event that lets it start, and one
    // event per phase that lets the phase's payload kernel start; made at the first such call
    hipStream_t meta_stream = nullptr;
    hipEvent_t ev_fork = nullptr;
    std::vector<hipEvent_t> ev_phase;
};

Ctx g;                                  // the default context

#define HIPCHK(expr)                                                       \
    do {                                                                   \
        hipError_t _e = (expr);                                            \
        if (_e != hipSuccess) { sh.last_hip_error = (int)_e; return TUNA_ERR_HIP; } \
    } while (0)

inline size_t align_up(size_t v, size_t a = kAlign) { return (v + a - 1) / a * a; }

// 64-bit words of the validation pass's partial results: at most 8 workgroups per compute unit
inline size_t vpart_words(int num_cus) { return (size_t)num_cus * 8 * kValPartial; }

// The library runs on the HIP device that is current at its first call.
int ensure_device() {
    if (sh.ready) {
        // the workspaces, the schedules and the status blocks live on the first call's device: refuse
        // to launch kernels on them from another one
        int dev = -1;
        HIPCHK(hipGetDevice(&dev));
        return dev == sh.device ? TUNA_OK : TUNA_ERR_ARG;
    }
    int ndev = 0;
    HIPCHK(hipGetDeviceCount(&ndev));
    if (ndev < 1) { sh.last_hip_error = (int)hipErrorNoDevice; return TUNA_ERR_HIP; }
    HIPCHK(hipGetDevice(&sh.device));
    hipDeviceProp_t prop;
    HIPCHK(hipGetDeviceProperties(&prop, sh.device));
    sh.num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    sh.ready = true;
    return TUNA_OK;
}

int ensure_ctx(Ctx& c) {
    const int rc = ensure_device();
    if (rc != TUNA_OK || c.ready) return rc;
    c.sb.num_cus = sh.num_cus;
    HIPCHK(hipMalloc((void**)&c.sb.d_status, align_up(sizeof(Status))));
    HIPCHK(hipHostMalloc((void**)&c.sb.h_status, sizeof(Status), hipHostMallocDefault));
    if (hipHostGetDevicePointer((void**)&c.sb.h_status_dev, c.sb.h_status, 0) != hipSuccess) {
        (void)hipGetLastError();
        c.sb.h_status_dev = nullptr;
    }
    HIPCHK(hipMalloc((void**)&c.sb.d_vpart, align_up(vpart_words(c.sb.num_cus) * 8)));
    HIPCHK(hipEventCreate(&c.ev_end));
    std::memset(&c.stats, 0, sizeof(c.stats));
    c.ready = true;
    return TUNA_OK;
}

void free_ctx(Ctx& c) {
    if (c.sb.d_status) (void)hipFree(c.sb.d_status);
    if (c.sb.h_status) (void)hipHostFree(c.sb.h_status);
    if (c.sb.d_vpart) (void)hipFree(c.sb.d_vpart);
    if (c.meta) (void)hipFree(c.meta);
    if (c.data) (void)hipFree(c.data);
    if (c.tiny_t) (void)hipFree(c.tiny_t);
    if (c.ev_end) (void)hipEventDestroy(c.ev_end);
    for (hipEvent_t e : c.ev_pool) (void)hipEventDestroy(e);
    for (hipEvent_t e : c.ev_phase) (void)hipEventDestroy(e);
    if (c.ev_fork) (void)hipEventDestroy(c.ev_fork);
    if (c.meta_stream) (void)hipStreamDestroy(c.meta_stream);
    c = Ctx{};
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
    unsigned long long* rank_bytes;
};

size_t meta_bytes_for(int P) {
    const size_t P2 = (size_t)P * P, ld = (size_t)P + 1;
    size_t b = 0;
    b += 2 * align_up(P2 * 4);
    b += 2 * (align_up(P * ld * 4) + align_up(P * 4) + align_up((P + 1) * 8) + align_up((P + 1) * 4) + align_up(4));
    b += align_up((size_t)P * 8);          // payload bytes per rank of the phase being laid out
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
    L.unit_chunks = kUnitChunks;
}

MetaBuffers carve_meta(Carver& cv, int P) {
    MetaBuffers m;
    m.cur = cv.take<int32_t>((size_t)P * P);
    m.nxt = cv.take<int32_t>((size_t)P * P);
    carve_layout(cv, P, m.Ls);
    carve_layout(cv, P, m.Lr);
    m.rank_bytes = cv.take<unsigned long long>(P);
    return m;
}

// metadata of exact-size T: per class the ranks' first chunks and part sizes and the class's place in
// T, per phase the blocks' offsets by slot index, and the same offsets in message order (one array for
// the phase being run, or one per phase when a plan keeps them)
size_t exact_t_meta_bytes_for(const PlanHost& pl, bool keep_all_phases) {
    const size_t nph = pl.phases.size(), P = (size_t)pl.P, ncls = (size_t)class_count((int)nph);
    return (keep_all_phases ? nph : 1) * align_up(P * (P + 1) * 4) + align_up(nph * P * P * 4) +
           align_up(ncls * P * 8) + align_up(ncls * P * 4) + align_up(ncls * 8);
}

struct Prepared;
void carve_exact_t(Carver& cv, const PlanHost& pl, bool keep_all_phases, Prepared& pr);

struct DataSizes {
    size_t unit_cap;        // wave units per layout (upper bound)
    size_t stage_chunks;    // chunks per staging buffer
    long long slots;        // T slots per rank
    long long slot_bytes;   // M rounded up to whole 128-byte lines
    size_t t_bytes;
    size_t total;
};

DataSizes data_sizes_for(const PlanHost& pl, long long M, unsigned long long total_chunks, bool fused,
                         bool staggered = false, bool dense = false, unsigned long long t_chunks = 0,
                         bool tiled = false) {
    // t_chunks: exact-size T as the host laid it out (colour_classes)
    DataSizes d{};
    const bool any_phase = !pl.phases.empty() && total_chunks > 0;
    // every rank's region of a staging buffer (and of a class of exact-size T) is rounded up to a 128-byte line
    const size_t rank_pad = (size_t)pl.P * kRankAlignChunks;
    d.stage_chunks = any_phase ? (size_t)total_chunks + rank_pad : 0;
    // fused rounds cut chunks at destination lines: up to one more chunk per moving block
    // the destination-tiled hop counts 16-byte pieces of R and T: a block owns at most its chunks plus the
    // 7 pieces from its line's start, 7 that complete the previous run's line, one for an unaligned end
    const size_t head_chunks = ((fused || staggered) ? (size_t)pl.P * pl.P : 0) * (tiled ? 16 : 1);
    d.unit_cap = any_phase ? (size_t)((total_chunks + head_chunks) / kUnitChunks) + pl.P + 1 : 0;
    d.slots = pl.slots;
    d.slot_bytes = (M + 127) / 128 * 128;     // whole 128-byte lines per slot
    d.t_bytes = any_phase ? (size_t)pl.P * (size_t)d.slots * (size_t)d.slot_bytes : 0;
    if (dense) {       // exact size: what waits in T at one time
        d.slots = 0;
        d.t_bytes = any_phase ? (size_t)t_chunks * 16 : 0;
    }
    // pl.slots already counts both copies of T when the plan is a fused one
    d.total = 2 * align_up(d.unit_cap * sizeof(int4)) + (fused ? 0 : 2 * align_up(d.stage_chunks * 16)) +
              align_up(d.t_bytes + kTailSlack);
    return d;
}

void free_device_plan(DevicePlan& dp) {
    if (!dp.borrowed) {
        for (auto* p : dp.d_seg_mem) (void)hipFree(p);
        for (auto* p : dp.d_zt) (void)hipFree(p);
        for (auto* p : dp.d_tord) (void)hipFree(p);
        for (auto* p : dp.d_tcls) (void)hipFree(p);
        if (dp.d_hm1) (void)hipFree(dp.d_hm1);
        if (dp.d_mask) (void)hipFree(dp.d_mask);
    }
    dp.d_seg_mem.clear(); dp.d_zt.clear(); dp.d_seg.clear(); dp.d_tord.clear(); dp.d_tcls.clear();
    dp.d_hm1 = nullptr; dp.d_mask = nullptr;
}

// Cached schedule of (P, Q, r_l, r_g, fused).  The host keeps scalars only; the per-phase tables are
// built on the device by k_build_phase_table, on the caller's stream (the kernels that read them
// are enqueued behind it).
// Radices clamped the way make_plan clamps them.
void clamp_radices(int Q, int N, int rl, int rg, int* crl, int* crg) {
    *crl = rl < 2 ? 2 : rl; *crg = rg < 2 ? 2 : rg;
    if (Q >= 2 && *crl > Q) *crl = Q;
    if (N >= 2 && *crg > N) *crg = N;
    if (Q < 2) *crl = 2;
    if (N < 2) *crg = 2;
}

int get_plan(int P, int Q, int rl, int rg, bool fused, hipStream_t s, DevicePlan** out) {
    const int N = P / Q;
    int crl, crg;
    clamp_radices(Q, N, rl, rg, &crl, &crg);
    auto key = std::make_tuple(P, Q, crl, crg, fused ? 1 : 0);
    auto it = sh.plans.find(key);
    if (it == sh.plans.end()) {
        DevicePlan dp;
        dp.host = make_plan(P, Q, crl, crg, fused, /*with_tables=*/false);
        if ((int)dp.host.phases.size() > TUNA_MAX_PHASES) return TUNA_ERR_TOO_LARGE;
        // a schedule that cannot be completed leaves nothing behind (its kernels may be in flight: wait)
        struct Guard {
            DevicePlan* dp; hipStream_t s;
            ~Guard() { if (dp) { (void)hipStreamSynchronize(s); free_device_plan(*dp); } }
        } guard{&dp, s};
        for (auto& ph : dp.host.phases) {
            // field-major table: e[], z[], src[], dst[], srcph[], srcseg[]
            const size_t stride = align_up((size_t)ph.nseg * 4) / 4;
            int32_t* dm = nullptr;
            int32_t* dz = nullptr;
            HIPCHK(hipMalloc((void**)&dm, 8 * stride * 4 + kAlign));
            dp.d_seg_mem.push_back(dm);
            HIPCHK(hipMalloc((void**)&dz, align_up((size_t)P * 4)));
            dp.d_zt.push_back(dz);
            hipLaunchKernelGGL(k_build_phase_table, dim3((unsigned)((P + 255) / 256)), dim3(256), 0, s, dp.host.sc,
                               phase_scalars(ph), dm, dm + stride, dm + 2 * stride, dm + 3 * stride, dm + 4 * stride,
                               dm + 5 * stride, dm + 6 * stride, dm + 7 * stride, dz);
            HIPCHK(hipGetLastError());
            dp.d_seg.push_back(SegDev{dm, dm + stride, dm + 2 * stride, dm + 3 * stride, dm + 4 * stride, dm + 5 * stride,
                                      dm + 6 * stride, dm + 7 * stride});
        }
        HIPCHK(hipMalloc((void**)&dp.d_hm1, align_up((size_t)P * 4)));
        HIPCHK(hipMalloc((void**)&dp.d_mask, align_up((size_t)P * 8)));
        hipLaunchKernelGGL(k_build_hops, dim3((unsigned)((P + 255) / 256)), dim3(256), 0, s, dp.host.sc, dp.d_hm1, dp.d_mask);
        HIPCHK(hipGetLastError());
        // the class tables of exact-size T come from the host (copied before the call returns: the
        // vectors are temporaries)
        std::vector<std::vector<int32_t>> tord;
        build_class_tables(dp.host, tord, dp.tcls);
        for (size_t i = 0; i < dp.host.phases.size(); ++i) {
            int32_t *d_o = nullptr, *d_c = nullptr;
            HIPCHK(hipMalloc((void**)&d_o, align_up(tord[i].size() * 4 + 4)));
            dp.d_tord.push_back(d_o);
            HIPCHK(hipMalloc((void**)&d_c, align_up(dp.tcls[i].size() * 4 + 4)));
            dp.d_tcls.push_back(d_c);
            if (!tord[i].empty()) HIPCHK(hipMemcpy(d_o, tord[i].data(), tord[i].size() * 4, hipMemcpyHostToDevice));
            if (!dp.tcls[i].empty()) HIPCHK(hipMemcpy(d_c, dp.tcls[i].data(), dp.tcls[i].size() * 4, hipMemcpyHostToDevice));
        }
        dp.built_on = s;
        guard.dp = nullptr;
        it = sh.plans.emplace(key, std::move(dp)).first;
    }
    // a cached schedule built on another stream: make sure its tables are complete
    if (it->second.built_on != s && !it->second.complete) {
        HIPCHK(hipStreamSynchronize(it->second.built_on));
        it->second.complete = true;
    }
    *out = &it->second;
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
    if (e != hipSuccess) { (void)hipGetLastError(); sh.last_hip_error = (int)e; *buf = nullptr; return TUNA_ERR_NOMEM; }
    *have = need;
    return TUNA_OK;
}

void mark(Ctx* c, hipStream_t s, int cat, int phase) {
    if (!c || !c->profile) return;
    const size_t k = c->marks.size();
    if (k >= c->ev_pool.size()) {
        hipEvent_t ev;
        if (hipEventCreate(&ev) != hipSuccess) return;
        c->ev_pool.push_back(ev);
    }
    if (hipEventRecord(c->ev_pool[k], s) != hipSuccess) return;
    c->marks.push_back(Mark{c->ev_pool[k], cat, phase});
}

// One-shot grid over an upper bound of wave units (4 per workgroup); waves past the device-side
// unit count exit immediately.
// Dynamic LDS that leaves room for `resident` workgroups of a copy kernel per compute unit (one wave
// per SIMD each; 8 is the kernels' own limit).  Nothing uses the memory: it only caps the occupancy.
// static_lds: the kernel's own LDS bytes.
size_t occupancy_padding(int resident, size_t static_lds) {
    constexpr size_t kLdsPerCu = 160 * 1024;
    if (resident >= 8) return 0;
    // more than 1 / (resident + 1) of the LDS each, rounded up to 1 KiB: resident + 1 workgroups no longer fit
    const size_t want = (kLdsPerCu / (size_t)(resident + 1) / 1024 + 1) * 1024;
    return want > static_lds ? want - static_lds : 0;
}

template <class K>
size_t static_lds_of(K kernel) {
    hipFuncAttributes at{};
    if (hipFuncGetAttributes(&at, reinterpret_cast<const void*>(kernel)) != hipSuccess) { (void)hipGetLastError(); return 0; }
    return at.sharedSizeBytes;
}

// resident: workgroups per compute unit the launch may keep resident (see occupancy_padding)
template <int MODE, bool DENSE>
int launch_copy_as(int gran, size_t unit_cap, const CopyArgs& a, hipStream_t s, int resident) {
    const size_t waves = kCopyThreads / kWave;
    // unit_cap counts the units of the whole launch, or of one rank's row when the launch has a row per rank
    const dim3 grid((unsigned)((unit_cap + waves - 1) / waves), a.batch_rows ? (unsigned)a.P : 1u), block(kCopyThreads);
    if (grid.x == 0) return TUNA_OK;
    if ((MODE == kPack || MODE == kFused) && gran == 128) {
        static const size_t lds = static_lds_of(k_copy<MODE, 128, DENSE>);
        hipLaunchKernelGGL((k_copy<MODE, 128, DENSE>), grid, block, occupancy_padding(resident, lds), s, a);   // sources are whole lines
    } else if (MODE == kExchange || gran >= 16) {
        static const size_t lds = static_lds_of(k_copy<MODE, 16, DENSE>);
        hipLaunchKernelGGL((k_copy<MODE, 16, DENSE>), grid, block, occupancy_padding(resident, lds), s, a);
    } else if (gran == 4) {
        static const size_t lds = static_lds_of(k_copy<MODE, 4, DENSE>);
        hipLaunchKernelGGL((k_copy<MODE, 4, DENSE>), grid, block, occupancy_padding(resident, lds), s, a);
    } else {
        static const size_t lds = static_lds_of(k_copy<MODE, 1, DENSE>);
        hipLaunchKernelGGL((k_copy<MODE, 1, DENSE>), grid, block, occupancy_padding(resident, lds), s, a);
    }
    HIPCHK(hipGetLastError());
    return TUNA_OK;
}

// exact_kernels: the variant that addresses T in exact size (it never looks at its T arguments when
// the schedule has no T-bound block, so it also serves schedules without T)
template <int MODE>
int launch_copy(int gran, size_t unit_cap, const CopyArgs& a, hipStream_t s, bool exact_kernels, int resident = 8) {
    if (MODE != kExchange && exact_kernels) return launch_copy_as<MODE, true>(gran, unit_cap, a, s, resident);
    return launch_copy_as<MODE, false>(gran, unit_cap, a, s, resident);
}

// Metadata of one digit phase: sizes exchanged, both staging layouts scanned, wave units cut.
int phase_metadata(const PhaseLayoutArgs& a, hipStream_t s, const ExactT& x, bool sizes_ready = false) {
    if (!a.inline_exchange && !sizes_ready) {
        hipLaunchKernelGGL(k_size_exchange, dim3((unsigned)((a.P + 255) / 256), (unsigned)((a.P + kExchangeRanks - 1) / kExchangeRanks)),
                           dim3(256), 0, s, a.cur, a.nxt, a.zt, a.P, a.Q, a.N, a.dim, a.rx);
        HIPCHK(hipGetLastError());
    }
    hipLaunchKernelGGL(k_phase_layout, dim3(a.P), dim3(kScanThreads), 0, s, a);
    HIPCHK(hipGetLastError());
    // layouts to scan: receive side, the send side where wanted, then the classes of exact-size T
    const int nl = a.want_send ? 2 : 1;
    hipLaunchKernelGGL(k_layout_base, dim3(nl + (a.want_tbound ? x.ncls : 0)), dim3(kScanThreads), 0, s, a.P, a.Lr, a.Ls, nl,
                       a.phase_chunks, a.want_send ? 1 : 0, x, a.rank_bytes, a.phase_bytes, a.phase_units);
    HIPCHK(hipGetLastError());
    const int lds_ints = a.nseg + 1 <= kUnitsLdsMaxInts ? a.nseg + 1 : 0;
    hipLaunchKernelGGL(k_layout_units, dim3(a.P, a.want_send ? 2 : 1), dim3(256), (size_t)lds_ints * 4, s, a.nseg, a.Lr,
                       a.Ls, lds_ints);
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

// Validation + sizing pass shared by tuna_alltoallv* and tuna_workspace_bytes: fills *sb.h_status.
int run_validate(const StatusBufs& sb, const int32_t* sendcounts, const int32_t* recvcounts, const int64_t* sdispls,
                 const int64_t* rdispls, int P, hipStream_t s, const DevicePlan* exact_t_for = nullptr) {
    // every field of the status block a call reads is written by the call's own kernels: no clearing
    const size_t t = (size_t)((P + kValTile - 1) / kValTile);
    const unsigned vgrid = (unsigned)(t * t < (size_t)sb.num_cus * 8 ? t * t : (size_t)sb.num_cus * 8);
    // with a schedule that has T: also the size of every class of exact-size T (summed into the status block)
    const int nph = exact_t_for ? (int)exact_t_for->host.phases.size() : 0;
    const int ncls = class_count(nph);
    if (ncls > 0) {
        hipLaunchKernelGGL(k_zero64, dim3((unsigned)((ncls + 255) / 256)), dim3(256), 0, s, sb.d_status->cls_chunks, ncls);
        HIPCHK(hipGetLastError());
    }
    hipLaunchKernelGGL(k_validate, dim3(vgrid), dim3(kValTile, 4), (size_t)ncls * 8, s, sendcounts, recvcounts, sdispls,
                       rdispls, P, sb.d_vpart, exact_t_for ? exact_t_for->d_hm1 : nullptr,
                       exact_t_for ? exact_t_for->host.Q : 1, exact_t_for ? exact_t_for->host.N : 1,
                       exact_t_for ? exact_t_for->d_mask : nullptr, nph, sb.d_status->cls_chunks);
    HIPCHK(hipGetLastError());
    hipLaunchKernelGGL(k_validate_finish, dim3(1), dim3(256), 0, s, sb.d_vpart, (int)vgrid, sb.d_status);
    HIPCHK(hipGetLastError());
    HIPCHK(hipMemcpyAsync(sb.h_status, sb.d_status, 64, hipMemcpyDeviceToHost, s));
    if (ncls > 0)
        HIPCHK(hipMemcpyAsync(sb.h_status->cls_chunks, sb.d_status->cls_chunks, (size_t)ncls * 8, hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));
    return TUNA_OK;
}

// What the data kernels of a call need, fixed once the counts have been validated and sized.
struct Prepared {
    int P = 0, Q = 0, N = 0;
    DevicePlan* dp = nullptr;
    StatusBufs sb;
    Ctx* ctx = nullptr;                 // where profiling marks go (none for the entry point that allocates nothing)
    Options opt;
    int32_t* debug_sizes = nullptr;     // host [phases + 1][P][P]: the block-size matrix before the first phase and after every phase (verification)
    bool fused = false, staggered = false;
    int gran = 1;
    const void* sendbuf = nullptr;
    void* recvbuf = nullptr;
    const int32_t* sendcounts = nullptr;
    const int32_t* recvcounts = nullptr;
    const int64_t* sdispls = nullptr;
    const int64_t* rdispls = nullptr;
    unsigned long long user_limit = 0;
    int max_count = 0;
    unsigned long long total_bytes = 0;
    DataSizes ds{};
    v4u* stage_s = nullptr;
    v4u* stage_r = nullptr;
    unsigned char* T = nullptr;
    // exact-size T: the prefix over the T-bound blocks (per phase, or one reused by every phase) and
    // the per-phase position tables; the classes' places in T come from the host (colour_classes), the
    // ranks' places inside a class are assigned on the device, phase by phase
    bool exact_t = false;               // T in exact size, and the schedule has T at all
    bool exact_kernels = false;         // T in exact size was asked for
    bool tiled = false;                 // one-kernel phases before the last run as the destination-tiled hop (k_copy_tiled) where they can
    bool tiled_final = false;           // and so does the last phase
    bool sizes_direct = false;          // one phase: the receivers' sizes were taken from recvcounts (run_one_pass), no size exchange
    std::vector<int*> tpre;             // per phase: the blocks' offsets in message order (one array shared, or one each)
    ExactT x{};
    long long* d_cbase = nullptr;       // [classes]: where the host placed every class in T
    std::vector<long long> cbase;       // the same on the host
    unsigned long long t_chunks = 0;    // chunks of exact-size T as laid out
    HopDev hop{};                       // one-kernel phases of a one-pass call: the resolved addresses of the phase being run
    // the ranks' own blocks: moved by the copy engine when blocks can be large (see launch_self_copy)
    bool self_engine = false;
    LayoutDev selfL{};
    HopDev selfH{};
    size_t self_units = 0;              // wave units to launch for: an upper bound, or the exact count of a plan
    int block_count = 0;                // rounds per batch of launches (0: all rounds of a phase at once)
    unsigned long long* rank_bytes = nullptr;   // [P] scratch of the metadata kernels
};

void carve_exact_t(Carver& cv, const PlanHost& pl, bool keep_all_phases, Prepared& pr) {
    const size_t nph = pl.phases.size(), P = (size_t)pl.P, ncls = (size_t)class_count((int)nph);
    pr.tpre.assign(nph, nullptr);
    for (size_t i = 0; i < nph; ++i)
        pr.tpre[i] = (i == 0 || keep_all_phases) ? cv.take<int>(P * (P + 1)) : pr.tpre[0];
    pr.x.tpos = cv.take<int>(nph * P * P);
    pr.x.tbase = cv.take<long long>(ncls * P);
    pr.x.csub = cv.take<int>(ncls * P);
    pr.d_cbase = cv.take<long long>(ncls);
    pr.x.cbase = pr.d_cbase;
}

// The classes' places in T go to the device through the pinned mirror of the status block (its class
// sums have been read by now); the copy is ordered on the stream before the kernels that read it.
int upload_cbase(const Prepared& pr, hipStream_t s) {
    const size_t ncls = pr.cbase.size();
    if (!pr.exact_t || !ncls) return TUNA_OK;
    long long* stage = reinterpret_cast<long long*>(pr.sb.h_status->cls_chunks);
    for (size_t k = 0; k < ncls; ++k) stage[k] = pr.cbase[k];
    HIPCHK(hipMemcpyAsync(pr.d_cbase, stage, ncls * 8, hipMemcpyHostToDevice, s));
    return TUNA_OK;
}

// the exact-size T arguments of phase i
ExactT exact_t_of(const Prepared& pr, size_t i) {
    ExactT x = pr.x;
    if (!pr.exact_t) return ExactT{};
    x.tpre = pr.tpre[i]; x.ld = pr.P + 1; x.phase = (int)i;
    x.tord = pr.dp->d_tord[i]; x.tcls = pr.dp->d_tcls[i]; x.ncls = (int)(pr.dp->tcls[i].size() / 3);
    return x;
}

bool phase_is_one_kernel(const Prepared& pr, const PhaseHost& ph) {
    return pr.fused || (pr.staggered && ph.dim == 1);
}

// Where the classes of exact-size T lie.  Class (f, y) holds the blocks stored when they arrive in
// phase f and forwarded in phase y; it needs its chunks (summed by the validation pass) plus a 128-byte
// line of rounding per rank, and it is alive from the kernel that stores it to the kernel that reads it:
// with three stages from the unpack of phase f to the pack of phase y, with one-kernel phases from the
// kernel of phase f to the kernel of phase y (which reads it while it stores the classes (y, .), so those
// must lie elsewhere).  A phase run in batches of rounds (`batched`) is like a one-kernel phase in this
// respect: the unpack of its first batch stores while the pack of its next batch still has to read.
// Every class is placed at the lowest offset where it overlaps no class alive at the same time (first
// fit).  Returns the chunks of T; cbase[class] = first chunk.
unsigned long long colour_classes(const PlanHost& pl, bool fused, bool staggered, bool batched,
                                  const unsigned long long* cls_chunks, std::vector<long long>& cbase) {
    const int nph = (int)pl.phases.size();
    struct Item { int cid, start, end; unsigned long long cap; long long off; };
    std::vector<Item> items;
    for (int f = 0; f < nph; ++f) {
        const bool one_kernel = fused || batched || (staggered && pl.phases[f].dim == 1);
        for (int y = f + 1; y < nph; ++y) {
            const int cid = class_id(f, y, nph);
            if (!cls_chunks[cid]) continue;
            const unsigned long long cap = (cls_chunks[cid] + (unsigned long long)pl.P * kRankAlignChunks + 15) / 16 * 16;
            items.push_back(Item{cid, 2 * f + (one_kernel ? 0 : 1), 2 * y, cap, 0});
        }
    }
    // First fit depends on the order of placement and no single order is best for every schedule: four
    // are tried (by first use, by size, by length of life, by size times length of life) and the
    // tightest result is kept (at most 12 % above the bytes alive at one time on the schedules measured).
    cbase.assign((size_t)class_count(nph), 0);
    unsigned long long best_extent = ~0ull;
    for (int order = 0; order < 4; ++order) {
        std::vector<Item> it = items;
        std::stable_sort(it.begin(), it.end(), [order](const Item& a, const Item& b) {
            const long long la = a.end - a.start + 1, lb = b.end - b.start + 1;
            switch (order) {
                case 0: return a.start != b.start ? a.start < b.start : a.cap > b.cap;
                case 1: return a.cap != b.cap ? a.cap > b.cap : a.start < b.start;
                case 2: return la != lb ? la > lb : a.cap > b.cap;
                default: {
                    const unsigned long long xa = a.cap * (unsigned long long)la, xb = b.cap * (unsigned long long)lb;
                    return xa != xb ? xa > xb : a.start < b.start;
                }
            }
        });
        unsigned long long extent = 0;
        for (size_t k = 0; k < it.size(); ++k) {
            std::vector<std::pair<long long, long long>> busy;   // ranges of the classes alive together with this one
            for (size_t m = 0; m < k; ++m)
                if (it[m].end >= it[k].start && it[m].start <= it[k].end)
                    busy.emplace_back(it[m].off, it[m].off + (long long)it[m].cap);
            std::sort(busy.begin(), busy.end());
            long long off = 0;
            for (const auto& b : busy) {
                if (off + (long long)it[k].cap <= b.first) break;
                off = std::max(off, b.second);
            }
            it[k].off = off;
            extent = std::max(extent, (unsigned long long)off + it[k].cap);
        }
        if (extent < best_extent) {
            best_extent = extent;
            for (const Item& x : it) cbase[(size_t)x.cid] = x.off;
        }
    }
    return items.empty() ? 0 : best_extent;
}

// T in exact size or in the paper's slots of M bytes.  Left to the library (option value 2), slots
// are kept when they would be at least 90 % full -- blocks of (nearly) one size, where the slot
// arithmetic is as dense as exact size and cheaper to address.  Otherwise both footprints are known
// from the validation pass: exact size is taken when it is not the larger one, or when it still fits
// into half of the device memory that is free (it is the faster layout: dense writes and reads);
// else the paper's slots.
bool choose_exact_t(int option, const PlanHost& pl, const Status& hs, unsigned long long exact_t_chunks) {
    if (option != 2) return option != 0;
    const double slot_bytes = (double)((hs.max_count + 127) / 128 * 128);
    if ((double)hs.total_bytes >= 0.9 * (double)pl.P * (double)pl.P * slot_bytes) return false;
    const double slots_t = (double)pl.P * (double)pl.slots * slot_bytes;
    const double exact_t = (double)exact_t_chunks * 16.0 + (double)pl.phases.size() * (double)pl.P * (double)pl.P * 4.0;
    if (exact_t <= slots_t) return true;
    size_t free_b = 0, total_b = 0;
    if (hipMemGetInfo(&free_b, &total_b) != hipSuccess) { (void)hipGetLastError(); return false; }
    return exact_t <= 0.5 * (double)free_b;
}

void fill_stats_header(const Prepared& pr, const Status& hs, tuna_stats_t& st) {
    const PlanHost& pl = pr.dp->host;
    std::memset(&st, 0, sizeof(st));
    st.P = pr.P; st.Q = pr.Q; st.N = pr.N; st.local_radix = pl.rl; st.global_radix = pl.rg;
    st.w_local = pl.w_l; st.w_global = pl.w_g; st.K_local = pl.K_l; st.K_global = pl.K_g;
    st.B_local = pl.B_l; st.B_global = pl.B_g; st.n_phases = (int)pl.phases.size();
    if (pr.staggered) st.K_global = pr.Q * (pr.N - 1);
    st.temp_slots_per_rank = pr.exact_t ? 0 : pl.slots;
    st.dense_t = pr.exact_kernels ? 1 : 0;
    st.fused = pr.fused ? 1 : 0;
    st.max_block_bytes = hs.max_count;
    st.total_payload_bytes = (int64_t)hs.total_bytes;
    st.granularity = pr.gran;
    for (size_t i = 0; i < pl.phases.size(); ++i) {
        const PhaseHost& ph = pl.phases[i];
        tuna_phase_stats_t& ps = st.phase[i];
        ps.dim = ph.dim; ps.x = ph.x; ps.radix = ph.r; ps.rounds = ph.nz;
        if (pr.staggered && ph.dim == 1) ps.rounds = pr.Q * (pr.N - 1);
        ps.blocks = (int64_t)ph.nseg * pr.P;
    }
}

// Problems beyond the kernels' 32-bit arithmetic.  Block sizes are rounded up to chunks and lines in
// int: the largest block must leave room for that.  Chunk prefixes are 32-bit per rank: what one rank
// stages in a phase is bounded both by all chunks there are and by P blocks of at most M bytes.
bool too_large(int P, const Status& hs) {
    if (hs.max_count > INT_MAX - 256) return true;
    const unsigned long long by_m = (unsigned long long)P * (unsigned long long)((hs.max_count + 15) / 16 + 1);
    const unsigned long long by_all = hs.total_chunks + (unsigned long long)P;
    return std::min(by_m, by_all) >= (1ull << 31);
}

constexpr int kTiledMinMeanBytes = 700;    // see prepare_sizes
constexpr int kTiledMinMeanBytesIntoT = 512;

// Validation + sizing pass of a call whose arguments, schedule and status buffers are in `pr` (one
// read-back).  On TUNA_OK with *empty == true there is nothing to move.
int prepare_sizes(Prepared& pr, int dense_option, hipStream_t s, Status& hs, bool* empty) {
    const int P = pr.P;
    const bool has_t = pr.dp->host.slots > 0;              // a schedule without T (r >= P - 1) has nothing to size
    int rc = run_validate(pr.sb, pr.sendcounts, pr.recvcounts, pr.sdispls, pr.rdispls, P, s,
                          (dense_option != 0 && has_t) ? pr.dp : nullptr);
    if (rc != TUNA_OK) return rc;
    hs = *pr.sb.h_status;
    if (pr.dp->built_on == s) pr.dp->complete = true;      // run_validate synchronised this stream
    if (hs.flags & 1u) return TUNA_ERR_NEGATIVE_COUNT;
    if (hs.flags & 2u) return TUNA_ERR_COUNT_MISMATCH;
    if (hs.flags & 4u) return TUNA_ERR_ARG;                 // a non-empty block at a negative displacement
    if (too_large(P, hs)) return TUNA_ERR_TOO_LARGE;
    if (dense_option != 0 && has_t)
        pr.t_chunks = colour_classes(pr.dp->host, pr.fused, pr.staggered, pr.block_count > 0, pr.sb.h_status->cls_chunks, pr.cbase);
    pr.exact_kernels = choose_exact_t(dense_option, pr.dp->host, hs, pr.t_chunks);
    pr.exact_t = pr.exact_kernels && has_t;
    *empty = hs.total_bytes == 0;
    if (*empty) return TUNA_OK;
    if (!pr.sendbuf || !pr.recvbuf) return TUNA_ERR_ARG;
    const unsigned int abits = hs.align_bits | (unsigned int)((uintptr_t)pr.sendbuf & 127u) |
                               (unsigned int)((uintptr_t)pr.recvbuf & 127u);
    pr.gran = (abits & 127u) == 0 ? 128 : ((abits & 15u) == 0 ? 16 : ((abits & 3u) == 0 ? 4 : 1));
    pr.max_count = hs.max_count;
    pr.total_bytes = hs.total_bytes;
    pr.user_limit = (unsigned long long)(uintptr_t)pr.sendbuf + hs.send_extent;
    // The destination-tiled hop: one-kernel phases over all rounds at once, receive regions dense (validation
    // flag), word- or chunk-granular data (whole-line data is as fast in the copy engine, byte-granular data
    // would need the pieces at block edges put together byte by byte), blocks that are not all tiny (those
    // have k_hop_small).
    // Into R it pays when the blocks are mostly pieces inside blocks, not edges: measured, 1 KiB blocks gain 8 %
    // per call at r = P and 512-byte blocks lose 2 %; Zipf sizes with four blocks in five under 256 bytes lose 11 %
    // in their last phase.  Hence, for a schedule's last phase (all its blocks are final), a mean block of at least
    // kTiledMinMeanBytes and at most a quarter of the blocks short.  Into T every block is whole chunks and
    // there are no edges: the phases before the last gain 6 to 10 % with those Zipf sizes and 2 to 4 % with a
    // mean block of 256 bytes, and lose 2 to 8 % below that: a mean block of kTiledMinMeanBytesIntoT.
    const unsigned long long P2 = (unsigned long long)P * (unsigned long long)P;
    pr.tiled = pr.fused && !pr.staggered && pr.block_count == 0 && !(hs.flags & 8u) && (pr.gran == 4 || pr.gran == 16) &&
               hs.max_count > kSmallBlockBytes && !pr.dp->host.phases.empty() &&
               hs.total_bytes >= (unsigned long long)kTiledMinMeanBytesIntoT * P2;
    pr.tiled_final = pr.tiled && hs.total_bytes >= (unsigned long long)kTiledMinMeanBytes * P2 && hs.short_blocks * 4 <= P2;
    pr.ds = data_sizes_for(pr.dp->host, hs.max_count, hs.total_chunks, pr.fused, pr.staggered, pr.exact_t, pr.t_chunks,
                           pr.tiled);
    return TUNA_OK;
}

// Argument checks, cached schedule, validation + sizing pass.
// One-kernel hops or the three stages.  Left to the library (TUNA_MODE_AUTO) it is the one-kernel hop:
// with every rank's buffers in one memory a hop needs no message, and moving a block straight from where
// its sender holds it to where its receiver keeps it reads and writes it once instead of three times
// (measured on every workload of the benchmark: 2.0 to 2.6 times faster per call, less memory).
bool mode_is_fused(const Options& o) { return o.mode != TUNA_MODE_STAGED; }

int prepare_call(Ctx& c, const Options& opt, const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls,
                 void* recvbuf, const int32_t* recvcounts, const int64_t* rdispls, int P, int ranks_per_node, int rl,
                 int rg, hipStream_t s, Prepared& pr, Status& hs, bool* empty) {
    int Q = 0;
    int rc = resolve_hierarchy(P, ranks_per_node, &Q);
    if (rc != TUNA_OK) return rc;
    if (rl < 2 || rg < 2) return TUNA_ERR_ARG;
    if (!sendcounts || !recvcounts || !sdispls || !rdispls) return TUNA_ERR_ARG;
    rc = ensure_ctx(c);
    if (rc != TUNA_OK) return rc;
    const int N = P / Q;
    pr.P = P; pr.Q = Q; pr.N = N;
    pr.sb = c.sb;
    pr.ctx = &c;
    pr.opt = opt;
    pr.fused = mode_is_fused(opt);
    // staggered inter-node schedule: one block per message, N - 1 node distances, straight from T
    pr.staggered = opt.staggered != 0 && N > 1;
    if (pr.staggered) rg = N;
    rc = get_plan(P, Q, rl, rg, pr.fused, s, &pr.dp);
    if (rc != TUNA_OK) return rc;
    pr.sendbuf = sendbuf; pr.recvbuf = recvbuf; pr.sendcounts = sendcounts; pr.recvcounts = recvcounts;
    pr.sdispls = sdispls; pr.rdispls = rdispls;
    pr.block_count = opt.block_count;
    return prepare_sizes(pr, opt.t_layout, s, hs, empty);
}

// One-kernel phases of problems whose blocks all fit into 64 bytes run k_hop_small (one thread per block)
// instead of the byte-balanced engine.
bool small_blocks(const Prepared& pr) { return pr.max_count > 0 && pr.max_count <= kSmallBlockBytes; }

// Phases that run as the destination-tiled hop: the last one (all its blocks are final) when the blocks are
// mostly interior, and with T in exact size the ones before it -- the blocks a rank stores into T lie back to
// back inside their class, so their destinations form runs just like those in R, and they are whole chunks.
// (T in slots keeps the copy engine: its slot tails are filled up to the line by a path of their own.)
bool phase_is_tiled(const Prepared& pr, size_t i) {
    return i + 1 == pr.dp->host.phases.size() ? pr.tiled_final : (pr.tiled && pr.exact_t);
}

// The last phase of a word-granular schedule as a tiled hop takes units of twice the size (k_copy_tiled<4, 8>):
// every block it writes has an edge piece, and what a wave spends on its edge pieces does not grow with the unit.
bool phase_has_wide_units(const Prepared& pr, size_t i) {
    return i + 1 == pr.dp->host.phases.size() && pr.tiled_final && pr.gran < 16;
}

// the receive-side layout of phase i with the unit size its payload kernel takes
LayoutDev layout_of_phase(const Prepared& pr, size_t i, const LayoutDev& Lr) {
    LayoutDev L = Lr;
    L.unit_chunks = phase_has_wide_units(pr, i) ? kWideUnitChunks : kUnitChunks;
    return L;
}

int launch_resolve(const Prepared& pr, size_t i, const int32_t* nxt, const HopDev& hop, hipStream_t s);

// The metadata of a phase that runs as the destination-tiled hop: the size exchange, the places in T of the
// blocks it stores there, every block's source and destination, then the layout of the 16-byte pieces of the
// destinations in place of the chunk scan.
int launch_tiled_metadata(const Prepared& pr, size_t i, const int32_t* cur, int32_t* nxt, const LayoutDev& Ls,
                          const LayoutDev& Lr_, const HopDev& hop, hipStream_t s) {
    const LayoutDev Lr = layout_of_phase(pr, i, Lr_);
    const PhaseHost& ph = pr.dp->host.phases[i];
    const int P = pr.P;
    const bool last = i + 1 == pr.dp->host.phases.size();
    if (!pr.sizes_direct) {
        hipLaunchKernelGGL(k_size_exchange, dim3((unsigned)((P + 255) / 256), (unsigned)((P + kExchangeRanks - 1) / kExchangeRanks)),
                           dim3(256), 0, s, cur, nxt, pr.dp->d_zt[i], P, pr.Q, pr.N, ph.dim, (int)ph.rx);
        HIPCHK(hipGetLastError());
    }
    if (!last) {
        // the blocks this phase stores into T: their places inside the classes (k_phase_layout's class scans,
        // which also count the phase's payload bytes) and the ranks' parts of the classes (k_layout_base)
        PhaseLayoutArgs m{};
        m.cur = cur; m.nxt = nxt; m.zt = pr.dp->d_zt[i]; m.seg = pr.dp->d_seg[i]; m.nseg = ph.nseg;
        m.P = P; m.Q = pr.Q; m.N = pr.N; m.dim = ph.dim; m.rx = (int)ph.rx;
        m.Ls = Ls; m.Lr = Lr; m.want_send = 0; m.want_tbound = 1; m.x = exact_t_of(pr, i);
        m.rank_bytes = pr.rank_bytes;
        m.phase_bytes = &pr.sb.d_status->phase_bytes[i]; m.phase_chunks = &pr.sb.d_status->phase_chunks[i];
        m.phase_units = pr.sb.d_status->phase_units[i];
        hipLaunchKernelGGL(k_phase_layout, dim3(P), dim3(kScanThreads), 0, s, m);
        HIPCHK(hipGetLastError());
        if (m.x.ncls > 0) {
            hipLaunchKernelGGL(k_layout_base, dim3(m.x.ncls), dim3(kScanThreads), 0, s, P, Lr, Ls, 0, m.phase_chunks, -1, m.x,
                               m.rank_bytes, m.phase_bytes, m.phase_units);
            HIPCHK(hipGetLastError());
        }
    }
    int rc = launch_resolve(pr, i, nxt, hop, s);
    if (rc != TUNA_OK) return rc;
    TiledLayoutArgs fa{};
    fa.hop = hop; fa.nseg = ph.nseg; fa.P = P; fa.Lr = Lr; fa.rank_bytes = last ? pr.rank_bytes : nullptr;
    hipLaunchKernelGGL(k_tiled_layout, dim3(P), dim3(kScanThreads), 0, s, fa);
    HIPCHK(hipGetLastError());
    hipLaunchKernelGGL(k_layout_base, dim3(1), dim3(kScanThreads), 0, s, P, Lr, Ls, 1, &pr.sb.d_status->phase_chunks[i], 0,
                       ExactT{}, pr.rank_bytes, &pr.sb.d_status->phase_bytes[i], pr.sb.d_status->phase_units[i]);
    HIPCHK(hipGetLastError());
    const int lds_ints = ph.nseg + 1 <= kUnitsLdsMaxInts ? ph.nseg + 1 : 0;
    hipLaunchKernelGGL(k_layout_units, dim3(P, 1), dim3(256), (size_t)lds_ints * 4, s, ph.nseg, Lr, Ls, lds_ints);
    HIPCHK(hipGetLastError());
    return TUNA_OK;
}

int launch_phase_metadata(const Prepared& pr, size_t i, const int32_t* cur, int32_t* nxt, const LayoutDev& Ls,
                          const LayoutDev& Lr, const HopDev& hop, hipStream_t s) {
    const PhaseHost& ph = pr.dp->host.phases[i];
    const bool one_kernel = phase_is_one_kernel(pr, ph);
    if (phase_is_tiled(pr, i)) return launch_tiled_metadata(pr, i, cur, nxt, Ls, Lr, hop, s);
    PhaseLayoutArgs m{};
    m.cur = cur; m.nxt = nxt; m.zt = pr.dp->d_zt[i]; m.seg = pr.dp->d_seg[i]; m.nseg = ph.nseg;
    m.P = pr.P; m.Q = pr.Q; m.N = pr.N; m.dim = ph.dim; m.rx = (int)ph.rx;
    m.Ls = Ls; m.Lr = Lr; m.want_send = one_kernel ? 0 : 1;
    if (pr.exact_t) { m.want_tbound = 1; m.x = exact_t_of(pr, i); }
    m.rank_bytes = pr.rank_bytes;
    m.phase_bytes = &pr.sb.d_status->phase_bytes[i]; m.phase_chunks = &pr.sb.d_status->phase_chunks[i];
    m.phase_units = pr.sb.d_status->phase_units[i];
    m.head_displs = one_kernel ? pr.rdispls : nullptr;
    m.head_base = (unsigned int)((uintptr_t)pr.recvbuf & 15u);
    // with few ranks a launch costs more than the kernel (measured: 19 us per call at P = 16, nothing at
    // P = 256, while at P = 4096 the separate kernel saves 44 us per phase): the scan kernel then
    // exchanges the sizes itself
    m.inline_exchange = (pr.P <= 128 && !pr.sizes_direct) ? 1 : 0;
    int rc = phase_metadata(m, s, exact_t_of(pr, i), pr.sizes_direct);
    if (rc != TUNA_OK || !one_kernel) return rc;
    return launch_resolve(pr, i, nxt, hop, s);
}

// one-kernel phase: where every block comes from and goes to, once per phase instead of once per wave
int launch_resolve(const Prepared& pr, size_t i, const int32_t* nxt, const HopDev& hop, hipStream_t s) {
    const PhaseHost& ph = pr.dp->host.phases[i];
    ResolveArgs ra{};
    ra.nxt = nxt; ra.seg = pr.dp->d_seg[i]; ra.nseg = ph.nseg;
    ra.P = pr.P; ra.Q = pr.Q; ra.N = pr.N; ra.dim = ph.dim; ra.rx = (int)ph.rx;
    ra.S = (const unsigned char*)pr.sendbuf; ra.sdispls = pr.sdispls;
    ra.R = (unsigned char*)pr.recvbuf; ra.rdispls = pr.rdispls;
    ra.slots = pr.ds.slots; ra.slot_bytes = pr.ds.slot_bytes;
    ra.x = exact_t_of(pr, i);
    ra.hop = hop;
    ra.exact_sizes = small_blocks(pr) ? 1 : 0;
    if (ph.nz >= kResolveTile) {     // many rounds: neighbouring segments come from neighbouring senders
        constexpr int per = 256 / kResolveTile;
        const dim3 grid((unsigned)((ph.nseg + per - 1) / per), (unsigned)((pr.P + kResolveTile - 1) / kResolveTile));
        if (pr.exact_kernels) hipLaunchKernelGGL((k_resolve_hop<true, kResolveTile>), grid, dim3(256), 0, s, ra);
        else hipLaunchKernelGGL((k_resolve_hop<false, kResolveTile>), grid, dim3(256), 0, s, ra);
    } else {
        const dim3 grid((unsigned)((ph.nseg + 255) / 256), (unsigned)pr.P);
        if (pr.exact_kernels) hipLaunchKernelGGL((k_resolve_hop<true, 1>), grid, dim3(256), 0, s, ra);
        else hipLaunchKernelGGL((k_resolve_hop<false, 1>), grid, dim3(256), 0, s, ra);
    }
    HIPCHK(hipGetLastError());
    return TUNA_OK;
}


// Resolved addresses of a one-kernel phase: row stride and bytes.
int hop_ld_for(int nseg) { return (nseg + 31) / 32 * 32; }
size_t hop_bytes_for(int P, int ld) { return 2 * align_up((size_t)P * ld * 8) + align_up((size_t)P * ld * 4); }
void carve_hop(Carver& cv, int P, int ld, HopDev& h) {
    h.ld = ld;
    h.src = cv.take<unsigned long long>((size_t)P * ld);
    h.dst = cv.take<unsigned long long>((size_t)P * ld);
    h.size = cv.take<int>((size_t)P * ld);
}
// largest row stride any one-kernel phase of the call needs (0: it has none)
int max_hop_ld(const Prepared& pr) {
    int ld = 0;
    for (const auto& ph : pr.dp->host.phases)
        if (phase_is_one_kernel(pr, ph)) ld = std::max(ld, hop_ld_for(ph.nseg));
    return ld;
}

// The block every rank keeps for itself (Section "Estimating temporary buffer size": one block is
// destined for the rank itself) goes straight from S to R.  Small blocks: one workgroup per rank.  When
// blocks can be large (M above 64 KiB) the own blocks are laid out as one more one-kernel phase and
// the byte-balanced copy engine moves them, so that a 1 GiB diagonal block is spread over the whole
// device like any other block.
constexpr int kSelfEngineMinM = 1 << 16;
bool self_uses_engine(const Prepared& pr) { return pr.max_count > kSelfEngineMinM; }
size_t self_unit_bound(const Prepared& pr) {
    // per rank at most ceil((15 + M + 15) / 16) chunks
    return (size_t)pr.P * (((size_t)pr.max_count / 16 + 2) / kUnitChunks + 1);
}
size_t self_meta_bytes(const Prepared& pr) {
    if (!self_uses_engine(pr)) return 0;
    const size_t P = (size_t)pr.P;
    return align_up(P * 2 * 4) + align_up(P * 4) + align_up((P + 1) * 8) + align_up((P + 1) * 4) + align_up(4) +
           align_up(self_unit_bound(pr) * sizeof(int4)) + 2 * align_up(P * 8) + align_up(P * 4);
}
void carve_self(Carver& cv, Prepared& pr) {
    pr.self_engine = self_uses_engine(pr);
    if (!pr.self_engine) return;
    const size_t P = (size_t)pr.P;
    LayoutDev& L = pr.selfL;
    L.ld = 2;
    L.pre = cv.take<int>(P * 2);
    L.tot = cv.take<int>(P);
    L.rank_base = cv.take<long long>(P + 1);
    L.unit_base = cv.take<int>(P + 1);
    L.n_units = cv.take<int>(1);
    L.unit_chunks = kUnitChunks;
    pr.self_units = self_unit_bound(pr);
    L.units = cv.take<int4>(pr.self_units);
    carve_hop(cv, pr.P, 1, pr.selfH);
}

// layout of the own blocks for the copy engine (nothing to do for the one-workgroup-per-rank form)
int launch_self_metadata(const Prepared& pr, hipStream_t s) {
    if (!pr.self_engine) return TUNA_OK;
    hipLaunchKernelGGL(k_self_layout, dim3((unsigned)((pr.P + 255) / 256)), dim3(256), 0, s,
                       (const unsigned char*)pr.sendbuf, pr.sendcounts, pr.sdispls, (unsigned char*)pr.recvbuf, pr.rdispls,
                       pr.P, pr.selfL, pr.selfH);
    HIPCHK(hipGetLastError());
    hipLaunchKernelGGL(k_layout_base, dim3(1), dim3(kScanThreads), 0, s, pr.P, pr.selfL, pr.selfL, 1,
                       (unsigned long long*)nullptr, -1, ExactT{}, (const unsigned long long*)nullptr,
                       (unsigned long long*)nullptr, &pr.sb.d_status->self_units);
    HIPCHK(hipGetLastError());
    hipLaunchKernelGGL(k_layout_units, dim3(pr.P, 1), dim3(256), 2 * sizeof(int), s, 1, pr.selfL, pr.selfL, 2);
    HIPCHK(hipGetLastError());
    return TUNA_OK;
}

int launch_self_copy(const Prepared& pr, hipStream_t s) {
    if (pr.self_engine) {
        CopyArgs a{};
        a.L = pr.selfL; a.hop = pr.selfH; a.nseg = 1; a.seg_lo = 0; a.seg_hi = 1;
        a.P = pr.P; a.Q = pr.Q; a.N = pr.N;
        a.user_limit = pr.user_limit;
        return launch_copy<kFused>(pr.gran, pr.self_units, a, s, pr.exact_kernels, 6);
    }
    hipLaunchKernelGGL(k_self_copy, dim3(pr.P, 1), dim3(256), 0, s, (const unsigned char*)pr.sendbuf,
                       pr.sendcounts, pr.sdispls, (unsigned char*)pr.recvbuf, pr.rdispls, pr.P);
    HIPCHK(hipGetLastError());
    return TUNA_OK;
}

// The payload kernels of digit phase i: pack, exchange, unpack -- or the one-kernel hop.
// unit_cap: number of wave units to launch for (an upper bound is fine).
int launch_phase_data(const Prepared& pr, size_t i, const LayoutDev& Ls, const LayoutDev& Lr, const HopDev& hop,
                      size_t unit_cap, hipStream_t s) {
    const PhaseHost& ph = pr.dp->host.phases[i];
    CopyArgs a{};
    a.seg = pr.dp->d_seg[i]; a.nseg = ph.nseg;
    a.T = pr.T; a.slots = pr.ds.slots; a.slot_bytes = pr.ds.slot_bytes;
    a.P = pr.P; a.Q = pr.Q; a.N = pr.N; a.dim = ph.dim; a.rx = (int)ph.rx;
    a.user_limit = pr.user_limit;
    a.x = exact_t_of(pr, i);
    // batches of rounds (Algorithm "Coalesced TuNA_l^g": block_count rounds are in flight at a time): the
    // rounds z0 .. z1-1 of a phase are the segments [below(z0), below(z1)) of every rank's message order
    const PhaseScalars ps = phase_scalars(ph);
    const long long mult = ph.dim == 0 ? pr.N : pr.Q;
    // Resident workgroups per compute unit of the three-stage kernels, measured on MI355X.  The kernels
    // keep many loads in flight per wave, and beyond some number of waves more of them only queue up in
    // the memory system.  Launches that move 2 GiB and more are fastest with 6 resident workgroups of 8
    // (blocks under 2 KiB: 2 to 4 % over 8 in pack, up to 7 % in the exchange, 10 % in unpack) or with 5
    // (larger blocks: another 3 to 8 %); short launches, where the ramp and the tail count, with 8 in pack
    // and 7 in the exchange and unpack.  Sizes are estimated from the mean block.  The one-kernel phases
    // hold 6 by their registers.
    const double mean_block = (double)pr.total_bytes / ((double)pr.P * (double)pr.P);
    const bool short_launch = mean_block * (double)ph.nseg * (double)pr.P < 2.0 * 1024 * 1024 * 1024;
    const int long_resident = mean_block < 2048.0 ? 6 : 5;
    const int pack_resident = short_launch ? 8 : long_resident;
    const int exchange_resident = short_launch ? 7 : long_resident;
    const int unpack_resident = short_launch ? 7 : long_resident;
    int per_batch = pr.block_count;                  // the staggered schedule counts single-block rounds: Q per node distance
    if (per_batch > 0 && pr.staggered && ph.dim == 1) per_batch = std::max(1, per_batch / pr.Q);
    const int step = (per_batch > 0 && per_batch < ph.nz) ? per_batch : ph.nz;
    for (int z0 = 1; z0 <= ph.nz; z0 += step) {
        const int z1 = std::min(z0 + step, ph.nz + 1);
        a.seg_lo = (int)(count_below_digit(ps, z0) * mult);
        a.seg_hi = (int)(count_below_digit(ps, z1) * mult);
        // a batch touches few units of every rank: at most its blocks times the chunks of the largest
        // block (one more per block when chunks are cut at destination lines), and the unit it starts
        // in.  One grid row per rank of that width, unless the whole unit list is shorter.
        size_t launch_units = unit_cap;
        a.batch_rows = 0;
        if (step < ph.nz) {
            const size_t cmax = (size_t)(pr.max_count + 15) / 16 + 1;
            const size_t row_units = ((size_t)(a.seg_hi - a.seg_lo) * cmax + kUnitChunks - 1) / kUnitChunks + 1;
            if (row_units * (size_t)pr.P < unit_cap) { launch_units = row_units; a.batch_rows = 1; }
        }
        int rc;
        if (phase_is_one_kernel(pr, ph) && small_blocks(pr)) {
            const dim3 grid((unsigned)((a.seg_hi - a.seg_lo + 255) / 256), (unsigned)pr.P);
            if (pr.gran >= 4) hipLaunchKernelGGL(k_hop_small<4>, grid, dim3(256), 0, s, hop, pr.T, a.seg_lo, a.seg_hi);
            else hipLaunchKernelGGL(k_hop_small<1>, grid, dim3(256), 0, s, hop, pr.T, a.seg_lo, a.seg_hi);
            HIPCHK(hipGetLastError());
            mark(pr.ctx, s, kCatPack, (int)i);
            continue;
        }
        if (phase_is_tiled(pr, i)) {
            // tiled over the 16-byte pieces of the destinations (k_copy_tiled); its time is reported as the
            // phase's unpack time, so that it can be told from the copy engine's one-kernel hops
            TiledCopyArgs fa{};
            fa.L = layout_of_phase(pr, i, Lr); fa.hop = hop; fa.nseg = ph.nseg; fa.T = pr.T; fa.user_limit = pr.user_limit;
            const dim3 grid((unsigned)((launch_units + kCopyThreads / kWave - 1) / (kCopyThreads / kWave)));
            if (grid.x) {
                const int resident = short_launch ? 8 : 7;
                if (pr.gran >= 16) {
                    static const size_t lds = static_lds_of(k_copy_tiled<16, kChunksPerLane>);
                    hipLaunchKernelGGL((k_copy_tiled<16, kChunksPerLane>), grid, dim3(kCopyThreads), occupancy_padding(resident, lds), s, fa);
                } else if (phase_has_wide_units(pr, i)) {
                    static const size_t lds = static_lds_of(k_copy_tiled<4, kWideChunksPerLane>);
                    hipLaunchKernelGGL((k_copy_tiled<4, kWideChunksPerLane>), grid, dim3(kCopyThreads), occupancy_padding(resident, lds), s, fa);
                } else {
                    static const size_t lds = static_lds_of(k_copy_tiled<4, kChunksPerLane>);
                    hipLaunchKernelGGL((k_copy_tiled<4, kChunksPerLane>), grid, dim3(kCopyThreads), occupancy_padding(resident, lds), s, fa);
                }
                HIPCHK(hipGetLastError());
            }
            mark(pr.ctx, s, kCatUnpack, (int)i);
            continue;
        }
        if (phase_is_one_kernel(pr, ph)) {
            // one hop in one kernel: S / T of the sender -> R / the other copy of T at the receiver
            a.stage = nullptr; a.L = Lr; a.hop = hop;
            // measured on the 16 GiB workload: a phase of many rounds gathers short pieces from many senders
            // and wants all the waves it can get (7 or 8 resident workgroups: 5.35 TB/s, 5 % less with 6); a
            // phase of few rounds streams long runs and is fastest with 6 (5.4 TB/s; 10 % less with 8)
            const int fused_resident = short_launch ? 8 : (ph.nz >= 32 ? 7 : 6);
            rc = launch_copy<kFused>(pr.gran, launch_units, a, s, pr.exact_kernels, fused_resident);
            if (rc != TUNA_OK) return rc;
            mark(pr.ctx, s, kCatPack, (int)i);
            continue;
        }
        // pack: S / T -> send staging
        a.stage = pr.stage_s; a.L = Ls; a.counts = nullptr;
        a.user = (unsigned char*)pr.sendbuf; a.displs = pr.sdispls;
        rc = launch_copy<kPack>(pr.gran, launch_units, a, s, pr.exact_kernels, pack_resident);
        if (rc != TUNA_OK) return rc;
        mark(pr.ctx, s, kCatPack, (int)i);
        // exchange: send staging of the partner -> receive staging
        a.stage = pr.stage_r; a.L = Lr; a.stage_src = pr.stage_s; a.Ls = Ls;
        rc = launch_copy<kExchange>(pr.gran, launch_units, a, s, pr.exact_kernels, exchange_resident);
        if (rc != TUNA_OK) return rc;
        mark(pr.ctx, s, kCatExchange, (int)i);
        // unpack: receive staging -> R / T
        a.counts = pr.recvcounts; a.user = (unsigned char*)pr.recvbuf; a.displs = pr.rdispls;
        rc = launch_copy<kUnpack>(pr.gran, launch_units, a, s, pr.exact_kernels, unpack_resident);
        if (rc != TUNA_OK) return rc;
        mark(pr.ctx, s, kCatUnpack, (int)i);
    }
    return TUNA_OK;
}

int run_two_pass(Ctx& c, const Prepared& prepared, hipStream_t s);
int run_pipelined(Ctx& c, const Prepared& prepared, hipStream_t s);
size_t plan_meta_bytes(const Prepared& pr);

// Immediate calls take the pipelined form (run_pipelined: one-kernel phases, not profiled) or the two-pass
// form (run_two_pass) from this many staged chunks on (64 MiB), when the schedule has at least two phases.
constexpr unsigned long long kTwoPassMinChunks = 1ull << 22;
bool use_two_pass(const PlanHost& pl, const Status& hs) {
    return pl.phases.size() >= 2 && hs.total_chunks >= kTwoPassMinChunks;
}

// Metadata bytes of a one-pass call: the two size matrices, one pair of layouts reused by every phase,
// the exact-size T tables and, for one-kernel phases, the resolved source, destination and size of every block.
size_t one_pass_meta_bytes(const Prepared& pr) {
    const int hld = max_hop_ld(pr);
    return meta_bytes_for(pr.P) + (pr.exact_t ? exact_t_meta_bytes_for(pr.dp->host, false) : 0) +
           (hld ? hop_bytes_for(pr.P, hld) : 0) + self_meta_bytes(pr);
}

// A call in one pass: rotation, the own blocks, then per digit phase its metadata kernels followed at
// once by its payload kernels, launched for an upper bound of work.  `mbase` holds one_pass_meta_bytes,
// `dbase` pr.ds.total bytes.
int run_one_pass(Prepared& pr, void* mbase, size_t mbytes, void* dbase, hipStream_t s, tuna_stats_t& st) {
    const PlanHost& pl = pr.dp->host;
    const DataSizes& ds = pr.ds;
    const int P = pr.P;
    Carver cm(mbase, mbytes);
    MetaBuffers mb = carve_meta(cm, P);
    pr.rank_bytes = mb.rank_bytes;
    if (pr.exact_t) carve_exact_t(cm, pl, false, pr);
    if (const int hld = max_hop_ld(pr)) carve_hop(cm, P, hld, pr.hop);
    carve_self(cm, pr);
    Carver cd(dbase, ds.total);
    mb.Ls.units = cd.take<int4>(ds.unit_cap);
    mb.Lr.units = cd.take<int4>(ds.unit_cap);
    pr.stage_s = cd.take<v4u>(pr.fused ? 0 : ds.stage_chunks);
    pr.stage_r = cd.take<v4u>(pr.fused ? 0 : ds.stage_chunks);
    pr.T = cd.take<unsigned char>(ds.t_bytes + kTailSlack);
    if (!cm.ok || !cd.ok) return TUNA_ERR_WORKSPACE_TOO_SMALL;
    int rc = upload_cbase(pr, s);
    if (rc != TUNA_OK) return rc;
    st.temp_bytes = (int64_t)ds.t_bytes;
    st.staging_bytes = pr.fused ? 0 : (int64_t)(2 * ds.stage_chunks * 16);
    st.workspace_bytes = (int64_t)(mbytes + ds.total);

    // ---- initial rotation (index only) and the own block ----------------------------------------
    const dim3 grot((unsigned)((P + 255) / 256), (unsigned)((P + kExchangeRanks - 1) / kExchangeRanks));
    // A schedule of one phase whose block sizes nobody asked to see: every block arrives in its only hop, so what
    // the phase's metadata exchange would leave in the receivers' size arrays is recvcounts, rotated (validation
    // has checked that it is the transpose of sendcounts): one kernel instead of the rotation and the exchange.
    pr.sizes_direct = pl.phases.size() == 1 && pr.fused && !pr.debug_sizes;
    if (pr.sizes_direct) hipLaunchKernelGGL(k_rotate_init, grot, dim3(256), 0, s, pr.recvcounts, mb.nxt, P, pr.Q, pr.N, 1);
    else hipLaunchKernelGGL(k_rotate_init, grot, dim3(256), 0, s, pr.sendcounts, mb.cur, P, pr.Q, pr.N, 0);
    HIPCHK(hipGetLastError());
    mark(pr.ctx, s, kCatPrepare, -1);
    rc = launch_self_metadata(pr, s);
    if (rc != TUNA_OK) return rc;
    rc = launch_self_copy(pr, s);
    if (rc != TUNA_OK) return rc;
    mark(pr.ctx, s, kCatSelf, -1);

    // ---- digit phases -----------------------------------------------------------------------------
    int32_t* cur = mb.cur;
    int32_t* nxt = mb.nxt;
    for (size_t i = 0; i < pl.phases.size(); ++i) {
        rc = launch_phase_metadata(pr, i, cur, nxt, mb.Ls, mb.Lr, pr.hop, s);
        if (rc != TUNA_OK) return rc;
        mark(pr.ctx, s, kCatMeta, (int)i);
        rc = launch_phase_data(pr, i, mb.Ls, mb.Lr, pr.hop, ds.unit_cap, s);
        if (rc != TUNA_OK) return rc;
        std::swap(cur, nxt);
    }
    return TUNA_OK;
}

int run_once(Ctx& c, const Options& opt, const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls,
             void* recvbuf, const int32_t* recvcounts, const int64_t* rdispls, int P, int ranks_per_node, int rl, int rg,
             void* stream);

// A whole call in one kernel launch (k_tiny_call) for problems of at most 64 ranks and 1 MiB of payload,
// where a call costs what its launches cost: about thirty launches and a synchronisation become one
// launch and a synchronisation.  Only when everything was left to the library (mode, no batches, no
// staggering, no profiling).  *done = false: the kernel declined (invalid counts, or not that small) and
// nothing has moved; the caller goes on with the general path.
constexpr size_t kTinyTBytes = 4u << 20;
int run_tiny(Ctx& c, const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls, void* recvbuf,
             const int32_t* recvcounts, const int64_t* rdispls, int P, int ranks_per_node, int rl, int rg,
             hipStream_t s, bool* done) {
    *done = false;
    int Q = 0;
    if (resolve_hierarchy(P, ranks_per_node, &Q) != TUNA_OK || rl < 2 || rg < 2) return TUNA_OK;   // the general path reports it
    if (!sendbuf || !recvbuf || !sendcounts || !recvcounts || !sdispls || !rdispls) return TUNA_OK;
    int rc = ensure_ctx(c);
    if (rc != TUNA_OK) return rc;
    DevicePlan* dp = nullptr;
    rc = get_plan(P, Q, rl, rg, /*fused=*/true, s, &dp);
    if (rc != TUNA_OK) return rc;
    const PlanHost& pl = dp->host;
    if ((int)pl.phases.size() > kTinyMaxPhases) return TUNA_OK;
    if (!c.tiny_t) {
        const hipError_t e = hipMalloc((void**)&c.tiny_t, kTinyTBytes);
        if (e != hipSuccess) { (void)hipGetLastError(); c.tiny_t = nullptr; return TUNA_OK; }
    }
    if (c.end_recorded && c.last_stream != s) HIPCHK(hipStreamWaitEvent(s, c.ev_end, 0));
    TinyArgs a{};
    a.S = (const unsigned char*)sendbuf; a.sendcounts = sendcounts; a.sdispls = sdispls;
    a.R = (unsigned char*)recvbuf; a.recvcounts = recvcounts; a.rdispls = rdispls;
    a.P = P; a.Q = Q; a.N = P / Q; a.nph = (int)pl.phases.size();
    for (int i = 0; i < a.nph; ++i) {
        const SegDev& sd = dp->d_seg[i];
        a.ph[i] = TinyPhase{sd.e, sd.z, sd.src, sd.dst, pl.phases[i].nseg, pl.phases[i].dim, (int)pl.phases[i].rx};
    }
    // the kernel writes its 64 bytes of status straight into the pinned host mirror: a copy command after it
    // would cost a fifth of the whole call
    a.T = c.tiny_t; a.slots = pl.slots; a.t_capacity = kTinyTBytes; a.st = c.sb.h_status_dev ? c.sb.h_status_dev : c.sb.d_status;
    c.sb.h_status->tiny_done = 0;
    // the kernel keeps the size and displacement matrices and every phase's tables in LDS: more than the
    // 64 KiB a kernel may use without asking
    int table_entries = 0;
    for (int i = 0; i < a.nph; ++i) table_entries += pl.phases[i].nseg;
    const size_t lds = tiny_lds_bytes(P, table_entries);
    static const hipError_t lds_allowed = hipFuncSetAttribute(reinterpret_cast<const void*>(k_tiny_call),
        hipFuncAttributeMaxDynamicSharedMemorySize, (int)tiny_lds_bytes(kTinyMaxRanks, kTinyMaxPhases * kTinyMaxRanks));
    if (lds_allowed != hipSuccess) { (void)hipGetLastError(); return TUNA_OK; }     // the general path does the call
    hipLaunchKernelGGL(k_tiny_call, dim3(1), dim3(kTinyThreads), lds, s, a);
    HIPCHK(hipGetLastError());
    if (!c.sb.h_status_dev) HIPCHK(hipMemcpyAsync(c.sb.h_status, c.sb.d_status, 64, hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));
    if (dp->built_on == s) dp->complete = true;
    const Status& hs = *c.sb.h_status;
    if (!hs.tiny_done) return TUNA_OK;
    // statistics: the schedule's numbers; nothing is timed
    Prepared pr;
    pr.P = P; pr.Q = Q; pr.N = P / Q; pr.dp = dp; pr.fused = true;
    const unsigned int abits = hs.align_bits | (unsigned int)((uintptr_t)sendbuf & 127u) | (unsigned int)((uintptr_t)recvbuf & 127u);
    pr.gran = (abits & 127u) == 0 ? 128 : ((abits & 15u) == 0 ? 16 : ((abits & 3u) == 0 ? 4 : 1));
    c.marks.clear();
    c.stats_plan = nullptr;
    fill_stats_header(pr, hs, c.stats);
    c.stats.temp_bytes = (int64_t)P * pl.slots * (((int64_t)hs.max_count + 15) / 16 * 16);
    c.stats.workspace_bytes = (int64_t)kTinyTBytes;
    c.end_recorded = false;
    c.last_stream = s;
    c.have_stats = true;
    *done = true;
    return TUNA_OK;
}

// An immediate call.  When the T layout was left to the library and exact-size T could not be
// allocated, the call is made again with the paper's slots before it gives up (nothing has moved yet).
int run(Ctx& c, const Options& opt, const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls,
        void* recvbuf, const int32_t* recvcounts, const int64_t* rdispls, int P, int ranks_per_node, int rl, int rg,
        void* stream) {
    if (P <= kTinyMaxRanks && opt.mode == TUNA_MODE_AUTO && opt.t_layout == TUNA_T_AUTO && !opt.staggered &&
        !opt.block_count && !opt.profile && !c.user_ws && c.tiny_declined != (const void*)sendcounts) {
        bool done = false;
        const int trc = run_tiny(c, sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P, ranks_per_node, rl, rg,
                                 (hipStream_t)stream, &done);
        if (trc != TUNA_OK || done) return trc;
        c.tiny_declined = sendcounts;
    }
    int rc = run_once(c, opt, sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P, ranks_per_node, rl, rg, stream);
    if (rc == TUNA_ERR_NOMEM && opt.t_layout == TUNA_T_AUTO && c.stats.dense_t) {
        Options o = opt;
        o.t_layout = TUNA_T_SLOTS;
        rc = run_once(c, o, sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P, ranks_per_node, rl, rg, stream);
    }
    return rc;
}

// An immediate call on context `c`.  Calls on one context share its workspace and status block: a call
// issued on another stream than the previous one first makes its stream wait for that call's end.
int run_once(Ctx& c, const Options& opt, const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls,
        void* recvbuf, const int32_t* recvcounts, const int64_t* rdispls, int P, int ranks_per_node, int rl, int rg,
        void* stream) {
    hipStream_t s = (hipStream_t)stream;
    if (c.ready && c.end_recorded && c.last_stream != s) HIPCHK(hipStreamWaitEvent(s, c.ev_end, 0));
    c.marks.clear();
    c.end_recorded = false;
    c.have_stats = false;
    c.stats_plan = nullptr;
    c.profile = opt.profile != 0;
    if (c.ready) mark(&c, s, -1, -1);
    Prepared pr;
    Status hs{};
    bool empty = false;
    int rc = prepare_call(c, opt, sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P, ranks_per_node, rl, rg,
                          s, pr, hs, &empty);
    if (rc != TUNA_OK) return rc;
    tuna_stats_t& st = c.stats;
    fill_stats_header(pr, hs, st);
    if (empty) { c.have_stats = true; return TUNA_OK; }
    const PlanHost& pl = pr.dp->host;
    if (use_two_pass(pl, hs) && pr.fused && !c.profile && !pr.debug_sizes) {
        rc = run_pipelined(c, pr, s);
    } else if (use_two_pass(pl, hs)) {
        rc = run_two_pass(c, pr, s);
    } else {
        // ---- workspace ---------------------------------------------------------------------------
        const size_t mbytes = one_pass_meta_bytes(pr);
        const DataSizes& ds = pr.ds;
        void *mbase, *dbase;
        if (c.user_ws) {
            if (mbytes + ds.total > c.user_ws_bytes) return TUNA_ERR_WORKSPACE_TOO_SMALL;
            mbase = c.user_ws;
            dbase = (char*)c.user_ws + mbytes;
        } else {
            rc = grow(&c.meta, &c.meta_bytes, mbytes);
            if (rc != TUNA_OK) return rc;
            rc = grow(&c.data, &c.data_bytes, ds.total);
            if (rc != TUNA_OK) return rc;
            mbase = c.meta;
            dbase = c.data;
        }
        rc = run_one_pass(pr, mbase, mbytes, dbase, s, st);
    }
    if (rc != TUNA_OK) return rc;
    HIPCHK(hipEventRecord(c.ev_end, s));
    c.end_recorded = true;
    c.last_stream = s;
    c.have_stats = true;
    return TUNA_OK;
}

// ---- persistent calls ------------------------------------------------------------------------------
// All metadata of a call (validation, sizing, every phase's size exchange, scans and unit lists) is
// computed once when the plan is made; starting it only launches the payload kernels.
struct Plan {
    Prepared pr;
    Ctx* ctx = nullptr;             // its statistics and profiling marks go here
    void* mem_meta = nullptr;       // cur / nxt and every phase's two layouts
    void* mem_data = nullptr;       // staging and T
    std::vector<LayoutDev> Ls, Lr;  // per phase
    std::vector<HopDev> hop;        // per phase (one-kernel phases only)
    std::vector<size_t> units;      // per phase: exact number of wave units (max of the two layouts)
    tuna_stats_t stats;
    unsigned long long phase_bytes[TUNA_MAX_PHASES];
    unsigned long long phase_chunks[TUNA_MAX_PHASES];
    bool empty = false;
};

size_t layout_bytes_for(int P, size_t unit_cap) {
    const size_t ld = (size_t)P + 1;
    return align_up((size_t)P * ld * 4) + align_up((size_t)P * 4) + align_up(((size_t)P + 1) * 8) +
           align_up(((size_t)P + 1) * 4) + align_up(4) + align_up(unit_cap * sizeof(int4));
}

void carve_full_layout(Carver& cv, int P, size_t unit_cap, LayoutDev& L) {
    carve_layout(cv, P, L);
    L.units = cv.take<int4>(unit_cap);
}

// Metadata memory of a plan: two size matrices, the per-rank byte sums, per phase two complete layouts.
size_t plan_meta_bytes(const Prepared& pr) {
    const PlanHost& pl = pr.dp->host;
    const size_t P2 = (size_t)pr.P * pr.P;
    size_t hop_bytes = 0;
    for (const auto& ph : pl.phases)
        if (phase_is_one_kernel(pr, ph)) hop_bytes += hop_bytes_for(pr.P, hop_ld_for(ph.nseg));
    return 2 * align_up(P2 * 4) + align_up((size_t)pr.P * 8) + pl.phases.size() * 2 * layout_bytes_for(pr.P, pr.ds.unit_cap) +
           (pr.exact_t ? exact_t_meta_bytes_for(pl, true) : 0) + hop_bytes + self_meta_bytes(pr);
}

// Every phase's metadata in `meta` (plan_meta_bytes of it), then one read-back: exact unit counts,
// per-phase bytes and chunks, and from them the payload memory the plan needs (*dbytes).
// with_marks: record the profiling marks of an immediate call.
// Carves a plan's metadata (plan_meta_bytes) out of `meta`: every phase gets layouts and hop arrays of its own.
bool plan_carve_meta(Plan* plan, void* meta, size_t mbytes, int32_t** cur, int32_t** nxt) {
    Prepared& pr = plan->pr;
    const PlanHost& pl = pr.dp->host;
    const size_t nph = pl.phases.size();
    const int P = pr.P;
    const size_t P2 = (size_t)P * P;
    Carver cm(meta, mbytes);
    *cur = cm.take<int32_t>(P2);
    *nxt = cm.take<int32_t>(P2);
    pr.rank_bytes = cm.take<unsigned long long>(P);
    plan->Ls.resize(nph); plan->Lr.resize(nph); plan->units.assign(nph, 0);
    for (size_t i = 0; i < nph; ++i) {
        carve_full_layout(cm, P, pr.ds.unit_cap, plan->Ls[i]);
        carve_full_layout(cm, P, pr.ds.unit_cap, plan->Lr[i]);
    }
    if (pr.exact_t) carve_exact_t(cm, pl, true, pr);
    plan->hop.assign(nph, HopDev{});
    for (size_t i = 0; i < nph; ++i)
        if (phase_is_one_kernel(pr, pl.phases[i])) carve_hop(cm, P, hop_ld_for(pl.phases[i].nseg), plan->hop[i]);
    carve_self(cm, pr);
    return cm.ok;
}

int plan_build_metadata(Plan* plan, void* meta, size_t mbytes, hipStream_t s, bool with_marks, size_t* stage_bytes,
                        size_t* dbytes) {
    Prepared& pr = plan->pr;
    const PlanHost& pl = pr.dp->host;
    const size_t nph = pl.phases.size();
    const int P = pr.P;
    const size_t P2 = (size_t)P * P;
    int32_t *cur = nullptr, *nxt = nullptr;
    if (!plan_carve_meta(plan, meta, mbytes, &cur, &nxt)) return TUNA_ERR_WORKSPACE_TOO_SMALL;
    int rc = upload_cbase(pr, s);
    if (rc != TUNA_OK) return rc;
    const dim3 grot((unsigned)((P + 255) / 256), (unsigned)((P + kExchangeRanks - 1) / kExchangeRanks));
    hipLaunchKernelGGL(k_rotate_init, grot, dim3(256), 0, s, pr.sendcounts, cur, P, pr.Q, pr.N, 0);
    HIPCHK(hipGetLastError());
    rc = launch_self_metadata(pr, s);
    if (rc != TUNA_OK) return rc;
    if (with_marks) mark(pr.ctx, s, kCatPrepare, -1);
    if (pr.debug_sizes) HIPCHK(hipMemcpyAsync(pr.debug_sizes, cur, P2 * 4, hipMemcpyDeviceToHost, s));
    for (size_t i = 0; i < nph; ++i) {
        rc = launch_phase_metadata(pr, i, cur, nxt, plan->Ls[i], plan->Lr[i], plan->hop[i], s);
        if (rc != TUNA_OK) return rc;
        if (with_marks) mark(pr.ctx, s, kCatMeta, (int)i);
        if (pr.debug_sizes) HIPCHK(hipMemcpyAsync(pr.debug_sizes + (i + 1) * P2, nxt, P2 * 4, hipMemcpyDeviceToHost, s));
        std::swap(cur, nxt);
    }
    // exact unit counts, bytes and staged chunks per phase: one read-back of the status block
    const Status* h_status = pr.sb.h_status;
    HIPCHK(hipMemcpyAsync(pr.sb.h_status, pr.sb.d_status, sizeof(Status), hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));
    unsigned long long max_chunks = 0;
    if (pr.self_engine) pr.self_units = h_status->self_units;     // exact from now on
    for (size_t i = 0; i < nph; ++i) {
        const bool one = phase_is_one_kernel(pr, pl.phases[i]);
        plan->units[i] = (size_t)std::max(h_status->phase_units[i][0], one ? 0u : h_status->phase_units[i][1]);
        plan->phase_bytes[i] = h_status->phase_bytes[i];
        plan->phase_chunks[i] = h_status->phase_chunks[i];
        plan->stats.phase[i].payload_bytes = (int64_t)plan->phase_bytes[i];
        plan->stats.phase[i].staged_bytes = (int64_t)plan->phase_chunks[i] * 16;
        if (!phase_is_one_kernel(pr, pl.phases[i])) max_chunks = std::max(max_chunks, plan->phase_chunks[i]);
    }
    // payload memory: staging sized by the largest phase; T by M and the slot count, or -- exact
    // size -- by the host's placement of the classes of waiting blocks (colour_classes)
    // (phase_chunks is the send side's total; the receive side holds the same blocks, but every rank's
    // region is rounded up to a line on its own, so its total may be up to one line per rank larger)
    *stage_bytes = max_chunks ? align_up(((size_t)max_chunks + (size_t)P * kRankAlignChunks) * 16) : 0;
    *dbytes = 2 * *stage_bytes + (pr.ds.t_bytes ? align_up(pr.ds.t_bytes + kTailSlack) : 0);
    plan->stats.temp_bytes = (int64_t)pr.ds.t_bytes;
    plan->stats.staging_bytes = (int64_t)(2 * *stage_bytes);
    plan->stats.workspace_bytes = (int64_t)(mbytes + *dbytes);
    return TUNA_OK;
}

void plan_carve_data(Plan* plan, void* data, size_t stage_bytes, size_t dbytes) {
    Prepared& pr = plan->pr;
    Carver cd(data, dbytes);
    pr.stage_s = cd.take<v4u>(stage_bytes / 16);
    pr.stage_r = cd.take<v4u>(stage_bytes / 16);
    pr.T = cd.take<unsigned char>(pr.ds.t_bytes ? pr.ds.t_bytes + kTailSlack : 0);
}

// The payload kernels of every phase, with exact grids.
int plan_launch_data(const Plan* plan, hipStream_t s) {
    const Prepared& pr = plan->pr;
    int rc = launch_self_copy(pr, s);
    if (rc != TUNA_OK) return rc;
    mark(pr.ctx, s, kCatSelf, -1);
    const size_t nph = pr.dp->host.phases.size();
    for (size_t i = 0; i < nph; ++i) {
        rc = launch_phase_data(pr, i, plan->Ls[i], plan->Lr[i], plan->hop[i], plan->units[i], s);
        if (rc != TUNA_OK) return rc;
    }
    return TUNA_OK;
}

int plan_create(Ctx& c, const Options& opt, const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls,
                void* recvbuf, const int32_t* recvcounts, const int64_t* rdispls, int P, int ranks_per_node, int rl, int rg,
                hipStream_t s, Plan** out, int32_t* debug_sizes = nullptr) {
    Plan* plan = new Plan();
    plan->ctx = &c;
    Prepared& pr = plan->pr;
    pr.debug_sizes = debug_sizes;
    Status hs{};
    c.profile = false;
    int rc = prepare_call(c, opt, sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P, ranks_per_node, rl, rg, s,
                          pr, hs, &plan->empty);
    if (rc != TUNA_OK) { delete plan; return rc; }
    fill_stats_header(pr, hs, plan->stats);
    if (plan->empty) { ++sh.live_plans; *out = plan; return TUNA_OK; }
    const size_t mbytes = plan_meta_bytes(pr);
    hipError_t e = hipMalloc(&plan->mem_meta, mbytes ? mbytes : kAlign);
    if (e != hipSuccess) { (void)hipGetLastError(); sh.last_hip_error = (int)e; delete plan; return TUNA_ERR_NOMEM; }
    auto fail = [&](int code) { (void)hipFree(plan->mem_meta); if (plan->mem_data) (void)hipFree(plan->mem_data); delete plan; return code; };
    size_t stage_bytes = 0, dbytes = 0;
    rc = plan_build_metadata(plan, plan->mem_meta, mbytes, s, /*with_marks=*/false, &stage_bytes, &dbytes);
    if (rc != TUNA_OK) return fail(rc == TUNA_ERR_WORKSPACE_TOO_SMALL ? TUNA_ERR_NOMEM : rc);
    if (dbytes) {
        e = hipMalloc(&plan->mem_data, dbytes);
        if (e != hipSuccess) { (void)hipGetLastError(); sh.last_hip_error = (int)e; return fail(TUNA_ERR_NOMEM); }
        plan_carve_data(plan, plan->mem_data, stage_bytes, dbytes);
    }
    ++sh.live_plans;
    *out = plan;
    return TUNA_OK;
}

// Starts of different plans share nothing but their context's statistics and profiling marks (the
// last start wins there); the plan's own memory holds everything its kernels touch.
int plan_start(Plan* plan, hipStream_t s) {
    Ctx& c = *plan->ctx;
    c.marks.clear();
    c.have_stats = false;
    c.stats = plan->stats;
    c.stats_plan = plan;
    c.profile = plan->pr.opt.profile != 0 || sh.defaults.profile != 0;
    if (plan->empty) { c.end_recorded = false; c.have_stats = true; return TUNA_OK; }
    mark(&c, s, -1, -1);
    mark(&c, s, kCatPrepare, -1);
    int rc = plan_launch_data(plan, s);
    if (rc != TUNA_OK) return rc;
    if (c.profile) {
        HIPCHK(hipEventRecord(c.ev_end, s));
        c.end_recorded = true;
        c.last_stream = s;
    }
    c.have_stats = true;
    return TUNA_OK;
}

// An immediate call in two passes: every phase's metadata first, one more read-back, then the
// payload kernels with exact grids and staging sized by the largest phase -- a transient plan in
// the library's (or the caller's) workspace.  Worth the second synchronisation when the payload
// is large and the schedule has several phases: the one-pass form launches every copy kernel for
// an upper bound of units, most of which are empty at small radices.
int run_two_pass(Ctx& c, const Prepared& prepared, hipStream_t s) {
    Plan plan;
    plan.pr = prepared;
    plan.ctx = &c;
    plan.stats = c.stats;
    const size_t mbytes = plan_meta_bytes(plan.pr);
    void* mbase = nullptr;
    int rc;
    if (c.user_ws) {
        if (mbytes > c.user_ws_bytes) return TUNA_ERR_WORKSPACE_TOO_SMALL;
        mbase = c.user_ws;
    } else {
        rc = grow(&c.meta, &c.meta_bytes, mbytes);
        if (rc != TUNA_OK) return rc;
        mbase = c.meta;
    }
    size_t stage_bytes = 0, dbytes = 0;
    rc = plan_build_metadata(&plan, mbase, mbytes, s, /*with_marks=*/true, &stage_bytes, &dbytes);
    if (rc != TUNA_OK) return rc;
    void* dbase = nullptr;
    if (c.user_ws) {
        if (mbytes + dbytes > c.user_ws_bytes) return TUNA_ERR_WORKSPACE_TOO_SMALL;
        dbase = (char*)c.user_ws + mbytes;
    } else if (dbytes) {
        rc = grow(&c.data, &c.data_bytes, dbytes);
        if (rc != TUNA_OK) return rc;
        dbase = c.data;
    }
    if (dbytes) plan_carve_data(&plan, dbase, stage_bytes, dbytes);
    c.stats = plan.stats;
    mark(&c, s, kCatPrepare, -1);                 // the read-back between the passes counts as preparation
    return plan_launch_data(&plan, s);
}

// A large call whose phases are all one-kernel hops, pipelined: the metadata kernels of every phase run back to
// back on a stream of the context's own (they depend on the block sizes only, never on the payload), the payload
// kernel of phase i runs on the caller's stream as soon as the metadata of phase i is complete (an event), with
// the grid of a one-pass call (an upper bound of units; the waves beyond the device's count leave at once).  The
// metadata of phase i + 1 is then computed while the payload of phase i moves, and the host waits for nothing
// after validation.  Every phase has metadata buffers of its own, as in a plan; T is sized from validation.
// Nothing a metadata kernel reads is written by a payload kernel, and a payload kernel reads only its own phase's
// buffers, S and T.  Not taken when the call is profiled (its per-kernel times are measured on one stream) or
// its size matrices are captured for verification.
int run_pipelined(Ctx& c, const Prepared& prepared, hipStream_t s) {
    Plan plan;
    plan.pr = prepared;
    plan.ctx = &c;
    Prepared& pr = plan.pr;
    const PlanHost& pl = pr.dp->host;
    const size_t nph = pl.phases.size();
    // the second stream and the events are made at the first such call; where the runtime refuses them the call
    // is made in two passes on the caller's stream instead
    bool have = true;
    if (!c.meta_stream && hipStreamCreateWithFlags(&c.meta_stream, hipStreamNonBlocking) != hipSuccess) { c.meta_stream = nullptr; have = false; }
    if (have && !c.ev_fork && hipEventCreateWithFlags(&c.ev_fork, hipEventDisableTiming) != hipSuccess) { c.ev_fork = nullptr; have = false; }
    while (have && c.ev_phase.size() < nph) {
        hipEvent_t e;
        if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) { have = false; break; }
        c.ev_phase.push_back(e);
    }
    if (!have) {
        (void)hipGetLastError();
        return run_two_pass(c, prepared, s);
    }
    const size_t mbytes = plan_meta_bytes(pr);
    const size_t dbytes = pr.ds.t_bytes ? align_up(pr.ds.t_bytes + kTailSlack) : 0;
    void *mbase = nullptr, *dbase = nullptr;
    int rc;
    if (c.user_ws) {
        if (mbytes + dbytes > c.user_ws_bytes) return TUNA_ERR_WORKSPACE_TOO_SMALL;
        mbase = c.user_ws;
        dbase = (char*)c.user_ws + mbytes;
    } else {
        rc = grow(&c.meta, &c.meta_bytes, mbytes);
        if (rc != TUNA_OK) return rc;
        if (dbytes) {
            rc = grow(&c.data, &c.data_bytes, dbytes);
            if (rc != TUNA_OK) return rc;
        }
        mbase = c.meta;
        dbase = c.data;
    }
    int32_t *cur = nullptr, *nxt = nullptr;
    if (!plan_carve_meta(&plan, mbase, mbytes, &cur, &nxt)) return TUNA_ERR_WORKSPACE_TOO_SMALL;
    if (dbytes) plan_carve_data(&plan, dbase, 0, dbytes);
    c.stats.temp_bytes = (int64_t)pr.ds.t_bytes;
    c.stats.staging_bytes = 0;
    c.stats.workspace_bytes = (int64_t)(mbytes + dbytes);
    hipStream_t m = c.meta_stream;
    // the metadata stream starts behind everything the caller's stream holds so far
    HIPCHK(hipEventRecord(c.ev_fork, s));
    HIPCHK(hipStreamWaitEvent(m, c.ev_fork, 0));
    rc = upload_cbase(pr, m);
    if (rc != TUNA_OK) return rc;
    const int P = pr.P;
    const dim3 grot((unsigned)((P + 255) / 256), (unsigned)((P + kExchangeRanks - 1) / kExchangeRanks));
    hipLaunchKernelGGL(k_rotate_init, grot, dim3(256), 0, m, pr.sendcounts, cur, P, pr.Q, pr.N, 0);
    HIPCHK(hipGetLastError());
    // the own blocks on the caller's stream, while the first phase's metadata is computed
    rc = launch_self_metadata(pr, s);
    if (rc != TUNA_OK) return rc;
    rc = launch_self_copy(pr, s);
    if (rc != TUNA_OK) return rc;
    for (size_t i = 0; i < nph; ++i) {
        rc = launch_phase_metadata(pr, i, cur, nxt, plan.Ls[i], plan.Lr[i], plan.hop[i], m);
        if (rc != TUNA_OK) break;
        HIPCHK(hipEventRecord(c.ev_phase[i], m));
        HIPCHK(hipStreamWaitEvent(s, c.ev_phase[i], 0));
        rc = launch_phase_data(pr, i, plan.Ls[i], plan.Lr[i], plan.hop[i], pr.ds.unit_cap, s);
        if (rc != TUNA_OK) break;
        std::swap(cur, nxt);
    }
    if (rc != TUNA_OK) {
        // whatever was launched on the metadata stream ends before the caller's stream goes on
        (void)hipEventRecord(c.ev_fork, m);
        (void)hipStreamWaitEvent(s, c.ev_fork, 0);
    }
    return rc;
}

}  // namespace
}  // namespace tuna

namespace tuna {
namespace {

// ---- the entry point that allocates nothing --------------------------------------------------------
// Same call as tuna_alltoallv_hier, one pass, with every buffer carved from the static device array
// `scratch`: no hipMalloc, no hipFree, no event or pinned-memory creation.  The schedule tables are
// rebuilt in scratch by every call (a few small kernels) instead of being cached in allocated memory.
constexpr int kMaxDevices = 64;
struct StaticState {
    unsigned char* ptr[kMaxDevices] = {};   // device address of `scratch` on each GPU (every GPU has its own copy)
    int num_cus[kMaxDevices] = {};
    Status h_status;                          // host mirror of the status block (pageable: no pinned allocation)
};
StaticState g_static;

int run_static(const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls, void* recvbuf,
               const int32_t* recvcounts, const int64_t* rdispls, int P, int ranks_per_node, int rl, int rg,
               hipStream_t s) {
    int Q = 0;
    int rc = resolve_hierarchy(P, ranks_per_node, &Q);
    if (rc != TUNA_OK) return rc;
    if (rl < 2 || rg < 2) return TUNA_ERR_ARG;
    if (!sendcounts || !recvcounts || !sdispls || !rdispls) return TUNA_ERR_ARG;
    const int N = P / Q;
    // set-up, once per device with that device current: the address of this GPU's copy of the array
    int dev = -1;
    HIPCHK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return TUNA_ERR_ARG;
    if (!g_static.ptr[dev]) {
        void* p = nullptr;
        HIPCHK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) { sh.last_hip_error = (int)hipErrorInvalidSymbol; return TUNA_ERR_HIP; }
        int cus = 0;
        HIPCHK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
        g_static.num_cus[dev] = cus > 0 ? cus : 256;
        g_static.ptr[dev] = (unsigned char*)p;
    }
    Carver cv(g_static.ptr[dev], (size_t)TUNA_NOALLOC_SCRATCH_BYTES);

    Prepared pr;
    pr.P = P; pr.Q = Q; pr.N = N;
    pr.sb.num_cus = g_static.num_cus[dev];
    pr.sb.d_status = cv.take<Status>(1);
    pr.sb.d_vpart = cv.take<unsigned long long>(vpart_words(pr.sb.num_cus));
    pr.sb.h_status = &g_static.h_status;
    pr.opt = sh.defaults;
    pr.opt.profile = 0;                       // no events are created here
    pr.fused = mode_is_fused(pr.opt);
    pr.staggered = pr.opt.staggered != 0 && N > 1;
    if (pr.staggered) rg = N;
    pr.block_count = pr.opt.block_count;
    pr.sendbuf = sendbuf; pr.recvbuf = recvbuf; pr.sendcounts = sendcounts; pr.recvcounts = recvcounts;
    pr.sdispls = sdispls; pr.rdispls = rdispls;

    // ---- the schedule, its tables in scratch (see get_plan for the cached form) ------------------------
    int crl, crg;
    clamp_radices(Q, N, rl, rg, &crl, &crg);
    DevicePlan dp;
    dp.host = make_plan(P, Q, crl, crg, pr.fused, /*with_tables=*/false);
    if ((int)dp.host.phases.size() > TUNA_MAX_PHASES) return TUNA_ERR_TOO_LARGE;
    dp.borrowed = true;                       // nothing of it is freed: it all lies in the static array
    std::vector<std::vector<int32_t>> tord;
    build_class_tables(dp.host, tord, dp.tcls);
    size_t table_bytes = align_up((size_t)P * 4) + align_up((size_t)P * 8);
    for (size_t i = 0; i < dp.host.phases.size(); ++i)
        table_bytes += 8 * align_up((size_t)dp.host.phases[i].nseg * 4) + align_up((size_t)P * 4) +
                       align_up(tord[i].size() * 4 + 4) + align_up(dp.tcls[i].size() * 4 + 4);
    if (cv.off + table_bytes > cv.cap) return TUNA_ERR_NOALLOC_LIMIT;     // before any kernel is launched
    for (size_t i = 0; i < dp.host.phases.size(); ++i) {
        const PhaseHost& ph = dp.host.phases[i];
        const size_t stride = align_up((size_t)ph.nseg * 4) / 4;
        int32_t* dm = cv.take<int32_t>(8 * stride);
        int32_t* dz = cv.take<int32_t>(P);
        hipLaunchKernelGGL(k_build_phase_table, dim3((unsigned)((P + 255) / 256)), dim3(256), 0, s, dp.host.sc,
                           phase_scalars(ph), dm, dm + stride, dm + 2 * stride, dm + 3 * stride, dm + 4 * stride,
                           dm + 5 * stride, dm + 6 * stride, dm + 7 * stride, dz);
        HIPCHK(hipGetLastError());
        dp.d_zt.push_back(dz);
        dp.d_seg.push_back(SegDev{dm, dm + stride, dm + 2 * stride, dm + 3 * stride, dm + 4 * stride, dm + 5 * stride,
                                  dm + 6 * stride, dm + 7 * stride});
        int32_t* d_o = cv.take<int32_t>(tord[i].size() + 1);
        int32_t* d_c = cv.take<int32_t>(dp.tcls[i].size() + 1);
        // pageable source: the copy has left the host arrays when the call returns
        if (!tord[i].empty()) HIPCHK(hipMemcpyAsync(d_o, tord[i].data(), tord[i].size() * 4, hipMemcpyHostToDevice, s));
        if (!dp.tcls[i].empty()) HIPCHK(hipMemcpyAsync(d_c, dp.tcls[i].data(), dp.tcls[i].size() * 4, hipMemcpyHostToDevice, s));
        dp.d_tord.push_back(d_o);
        dp.d_tcls.push_back(d_c);
    }
    dp.d_hm1 = cv.take<int32_t>(P);
    dp.d_mask = cv.take<unsigned long long>(P);
    hipLaunchKernelGGL(k_build_hops, dim3((unsigned)((P + 255) / 256)), dim3(256), 0, s, dp.host.sc, dp.d_hm1, dp.d_mask);
    HIPCHK(hipGetLastError());
    dp.built_on = s;
    pr.dp = &dp;

    // ---- validation and sizing (one read-back), then the one-pass call ---------------------------------
    Status hs{};
    bool empty = false;
    rc = prepare_sizes(pr, pr.opt.t_layout, s, hs, &empty);
    if (rc != TUNA_OK) return rc;
    // the statistics on file (header only: nothing here is timed) are the default context's
    g.marks.clear();
    g.end_recorded = false;
    g.stats_plan = nullptr;
    fill_stats_header(pr, hs, g.stats);
    g.have_stats = true;
    if (empty) return TUNA_OK;
    const size_t mbytes = one_pass_meta_bytes(pr);
    if (cv.off + mbytes + pr.ds.total > cv.cap) return TUNA_ERR_NOALLOC_LIMIT;
    char* mbase = cv.base + cv.off;
    return run_one_pass(pr, mbase, mbytes, mbase + mbytes, s, g.stats);
}

// ---- cost model of a call and its calibration ----------------------------------------------------------
// The paper chooses the radix from P and the block size because each of its K rounds pays a network
// latency (Section "Performance analysis of TuNA", "Radix selection").  In one HBM a round has no latency
// of its own; what a call costs is a fixed part, a part per digit phase (its launches), a part per entry
// of the P x P matrices (validation, rotation), the bytes its hops move and a part per moving block
// (metadata; the whole cost when blocks are tiny):
//     ms = c0 + c1 * phases + c2 * (phases + 1) * P^2 / 1e6 + c3 * hop bytes / 1e9 + c4 * moving blocks / 1e6
// with hop bytes = sum over phases of the payload bytes that move, moving blocks likewise.  One set of
// constants per mode (three-stage, one-kernel).  One-kernel phases of problems whose blocks all fit into
// 64 bytes run another kernel (k_hop_small, one thread per block), whose blocks and bytes are priced by
// constants of their own, c5 and c6, in place of c4 and c3.  The built-in constants were fitted to
// immediate calls on MI355X by tuna_calibrate; calling it replaces them by a fit to calls timed on the
// device at hand.
constexpr int kModelTerms = 7;
static_assert(kModelTerms + 3 == TUNA_MODEL_CONSTANTS, "tuna_model_constants reports the terms and the three factors");
struct Model {
    double c[kModelTerms];
};
struct ModelSet {
    Model m[2] = {{{0.0393, 0.0360, 0.0071, 1.0192, 0.0412, 0.0, 0.0}},            // [0] three stages
                  {{0.0368, 0.0312, 0.0061, 0.3481, 0.0398, 0.0150, 1.4108}}};    // [1] one-kernel hops
    // T in the paper's slots of M bytes: the bytes that pass through T cost more the emptier the slots are
    // (sparse writes and reads): their share of the byte term is scaled by 1 + k * (1 - mean / M)
    double slot_penalty[2] = {0.25, 0.45};
    // byte-granular problems (some count, displacement or buffer address is not a multiple of 4) run the
    // kernel variants that load and store single bytes at block edges: their byte term is scaled by this
    double byte_granular[2] = {1.15, 1.38};
    // line-granular problems (every count, displacement and buffer address is a multiple of 128) run the kernel
    // variants that read their sources with streaming loads, and no block shares a line with its neighbour:
    // their byte and block terms are scaled by this
    double line_granular[2] = {0.90, 0.79};
    bool calibrated = false;
};
ModelSet g_model;

struct Features {
    double phases, p2, hop_gb, mblocks, msmall, small_gb, t_share;    // t_share: share of the hop bytes that is written to or read from T
};

// small: the problem's one-kernel phases run k_hop_small (one-kernel mode and no block above 64 bytes)
Features features_of(const PlanHost& pl, double payload_bytes, bool small) {
    Features f{};
    const double P = (double)pl.P;
    f.phases = (double)pl.phases.size();
    f.p2 = (f.phases + 1.0) * P * P / 1e6;      // the passes over the P x P size matrix: one per phase, one for validation and rotation
    double moving = 0.0;
    for (const auto& ph : pl.phases) moving += (double)ph.nseg * P;
    (small ? f.msmall : f.mblocks) = moving / 1e6;
    // sizes are taken to be independent of the rank distance: every slot index carries payload / P^2
    (small ? f.small_gb : f.hop_gb) = P > 0 ? payload_bytes * (moving / (P * P)) / 1e9 : 0.0;
    // a block of h hops passes through T h - 1 times: it is written there h - 1 times and read h - 1 times,
    // of 2 h accesses in all
    const double hops = P > 0 ? moving / P : 0.0;                    // sum over slot indices of their hops
    const double through_t = hops - (P - 1.0);                       // sum of (h - 1) over the P - 1 moving indices
    f.t_share = hops > 0 ? (through_t > 0 ? through_t / hops : 0.0) : 0.0;
    return f;
}

double model_ms(const Model& m, const Features& f) {
    return m.c[0] + m.c[1] * f.phases + m.c[2] * f.p2 + m.c[3] * f.hop_gb + m.c[4] * f.mblocks + m.c[5] * f.msmall +
           m.c[6] * f.small_gb;
}

// the model's byte term
double bytes_ms(const Model& m, const Features& f) { return m.c[3] * f.hop_gb + m.c[6] * f.small_gb; }

// the model's byte and block terms: what depends on the payload
double data_ms(const Model& m, const Features& f) { return bytes_ms(m, f) + m.c[4] * f.mblocks + m.c[5] * f.msmall; }

bool small_block_path(bool fused, int64_t max_block) { return fused && max_block > 0 && max_block <= kSmallBlockBytes; }

double predict_ms(int P, int Q, int rl, int rg, bool fused, int t_layout, int64_t payload_bytes, int64_t max_block,
                  int granularity) {
    const PlanHost pl = make_plan(P, Q, rl, rg, false, /*with_tables=*/false);
    Features f = features_of(pl, (double)payload_bytes, small_block_path(fused, max_block));
    const Model& m = g_model.m[fused ? 1 : 0];
    double ms = model_ms(m, f);
    if (granularity > 0 && granularity < 4) ms += bytes_ms(m, f) * (g_model.byte_granular[fused ? 1 : 0] - 1.0);
    if (granularity >= 128) ms += data_ms(m, f) * (g_model.line_granular[fused ? 1 : 0] - 1.0);
    if (t_layout == TUNA_T_SLOTS && max_block > 0 && pl.slots > 0) {
        const double mean = (double)payload_bytes / ((double)P * (double)P);
        const double m128 = (double)((max_block + 127) / 128 * 128);
        const double empty = 1.0 - std::min(1.0, mean / m128);
        ms += bytes_ms(m, f) * f.t_share * g_model.slot_penalty[fused ? 1 : 0] * empty;
    }
    return ms;
}

// Least squares for the constants from timed calls, weighted for relative error; a constant that
// comes out negative is set to zero and the others are fitted again.  A term that no call exercises
// (the small-block term of the three-stage mode) is zero from the start.
bool fit_model(const std::vector<Features>& X, const std::vector<double>& y, Model* out) {
    constexpr int n = kModelTerms;
    bool fixed[n] = {};
    auto row_of = [](const Features& f, double* row) {
        row[0] = 1.0; row[1] = f.phases; row[2] = f.p2; row[3] = f.hop_gb; row[4] = f.mblocks; row[5] = f.msmall;
        row[6] = f.small_gb;
    };
    for (int i = 0; i < n; ++i) {
        bool used = false;
        for (const Features& f : X) { double row[n]; row_of(f, row); used = used || row[i] != 0.0; }
        fixed[i] = !used;
    }
    for (int round = 0; round < n; ++round) {
        double A[n][n + 1] = {};
        for (size_t k = 0; k < X.size(); ++k) {
            const double w = 1.0 / (y[k] * y[k]);
            double row[n];
            row_of(X[k], row);
            for (int i = 0; i < n; ++i) {
                if (fixed[i]) continue;
                for (int j = 0; j < n; ++j)
                    if (!fixed[j]) A[i][j] += w * row[i] * row[j];
                A[i][n] += w * row[i] * y[k];
            }
        }
        for (int i = 0; i < n; ++i)
            if (fixed[i]) A[i][i] = 1.0;              // x_i = 0
        // Gaussian elimination with partial pivoting
        int perm[n];
        for (int i = 0; i < n; ++i) perm[i] = i;
        for (int col = 0; col < n; ++col) {
            int piv = col;
            for (int r = col + 1; r < n; ++r)
                if (std::fabs(A[perm[r]][col]) > std::fabs(A[perm[piv]][col])) piv = r;
            std::swap(perm[col], perm[piv]);
            const double d = A[perm[col]][col];
            if (std::fabs(d) < 1e-300) return false;
            for (int r = col + 1; r < n; ++r) {
                const double fct = A[perm[r]][col] / d;
                for (int c2 = col; c2 <= n; ++c2) A[perm[r]][c2] -= fct * A[perm[col]][c2];
            }
        }
        double x[n];
        for (int i = n - 1; i >= 0; --i) {
            double v = A[perm[i]][n];
            for (int j = i + 1; j < n; ++j) v -= A[perm[i]][j] * x[j];
            x[i] = v / A[perm[i]][i];
        }
        int worst = -1;
        for (int i = 0; i < n; ++i)
            if (!fixed[i] && x[i] < 0 && (worst < 0 || x[i] < x[worst])) worst = i;
        if (worst < 0) {
            for (int i = 0; i < n; ++i) out->c[i] = fixed[i] ? 0.0 : x[i];
            return true;
        }
        fixed[worst] = true;
    }
    return false;
}

// Times immediate calls of dense problems with equal blocks (P x P blocks of S bytes) on a context of
// their own and fits the model to them.  Allocates the problems' buffers (up to about 2.3 GiB, plus
// the calls' workspaces) and frees them again; synchronises.
int calibrate(hipStream_t s) {
    int rc = ensure_device();
    if (rc != TUNA_OK) return rc;
    struct Problem { int P, S; int radices[3]; };
    // byte-granular: fitted after the others, as a factor on the byte term; large enough for that term to be
    // most of the call's time
    const Problem odd = {1024, 515, {2, 32, 1024}};
    // line-granular: fitted after the others too, as a factor on the byte and block terms
    const Problem lines = {2048, 256, {8, 2048, 0}};
    // tiny (fixed costs), many tiny blocks (per-block and per-entry costs), large blocks beyond the caches
    // (bytes), and a mix; S is 4 bytes off a multiple of 16, the usual alignment of float payloads
    const Problem problems[] = {{32, 68, {2, 6, 32}}, {256, 516, {2, 16, 256}}, {1024, 20, {2, 32, 1024}}, {2048, 36, {8, 2048, 0}},
                                {2048, 4, {2, 2048, 0}}, {1024, 60, {4, 1024, 0}},
                                {512, 4100, {2, 23, 512}}, {2048, 260, {8, 2048, 0}}};
    size_t max_entries = 0, max_bytes = 0;
    for (const Problem& pb : problems) {
        max_entries = std::max(max_entries, (size_t)pb.P * pb.P);
        max_bytes = std::max(max_bytes, (size_t)pb.P * pb.P * pb.S);
    }
    max_bytes = std::max(max_bytes, (size_t)odd.P * odd.P * odd.S);
    int32_t *sc = nullptr, *rc_ = nullptr;
    int64_t *sd = nullptr, *rd = nullptr;
    unsigned char *send = nullptr, *recv = nullptr;
    Ctx* c = new Ctx();
    auto cleanup = [&]() {
        (void)hipDeviceSynchronize();
        for (void* ptr : {(void*)sc, (void*)rc_, (void*)sd, (void*)rd, (void*)send, (void*)recv})
            if (ptr) (void)hipFree(ptr);
        free_ctx(*c);
        delete c;
    };
    auto alloc = [&](void** ptr, size_t bytes) {
        const hipError_t e = hipMalloc(ptr, bytes);
        if (e != hipSuccess) { (void)hipGetLastError(); sh.last_hip_error = (int)e; *ptr = nullptr; return false; }
        return true;
    };
    if (!alloc((void**)&sc, max_entries * 4) || !alloc((void**)&rc_, max_entries * 4) || !alloc((void**)&sd, max_entries * 8) ||
        !alloc((void**)&rd, max_entries * 8) || !alloc((void**)&send, max_bytes + 256) || !alloc((void**)&recv, max_bytes + 256)) {
        cleanup();
        return TUNA_ERR_NOMEM;
    }
    if (hipMemsetAsync(send, 0x5a, max_bytes + 256, s) != hipSuccess) { (void)hipGetLastError(); cleanup(); return TUNA_ERR_HIP; }
    std::vector<Features> X[2], Xo[2], Xl[2];
    std::vector<double> y[2], yo[2], yl[2];
    std::vector<Problem> all(std::begin(problems), std::end(problems));
    all.push_back(odd);
    all.push_back(lines);
    for (const Problem& pb : all) {
        const bool is_odd = (pb.S & 3) != 0, is_lines = (pb.S & 127) == 0;
        const size_t entries = (size_t)pb.P * pb.P;
        hipLaunchKernelGGL(k_fill_uniform, dim3((unsigned)((entries + 255) / 256)), dim3(256), 0, s, sc, sd, rc_, rd, pb.P, pb.S);
        if (hipGetLastError() != hipSuccess || hipStreamSynchronize(s) != hipSuccess) { cleanup(); return TUNA_ERR_HIP; }
        for (int r : pb.radices) {
            if (r < 2) continue;
            for (int fused = 0; fused < 2; ++fused) {
                Options o;
                o.mode = fused ? TUNA_MODE_FUSED : TUNA_MODE_STAGED;
                o.t_layout = TUNA_T_EXACT;
                constexpr int kReps = 6;
                double t[kReps];
                for (int it = 0; it < kReps; ++it) {     // the first call warms up (allocations, schedule tables)
                    const auto t0 = std::chrono::steady_clock::now();
                    rc = run(*c, o, send, sc, sd, recv, rc_, rd, pb.P, 0, r, r, s);
                    if (rc == TUNA_OK && hipStreamSynchronize(s) != hipSuccess) rc = TUNA_ERR_HIP;
                    if (rc != TUNA_OK) { cleanup(); return rc; }
                    t[it] = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
                }
                std::sort(t + 1, t + kReps);
                const PlanHost pl = make_plan(pb.P, pb.P, r, r, false, false);
                (is_odd ? Xo : is_lines ? Xl : X)[fused].push_back(features_of(pl, (double)entries * pb.S, small_block_path(fused != 0, pb.S)));
                (is_odd ? yo : is_lines ? yl : y)[fused].push_back(t[1 + (kReps - 1) / 2]);      // median of the timed calls
            }
        }
    }
    cleanup();
    ModelSet fitted = g_model;
    for (int fused = 0; fused < 2; ++fused) {
        if (!fit_model(X[fused], y[fused], &fitted.m[fused])) return TUNA_ERR_HIP;
        // the factor on the byte term that explains the byte-granular calls best (least squares)
        double num = 0.0, den = 0.0;
        for (size_t k = 0; k < Xo[fused].size(); ++k) {
            const double bms = bytes_ms(fitted.m[fused], Xo[fused][k]);
            const double rest = model_ms(fitted.m[fused], Xo[fused][k]) - bms;
            num += (yo[fused][k] - rest) * bms;
            den += bms * bms;
        }
        if (den > 0) fitted.byte_granular[fused] = std::max(1.0, num / den);
        // likewise the factor on the byte and block terms for the line-granular calls
        num = den = 0.0;
        for (size_t k = 0; k < Xl[fused].size(); ++k) {
            const double dms = data_ms(fitted.m[fused], Xl[fused][k]);
            const double rest = model_ms(fitted.m[fused], Xl[fused][k]) - dms;
            num += (yl[fused][k] - rest) * dms;
            den += dms * dms;
        }
        if (den > 0) fitted.line_granular[fused] = std::min(1.0, std::max(0.5, num / den));
    }
    fitted.calibrated = true;
    g_model = fitted;
    return TUNA_OK;
}

}  // namespace
}  // namespace tuna

using namespace tuna;

extern "C" {

// Options of a call: the caller's struct where given (checked), else the process-wide defaults.
static int options_from(const tuna_opts_t* o, Options* out) {
    *out = sh.defaults;
    if (!o) return TUNA_OK;
    if (o->struct_size != (int32_t)sizeof(tuna_opts_t)) return TUNA_ERR_ARG;
    if (o->mode < TUNA_MODE_AUTO || o->mode > TUNA_MODE_FUSED || o->t_layout < TUNA_T_SLOTS || o->t_layout > TUNA_T_AUTO ||
        o->block_count < 0)
        return TUNA_ERR_ARG;
    out->profile = o->profile ? 1 : 0; out->mode = o->mode; out->staggered = o->staggered ? 1 : 0;
    out->t_layout = o->t_layout; out->block_count = o->block_count;
    return TUNA_OK;
}

// The schedule queries describe the tables of the one-kernel hops (T in slots laid out twice) only when
// that mode was asked for by name; left to the library they describe the paper's single T.
static bool query_fused() { return sh.defaults.mode == TUNA_MODE_FUSED; }

static Ctx* ctx_of(tuna_ctx_t ctx) { return ctx ? reinterpret_cast<Ctx*>(ctx) : &g; }

// radix 0 = left to the library: the linear schedule in both dimensions (see tuna_select)
static int auto_radix(int radix, int P) { return radix == TUNA_RADIX_AUTO ? (P > 2 ? P : 2) : radix; }

int tuna_alltoallv(const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls, void* recvbuf,
                   const int32_t* recvcounts, const int64_t* rdispls, int P, int radix, int ranks_per_node,
                   void* stream) {
    radix = auto_radix(radix, P);
    if (radix < 2) return TUNA_ERR_ARG;
    return run(g, sh.defaults, sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P, ranks_per_node, radix,
               radix, stream);
}

int tuna_alltoallv_hier(const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls, void* recvbuf,
                        const int32_t* recvcounts, const int64_t* rdispls, int P, int ranks_per_node,
                        int local_radix, int global_radix, void* stream) {
    local_radix = auto_radix(local_radix, P); global_radix = auto_radix(global_radix, P);
    if (local_radix < 2 || global_radix < 2) return TUNA_ERR_ARG;
    return run(g, sh.defaults, sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P, ranks_per_node,
               local_radix, global_radix, stream);
}

int tuna_alltoallv_ex(tuna_ctx_t ctx, const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls,
                      void* recvbuf, const int32_t* recvcounts, const int64_t* rdispls, int P, int ranks_per_node,
                      int local_radix, int global_radix, const tuna_opts_t* opts, void* stream) {
    Options o;
    const int rc = options_from(opts, &o);
    if (rc != TUNA_OK) return rc;
    local_radix = auto_radix(local_radix, P); global_radix = auto_radix(global_radix, P);
    if (local_radix < 2 || global_radix < 2) return TUNA_ERR_ARG;
    return run(*ctx_of(ctx), o, sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P, ranks_per_node,
               local_radix, global_radix, stream);
}

int tuna_alltoallv_noalloc(const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls, void* recvbuf,
                           const int32_t* recvcounts, const int64_t* rdispls, int P, int ranks_per_node,
                           int local_radix, int global_radix, void* stream) {
    return run_static(sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P, ranks_per_node,
                      auto_radix(local_radix, P), auto_radix(global_radix, P), (hipStream_t)stream);
}

int tuna_alltoallv_init_ex(tuna_ctx_t ctx, const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls,
                           void* recvbuf, const int32_t* recvcounts, const int64_t* rdispls, int P, int ranks_per_node,
                           int local_radix, int global_radix, const tuna_opts_t* opts, void* stream, tuna_plan_t* plan) {
    if (!plan) return TUNA_ERR_ARG;
    *plan = nullptr;
    Options o;
    int rc = options_from(opts, &o);
    if (rc != TUNA_OK) return rc;
    local_radix = auto_radix(local_radix, P); global_radix = auto_radix(global_radix, P);
    if (local_radix < 2 || global_radix < 2) return TUNA_ERR_ARG;
    Plan* p = nullptr;
    rc = plan_create(*ctx_of(ctx), o, sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P, ranks_per_node,
                     local_radix, global_radix, (hipStream_t)stream, &p);
    if (rc == TUNA_ERR_NOMEM && o.t_layout == TUNA_T_AUTO) {     // exact-size T did not fit: the paper's slots may
        o.t_layout = TUNA_T_SLOTS;
        rc = plan_create(*ctx_of(ctx), o, sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P, ranks_per_node,
                         local_radix, global_radix, (hipStream_t)stream, &p);
    }
    if (rc == TUNA_OK) *plan = reinterpret_cast<tuna_plan_t>(p);
    return rc;
}

int tuna_alltoallv_init(const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls, void* recvbuf,
                        const int32_t* recvcounts, const int64_t* rdispls, int P, int ranks_per_node,
                        int local_radix, int global_radix, void* stream, tuna_plan_t* plan) {
    return tuna_alltoallv_init_ex(nullptr, sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P, ranks_per_node,
                                  local_radix, global_radix, nullptr, stream, plan);
}

int tuna_debug_phase_sizes(const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls, void* recvbuf,
                           const int32_t* recvcounts, const int64_t* rdispls, int P, int ranks_per_node,
                           int local_radix, int global_radix, void* stream, int32_t* sizes, int capacity_phases) {
    if (!sizes) return TUNA_ERR_ARG;
    tuna_plan_info_t info;
    int rc = tuna_plan_info(P, ranks_per_node, local_radix, global_radix, &info);
    if (rc != TUNA_OK) return rc;
    if (capacity_phases < info.n_phases + 1) return TUNA_ERR_ARG;
    Plan* p = nullptr;
    rc = plan_create(g, sh.defaults, sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P, ranks_per_node,
                     local_radix, global_radix, (hipStream_t)stream, &p, sizes);
    if (rc != TUNA_OK) return rc;
    return tuna_plan_free(reinterpret_cast<tuna_plan_t>(p));     // waits for the device: the copies have arrived
}

int tuna_start(tuna_plan_t plan, void* stream) {
    if (!plan) return TUNA_ERR_ARG;
    const int rc = ensure_device();        // the plan's memory lives on the library's device
    if (rc != TUNA_OK) return rc;
    return plan_start(reinterpret_cast<Plan*>(plan), (hipStream_t)stream);
}

int tuna_plan_free(tuna_plan_t plan) {
    if (!plan) return TUNA_OK;
    Plan* p = reinterpret_cast<Plan*>(plan);
    if (p->ctx && p->ctx->stats_plan == p) p->ctx->stats_plan = nullptr;
    // the plan goes away whatever the wait for the device says: its memory is released and the count of
    // live plans drops, then the error (if any) is reported
    const hipError_t e = hipDeviceSynchronize();
    if (p->mem_meta) (void)hipFree(p->mem_meta);
    if (p->mem_data) (void)hipFree(p->mem_data);
    delete p;
    --sh.live_plans;
    if (e != hipSuccess) { sh.last_hip_error = (int)e; return TUNA_ERR_HIP; }
    return TUNA_OK;
}

int tuna_ctx_create(tuna_ctx_t* ctx) {
    if (!ctx) return TUNA_ERR_ARG;
    *ctx = nullptr;
    Ctx* c = new Ctx();
    const int rc = ensure_ctx(*c);
    if (rc != TUNA_OK) { free_ctx(*c); delete c; return rc; }
    ++sh.live_contexts;
    *ctx = reinterpret_cast<tuna_ctx_t>(c);
    return TUNA_OK;
}

int tuna_ctx_destroy(tuna_ctx_t ctx) {
    if (!ctx) return TUNA_OK;
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    const hipError_t e = hipDeviceSynchronize();
    free_ctx(*c);
    delete c;
    --sh.live_contexts;
    if (e != hipSuccess) { sh.last_hip_error = (int)e; return TUNA_ERR_HIP; }
    return TUNA_OK;
}

int tuna_opts_init(tuna_opts_t* opts) {
    if (!opts) return TUNA_ERR_ARG;
    std::memset(opts, 0, sizeof(*opts));
    opts->struct_size = (int32_t)sizeof(tuna_opts_t);
    opts->mode = sh.defaults.mode; opts->staggered = sh.defaults.staggered; opts->t_layout = sh.defaults.t_layout;
    opts->block_count = sh.defaults.block_count; opts->profile = sh.defaults.profile;
    return TUNA_OK;
}

int tuna_workspace_bytes(const int32_t* sendcounts, int P, int ranks_per_node, int local_radix, int global_radix,
                         size_t* bytes) {
    if (!bytes || !sendcounts || local_radix < 2 || global_radix < 2) return TUNA_ERR_ARG;
    int Q = 0;
    int rc = resolve_hierarchy(P, ranks_per_node, &Q);
    if (rc != TUNA_OK) return rc;
    rc = ensure_ctx(g);
    if (rc != TUNA_OK) return rc;
    const int N = P / Q;
    const Options& o = sh.defaults;
    const bool fused = mode_is_fused(o);
    const bool staggered = o.staggered != 0 && N > 1;
    DevicePlan* dp = nullptr;
    rc = get_plan(P, Q, local_radix, staggered ? N : global_radix, fused, nullptr, &dp);
    if (rc != TUNA_OK) return rc;
    const PlanHost& pl = dp->host;
    rc = run_validate(g.sb, sendcounts, nullptr, nullptr, nullptr, P, nullptr, (o.t_layout != 0 && pl.slots > 0) ? dp : nullptr);
    if (rc != TUNA_OK) return rc;
    const Status* h_status = g.sb.h_status;
    std::vector<long long> cbase;
    const unsigned long long t_chunks = (o.t_layout != 0 && pl.slots > 0)
        ? colour_classes(pl, fused, staggered, o.block_count > 0, h_status->cls_chunks, cbase) : 0;
    const bool exact_t = choose_exact_t(o.t_layout, pl, *h_status, t_chunks) && pl.slots > 0;
    dp->complete = true;                                  // run_validate synchronised the stream the tables were built on
    if (h_status->flags & 1u) return TUNA_ERR_NEGATIVE_COUNT;
    if (too_large(P, *h_status)) return TUNA_ERR_TOO_LARGE;
    const DataSizes ds = data_sizes_for(pl, h_status->max_count, h_status->total_chunks, fused, staggered,
                                        exact_t, t_chunks, fused && !staggered && o.block_count == 0);
    Prepared pr;
    pr.P = P; pr.Q = Q; pr.N = N; pr.dp = dp; pr.ds = ds; pr.exact_t = exact_t;
    pr.fused = fused; pr.staggered = staggered; pr.max_count = h_status->max_count;
    *bytes = one_pass_meta_bytes(pr) + ds.total;
    if (use_two_pass(pl, *h_status)) {
        // the two-pass form keeps every phase's layouts; its staging is at most the one-pass form's
        *bytes = plan_meta_bytes(pr) + (pr.fused ? 0 : 2 * align_up(ds.stage_chunks * 16)) +
                 (ds.t_bytes ? align_up(ds.t_bytes + kTailSlack) : 0);
    }
    return TUNA_OK;
}

int tuna_plain_copy(const void* src, void* dst, size_t bytes, void* stream) {
    if (!src || !dst || (bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return TUNA_ERR_ARG;
    int rc = ensure_device();
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
    if (!sh.ready) return TUNA_OK;
    if (sh.live_plans > 0) return TUNA_ERR_ARG;      // persistent plans use the cached schedules
    HIPCHK(hipDeviceSynchronize());
    if (g.meta) { HIPCHK(hipFree(g.meta)); g.meta = nullptr; g.meta_bytes = 0; }
    if (g.data) { HIPCHK(hipFree(g.data)); g.data = nullptr; g.data_bytes = 0; }
    for (auto& kv : sh.plans) free_device_plan(kv.second);
    sh.plans.clear();
    return TUNA_OK;
}

int tuna_set_option(int option, int value) {
    Options& d = sh.defaults;
    if (option == TUNA_OPT_PROFILE) { d.profile = value ? 1 : 0; return TUNA_OK; }
    if (option == TUNA_OPT_FUSED) {      // 0: three stages, 1: one-kernel hops, 2: left to the library
        if (value < 0 || value > 2) return TUNA_ERR_ARG;
        d.mode = value == 0 ? TUNA_MODE_STAGED : (value == 1 ? TUNA_MODE_FUSED : TUNA_MODE_AUTO);
        return TUNA_OK;
    }
    if (option == TUNA_OPT_STAGGERED) { d.staggered = value ? 1 : 0; return TUNA_OK; }
    if (option == TUNA_OPT_DENSE_T) { if (value < 0 || value > 2) return TUNA_ERR_ARG; d.t_layout = value; return TUNA_OK; }
    if (option == TUNA_OPT_BLOCK_COUNT) { if (value < 0) return TUNA_ERR_ARG; d.block_count = value; return TUNA_OK; }
    return TUNA_ERR_ARG;
}

int tuna_get_stats(tuna_stats_t* out) { return tuna_ctx_get_stats(nullptr, out); }

int tuna_ctx_get_stats(tuna_ctx_t ctx, tuna_stats_t* out) {
    Ctx& g = *ctx_of(ctx);               // the context whose statistics are asked for
    if (!out) return TUNA_ERR_ARG;
    if (!g.have_stats) { std::memset(out, 0, sizeof(*out)); out->last_hip_error = sh.last_hip_error; return TUNA_OK; }
    tuna_stats_t& st = g.stats;
    if (g.end_recorded) {
        HIPCHK(hipEventSynchronize(g.ev_end));
        if (!g.stats_plan) {   // a persistent plan knows its per-phase bytes since it was made
            HIPCHK(hipMemcpy(g.sb.h_status, g.sb.d_status, sizeof(Status), hipMemcpyDeviceToHost));
            for (int i = 0; i < st.n_phases; ++i) {
                st.phase[i].payload_bytes = (int64_t)g.sb.h_status->phase_bytes[i];
                st.phase[i].staged_bytes = (int64_t)g.sb.h_status->phase_chunks[i] * 16;
            }
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
    out->last_hip_error = sh.last_hip_error;
    return TUNA_OK;
}

int tuna_plan_info(int P, int ranks_per_node, int local_radix, int global_radix, tuna_plan_info_t* out) {
    if (!out || local_radix < 2 || global_radix < 2) return TUNA_ERR_ARG;
    int Q = 0;
    int rc = resolve_hierarchy(P, ranks_per_node, &Q);
    if (rc != TUNA_OK) return rc;
    if (sh.defaults.staggered && P / Q > 1) global_radix = P / Q;
    const PlanHost pl = make_plan(P, Q, local_radix, global_radix, query_fused(), /*with_tables=*/false);
    out->P = P; out->Q = Q; out->N = pl.N;
    out->local_radix = pl.rl; out->global_radix = pl.rg;
    out->w_local = pl.w_l; out->w_global = pl.w_g;
    out->K_local = pl.K_l; out->K_global = (sh.defaults.staggered && pl.N > 1) ? Q * (pl.N - 1) : pl.K_g;
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
    const PlanHost pl = make_plan(P, Q, local_radix, global_radix, query_fused());
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

int tuna_plan_phase_device(int P, int ranks_per_node, int local_radix, int global_radix, int phase, int32_t* seg,
                           int seg_capacity) {
    if (!seg || local_radix < 2 || global_radix < 2 || phase < 0 || seg_capacity < 0) return TUNA_ERR_ARG;
    int Q = 0;
    int rc = resolve_hierarchy(P, ranks_per_node, &Q);
    if (rc != TUNA_OK) return rc;
    rc = ensure_device();
    if (rc != TUNA_OK) return rc;
    if (sh.defaults.staggered && P / Q > 1) global_radix = P / Q;
    DevicePlan* dp = nullptr;
    rc = get_plan(P, Q, local_radix, global_radix, query_fused(), nullptr, &dp);
    if (rc != TUNA_OK) return rc;
    if (phase >= (int)dp->host.phases.size()) return TUNA_ERR_ARG;
    HIPCHK(hipDeviceSynchronize());
    dp->complete = true;
    const int nseg = dp->host.phases[phase].nseg;
    const int n = seg_capacity < nseg ? seg_capacity : nseg;
    std::vector<int32_t> f((size_t)n);
    const int32_t* src[4] = {dp->d_seg[phase].e, dp->d_seg[phase].z, dp->d_seg[phase].src, dp->d_seg[phase].dst};
    for (int c = 0; c < 4; ++c) {
        if (n) HIPCHK(hipMemcpy(f.data(), src[c], (size_t)n * 4, hipMemcpyDeviceToHost));
        for (int k = 0; k < n; ++k) seg[(size_t)k * 4 + c] = f[k];
    }
    return TUNA_OK;
}

int tuna_plan_phase_sources(int P, int ranks_per_node, int local_radix, int global_radix, int phase,
                            int on_device, int32_t* out, int capacity) {
    if (!out || local_radix < 2 || global_radix < 2 || phase < 0 || capacity < 0) return TUNA_ERR_ARG;
    int Q = 0;
    int rc = resolve_hierarchy(P, ranks_per_node, &Q);
    if (rc != TUNA_OK) return rc;
    if (!on_device) {
        const PlanHost pl = make_plan(P, Q, local_radix, global_radix, query_fused());
        if (phase >= (int)pl.phases.size()) return TUNA_ERR_ARG;
        const PhaseHost& ph = pl.phases[phase];
        const int n = capacity < ph.nseg ? capacity : ph.nseg;
        for (int k = 0; k < n; ++k) { out[2 * k] = ph.seg[k].src_phase; out[2 * k + 1] = ph.seg[k].src_seg; }
        return TUNA_OK;
    }
    rc = ensure_device();
    if (rc != TUNA_OK) return rc;
    if (sh.defaults.staggered && P / Q > 1) global_radix = P / Q;
    DevicePlan* dp = nullptr;
    rc = get_plan(P, Q, local_radix, global_radix, query_fused(), nullptr, &dp);
    if (rc != TUNA_OK) return rc;
    if (phase >= (int)dp->host.phases.size()) return TUNA_ERR_ARG;
    HIPCHK(hipDeviceSynchronize());
    dp->complete = true;
    const int nseg = dp->host.phases[phase].nseg;
    const int n = capacity < nseg ? capacity : nseg;
    std::vector<int32_t> f((size_t)n);
    const int32_t* src[2] = {dp->d_seg[phase].srcph, dp->d_seg[phase].srcseg};
    for (int c = 0; c < 2; ++c) {
        if (n) HIPCHK(hipMemcpy(f.data(), src[c], (size_t)n * 4, hipMemcpyDeviceToHost));
        for (int k = 0; k < n; ++k) out[(size_t)k * 2 + c] = f[k];
    }
    return TUNA_OK;
}

int tuna_predict_ms(int P, int ranks_per_node, int local_radix, int global_radix, int mode, int t_layout,
                    int64_t payload_bytes, int64_t max_block_bytes, int granularity, double* ms) {
    if (!ms || payload_bytes < 0 || max_block_bytes < 0 || granularity < 0 || mode < TUNA_MODE_AUTO || mode > TUNA_MODE_FUSED ||
        t_layout < TUNA_T_SLOTS || t_layout > TUNA_T_AUTO)
        return TUNA_ERR_ARG;
    int Q = 0;
    const int rc = resolve_hierarchy(P, ranks_per_node, &Q);
    if (rc != TUNA_OK) return rc;
    local_radix = auto_radix(local_radix, P); global_radix = auto_radix(global_radix, P);
    if (local_radix < 2 || global_radix < 2) return TUNA_ERR_ARG;
    *ms = predict_ms(P, Q, local_radix, global_radix, mode != TUNA_MODE_STAGED, t_layout, payload_bytes, max_block_bytes,
                     granularity);
    return TUNA_OK;
}

int tuna_select(int P, int ranks_per_node, int64_t payload_bytes, int64_t max_block_bytes, int granularity,
                tuna_choice_t* out) {
    if (!out || payload_bytes < 0 || max_block_bytes < 0 || granularity < 0) return TUNA_ERR_ARG;
    int Q = 0;
    const int rc = resolve_hierarchy(P, ranks_per_node, &Q);
    if (rc != TUNA_OK) return rc;
    const int N = P / Q;
    auto candidates = [](int size) {
        std::vector<int> c;
        if (size < 2) { c.push_back(2); return c; }
        for (long long r = 2; r < size; r *= 2) c.push_back((int)r);
        int sq = 2;
        while ((long long)sq * sq < size) ++sq;
        c.push_back(sq);
        c.push_back(size);
        return c;
    };
    std::memset(out, 0, sizeof(*out));
    double best = -1.0;
    for (int rl : candidates(Q))
        for (int rg : candidates(N))
            for (int fused = 1; fused >= 0; --fused)
                for (int tl = TUNA_T_EXACT; tl >= TUNA_T_SLOTS; --tl) {
                    const double t = predict_ms(P, Q, rl, rg, fused != 0, tl, payload_bytes, max_block_bytes, granularity);
                    if (best < 0 || t < best * (1.0 - 1e-9)) {
                        best = t;
                        out->local_radix = rl; out->global_radix = rg;
                        out->mode = fused ? TUNA_MODE_FUSED : TUNA_MODE_STAGED; out->t_layout = tl;
                    }
                }
    out->predicted_ms = best;
    out->calibrated = g_model.calibrated ? 1 : 0;
    return TUNA_OK;
}

int tuna_calibrate(void* stream) { return calibrate((hipStream_t)stream); }

int tuna_model_constants(int mode, double* c, int capacity) {
    if (!c || capacity < TUNA_MODEL_CONSTANTS || (mode != TUNA_MODE_STAGED && mode != TUNA_MODE_FUSED)) return TUNA_ERR_ARG;
    const int k = mode == TUNA_MODE_FUSED ? 1 : 0;
    for (int i = 0; i < kModelTerms; ++i) c[i] = g_model.m[k].c[i];
    c[kModelTerms] = g_model.slot_penalty[k];
    c[kModelTerms + 1] = g_model.byte_granular[k];
    c[kModelTerms + 2] = g_model.line_granular[k];
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
        case TUNA_ERR_NOALLOC_LIMIT: return "problem needs more than the static scratch of tuna_alltoallv_noalloc";
        default: return "unknown error";
    }
}

int tuna_version(void) { return kVersion; }

#ifndef TUNA_BUILD_ID
#define TUNA_BUILD_ID "unknown"
#endif
// the prefix lets the build id be read from the library file without loading it
static const char kBuildId[] = "tuna-build-id:" TUNA_BUILD_ID;
const char* tuna_build_id(void) { return kBuildId + sizeof("tuna-build-id:") - 1; }

}  // extern "C"
