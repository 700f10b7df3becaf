/*
 * tuna.h -- C ABI of the MI355X (gfx950) tunable-radix non-uniform all-to-all library.
 *
 * The library runs TuNA (Section "Tunable-radix Non-uniform All-to-all", Algorithm "TuNA") and
 * its hierarchical coalesced variant TuNA_l^g (Section "Hierarchical Tunable Non-uniform
 * All-to-all", Algorithm "Coalesced TuNA_l^g") for P *virtual ranks* whose send and receive
 * buffers all live in one GPU's memory.  Every digit phase is device work: metadata (block
 * size) exchange, size/displacement scan, and the move of the blocks whose base-r digit is
 * non-zero -- either as the paper's three steps (gather-pack, the exchange as an HBM-to-HBM move of
 * the packed messages, scatter-unpack into the receive buffer R or the temporary buffer T) or, by
 * default, as one hop per block straight from where its sender holds it to where its receiver
 * keeps it.
 *
 * Conventions for every entry point
 *   - Pointers named `sendbuf`, `recvbuf`, `*counts`, `*displs`, `workspace` are DEVICE pointers.
 *     Pointers to result structs / size_t outputs are HOST pointers.
 *   - Count and displacement matrices are row-major P x P, row = owning virtual rank:
 *       sendcounts[i*P + j], sdispls[i*P + j] : the block rank i sends to rank j
 *       recvcounts[j*P + i], rdispls[j*P + i] : where rank j receives the block from rank i
 *     Counts are BYTES (int32, >= 0); displacements are BYTES (int64, >= 0 for every non-empty
 *     block) from `sendbuf` / `recvbuf`,
 *     one allocation each holding all P ranks' buffers; regions may come in any order, with gaps.
 *     Receive regions must not overlap each other.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - The caller owns all arrays and keeps them alive until the stream work has completed.
 *     The library never writes `sendbuf` or the four matrices, and writes `recvbuf` only inside
 *     the receive regions (MPI_Alltoallv semantics).
 *   - Return value: TUNA_OK (0) or a negative TUNA_ERR_* code.  Nothing throws or aborts.  When
 *     an error is returned no payload byte has been moved.
 *   - sendbuf and recvbuf must not overlap.  The library uses the HIP device that is current at
 *     its first call; a compute call made while another device is current returns TUNA_ERR_ARG.
 *   - A context (tuna_ctx_t) holds what an immediate call uses besides the caller's arrays: a grow-only
 *     workspace, a small status block and the statistics of its last call.  The entry points without a
 *     context argument use the process's default context.  Calls on one context share its workspace:
 *     a call issued on another stream than the context's previous call makes its stream wait for that
 *     call first, so they do not race (and do not overlap).  Calls on different contexts share nothing
 *     but the read-only cached schedules and may overlap.  A context is not thread-safe: one host
 *     thread at a time per context; the process-wide defaults (tuna_set_option) are plain variables.
 *   - There is no CPU fallback: without a HIP device every compute entry point returns
 *     TUNA_ERR_HIP.
 */
#ifndef TUNA_H
#define TUNA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TUNA_OK 0
#define TUNA_ERR_ARG -1              /* null pointer, P < 1, radix < 2, ranks_per_node does not divide P,
                                        a non-empty block at a negative displacement */
#define TUNA_ERR_COUNT_MISMATCH -2   /* recvcounts[j][i] != sendcounts[i][j] for some i, j */
#define TUNA_ERR_NEGATIVE_COUNT -3   /* a negative count */
#define TUNA_ERR_NOMEM -4            /* the library could not allocate its workspace */
#define TUNA_ERR_WORKSPACE_TOO_SMALL -5 /* a caller-supplied workspace is smaller than needed */
#define TUNA_ERR_HIP -6              /* a HIP call failed; tuna_stats_t.last_hip_error has the code */
#define TUNA_ERR_TOO_LARGE -7        /* P, a block or a per-rank byte total exceeds the supported range */
#define TUNA_ERR_NOALLOC_LIMIT -8    /* tuna_alltoallv_noalloc: the call needs more than TUNA_NOALLOC_SCRATCH_BYTES */

#define TUNA_RADIX_AUTO 0            /* as a radix argument: left to the library (the linear schedule, see tuna_select) */

#define TUNA_MAX_PHASES 64
#define TUNA_MAX_RANKS 32768

/* One digit phase x: all rounds (x, z), 1 <= z < r, z*r^x below the dimension's size.  They
 * touch disjoint index sets and are issued together (Section "Tunable Radix"). */
typedef struct tuna_phase_stats {
    int32_t dim;            /* 0: local / flat phase over the Q ranks of a node; 1: global phase over the N nodes */
    int32_t x;              /* digit position */
    int32_t radix;          /* r of this phase */
    int32_t rounds;         /* number of point-to-point rounds (valid z) in this phase */
    int64_t blocks;         /* blocks moved, all ranks, empty ones included */
    int64_t payload_bytes;  /* b_x: payload bytes of those blocks */
    int64_t staged_bytes;   /* bytes they occupy in a staging buffer (every block padded to 16 B) */
    float ms_metadata;      /* metadata exchange + scans (profiling mode only, else 0) */
    float ms_pack;          /* one-kernel phases have one payload kernel: the copy engine's hop is reported here, */
    float ms_exchange;
    float ms_unpack;        /* the destination-tiled hop here */
} tuna_phase_stats_t;

typedef struct tuna_stats {
    int32_t P, Q, N;                 /* ranks, ranks per node, nodes (flat: Q = P, N = 1) */
    int32_t local_radix, global_radix;
    int32_t w_local, w_global;       /* digits: ceil(log_r Q), ceil(log_r N) */
    int32_t K_local, K_global;       /* point-to-point rounds */
    int32_t B_local, B_global;       /* T slots of the paper's bound, B = size - (K + 1), per dimension */
    int32_t n_phases;
    int32_t granularity;             /* 128, 16, 4 or 1: common divisor of all counts/displacements/base addresses */
    int32_t fused;                   /* 1 when the fused single-kernel rounds were used */
    int32_t last_hip_error;
    int32_t dense_t;                 /* 1 when T was addressed in exact size, 0 in slots of M bytes (TUNA_OPT_DENSE_T) */
    int64_t max_block_bytes;         /* M (Algorithm "TuNA", line 1) */
    int64_t total_payload_bytes;     /* sum of sendcounts */
    int64_t temp_slots_per_rank;     /* slots of T actually laid out per rank */
    int64_t temp_bytes;              /* bytes of T */
    int64_t staging_bytes;           /* bytes of the send + receive staging buffers */
    int64_t workspace_bytes;         /* total device bytes the call needed */
    float ms_prepare;                /* validation, sizing, initial rotation (profiling mode only) */
    float ms_self;                   /* own-block copy */
    float ms_total;                  /* first to last kernel of the call */
    float reserved_f;
    tuna_phase_stats_t phase[TUNA_MAX_PHASES];
} tuna_stats_t;

/* Host-only description of the schedule for (P, ranks_per_node, radices); no GPU is touched.
 * Section "Tunable Radix" (w, K), Section "Estimating temporary buffer size" (B, the T map). */
typedef struct tuna_plan_info {
    int32_t P, Q, N;
    int32_t local_radix, global_radix;   /* after clamping to [2, Q] and [2, N] */
    int32_t w_local, w_global;
    int32_t K_local, K_global;
    int32_t B_local, B_global;
    int32_t n_phases;
    int64_t temp_slots_per_rank;
    int64_t blocks_sent_per_rank;        /* D for one rank: one send per non-zero digit of each index */
} tuna_plan_info_t;

/*
 * The non-uniform all-to-all, MPI_Alltoallv's statement of the problem (abstract; Section
 * "Graph Mining": same function signature as MPI_Alltoallv plus the tunables): when the work
 * enqueued on `stream` has completed,
 *     recvbuf[rdispls[j][i] .. +recvcounts[j][i])  ==  sendbuf[sdispls[i][j] .. +sendcounts[i][j])
 * for all ranks i, j.
 *   radix           r of Algorithm "TuNA", 2..P; larger values are clamped to P (r = P is the
 *                   linear algorithm: one block per round, no temporary buffer).
 *   ranks_per_node  Q.  0, 1 or P: flat TuNA over all P ranks.  Otherwise Q must divide P, rank
 *                   p lives on node p / Q with local id p % Q, and the hierarchical variant runs
 *                   with local radix min(radix, Q) and global radix min(radix, N), N = P / Q.
 * The call validates the counts on the device, reads a few integers back (one stream
 * synchronisation), sizes or grows the workspace, then enqueues all phases on `stream` and
 * returns without waiting for them.  Payloads of 64 MiB and more with at least two digit phases:
 * with one-kernel hops (the default) the block-size exchanges and scans of all phases run on a
 * second stream owned by the context while `stream` moves the payload, each phase's payload kernel
 * behind an event of its metadata; work enqueued on `stream` after the call is ordered behind all
 * of it as usual.  With three-stage phases, or when the call is profiled, such a call is done in two
 * passes instead -- the metadata of every phase first, a second read-back of the phases' exact
 * work-list lengths, then the payload kernels -- which costs one more synchronisation and saves
 * launching every copy kernel for an upper bound of work.
 * Problems of at most 64 ranks, 1 MiB of payload and 8 digit phases are done by one kernel launch
 * (validation, all phases and the own blocks in one workgroup; options at their defaults, no
 * profiling): there the launches, not the bytes, are what a call costs.  It returns after that
 * kernel has finished.
 */
int tuna_alltoallv(const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls,
                   void* recvbuf, const int32_t* recvcounts, const int64_t* rdispls,
                   int P, int radix, int ranks_per_node, void* stream);

/*
 * The same with the two radices chosen separately (Section "Hierarchical TuNA": the intra-node
 * phase is TuNA with a radix up to Q; the inter-node phase exchanges the Q-block super-blocks
 * between ranks of equal local id).  global_radix >= N gives the paper's coalesced schedule
 * (N - 1 rounds, Q blocks per message); a smaller global_radix runs the same digit rounds over
 * the N node-ranks with super-blocks as the unit.
 */
int tuna_alltoallv_hier(const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls,
                        void* recvbuf, const int32_t* recvcounts, const int64_t* rdispls,
                        int P, int ranks_per_node, int local_radix, int global_radix, void* stream);

/*
 * Options of one call or plan.  tuna_opts_init fills the struct with the process-wide defaults (as
 * tuna_set_option left them) and its size; a caller then changes what it wants and passes the struct
 * to tuna_alltoallv_ex / tuna_alltoallv_init_ex.  A NULL options pointer means the defaults.
 *   mode         TUNA_MODE_AUTO (default): left to the library, which takes the one-kernel hops --
 *                with all ranks in one memory a hop needs no message, and moving a block straight from
 *                where its sender holds it to where its receiver keeps it reads and writes it once
 *                instead of three times.  When the receive regions are dense (every rank's blocks back to
 *                back in source order) and sizes, displacements and buffer addresses are multiples of 4,
 *                a phase is tiled over its destinations in 128-byte lines: the last phase of a schedule
 *                (all its blocks go into the receive buffer) when the blocks are mostly longer than a few
 *                lines (mean of 700 bytes or more, at most a quarter of them under 256 bytes), the phases
 *                before it (which store whole 16-byte chunks into T) when T is kept in exact size and
 *                the mean block is 512 bytes or more; otherwise (and always for T in slots, batches of
 *                rounds and the staggered schedule) over the blocks.  Which of the two ran changes no byte.
 *                TUNA_MODE_STAGED: pack -> exchange -> unpack, the paper's three steps as three kernels.
 *                TUNA_MODE_FUSED: the one-kernel hops.
 *   staggered, t_layout, block_count, profile: as TUNA_OPT_STAGGERED, TUNA_OPT_DENSE_T,
 *                TUNA_OPT_BLOCK_COUNT, TUNA_OPT_PROFILE below.
 */
#define TUNA_MODE_AUTO 0
#define TUNA_MODE_STAGED 1
#define TUNA_MODE_FUSED 2
#define TUNA_T_SLOTS 0
#define TUNA_T_EXACT 1
#define TUNA_T_AUTO 2
typedef struct tuna_opts {
    int32_t struct_size;    /* sizeof(tuna_opts_t), set by tuna_opts_init */
    int32_t mode;
    int32_t staggered;
    int32_t t_layout;
    int32_t block_count;
    int32_t profile;
    int32_t reserved[2];
} tuna_opts_t;
int tuna_opts_init(tuna_opts_t* opts);

/* A context of its own: workspace, status block, statistics.  tuna_ctx_create allocates a few hundred
 * KiB and an event; tuna_ctx_destroy waits for the device and frees everything the context owns.
 * NULL stands for the default context wherever a tuna_ctx_t is taken. */
typedef struct tuna_ctx_s* tuna_ctx_t;
int tuna_ctx_create(tuna_ctx_t* ctx);
int tuna_ctx_destroy(tuna_ctx_t ctx);
int tuna_ctx_get_stats(tuna_ctx_t ctx, tuna_stats_t* out);

/* tuna_alltoallv_hier on a given context with given options (Section "Hierarchical TuNA"; the radices
 * may be TUNA_RADIX_AUTO). */
int tuna_alltoallv_ex(tuna_ctx_t ctx, const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls,
                      void* recvbuf, const int32_t* recvcounts, const int64_t* rdispls,
                      int P, int ranks_per_node, int local_radix, int global_radix,
                      const tuna_opts_t* opts, void* stream);

/*
 * For callers that cannot allocate device memory when they call -- code under HIP graph capture
 * rules, tight serving loops, harnesses that forbid hipMalloc: the same call as
 * tuna_alltoallv_hier (same arguments, same result, the options in force apply, TUNA_OPT_PROFILE
 * excepted), done in one pass with every internal buffer -- status block, schedule tables, size
 * matrices, scans, work lists, staging buffers, T -- carved from one static device array of
 * TUNA_NOALLOC_SCRATCH_BYTES bytes that each GPU the library runs on holds until the process ends.
 * The call itself calls no hipMalloc, hipFree, hipHostMalloc or hipEventCreate (it still reads a
 * few integers back and synchronises `stream` once, like tuna_alltoallv).  A problem that needs
 * more than the array returns TUNA_ERR_NOALLOC_LIMIT before any payload byte has moved: the need
 * is about 26 P^2 bytes of tables and scans per phase-independent part, 24 bytes per moving block
 * and phase of schedule tables, twice the payload for the staging buffers of three-stage phases
 * and the bytes waiting in T -- e.g. P = 256 with 8 MiB of payload fits at every radix.
 * It uses the device that is current and works on any device.  All calls on one GPU share that
 * GPU's array, which keeps the previous call's contents (every call writes whatever it reads):
 * two calls that overlap in time on one GPU race, also with different streams.
 */
#define TUNA_NOALLOC_SCRATCH_BYTES (64u << 20)
int tuna_alltoallv_noalloc(const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls,
                           void* recvbuf, const int32_t* recvcounts, const int64_t* rdispls,
                           int P, int ranks_per_node, int local_radix, int global_radix, void* stream);

/*
 * Persistent form, after MPI's persistent collectives (MPI_Alltoallv_init / MPI_Start): for
 * callers that repeat an exchange with the same counts, displacements and buffers.
 * tuna_alltoallv_init does everything that depends only on the counts -- validation, sizing,
 * every phase's block-size exchange, scans and work lists -- keeps the result in device memory
 * owned by the plan (it allocates and synchronises), and fixes the options in force
 * (TUNA_OPT_FUSED, TUNA_OPT_STAGGERED, TUNA_OPT_DENSE_T).  tuna_start only enqueues the payload kernels on
 * `stream`: no allocation, no host synchronisation, no host-visible dependence on device data,
 * so it may be captured into a HIP graph (unless TUNA_OPT_PROFILE is on) and replayed.  The six
 * arrays must stay alive and unchanged while the plan exists; the contents of sendbuf may change
 * between starts.  Two starts of one plan must not overlap in time.  tuna_plan_free waits for
 * the device and releases the plan's memory.
 */
typedef struct tuna_plan_s* tuna_plan_t;
int tuna_alltoallv_init(const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls,
                        void* recvbuf, const int32_t* recvcounts, const int64_t* rdispls,
                        int P, int ranks_per_node, int local_radix, int global_radix,
                        void* stream, tuna_plan_t* plan);
/* The same with options and a context (which receives the plan's statistics and profiling events; the
 * plan's device memory is its own either way). */
int tuna_alltoallv_init_ex(tuna_ctx_t ctx, const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls,
                           void* recvbuf, const int32_t* recvcounts, const int64_t* rdispls,
                           int P, int ranks_per_node, int local_radix, int global_radix,
                           const tuna_opts_t* opts, void* stream, tuna_plan_t* plan);
int tuna_start(tuna_plan_t plan, void* stream);
int tuna_plan_free(tuna_plan_t plan);

/*
 * Device bytes a call with these counts and parameters needs under the options in force
 * (Algorithm "TuNA", lines 1-2: maximum block size M by a reduction over all ranks, T sized from
 * it -- or from the blocks' sizes and hop counts when T is kept in exact size).  The reduction
 * runs on the device; the call synchronises.  *bytes is a host pointer.
 */
int tuna_workspace_bytes(const int32_t* sendcounts, int P, int ranks_per_node,
                         int local_radix, int global_radix, size_t* bytes);

/*
 * Plain device-to-device copy of `bytes` bytes (a multiple of 16; both pointers 16-byte
 * aligned) with one 16-byte load and store per thread, enqueued on `stream`.  Not part of the
 * algorithm: it is the measured HBM copy ceiling the benchmark quotes next to the 8 TB/s peak,
 * and the known-size kernel that hardware byte counters are calibrated against.
 */
int tuna_plain_copy(const void* src, void* dst, size_t bytes, void* stream);

/*
 * Optional caller-owned workspace of the default context (device memory, 256-byte aligned).  While
 * set, calls on that context allocate nothing and return TUNA_ERR_WORKSPACE_TOO_SMALL when it does
 * not suffice.
 * tuna_set_workspace(NULL, 0) returns to the library-owned, grow-only workspace.
 */
int tuna_set_workspace(void* workspace, size_t bytes);

/* Frees the library-owned workspace and cached schedules (waits for the device first).  Returns
 * TUNA_ERR_ARG while persistent plans exist: free them first. */
int tuna_release(void);

/*
 * Options.  TUNA_OPT_PROFILE: 1 = bracket every kernel with HIP events on the call's stream so
 * that tuna_get_stats reports per-phase times (the breakdown categories of Section "Performance
 * analysis of coalesced and staggered TuNA_l^g": prepare, metadata, data, replace).
 * TUNA_OPT_FUSED: 1 = move every block of a phase straight from its source (S or T) to its
 * destination (R or T; with T in slots, the other of two copies of T) in one kernel instead of
 * pack -> exchange -> unpack; 0 = the three kernels; 2 (default) = left to the library (tuna_opts_t.mode).
 * TUNA_OPT_STAGGERED: 1 = the staggered inter-node schedule of Algorithm "Staggered TuNA_l^g"
 * for hierarchical calls: after the intra-node phase every one of the Q (N - 1) blocks bound
 * for another node is its own message and goes straight from where it lies (its T slot, or S)
 * to R of its destination -- no rearrangement of T, no packing; the global radix is N.
 * TUNA_OPT_DENSE_T: 1 = T in exact size, 0 = T in the paper's slots, 2 (default) = left to the
 * library: slots when they would be at least 90 % full (blocks of nearly one size, where the slot
 * arithmetic is just as dense and cheaper to address), else exact size when it is not the larger
 * of the two or still fits into half of the free device memory, else slots.  Exact size: Section
 * "Estimating temporary buffer size" bounds T by B slots of M bytes, M the largest block of all;
 * with skewed sizes nearly all of that is padding.  Here every block size is on the device before
 * the first round, so the blocks that wait in T lie back to back, each padded to 16 bytes.  A
 * block stored in phase f and forwarded in phase y occupies T from f to y; the blocks of one
 * (f, y) pair form a class whose size the validation pass sums, and classes whose waits do not
 * overlap share memory (with one-kernel hops a phase must not store where it reads, so the
 * classes a phase stores and the classes it forwards count as overlapping).  T then takes about
 * the largest number of bytes that wait at one time (at most 1.12 times that on the benchmark
 * workloads: 1.1 times the payload at r = 2 with three-stage phases, 1.7 times with one-kernel
 * hops, less at larger radices), whatever M is.
 * TUNA_OPT_BLOCK_COUNT: k > 0 = at most k rounds of a digit phase are moved per set of kernel
 * launches, in ascending round order; 0 (default) = all rounds of a phase at once.  This is the
 * block_count of Algorithms "Staggered TuNA_l^g" and "Coalesced TuNA_l^g" (the number of
 * point-to-point rounds in flight between two waits; Section "Performance analysis of coalesced
 * and staggered TuNA_l^g": 1 .. N - 1 for the coalesced schedule, 1 .. (N - 1) Q for the
 * staggered one, where a round carries one block -- there k is rounded down to whole node
 * distances of Q rounds each, at least one).  With the linear schedule r = P it gives the
 * scattered algorithm of Section "Background".  On a network it bounds congestion; in one HBM
 * it moves the same bytes with more launches.
 */
#define TUNA_OPT_PROFILE 1
#define TUNA_OPT_FUSED 2
#define TUNA_OPT_STAGGERED 3
#define TUNA_OPT_DENSE_T 4
#define TUNA_OPT_BLOCK_COUNT 5
int tuna_set_option(int option, int value);

/* Statistics of the last tuna_alltoallv* call on the default context (host struct).  Synchronises
 * with that call's stream work. */
int tuna_get_stats(tuna_stats_t* out);

/* Schedule description, host only. */
int tuna_plan_info(int P, int ranks_per_node, int local_radix, int global_radix,
                   tuna_plan_info_t* out);

/* Host only: phase `phase` (0 <= phase < n_phases) of the schedule.  header[0..5] receives
 * {dim, x, radix, rounds, moving blocks per rank, r^x}; when `seg` is not NULL it receives, for
 * the first min(seg_capacity, moving blocks) blocks in message order (digit value z ascending,
 * then slot index ascending; Algorithm "TuNA", lines 8-11), six int32 each:
 * {slot index e = j*Q + l, j, l, z, source T slot or -1 (send buffer), destination T slot or
 * -1 (final: receive buffer)}. */
int tuna_plan_phase(int P, int ranks_per_node, int local_radix, int global_radix, int phase,
                    int32_t* header, int32_t* seg, int seg_capacity);

/* Host only (on_device = 0) or read back from the device's tables (on_device = 1; needs a GPU,
 * synchronises): where every moving block of phase `phase` last moved before it -- two int32
 * per block in message order, {phase in which it arrived in T, its position in that phase's
 * message order}, or {-1, 0} for a block still in the send buffer.  Exact-size T finds a
 * block through this pair. */
int tuna_plan_phase_sources(int P, int ranks_per_node, int local_radix, int global_radix, int phase,
                            int on_device, int32_t* out, int capacity);

/* The same table as the device holds it (the kernels read tables that k_build_phase_table built
 * on the GPU with the same index arithmetic): four int32 per moving block in message order,
 * {e, z, source slot, destination slot}.  Needs a GPU; synchronises.  For verification. */
int tuna_plan_phase_device(int P, int ranks_per_node, int local_radix, int global_radix, int phase,
                           int32_t* seg, int seg_capacity);

/*
 * For verification: the device's block-size matrix as the metadata exchange leaves it (Section
 * "Two-phase communication": the sizes travel ahead of the blocks).  Builds a persistent plan for the
 * problem, copies the P x P int32 matrix of current block sizes to the host array `sizes` before the
 * first digit phase (entry 0: the initial rotation) and after every phase (entries 1 .. n_phases), row =
 * rank, column = slot index j * Q + l, and frees the plan again.  `sizes` must hold capacity_phases >=
 * n_phases + 1 matrices.  Allocates and synchronises; moves no payload.  With the staggered schedule
 * (TUNA_OPT_STAGGERED) the global radix of the plan is N.
 */
int tuna_debug_phase_sizes(const void* sendbuf, const int32_t* sendcounts, const int64_t* sdispls,
                           void* recvbuf, const int32_t* recvcounts, const int64_t* rdispls,
                           int P, int ranks_per_node, int local_radix, int global_radix, void* stream,
                           int32_t* sizes, int capacity_phases);

/*
 * Radix, mode and T layout for one GPU, from a cost model fitted to timed calls.  The paper picks r
 * from P and the block size because each of its K rounds pays a network latency (Section "Performance
 * analysis of TuNA", "Radix selection": small blocks -> r near 2, medium -> r near sqrt(P), large -> r
 * near P).  In one HBM a round has no latency of its own; the model of an immediate call is
 *     ms = c0 + c1 * phases + c2 * (phases + 1) * P^2 / 1e6 + c3 * hop bytes / 1e9 + c4 * moving blocks / 1e6,
 * phases = digits of the two radices (every phase, and the validation, passes once over the P x P block sizes), hop bytes = payload bytes times the average number of hops of a
 * block (the share of rank distances whose digit is non-zero, summed over the digit positions), moving
 * blocks = the same count in blocks; one set of constants for three-stage phases and one for one-kernel
 * hops; T in the paper's slots adds to the byte term by how empty the slots are (mean block / M).  When no
 * block exceeds 64 bytes the one-kernel hops run a kernel of their own (one thread per block), whose
 * blocks and bytes are priced by constants of their own, c5 and c6, in place of c4 and c3.
 *   tuna_calibrate   times about sixty immediate calls of dense synthetic problems on the current
 *                    device (a few hundred milliseconds; allocates up to about 8 GiB and frees it;
 *                    synchronises) and fits the constants to them.  Without it the constants are the
 *                    built-in ones, fitted the same way on an MI355X.
 *   tuna_predict_ms  the model's time for one setting.  max_block_bytes = 0: unknown (slots taken as full).
 *                    granularity: the largest of 1, 4, 16, 128 that divides every count, displacement
 *                    and both buffer addresses (tuna_stats_t.granularity), 0 = unknown (taken as 4);
 *                    byte-granular problems run kernel variants whose byte term costs a fitted factor more,
 *                    line-granular ones (128) variants whose byte and block terms cost a fitted factor less.
 *   tuna_select      evaluates the model for the radices 2, 4, 8, ..., ceil(sqrt(size)), size of each
 *                    dimension, both modes and both T layouts and returns the minimiser.  Every term
 *                    falls as r grows and one-kernel hops move a third of the bytes, so the answer on
 *                    one GPU is the linear schedule (r = Q, r = N) with one-kernel hops for every
 *                    payload; the function exists so that callers do not hard-code that, and so that
 *                    the model can be checked against measurements (the GPU tests do).
 * All three are host functions; only tuna_calibrate touches the GPU.  The model covers calls that take
 * the general path; the single-launch path of tuna_alltoallv for tiny problems is not modelled.
 */
typedef struct tuna_choice {
    int32_t local_radix, global_radix;
    int32_t mode;            /* TUNA_MODE_STAGED or TUNA_MODE_FUSED */
    int32_t t_layout;        /* TUNA_T_EXACT or TUNA_T_SLOTS */
    int32_t calibrated;      /* 1: constants fitted by tuna_calibrate in this process; 0: the built-in ones */
    int32_t reserved;
    double predicted_ms;     /* of one immediate call with this setting */
} tuna_choice_t;
int tuna_calibrate(void* stream);
/* Host only: the model's constants for `mode` (TUNA_MODE_STAGED or TUNA_MODE_FUSED) as they stand -- built in,
 * or fitted by tuna_calibrate: c[0..6] = c0 .. c6 above, c[7] = the factor on the byte term's share that
 * passes through T in slots, per unit of emptiness, c[8] = the factor on the byte term of byte-granular
 * problems, c[9] = the factor on the byte and block terms of line-granular problems.
 * capacity >= TUNA_MODEL_CONSTANTS. */
#define TUNA_MODEL_CONSTANTS 10
int tuna_model_constants(int mode, double* c, int capacity);
int tuna_predict_ms(int P, int ranks_per_node, int local_radix, int global_radix, int mode, int t_layout,
                    int64_t payload_bytes, int64_t max_block_bytes, int granularity, double* ms);
int tuna_select(int P, int ranks_per_node, int64_t payload_bytes, int64_t max_block_bytes, int granularity,
                tuna_choice_t* out);

/* Slot of block index o (1 <= o, not a direct block) in T for radix r:
 * t = o - 1 - dx (r - 1) - dz with dx the position and dz the value of o's highest base-r digit
 * (Section "Estimating temporary buffer size").  Returns -1 for o <= 0 or a direct block. */
int tuna_t_index(int o, int radix);

const char* tuna_strerror(int code);
int tuna_version(void);
/* Hash of the sources this library was built from (set by the build script; "unknown" otherwise). */
const char* tuna_build_id(void);

#ifdef __cplusplus
}
#endif
#endif /* TUNA_H */
