/*
 * C-ABI check: a plain C program (no Python, no torch) that drives libtuna.so through
 * include/tuna.h with memory from hipMalloc and compares the result with the CPU oracle
 * (liboracle.so).  Built by __graft_entry__.build(); run by tests/test_gpu_c_abi.py.
 * Usage: c_abi_check P radix ranks_per_node   -> prints "ok ..." and exits 0, or a message and 1.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../include/tuna.h"

int oracle_alltoallv(const unsigned char* send, const int32_t* sendcounts, const int64_t* sdispls,
                     unsigned char* recv, const int32_t* recvcounts, const int64_t* rdispls, int P);

#define HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %d at line %d\n", (int)e_, __LINE__); return 1; } } while (0)

static uint64_t lcg(uint64_t* s) { *s = *s * 6364136223846793005ull + 1442695040888963407ull; return *s >> 33; }

int main(int argc, char** argv) {
    const int P = argc > 1 ? atoi(argv[1]) : 12;
    const int radix = argc > 2 ? atoi(argv[2]) : 3;
    const int rpn = argc > 3 ? atoi(argv[3]) : 0;
    const size_t PP = (size_t)P * P;
    int32_t* sc = malloc(PP * 4); int32_t* rc = malloc(PP * 4);
    int64_t* sd = malloc(PP * 8); int64_t* rd = malloc(PP * 8);
    uint64_t seed = 0x241102581ull + (uint64_t)P * 131 + (uint64_t)radix;
    size_t sbytes = 5, rbytes = 7;                       /* leading gaps */
    for (size_t k = 0; k < PP; ++k) { sc[k] = (int32_t)(lcg(&seed) % 700); if (lcg(&seed) % 4 == 0) sc[k] = 0; }
    for (int i = 0; i < P; ++i) for (int j = 0; j < P; ++j) { sd[(size_t)i * P + j] = (int64_t)sbytes; sbytes += (size_t)sc[(size_t)i * P + j] + 3; }
    for (int j = 0; j < P; ++j) for (int i = 0; i < P; ++i) {
        rc[(size_t)j * P + i] = sc[(size_t)i * P + j];
        rd[(size_t)j * P + i] = (int64_t)rbytes; rbytes += (size_t)rc[(size_t)j * P + i] + 2;
    }
    unsigned char* send = malloc(sbytes); unsigned char* want = malloc(rbytes); unsigned char* got = malloc(rbytes);
    for (size_t k = 0; k < sbytes; ++k) send[k] = (unsigned char)(lcg(&seed));
    memset(want, 0xD2, rbytes);
    if (oracle_alltoallv(send, sc, sd, want, rc, rd, P) != 0) { printf("oracle failed\n"); return 1; }

    void *d_send, *d_recv, *d_sc, *d_rc, *d_sd, *d_rd;
    HIP(hipMalloc(&d_send, sbytes)); HIP(hipMalloc(&d_recv, rbytes));
    HIP(hipMalloc(&d_sc, PP * 4)); HIP(hipMalloc(&d_rc, PP * 4)); HIP(hipMalloc(&d_sd, PP * 8)); HIP(hipMalloc(&d_rd, PP * 8));
    HIP(hipMemcpy(d_send, send, sbytes, hipMemcpyHostToDevice));
    HIP(hipMemset(d_recv, 0xD2, rbytes));
    HIP(hipMemcpy(d_sc, sc, PP * 4, hipMemcpyHostToDevice)); HIP(hipMemcpy(d_rc, rc, PP * 4, hipMemcpyHostToDevice));
    HIP(hipMemcpy(d_sd, sd, PP * 8, hipMemcpyHostToDevice)); HIP(hipMemcpy(d_rd, rd, PP * 8, hipMemcpyHostToDevice));
    hipStream_t stream;
    HIP(hipStreamCreate(&stream));

    int code = tuna_alltoallv(d_send, d_sc, d_sd, d_recv, d_rc, d_rd, P, radix, rpn, stream);
    if (code != TUNA_OK) { printf("tuna_alltoallv: %s\n", tuna_strerror(code)); return 1; }
    HIP(hipStreamSynchronize(stream));
    HIP(hipMemcpy(got, d_recv, rbytes, hipMemcpyDeviceToHost));
    if (memcmp(got, want, rbytes) != 0) { printf("immediate call differs from the oracle\n"); return 1; }
    tuna_stats_t st;
    if (tuna_get_stats(&st) != TUNA_OK || st.P != P) { printf("stats\n"); return 1; }

    /* persistent form, two starts */
    tuna_plan_t plan = NULL;
    code = tuna_alltoallv_init(d_send, d_sc, d_sd, d_recv, d_rc, d_rd, P, rpn, radix, radix, stream, &plan);
    if (code != TUNA_OK) { printf("tuna_alltoallv_init: %s\n", tuna_strerror(code)); return 1; }
    for (int rep = 0; rep < 2; ++rep) {
        HIP(hipMemset(d_recv, 0xD2, rbytes));
        code = tuna_start(plan, stream);
        if (code != TUNA_OK) { printf("tuna_start: %s\n", tuna_strerror(code)); return 1; }
        HIP(hipStreamSynchronize(stream));
        HIP(hipMemcpy(got, d_recv, rbytes, hipMemcpyDeviceToHost));
        if (memcmp(got, want, rbytes) != 0) { printf("start %d differs from the oracle\n", rep); return 1; }
    }
    if (tuna_plan_free(plan) != TUNA_OK || tuna_release() != TUNA_OK) { printf("teardown\n"); return 1; }
    printf("ok P=%d radix=%d ranks_per_node=%d payload=%lld w=%d K=%d\n", P, radix, rpn,
           (long long)st.total_payload_bytes, st.w_local + st.w_global, st.K_local + st.K_global);
    return 0;
}
