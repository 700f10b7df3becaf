/*
 * TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.
 *
 * Plain CPU oracle for the non-uniform all-to-all.  The tunable-radix algorithm reaches,
 * in fewer and larger exchanges, exactly the result MPI_Alltoallv defines (abstract;
 * Section "Hierarchical TuNA", paragraph "Intra-node communication": every rank p sends
 * data block i to rank i and receives data block p from rank i).  So the oracle is that
 * definition written out: for every sender i and receiver j,
 *
 *     recv[ rdispls[j][i] .. +sendcounts[i][j] )  =  send[ sdispls[i][j] .. +sendcounts[i][j] )
 *
 * Two nested loops and a memcpy; no radix, no rounds, no temporary buffer, no blocking.
 * It shares no code with the GPU library and only tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.
 *
 * Matrices are row-major P x P, row = owning rank.  Counts in bytes (int32),
 * displacements in bytes (int64) from the start of one allocation that holds all ranks'
 * buffers.  Bytes of `recv` outside every receive region are never written.
 *
 * Pins (tests/test_oracle_pins.py): element-wise decode of a traceable payload on tiny
 * P, numpy's transpose for the uniform case, byte conservation, untouched canary gaps.
 */
#include <stdint.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_ERR_ARG -1
#define ORACLE_ERR_COUNT_MISMATCH -2
#define ORACLE_ERR_NEGATIVE_COUNT -3

/* MPI requires recvcounts[j][i] == sendcounts[i][j]; nothing is written when that fails. */
int oracle_check_counts(const int32_t* sendcounts, const int32_t* recvcounts, int P) {
    if (P < 1 || !sendcounts || !recvcounts) return ORACLE_ERR_ARG;
    for (int i = 0; i < P; ++i)
        for (int j = 0; j < P; ++j) {
            int32_t c = sendcounts[(size_t)i * P + j];
            if (c < 0) return ORACLE_ERR_NEGATIVE_COUNT;
            if (recvcounts[(size_t)j * P + i] != c) return ORACLE_ERR_COUNT_MISMATCH;
        }
    return ORACLE_OK;
}

int oracle_alltoallv(const unsigned char* send, const int32_t* sendcounts, const int64_t* sdispls,
                     unsigned char* recv, const int32_t* recvcounts, const int64_t* rdispls, int P) {
    int rc = oracle_check_counts(sendcounts, recvcounts, P);
    if (rc != ORACLE_OK) return rc;
    for (int i = 0; i < P; ++i)          /* sender   */
        for (int j = 0; j < P; ++j) {    /* receiver */
            size_t n = (size_t)sendcounts[(size_t)i * P + j];
            if (n == 0) continue;
            memcpy(recv + rdispls[(size_t)j * P + i], send + sdispls[(size_t)i * P + j], n);
        }
    return ORACLE_OK;
}

/* The same definition restricted to a list of receiving ranks: what those ranks must hold
 * afterwards.  Used to check samples of problems too large to transpose whole on the host. */
int oracle_alltoallv_receivers(const unsigned char* send, const int32_t* sendcounts,
                               const int64_t* sdispls, unsigned char* recv,
                               const int32_t* recvcounts, const int64_t* rdispls, int P,
                               const int32_t* receivers, int n_receivers) {
    if (P < 1 || n_receivers < 0 || (n_receivers > 0 && !receivers)) return ORACLE_ERR_ARG;
    for (int t = 0; t < n_receivers; ++t) {
        int j = receivers[t];
        if (j < 0 || j >= P) return ORACLE_ERR_ARG;
        for (int i = 0; i < P; ++i) {
            int32_t c = sendcounts[(size_t)i * P + j];
            if (c < 0) return ORACLE_ERR_NEGATIVE_COUNT;
            if (recvcounts[(size_t)j * P + i] != c) return ORACLE_ERR_COUNT_MISMATCH;
        }
    }
    for (int t = 0; t < n_receivers; ++t) {
        int j = receivers[t];
        for (int i = 0; i < P; ++i) {
            size_t n = (size_t)sendcounts[(size_t)i * P + j];
            if (n == 0) continue;
            memcpy(recv + rdispls[(size_t)j * P + i], send + sdispls[(size_t)i * P + j], n);
        }
    }
    return ORACLE_OK;
}
