/*
 * CPU oracle, C twin of the plain definition (Section 2 of the paper):
 *
 *   all-to-all : recv[R][i] = send[R (-) C^i][i]
 *   allgather  : recv[R][i] = send[R (-) C^i]
 *
 * where R (-) C subtracts component-wise with wrap-around in a d-dimensional
 * torus, ranks are row-major with the last dimension fastest, and blocks of m
 * bytes sit in neighbour order in the buffers.
 *
 * TEST INFRASTRUCTURE ONLY: used by the tests and as the timed CPU baseline of
 * the benchmark.  It is a separate translation unit that shares no header or
 * helper with the GPU library.  Plain loops and one memcpy per block; the loop
 * over processes is an OpenMP parallel-for.  Not tuned.
 */
#include <stdint.h>
#include <string.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ISO_ORACLE_MAX_DIMS 64

static int64_t source_rank(int d, const int32_t *dims, int64_t R, const int32_t *C)
{
    int64_t coord[ISO_ORACLE_MAX_DIMS];
    int64_t rem = R;
    for (int j = d - 1; j >= 0; --j) {
        coord[j] = rem % dims[j];
        rem /= dims[j];
    }
    int64_t src = 0;
    for (int j = 0; j < d; ++j) {
        int64_t x = (coord[j] - (int64_t)C[j]) % dims[j];
        if (x < 0) x += dims[j];
        src = src * dims[j] + x;
    }
    return src;
}

static int64_t n_ranks(int d, const int32_t *dims)
{
    int64_t p = 1;
    for (int j = 0; j < d; ++j) p *= dims[j];
    return p;
}

/* returns the number of threads used, or -1 on bad arguments */
int iso_oracle_alltoall(int d, const int32_t *dims, int s, const int32_t *offsets,
                        size_t m, const void *sendbuf, void *recvbuf, int threads)
{
    if (d <= 0 || d > ISO_ORACLE_MAX_DIMS || s < 0) return -1;
    const int64_t p = n_ranks(d, dims);
    const char *send = (const char *)sendbuf;
    char *recv = (char *)recvbuf;
    int used = 1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
    used = omp_get_max_threads();
#endif
#pragma omp parallel for schedule(static)
    for (int64_t R = 0; R < p; ++R) {
        for (int i = 0; i < s; ++i) {
            int64_t src = source_rank(d, dims, R, offsets + (size_t)i * d);
            memcpy(recv + ((size_t)R * s + i) * m, send + ((size_t)src * s + i) * m, m);
        }
    }
    return used;
}

int iso_oracle_allgather(int d, const int32_t *dims, int s, const int32_t *offsets,
                         size_t m, const void *sendbuf, void *recvbuf, int threads)
{
    if (d <= 0 || d > ISO_ORACLE_MAX_DIMS || s < 0) return -1;
    const int64_t p = n_ranks(d, dims);
    const char *send = (const char *)sendbuf;
    char *recv = (char *)recvbuf;
    int used = 1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
    used = omp_get_max_threads();
#endif
#pragma omp parallel for schedule(static)
    for (int64_t R = 0; R < p; ++R) {
        for (int i = 0; i < s; ++i) {
            int64_t src = source_rank(d, dims, R, offsets + (size_t)i * d);
            memcpy(recv + ((size_t)R * s + i) * m, send + (size_t)src * m, m);
        }
    }
    return used;
}
