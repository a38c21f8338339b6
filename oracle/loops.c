/* Oracle loops in plain C -- TEST INFRASTRUCTURE ONLY.
 *
 * The same definitions as oracle/collective.py and oracle/gemm.py, written as plain
 * sequential loops (optionally split over host threads with OpenMP) so that the
 * oracle can be timed on the host cores.  No intrinsics, no BLAS, no blocking.
 * Shares nothing with the HIP library.
 *
 *   reduce-copy : dst_d[i] = round(((src_0[i] + src_1[i]) + ...) ), fp32 adds in
 *                 source order, one rounding (paper Sec. 3.2: the local step of a
 *                 chunked collective; the result does not depend on NC, NT, C)
 *   gather-copy : dst[r*n + i] = src_r[i]
 *   gemm        : C[m,n] = sum_k A[m,k] * B[n,k], bf16 inputs, fp64 accumulation,
 *                 k ascending
 */
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline float bf16_widen(uint16_t h) {
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round to nearest, ties to even; NaN keeps a quiet payload */
static inline uint16_t bf16_round(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t upper = u >> 16, lower = u & 0xffffu;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u))) upper += 1u;
    return (uint16_t)upper;
}

int oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_reduce_copy_f32(const float* const* srcs, int nsrc, float* const* dsts, int ndst,
                            int64_t n, int threads) {
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        float acc = srcs[0][i];
        for (int s = 1; s < nsrc; ++s) acc = acc + srcs[s][i];
        for (int d = 0; d < ndst; ++d) dsts[d][i] = acc;
    }
}

void oracle_reduce_copy_bf16(const uint16_t* const* srcs, int nsrc, uint16_t* const* dsts, int ndst,
                             int64_t n, int threads) {
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        float acc = bf16_widen(srcs[0][i]);
        for (int s = 1; s < nsrc; ++s) acc = acc + bf16_widen(srcs[s][i]);
        uint16_t r = bf16_round(acc);
        for (int d = 0; d < ndst; ++d) dsts[d][i] = r;
    }
}

/* byte-wise, any element type: n_bytes per shard */
void oracle_gather_copy(const uint8_t* const* srcs, int nsrc, uint8_t* const* dsts, int ndst,
                        int64_t n_bytes, int threads) {
    for (int r = 0; r < nsrc; ++r) {
#pragma omp parallel for num_threads(threads) schedule(static)
        for (int64_t i = 0; i < n_bytes; ++i) {
            uint8_t v = srcs[r][i];
            for (int d = 0; d < ndst; ++d) dsts[d][(int64_t)r * n_bytes + i] = v;
        }
    }
}

/* rows [row_lo, row_hi) of the product, stored as C[(m - row_lo), n] (fp64, row-major, N columns);
 * A [M,K]; B [N,K] if b_is_nk else [K,N] */
void oracle_gemm_bf16(const uint16_t* A, const uint16_t* B, double* C, int64_t M, int64_t N, int64_t K,
                      int b_is_nk, int64_t row_lo, int64_t row_hi, int threads) {
    (void)M;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t m = row_lo; m < row_hi; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double a = (double)bf16_widen(A[m * K + k]);
                double b = (double)bf16_widen(b_is_nk ? B[n * K + k] : B[k * N + n]);
                acc = acc + a * b;
            }
            C[(m - row_lo) * N + n] = acc;
        }
    }
}
