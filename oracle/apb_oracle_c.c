/* CPU oracle, plain C part -- TEST INFRASTRUCTURE ONLY.
 *
 * The same steps as the numpy oracle beside this file, as plain loops, so that
 * full-size layers finish in seconds and the benchmark can time a CPU baseline.
 * Nothing here is shared with, or called by, the HIP library.
 *
 * Notation: W is N x K, X is K x M, Y is N x M; sigma = +1/-1 sign of a weight
 * (Sec. III Eq. 1); c = integer activation value, +-1 for 1-bit activations,
 * the level index p in 0..3 for 2-bit ones (Sec. IV, "1/1" and "1/2").
 *
 *   int part, unpacked   D[n,m] = sum_k sigma[n,k]*c[k,m]
 *   int part, packed     Sec. IV Eq. 16 (xor + popcount) for 1 bit; for 2 bits the
 *                        bit-plane form sum_b 2^b (2*pc(w & P_b)) - colsum, which is
 *                        Eqs. 18-19 with the masks folded into the two planes
 *   sparse part          A^full * B of Sec. III Eqs. 12-13, float64
 *   epilogue             Y = alpha*s*D + R, float64, rounded once to float32
 *
 * Packed activation buffer: Kw = ceil(K/32), Mp = 64*ceil(M/64); uint32 planes
 * [bits][Kw][Mp], then int32 colsum[Mp]; bit i of word j <-> k = 32*j+i.
 * Sign words: uint32 [N][Kw], same bit order, bit 1 <-> +1, pad bits 0.
 */
#include <stdint.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int pc32(uint32_t v) { return __builtin_popcount(v); }

int apb_oracle_c_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void apb_oracle_c_int_unpacked(const uint8_t* bit, const int8_t* c, int N, int K, int M, int32_t* D) {
    for (int n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m) {
            int64_t acc = 0;
            for (int k = 0; k < K; ++k) {
                int sigma = bit[(size_t)n * K + k] ? 1 : -1;
                acc += sigma * (int)c[(size_t)k * M + m];
            }
            D[(size_t)n * M + m] = (int32_t)acc;
        }
}

void apb_oracle_c_int_packed(const uint32_t* sign_words, const uint32_t* packed, int N, int K, int M,
                             int bits, int32_t* D, int threads) {
    const int Kw = (K + 31) / 32;
    const size_t Mp = 64 * (size_t)((M + 63) / 64);
    const uint32_t* planes = packed;
    const int32_t* colsum = (const int32_t*)(packed + (size_t)bits * Kw * Mp);
    (void)threads;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int n = 0; n < N; ++n) {
        const uint32_t* w = sign_words + (size_t)n * Kw;
        for (int m = 0; m < M; ++m) {
            if (bits == 1) {
                int diff = 0;
                for (int j = 0; j < Kw; ++j) diff += pc32(w[j] ^ planes[(size_t)j * Mp + m]);
                D[(size_t)n * M + m] = K - 2 * diff;
            } else {
                int pos = 0;
                for (int b = 0; b < bits; ++b)
                    for (int j = 0; j < Kw; ++j)
                        pos += (1 << b) * pc32(w[j] & planes[((size_t)b * Kw + j) * Mp + m]);
                D[(size_t)n * M + m] = 2 * pos - colsum[m];
            }
        }
    }
}

void apb_oracle_c_sparse(const int32_t* row_ptr, const int32_t* col_idx, const float* val, const int8_t* c,
                         float step, int N, int M, double* R, int threads) {
    const double s = (double)step;
    (void)threads;
#pragma omp parallel for num_threads(threads) schedule(dynamic, 1)
    for (int n = 0; n < N; ++n) {
        double* r = R + (size_t)n * M;
        for (int m = 0; m < M; ++m) r[m] = 0.0;
        for (int j = row_ptr[n]; j < row_ptr[n + 1]; ++j) {
            const double v = (double)val[j];
            const int8_t* x = c + (size_t)col_idx[j] * M;
            for (int m = 0; m < M; ++m) r[m] += v * ((double)x[m] * s);
        }
    }
}

void apb_oracle_c_epilogue(float alpha, float step, const int32_t* D, const double* R, size_t count, float* Y) {
    const double as = (double)alpha * (double)step;
    for (size_t i = 0; i < count; ++i) Y[i] = (float)(as * (double)D[i] + R[i]);
}

/* Steps 3-5 in one call (what the benchmark's CPU-baseline leg times). R is caller scratch, N*M doubles. */
void apb_oracle_c_forward(const uint32_t* sign_words, const int32_t* row_ptr, const int32_t* col_idx,
                          const float* val, float alpha, const uint32_t* packed, const int8_t* c, int N, int K,
                          int M, int bits, float step, int32_t* D, double* R, float* Y, int threads) {
    apb_oracle_c_int_packed(sign_words, packed, N, K, M, bits, D, threads);
    apb_oracle_c_sparse(row_ptr, col_idx, val, c, step, N, M, R, threads);
    apb_oracle_c_epilogue(alpha, step, D, R, (size_t)N * M, Y);
}
