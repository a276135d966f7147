// Kernels behind apb_compress: the partition of Sec. III Eq. 3, the sign bits of Eq. 1 packed
// for every weight ("fully represented" binary matrix), and the CSR of residuals of Eq. 12.
#include "apb_internal.h"

namespace apb {

namespace {

constexpr int kBlock = 256;

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// Sum of |w| and count over the binarized set {|w| <= delta}; one (sum, count) pair per block.
__global__ __launch_bounds__(kBlock) void k_inlier_abs_sum(const float* __restrict__ W, long long count,
                                                           float delta, double* __restrict__ part_sum,
                                                           long long* __restrict__ part_cnt) {
    __shared__ double s_sum[kBlock / kWave];
    __shared__ long long s_cnt[kBlock / kWave];
    double sum = 0.0;
    long long cnt = 0;
    const long long stride = (long long)gridDim.x * kBlock;
    for (long long i = (long long)blockIdx.x * kBlock + threadIdx.x; i < count; i += stride) {
        const float a = fabsf(W[i]);
        if (!(a > delta)) {
            sum += (double)a;
            ++cnt;
        }
    }
    for (int off = kWave / 2; off > 0; off >>= 1) {
        sum += __shfl_down(sum, off, kWave);
        cnt += __shfl_down(cnt, off, kWave);
    }
    if (lane_id() == 0) {
        s_sum[threadIdx.x / kWave] = sum;
        s_cnt[threadIdx.x / kWave] = cnt;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        long long c = 0;
        for (int w = 0; w < kBlock / kWave; ++w) {
            t += s_sum[w];
            c += s_cnt[w];
        }
        part_sum[blockIdx.x] = t;
        part_cnt[blockIdx.x] = c;
    }
}

// One block per weight row: ballot-pack the sign bits (bit 1 <-> w >= 0), count the residuals
// and sum the signs.  A wave's 64-bit ballot is exactly two output words.
__global__ __launch_bounds__(kBlock) void k_sign_pack_count(const float* __restrict__ W, int K, int Kw,
                                                            float delta, uint32_t* __restrict__ sign,
                                                            int32_t* __restrict__ counts,
                                                            int32_t* __restrict__ rowsum) {
    __shared__ int s_out[kBlock / kWave];
    __shared__ int s_pos[kBlock / kWave];
    const int n = blockIdx.x;
    const float* row = W + (size_t)n * K;
    uint32_t* srow = sign + (size_t)n * Kw;
    const int wave = threadIdx.x / kWave;
    int n_out = 0, n_pos = 0;
    for (int c0 = 0; c0 < K; c0 += kBlock) {
        const int k = c0 + threadIdx.x;
        const bool in = k < K;
        const float w = in ? row[k] : -1.0f;
        const unsigned long long pos = __ballot(in && w >= 0.0f);
        const unsigned long long out = __ballot(in && fabsf(w) > delta);
        n_pos += __popcll(pos);
        n_out += __popcll(out);
        if (lane_id() == 0) {
            const int j = (c0 + wave * kWave) / 32;
            if (j < Kw) srow[j] = (uint32_t)pos;
            if (j + 1 < Kw) srow[j + 1] = (uint32_t)(pos >> 32);
        }
    }
    if (lane_id() == 0) {
        s_out[wave] = n_out;
        s_pos[wave] = n_pos;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int o = 0, p = 0;
        for (int w = 0; w < kBlock / kWave; ++w) {
            o += s_out[w];
            p += s_pos[w];
        }
        counts[n] = o;
        rowsum[n] = 2 * p - K;
    }
}

// One wave per row: residuals in ascending column order via ballot + lane prefix count.
__global__ __launch_bounds__(kBlock) void k_scatter_csr(const float* __restrict__ W, int N, int K, float delta,
                                                        float alpha, const int32_t* __restrict__ row_ptr,
                                                        int32_t* __restrict__ col_idx, float* __restrict__ val,
                                                        double* __restrict__ vald) {
    const int n = blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
    if (n >= N) return;
    const float* row = W + (size_t)n * K;
    const int lane = lane_id();
    int base = row_ptr[n];
    for (int c0 = 0; c0 < K; c0 += kWave) {
        const int k = c0 + lane;
        const bool in = k < K;
        const float w = in ? row[k] : 0.0f;
        const bool out = in && fabsf(w) > delta;
        const unsigned long long mask = __ballot(out);
        if (out) {
            const int before = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                         __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
            const float signed_alpha = (w >= 0.0f) ? alpha : -alpha;
            col_idx[base + before] = k;
            const float residual = w - signed_alpha;        // one float subtraction (Eq. 12)
            val[base + before] = residual;
            vald[base + before] = (double)residual;
        }
        base += __popcll(mask);
    }
}

// signT[j][i] = word j of the row served by launch slot i (0 for padding slots).
__global__ __launch_bounds__(kBlock) void k_slot_major_signs(const uint32_t* __restrict__ sign,
                                                             const int32_t* __restrict__ perm, int Np, int Kw,
                                                             int rows_out, uint32_t* __restrict__ signT) {
    const long long t = (long long)blockIdx.x * kBlock + threadIdx.x;
    if (t >= (long long)Np * rows_out) return;
    const int j = (int)(t / Np), i = (int)(t % Np);
    const int n = perm ? perm[i] : i;                          // no permutation: plain transpose
    signT[t] = (n >= 0 && j < Kw) ? sign[(size_t)n * Kw + j] : 0u;   // word rows past Kw are zero padding
}

// Sec. IV "2/2": level index q = clamp(floor(w / s_w) + 2, 0, 3) of every weight (the weight it
// stands for is (q - 3/2) * s_w), packed as two bit-planes.  One thread per (row, word): it reads
// its 32 weights and writes the word of each plane twice, in the canonical [2][N][Kw] order and in
// the word-major [2][Kw2][N] order the matrix-core kernel reads (pad word row = 0).  Offline work.
__global__ __launch_bounds__(kBlock) void k_w2_pack(const float* __restrict__ W, int N, int K, int Kw, int Kw2,
                                                    float inv_step, uint32_t* __restrict__ planes,
                                                    uint32_t* __restrict__ planesC) {
    const long long t = (long long)blockIdx.x * kBlock + threadIdx.x;
    if (t >= (long long)N * Kw2) return;
    const int j = (int)(t / N), n = (int)(t % N);
    uint32_t w0 = 0, w1 = 0;
    if (j < Kw) {
        const float* src = W + (size_t)n * K + 32 * j;
        const int valid = min(32, K - 32 * j);
        for (int i = 0; i < valid; ++i) {
            const uint32_t q = (uint32_t)(int)fminf(3.0f, fmaxf(0.0f, floorf(src[i] * inv_step) + 2.0f));
            w0 |= (q & 1u) << i;
            w1 |= (q >> 1) << i;
        }
        planes[(size_t)n * Kw + j] = w0;
        planes[((size_t)N + n) * Kw + j] = w1;
    }
    planesC[(size_t)j * N + n] = w0;
    planesC[((size_t)Kw2 + j) * N + n] = w1;
}

// chunk_ptr[c][i]: index of the first residual of the row in slot i whose column is >= 256*c
// (lower bound in the ascending column list); slot_valsum[i]: float64 sum of that row's residuals.
__global__ __launch_bounds__(kBlock) void k_slot_tables(const int32_t* __restrict__ perm,
                                                        const int32_t* __restrict__ row_ptr,
                                                        const int32_t* __restrict__ col_idx,
                                                        const float* __restrict__ val, int Np, int nchunks,
                                                        int32_t* __restrict__ chunk_ptr,
                                                        double* __restrict__ slot_valsum) {
    const long long t = (long long)blockIdx.x * kBlock + threadIdx.x;
    if (t >= (long long)Np * (nchunks + 1)) return;
    const int c = (int)(t / Np), i = (int)(t % Np);
    const int n = perm[i];
    if (n < 0) {
        chunk_ptr[t] = 0;
        if (c == 0) slot_valsum[i] = 0.0;
        return;
    }
    int lo = row_ptr[n], hi = row_ptr[n + 1];
    if (c == 0) {
        double sum = 0.0;
        for (int q = lo; q < hi; ++q) sum += (double)val[q];
        slot_valsum[i] = sum;
    }
    const int bound = c * kChunkK;
    while (lo < hi) {
        const int mid = lo + (hi - lo) / 2;
        if (col_idx[mid] < bound) lo = mid + 1; else hi = mid;
    }
    chunk_ptr[t] = lo;
}

}  // namespace

int launch_slot_tables(const int32_t* perm, const int32_t* row_ptr, const int32_t* col_idx, const float* val, int Np,
                       int nchunks, int32_t* chunk_ptr, double* slot_valsum, hipStream_t s) {
    const long long total = (long long)Np * (nchunks + 1);
    hipLaunchKernelGGL(k_slot_tables, dim3((unsigned)((total + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, perm,
                       row_ptr, col_idx, val, Np, nchunks, chunk_ptr, slot_valsum);
    APB_HIP(hipGetLastError());
    return APB_OK;
}

int launch_inlier_abs_sum(const float* W, long long count, float delta, double* part_sum, long long* part_cnt,
                          int parts, hipStream_t s) {
    hipLaunchKernelGGL(k_inlier_abs_sum, dim3(parts), dim3(kBlock), 0, s, W, count, delta, part_sum, part_cnt);
    APB_HIP(hipGetLastError());
    return APB_OK;
}

int launch_w2_pack(const float* W, int N, int K, float inv_step, uint32_t* planes, uint32_t* planesC, hipStream_t s) {
    const int Kw = (K + 31) / 32, Kw2 = 2 * ((Kw + 1) / 2);
    const long long total = (long long)N * Kw2;
    hipLaunchKernelGGL(k_w2_pack, dim3((unsigned)((total + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, W, N, K, Kw,
                       Kw2, inv_step, planes, planesC);
    APB_HIP(hipGetLastError());
    return APB_OK;
}

int launch_sign_pack_count(const float* W, int N, int K, int Kw, float delta, uint32_t* sign, int32_t* counts,
                           int32_t* rowsum, hipStream_t s) {
    hipLaunchKernelGGL(k_sign_pack_count, dim3(N), dim3(kBlock), 0, s, W, K, Kw, delta, sign, counts, rowsum);
    APB_HIP(hipGetLastError());
    return APB_OK;
}

int launch_scatter_csr(const float* W, int N, int K, float delta, float alpha, const int32_t* row_ptr,
                       int32_t* col_idx, float* val, double* vald, hipStream_t s) {
    const int rows_per_block = kBlock / kWave;
    hipLaunchKernelGGL(k_scatter_csr, dim3((N + rows_per_block - 1) / rows_per_block), dim3(kBlock), 0, s, W, N,
                       K, delta, alpha, row_ptr, col_idx, val, vald);
    APB_HIP(hipGetLastError());
    return APB_OK;
}

int launch_slot_major_signs(const uint32_t* sign, const int32_t* perm, int Np, int Kw, int rows_out,
                            uint32_t* signT, hipStream_t s) {
    const long long total = (long long)Np * rows_out;
    hipLaunchKernelGGL(k_slot_major_signs, dim3((unsigned)((total + kBlock - 1) / kBlock)), dim3(kBlock), 0, s,
                       sign, perm, Np, Kw, rows_out, signT);
    APB_HIP(hipGetLastError());
    return APB_OK;
}

}  // namespace apb
