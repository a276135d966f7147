// apb_quantize_acts: quantize K x M float activations to 1 or 2 bits (Sec. IV, "1/1": +-beta;
// "1/2": a_p = p*s, p in 0..3) and pack them K-wise into bit-planes [bits][Kw][Mp], plus the
// per-column code sums (the Theta(n^2) term hoisted out of the product, Sec. IV "1/2").
//
// HBM-bound: reads 4*K*M bytes once, writes bits*K*M/8.  Lanes run along m.  In the main kernel a
// lane owns four adjacent columns, so every load is a 16-byte vector and a wave's load covers one
// contiguous kilobyte of a row of X; a lane builds, for 32 consecutive k, four words per plane and
// stores them as one 16-byte vector.  A workgroup of four waves walks a slab of K for one strip of
// 256 columns, adds its per-column code sums up in LDS and writes them once -- with a plain store
// when the slab is all of K (no zero-fill launch, no atomics), with an integer atomic otherwise.
#include "apb_internal.h"

namespace apb {

namespace {

constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kColsPerLane = 4;
constexpr int kStrip = kWave * kColsPerLane;                   // columns per workgroup

__global__ __launch_bounds__(kBlock) void k_zero_i32(int32_t* __restrict__ p, int count) {
    const int i = blockIdx.x * kBlock + threadIdx.x;
    if (i < count) p[i] = 0;
}

// p = clamp(rint(x / s), 0, 3): one float multiply by the precomputed 1/s, ties to even; NaN -> 0.
__device__ __forceinline__ uint32_t code2(float x, float inv_step) {
    return (uint32_t)(int)fminf(3.0f, fmaxf(0.0f, rintf(x * inv_step)));
}

// Main kernel: needs M % 4 == 0 (16-byte aligned rows of X).
template <int BITS>
__global__ __launch_bounds__(kBlock) void k_quantize_pack4(const float* __restrict__ X, int K, int M, int Kw,
                                                           int Mp, float inv_step, int words_per_slab,
                                                           uint32_t* __restrict__ planes,
                                                           int32_t* __restrict__ colsum) {
    __shared__ int s_sum[kWavesPerBlock][kStrip];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int m0 = blockIdx.x * kStrip + lane * kColsPerLane;      // first of this lane's four columns
    const bool col_ok = m0 < M;                                     // M % 4 == 0: all four or none
    const int j_begin = blockIdx.y * words_per_slab;
    const int j_end = min(Kw, j_begin + words_per_slab);
    int sum[kColsPerLane] = {0, 0, 0, 0};

    for (int j = j_begin + wave; j < j_end; j += kWavesPerBlock) {
        uint32_t w0[kColsPerLane] = {0, 0, 0, 0}, w1[kColsPerLane] = {0, 0, 0, 0};
        const int k0 = j * 32;
        // Loads are unconditional (addresses clamped into the matrix, results masked afterwards):
        // a branch around each load would make every load wait for the one before.
        const float* src = X + min(m0, M - kColsPerLane);
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            float4 xv[16];                                       // 16 independent 16-byte loads in flight
#pragma unroll
            for (int i = 0; i < 16; ++i)
                xv[i] = *reinterpret_cast<const float4*>(src + (size_t)min(k0 + 16 * half + i, K - 1) * M);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float xs[kColsPerLane] = {xv[i].x, xv[i].y, xv[i].z, xv[i].w};
                const int bit = 16 * half + i;
#pragma unroll
                for (int q = 0; q < kColsPerLane; ++q) {
                    if (BITS == 1) {
                        w0[q] |= (xs[q] >= 0.0f ? 1u : 0u) << bit;
                    } else {
                        const uint32_t p = code2(xs[q], inv_step);
                        w0[q] |= (p & 1u) << bit;
                        w1[q] |= (p >> 1) << bit;
                    }
                }
            }
        }
        // Bits of k >= K (last word) and of columns >= M are cleared here, in one go; the code sums
        // come from popcounts of the finished words.
        const int valid = K - k0;
        const uint32_t keep = !col_ok ? 0u : (valid >= 32 ? 0xffffffffu : ((1u << valid) - 1u));
#pragma unroll
        for (int q = 0; q < kColsPerLane; ++q) {
            w0[q] &= keep;
            w1[q] &= keep;
            sum[q] += __builtin_popcount(w0[q]) + 2 * __builtin_popcount(w1[q]);
        }
        if (m0 < Mp) {
            *reinterpret_cast<uint4*>(planes + (size_t)j * Mp + m0) = make_uint4(w0[0], w0[1], w0[2], w0[3]);
            if (BITS == 2)
                *reinterpret_cast<uint4*>(planes + ((size_t)Kw + j) * Mp + m0) = make_uint4(w1[0], w1[1], w1[2], w1[3]);
        }
    }
#pragma unroll
    for (int q = 0; q < kColsPerLane; ++q) s_sum[wave][lane * kColsPerLane + q] = sum[q];
    __syncthreads();
    const int m = blockIdx.x * kStrip + threadIdx.x;                // one column per thread now
    if (m < Mp) {
        int total = 0;
#pragma unroll
        for (int w = 0; w < kWavesPerBlock; ++w) total += s_sum[w][threadIdx.x];
        if (gridDim.y == 1) colsum[m] = total;
        else if (total != 0) atomicAdd(&colsum[m], total);
    }
}

// Fallback for M % 4 != 0: one column per lane, one word of K per wave, atomics into a zeroed colsum.
template <int BITS>
__global__ __launch_bounds__(kBlock) void k_quantize_pack1(const float* __restrict__ X, int K, int M, int Kw,
                                                           int Mp, float inv_step,
                                                           uint32_t* __restrict__ planes,
                                                           int32_t* __restrict__ colsum) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int m = blockIdx.x * kWave + lane;
    const int j = blockIdx.y * kWavesPerBlock + wave;          // word index along K
    if (j >= Kw) return;
    const bool col_ok = m < M;
    const int k0 = j * 32;
    uint32_t w0 = 0, w1 = 0;
    int sum = 0;
    const float* src = X + (size_t)k0 * M + m;
#pragma unroll 8
    for (int i = 0; i < 32; ++i) {
        const bool ok = col_ok && (k0 + i) < K;
        const float x = ok ? src[(size_t)i * M] : -1.0f;
        if (BITS == 1) {
            const uint32_t b = (ok && x >= 0.0f) ? 1u : 0u;
            w0 |= b << i;
            sum += (int)b;
        } else {
            const uint32_t p = ok ? code2(x, inv_step) : 0u;
            w0 |= (p & 1u) << i;
            w1 |= (p >> 1) << i;
            sum += (int)p;
        }
    }
    planes[(size_t)j * Mp + m] = w0;
    if (BITS == 2) planes[((size_t)Kw + j) * Mp + m] = w1;
    if (col_ok && sum != 0) atomicAdd(&colsum[m], sum);
}

}  // namespace

int launch_quantize(const float* X, int K, int M, int bits, float inv_step, uint32_t* planes, int32_t* colsum,
                    hipStream_t s) {
    const int Kw = (K + 31) / 32;
    const int Mp = kWave * ((M + kWave - 1) / kWave);
    auto zero_colsum = [&]() {
        hipLaunchKernelGGL(k_zero_i32, dim3((Mp + kBlock - 1) / kBlock), dim3(kBlock), 0, s, colsum, Mp);
    };
    if (M % kColsPerLane == 0 && ((reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(planes)) & 15u) == 0) {
        const int strips = (Mp + kStrip - 1) / kStrip;
        // Split K into slabs only when the strips alone cannot fill the chip (256 CUs x 8 waves).
        int slabs = 1;
        while ((long long)strips * kWavesPerBlock * slabs < 2048 && slabs * kWavesPerBlock < Kw) slabs *= 2;
        const int words_per_slab = (Kw + slabs - 1) / slabs;
        slabs = (Kw + words_per_slab - 1) / words_per_slab;
        if (slabs > 1) {
            zero_colsum();
            APB_HIP(hipGetLastError());
        }
        const dim3 grid(strips, slabs);
        if (bits == 1)
            hipLaunchKernelGGL(k_quantize_pack4<1>, grid, dim3(kBlock), 0, s, X, K, M, Kw, Mp, inv_step, words_per_slab,
                               planes, colsum);
        else
            hipLaunchKernelGGL(k_quantize_pack4<2>, grid, dim3(kBlock), 0, s, X, K, M, Kw, Mp, inv_step, words_per_slab,
                               planes, colsum);
    } else {
        zero_colsum();
        APB_HIP(hipGetLastError());
        const dim3 grid(Mp / kWave, (Kw + kWavesPerBlock - 1) / kWavesPerBlock);
        if (bits == 1)
            hipLaunchKernelGGL(k_quantize_pack1<1>, grid, dim3(kBlock), 0, s, X, K, M, Kw, Mp, inv_step, planes, colsum);
        else
            hipLaunchKernelGGL(k_quantize_pack1<2>, grid, dim3(kBlock), 0, s, X, K, M, Kw, Mp, inv_step, planes, colsum);
    }
    APB_HIP(hipGetLastError());
    return APB_OK;
}

}  // namespace apb
