// apb_quantize_acts: quantize K x M float activations to 1 or 2 bits (Sec. IV, "1/1": +-beta;
// "1/2": a_p = p*s, p in 0..3) and pack them K-wise into bit-planes [bits][Kw][Mp], plus the
// per-column code sums (the Theta(n^2) term hoisted out of the product, Sec. IV "1/2").
//
// HBM-bound: reads 4*K*M bytes once, writes bits*K*M/8.  Lanes run along m, so every load is
// one contiguous 256-byte row segment per wave; each lane builds one 32-bit word per plane
// from 32 consecutive k and stores it (again contiguous across the wave).
#include "apb_internal.h"

namespace apb {

namespace {

constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / kWave;

__global__ __launch_bounds__(kBlock) void k_zero_i32(int32_t* __restrict__ p, int count) {
    const int i = blockIdx.x * kBlock + threadIdx.x;
    if (i < count) p[i] = 0;
}

template <int BITS>
__global__ __launch_bounds__(kBlock) void k_quantize_pack(const float* __restrict__ X, int K, int M, int Kw,
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
            // p = clamp(rint(x / s), 0, 3): one float multiply by the precomputed 1/s, ties to even.
            const float r = fminf(3.0f, fmaxf(0.0f, rintf(x * inv_step)));
            const uint32_t p = ok ? (uint32_t)(int)r : 0u;
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
    hipLaunchKernelGGL(k_zero_i32, dim3((Mp + kBlock - 1) / kBlock), dim3(kBlock), 0, s, colsum, Mp);
    APB_HIP(hipGetLastError());
    const dim3 grid(Mp / kWave, (Kw + kWavesPerBlock - 1) / kWavesPerBlock);
    if (bits == 1)
        hipLaunchKernelGGL(k_quantize_pack<1>, grid, dim3(kBlock), 0, s, X, K, M, Kw, Mp, inv_step, planes, colsum);
    else
        hipLaunchKernelGGL(k_quantize_pack<2>, grid, dim3(kBlock), 0, s, X, K, M, Kw, Mp, inv_step, planes, colsum);
    APB_HIP(hipGetLastError());
    return APB_OK;
}

}  // namespace apb
