// Training-side operators of APB (Sec. III Eqs. 3-9) for one layer's latent weights:
//   forward   out[i] = APB(w[i]) = sign(w[i]) * alpha  if |w[i]| <= alpha + delta,  w[i] otherwise   (Eq. 3)
//   backward  grad_w = g (Eq. 4 with the identity as surrogate: the straight-through gradient), and the two
//             masked reductions over the binarized set chi_B = 1(|w| <= alpha + delta) (Eq. 6), with
//             dL/dw_hat = delta * sign(w) * g (Eq. 9):
//                 dL/ddelta =  1 / (delta^2 n) * sum dL/dw_hat * (alpha - |w|) * chi_B          (Eq. 7)
//                 dL/dalpha = -1 / (delta n)   * sum dL/dw_hat * chi_B                          (Eq. 8)
// Both are one pass over the weights: HBM-bound (forward 8 bytes per weight, backward 12, or 8 without
// grad_w).  The sums are float64 and deterministic: every workgroup reduces a fixed slice in a fixed order
// into one slot of the workspace, and a second, single-workgroup launch adds the slots in order.
#include <algorithm>
#include <cmath>

#include "apb_internal.h"

namespace apb {
namespace {

constexpr int kTrainThreads = 256;
constexpr int kTrainBlocks = 2048;                 // 8 workgroups of 4 waves per compute unit
constexpr int kPartials = 3;                       // sum for alpha, sum for delta, size of the binarized set

struct f4 {
    float x, y, z, w;
};

__device__ __forceinline__ float apb_of(float w, float alpha, float lim) {
    return fabsf(w) <= lim ? (w >= 0.0f ? alpha : -alpha) : w;
}

// VEC: 4 weights per load (pointers 16-byte aligned and n a multiple of 4) or 1.  Every lane keeps kUnroll loads
// in flight (each array is used exactly once: non-temporal, so that the stream does not push other data out of
// the caches).
constexpr int kUnroll = 4;

template <int VEC>
__global__ __launch_bounds__(kTrainThreads) void k_apb_operator(const float* __restrict__ W, long long n, float alpha,
                                                               float lim, float* __restrict__ out) {
    const long long stride = (long long)gridDim.x * kTrainThreads;
    const long long items = n / VEC;
    long long i = (long long)blockIdx.x * kTrainThreads + threadIdx.x;
    if (VEC == 4) {
        for (; i + (kUnroll - 1) * stride < items; i += kUnroll * stride) {
            f4 w[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const f4* src = reinterpret_cast<const f4*>(W) + i + u * stride;
                w[u].x = __builtin_nontemporal_load(&src->x);
                w[u].y = __builtin_nontemporal_load(&src->y);
                w[u].z = __builtin_nontemporal_load(&src->z);
                w[u].w = __builtin_nontemporal_load(&src->w);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                f4 o;
                o.x = apb_of(w[u].x, alpha, lim);
                o.y = apb_of(w[u].y, alpha, lim);
                o.z = apb_of(w[u].z, alpha, lim);
                o.w = apb_of(w[u].w, alpha, lim);
                reinterpret_cast<f4*>(out)[i + u * stride] = o;
            }
        }
    }
    for (; i < items; i += stride) {
        if (VEC == 4) {
            const f4 w = reinterpret_cast<const f4*>(W)[i];
            f4 o;
            o.x = apb_of(w.x, alpha, lim);
            o.y = apb_of(w.y, alpha, lim);
            o.z = apb_of(w.z, alpha, lim);
            o.w = apb_of(w.w, alpha, lim);
            reinterpret_cast<f4*>(out)[i] = o;
        } else {
            out[i] = apb_of(W[i], alpha, lim);
        }
    }
}

struct Sums {
    double s_alpha, s_delta;
    long long count;
};

__device__ __forceinline__ void add_term(float w, float g, double alpha, double delta, float lim, Sums& s) {
    if (fabsf(w) <= lim) {                                       // chi_B
        const double t = delta * (w >= 0.0f ? 1.0 : -1.0) * (double)g;      // dL/dw_hat, Eq. 9
        s.s_alpha += t;
        s.s_delta += t * (alpha - (double)fabsf(w));
        s.count += 1;
    }
}

template <int VEC>
__global__ __launch_bounds__(kTrainThreads) void k_apb_backward(const float* __restrict__ W, const float* __restrict__ G,
                                                               long long n, float alpha, float delta, float lim,
                                                               float* __restrict__ grad_w, double* __restrict__ partial) {
    __shared__ double red[kTrainThreads / kWave][kPartials];
    Sums s{0.0, 0.0, 0};
    const long long stride = (long long)gridDim.x * kTrainThreads;
    const long long items = n / VEC;
    // (one load of each array per pass: two in flight per lane measured slower here)
    long long i = (long long)blockIdx.x * kTrainThreads + threadIdx.x;
    for (; i < items; i += stride) {
        if (VEC == 4) {
            const f4 w = reinterpret_cast<const f4*>(W)[i];
            const f4 g = reinterpret_cast<const f4*>(G)[i];
            if (grad_w) reinterpret_cast<f4*>(grad_w)[i] = g;    // straight-through
            add_term(w.x, g.x, alpha, delta, lim, s);
            add_term(w.y, g.y, alpha, delta, lim, s);
            add_term(w.z, g.z, alpha, delta, lim, s);
            add_term(w.w, g.w, alpha, delta, lim, s);
        } else {
            const float w = W[i], g = G[i];
            if (grad_w) grad_w[i] = g;
            add_term(w, g, alpha, delta, lim, s);
        }
    }
    // lanes of a wave, then the waves of the workgroup, always in the same order
    double v[kPartials] = {s.s_alpha, s.s_delta, (double)s.count};
#pragma unroll
    for (int q = 0; q < kPartials; ++q)
#pragma unroll
        for (int off = kWave / 2; off > 0; off >>= 1) v[q] += __shfl_xor(v[q], off, kWave);
    const int wave = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0)
#pragma unroll
        for (int q = 0; q < kPartials; ++q) red[wave][q] = v[q];
    __syncthreads();
    if (threadIdx.x < kPartials) {
        double t = 0.0;
        for (int w = 0; w < kTrainThreads / kWave; ++w) t += red[w][threadIdx.x];
        partial[(size_t)blockIdx.x * kPartials + threadIdx.x] = t;
    }
}

// One workgroup: adds the slots in order and applies the factors of Eqs. 7-8.
__global__ __launch_bounds__(kTrainThreads) void k_apb_backward_finish(const double* __restrict__ partial, int slots,
                                                                       long long n, float delta,
                                                                       double* __restrict__ grad_alpha_delta,
                                                                       long long* __restrict__ n_binarized) {
    __shared__ double red[kTrainThreads][kPartials];
    double v[kPartials] = {0.0, 0.0, 0.0};
    for (int i = threadIdx.x; i < slots; i += kTrainThreads)
#pragma unroll
        for (int q = 0; q < kPartials; ++q) v[q] += partial[(size_t)i * kPartials + q];
#pragma unroll
    for (int q = 0; q < kPartials; ++q) red[threadIdx.x][q] = v[q];
    __syncthreads();
    if (threadIdx.x == 0) {
        double t[kPartials] = {0.0, 0.0, 0.0};
        for (int i = 0; i < kTrainThreads; ++i)
#pragma unroll
            for (int q = 0; q < kPartials; ++q) t[q] += red[i][q];
        const double d = (double)delta, nn = (double)n;
        grad_alpha_delta[0] = -t[0] / (d * nn);                 // Eq. 8
        grad_alpha_delta[1] = t[1] / (d * d * nn);              // Eq. 7
        if (n_binarized) *n_binarized = (long long)t[2];        // exact: counts below 2^53
    }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace
}  // namespace apb

using namespace apb;

extern "C" {

size_t apb_train_workspace_bytes(void) { return (size_t)kTrainBlocks * kPartials * sizeof(double); }

int apb_train_forward(const float* W, long long n, float alpha, float delta, float* out, void* stream) {
    if (!W || !out) return APB_ERR_NULL;
    if (n <= 0 || n >= (1LL << 40)) return APB_ERR_SHAPE;
    if (!(alpha >= 0.0f) || !(delta >= 0.0f) || std::isinf(alpha) || std::isinf(delta)) return APB_ERR_VALUE;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const float lim = alpha + delta;                             // the interval's half-width is ONE float addition
    const bool vec = n % 4 == 0 && aligned16(W) && aligned16(out);
    const long long items = vec ? n / 4 : n;
    const int blocks = (int)std::min<long long>(kTrainBlocks * 4, (items + kTrainThreads - 1) / kTrainThreads);
    if (vec) hipLaunchKernelGGL(k_apb_operator<4>, dim3(blocks), dim3(kTrainThreads), 0, s, W, n, alpha, lim, out);
    else hipLaunchKernelGGL(k_apb_operator<1>, dim3(blocks), dim3(kTrainThreads), 0, s, W, n, alpha, lim, out);
    APB_HIP(hipGetLastError());
    return APB_OK;
}

int apb_train_backward(const float* W, const float* G, long long n, float alpha, float delta, float* grad_w,
                       double* grad_alpha_delta, long long* n_binarized, void* workspace, void* stream) {
    if (!W || !G || !grad_alpha_delta || !workspace) return APB_ERR_NULL;
    if (n <= 0 || n >= (1LL << 40)) return APB_ERR_SHAPE;
    if (!(alpha >= 0.0f) || !(delta > 0.0f) || std::isinf(alpha) || std::isinf(delta)) return APB_ERR_VALUE;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const float lim = alpha + delta;
    const bool vec = n % 4 == 0 && aligned16(W) && aligned16(G) && (!grad_w || aligned16(grad_w));
    const long long items = vec ? n / 4 : n;
    const int blocks = (int)std::min<long long>(kTrainBlocks, (items + kTrainThreads - 1) / kTrainThreads);
    double* partial = static_cast<double*>(workspace);
    if (vec)
        hipLaunchKernelGGL(k_apb_backward<4>, dim3(blocks), dim3(kTrainThreads), 0, s, W, G, n, alpha, delta, lim, grad_w,
                           partial);
    else
        hipLaunchKernelGGL(k_apb_backward<1>, dim3(blocks), dim3(kTrainThreads), 0, s, W, G, n, alpha, delta, lim, grad_w,
                           partial);
    hipLaunchKernelGGL(k_apb_backward_finish, dim3(1), dim3(kTrainThreads), 0, s, partial, blocks, n, delta,
                       grad_alpha_delta, n_binarized);
    APB_HIP(hipGetLastError());
    return APB_OK;
}

}  // extern "C"
