// Register-only instruction-rate probes: what this chip sustains for the instruction mixes the forward
// kernels are made of, measured rather than taken from a data sheet.  Each kernel keeps 8 waves per SIMD
// busy with one mix in an unrolled loop and writes one word per lane at the end, so nothing but the
// instruction issue is timed.  The benchmark divides the work below by the kernel time.
#include "apb_fp4_expand.h"
#include "apb_internal.h"

namespace apb {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kBlocks = 256 * 8;       // 8 workgroups of 4 waves on each of the 256 compute units
constexpr int kThreads = 256;

// FP4 matrix instruction, 32x32x64: 4 independent accumulator tiles per wave.
__global__ __launch_bounds__(kThreads) void k_probe_mfma_fp4(int iters, int seed, float* out) {
    v8i a, b;
#pragma unroll
    for (int d = 0; d < 8; ++d) {
        a[d] = d < 4 ? (int)((seed * 0x9e3779b9u + threadIdx.x * 7u + d) & kNib) : 0;
        b[d] = d < 4 ? (int)((seed * 0x85ebca6bu + threadIdx.x * 13u + d) & (kNib * 3u)) : 0;
    }
    v16f c[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) c[t][r] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 4; ++t) c[t] = mfma_fp4(a, b, c[t]);
    }
    float s = 0.0f;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += c[t][r];
    out[blockIdx.x * kThreads + threadIdx.x] = s;
}

// int8 matrix instruction, 32x32x32.
__global__ __launch_bounds__(kThreads) void k_probe_mfma_i8(int iters, int seed, int* out) {
    v4i a = {seed, seed + 1, seed + 2, seed + 3}, b = {seed * 3, seed * 5, seed * 7, seed * 11};
    v16i c[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) c[t][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 4; ++t) c[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c[t], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += c[t][r];
    out[blockIdx.x * kThreads + threadIdx.x] = s;
}

// The popcount formulation's pair: one logic op + one accumulating popcount per 32 binary products.
// 16 pairs per loop pass (plus one multiply-add of bookkeeping, not counted as work).
__global__ __launch_bounds__(kThreads) void k_probe_and_bcnt(int iters, int seed, uint32_t* out) {
    uint32_t x = (uint32_t)seed + threadIdx.x, a[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) a[i] = i;
    const uint32_t w = (uint32_t)seed * 2654435761u;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) a[i] += __builtin_popcount((w + i * 0x9e3779b9u) & x);
        x = x * 3 + 1;
    }
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += a[i];
    out[blockIdx.x * kThreads + threadIdx.x] = s;
}

// float64 fused multiply-add on the vector ALU: 16 independent chains.
__global__ __launch_bounds__(kThreads) void k_probe_fma_f64(int iters, int seed, double* out) {
    double a[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) a[i] = i;
    const double x = 1.0 + (seed + threadIdx.x) * 1e-9;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) a[i] = fma(a[i], x, 1.0);
    }
    double s = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += a[i];
    out[blockIdx.x * kThreads + threadIdx.x] = s;
}

// Byte reads from an LDS table whose rows (one per lane) are 260 bytes apart, all lanes reading the same
// column: the access pattern of the residual loop's code table.
__global__ __launch_bounds__(kThreads) void k_probe_lds_u8(int iters, int seed, uint32_t* out) {
    __shared__ uint8_t t[64 * 260];
    for (int i = threadIdx.x; i < 64 * 260; i += kThreads) t[i] = (uint8_t)(i * 7 + seed);
    __syncthreads();
    const uint8_t* row = t + (threadIdx.x & 63) * 260;
    uint32_t s = 0;
    int c = seed & 255;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) s += row[(c + i * 13) & 255];
        c = __builtin_amdgcn_readfirstlane((c * 5 + 1) & 255);
    }
    out[blockIdx.x * kThreads + threadIdx.x] = s;
}


// The loop skeleton of the matrix-core kernel whose waves share an operand through LDS, piece by piece:
//   kLds            four 16-byte LDS reads per lane and pass, nothing else (bytes / s)
//   kLdsMfma        those reads feed four FP4 matrix instructions
//   kLdsMfmaBarrier ... and every pass ends with a 16-byte LDS write and a workgroup barrier
//   kLdsMfmaBarrierValu ... with 32 vector-ALU instructions (the operand expansion's mix) in the shadow as well
enum LdsMode { kLds = 0, kLdsMfma = 1, kLdsMfmaBarrier = 2, kLdsMfmaBarrierValu = 3 };

template <int MODE>
__global__ __launch_bounds__(kThreads) void k_probe_mfma_lds(int iters, int seed, uint32_t* out) {
    typedef uint32_t v4u __attribute__((ext_vector_type(4)));
    __shared__ v4u buf[4][4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < 4 * 4 * 64; i += kThreads)
        (&buf[0][0][0])[i] = v4u{(uint32_t)(i * 7 + seed) & kNib, (uint32_t)i & kNib, 0u, kNib};
    __syncthreads();
    v16f c[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) c[t][r] = 0.0f;
    v8i a;
#pragma unroll
    for (int d = 0; d < 8; ++d) a[d] = d < 4 ? (int)((seed * 0x9e3779b9u + threadIdx.x * 7u + d) & kNib) : 0;
    uint32_t x[8], acc = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) x[j] = lane * 77u + j + seed;
    for (int it = 0; it < iters; ++it) {
        int idx = it & 3;
        asm volatile("" : "+v"(idx));                           // (keeps the reads inside the loop)
        v4u b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) b[u] = buf[idx][u][lane];
        if (MODE == kLdsMfmaBarrierValu) {
#pragma unroll
            for (int j = 0; j < 16; ++j) x[j & 7] = ((x[j & 7] >> 1) & kNib) | (x[(j + 1) & 7] & (kNib << 1));
        }
        if (MODE >= kLdsMfmaBarrier) buf[(idx + 1) & 3][wave][lane] = v4u{x[0], x[1], x[2], x[3]};
        if (MODE == kLds) {
#pragma unroll
            for (int u = 0; u < 4; ++u) acc ^= b[u][0] ^ b[u][1] ^ b[u][2] ^ b[u][3];
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const v8i fb = {(int)b[u][0], (int)b[u][1], (int)b[u][2], (int)b[u][3], 0, 0, 0, 0};
                c[u] = mfma_fp4(a, fb, c[u]);
            }
        }
        if (MODE >= kLdsMfmaBarrier) __syncthreads();
    }
    float s = 0.0f;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += c[t][r];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc ^= x[j];
    out[blockIdx.x * kThreads + threadIdx.x] = acc ^ (uint32_t)s;
}

}  // namespace
}  // namespace apb

using namespace apb;

extern "C" {

size_t apb_probe_out_bytes(void) { return (size_t)kBlocks * kThreads * sizeof(double); }

int apb_probe_rate(int kind, int iters, void* out, double* work_per_launch, void* stream) {
    if (!out || !work_per_launch) return APB_ERR_NULL;
    if (iters <= 0 || iters > (1 << 20)) return APB_ERR_SHAPE;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const double lanes = (double)kBlocks * kThreads, waves = lanes / kWave;
    switch (kind) {
        case APB_PROBE_MFMA_FP4:
            hipLaunchKernelGGL(k_probe_mfma_fp4, dim3(kBlocks), dim3(kThreads), 0, s, iters, 3, static_cast<float*>(out));
            *work_per_launch = waves * iters * 4.0 * 2.0 * 32 * 32 * 64;
            break;
        case APB_PROBE_MFMA_I8:
            hipLaunchKernelGGL(k_probe_mfma_i8, dim3(kBlocks), dim3(kThreads), 0, s, iters, 3, static_cast<int*>(out));
            *work_per_launch = waves * iters * 4.0 * 2.0 * 32 * 32 * 32;
            break;
        case APB_PROBE_AND_BCNT:
            hipLaunchKernelGGL(k_probe_and_bcnt, dim3(kBlocks), dim3(kThreads), 0, s, iters, 12345, static_cast<uint32_t*>(out));
            *work_per_launch = lanes * iters * 32.0;      // the pairs alone; the loop's own bookkeeping is not counted
            break;
        case APB_PROBE_FMA_F64:
            hipLaunchKernelGGL(k_probe_fma_f64, dim3(kBlocks), dim3(kThreads), 0, s, iters, 5, static_cast<double*>(out));
            *work_per_launch = lanes * iters * 16.0;
            break;
        case APB_PROBE_LDS_U8:
            hipLaunchKernelGGL(k_probe_lds_u8, dim3(kBlocks), dim3(kThreads), 0, s, iters, 9, static_cast<uint32_t*>(out));
            *work_per_launch = lanes * iters * 16.0;
            break;
        case APB_PROBE_LDS_B128:
            hipLaunchKernelGGL(k_probe_mfma_lds<kLds>, dim3(kBlocks), dim3(kThreads), 0, s, iters, 7, static_cast<uint32_t*>(out));
            *work_per_launch = lanes * iters * 4.0 * 16.0;                       // bytes
            break;
        case APB_PROBE_MFMA_FP4_LDS:
            hipLaunchKernelGGL(k_probe_mfma_lds<kLdsMfma>, dim3(kBlocks), dim3(kThreads), 0, s, iters, 7, static_cast<uint32_t*>(out));
            *work_per_launch = waves * iters * 4.0 * 2.0 * 32 * 32 * 64;
            break;
        case APB_PROBE_MFMA_FP4_LDS_BARRIER:
            hipLaunchKernelGGL(k_probe_mfma_lds<kLdsMfmaBarrier>, dim3(kBlocks), dim3(kThreads), 0, s, iters, 7,
                               static_cast<uint32_t*>(out));
            *work_per_launch = waves * iters * 4.0 * 2.0 * 32 * 32 * 64;
            break;
        case APB_PROBE_MFMA_FP4_LDS_BARRIER_VALU:
            hipLaunchKernelGGL(k_probe_mfma_lds<kLdsMfmaBarrierValu>, dim3(kBlocks), dim3(kThreads), 0, s, iters, 7,
                               static_cast<uint32_t*>(out));
            *work_per_launch = waves * iters * 4.0 * 2.0 * 32 * 32 * 64;
            break;
        default:
            return APB_ERR_VALUE;
    }
    APB_HIP(hipGetLastError());
    return APB_OK;
}

}  // extern "C"
