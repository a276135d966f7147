// apb_forward: Y = alpha*s*D + s * sum_j val_j * c[col_j, :]   (Sec. III Eq. 13)
//
// Integer part D (Sec. IV Eq. 16 for 1-bit activations; for 2-bit ones the two stored bit-planes
// P0, P1 of the level index p stand in for the paper's (t, h, m) vectors of Eqs. 18-19:
//   D[n,m] = sum_k sigma[n,k]*p[k,m] = 2 * sum_b 2^b * popcount(w & P_b) - colsum[m]).
//
// Mapping: lanes run along m (one output column per lane), so a wave's activation word load is one
// contiguous 256-byte segment of a plane row, and the weight words of the kRowTile rows a wave owns
// are wave-uniform -> they travel through the scalar path and feed v_and/v_xor as SGPR operands.
// Per 32 binary multiply-adds the inner loop issues one logic op and one v_bcnt_u32_b32 (popcount
// with accumulate), the CDNA counterpart of the paper's xor/popcount/add port analysis.
#include "apb_internal.h"

namespace apb {

namespace {

constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / kWave;

template <int BITS, bool INT_ONLY>
__global__ __launch_bounds__(kBlock) void k_forward_valu(
    const uint32_t* __restrict__ signT, int Np, int Kw, int K, const uint32_t* __restrict__ planes,
    const int32_t* __restrict__ colsum, int Mp, int M, const int32_t* __restrict__ perm,
    const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx, const float* __restrict__ val,
    double alpha, double step, int row_tiles, long long tasks, float* __restrict__ Y, int32_t* __restrict__ D) {
    constexpr int TN = kRowTile;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const long long task = (long long)blockIdx.x * kWavesPerBlock + wave;
    if (task >= tasks) return;
    const int tile = (int)(task % row_tiles);                  // waves of a block share the column strip
    const int strip = (int)(task / row_tiles);
    const int slot0 = tile * TN;
    const int m = strip * kWave + lane;

    int acc[BITS][TN];
#pragma unroll
    for (int b = 0; b < BITS; ++b)
#pragma unroll
        for (int r = 0; r < TN; ++r) acc[b][r] = 0;

    const uint32_t* wp = signT + slot0;
    const uint32_t* xp = planes + m;
    const size_t plane_stride = (size_t)Kw * Mp;
    for (int j = 0; j < Kw; ++j) {
        const uint32_t x0 = xp[(size_t)j * Mp];
        const uint32_t x1 = BITS == 2 ? xp[plane_stride + (size_t)j * Mp] : 0u;
        const uint32_t* w = wp + (size_t)j * Np;
#pragma unroll
        for (int r = 0; r < TN; ++r) {
            const uint32_t wr = w[r];
            if (BITS == 1) {
                acc[0][r] += __builtin_popcount(wr ^ x0);
            } else {
                acc[0][r] += __builtin_popcount(wr & x0);
                acc[1][r] += __builtin_popcount(wr & x1);
            }
        }
    }

    const int cs = BITS == 2 ? colsum[m] : 0;
    const bool col_ok = m < M;
#pragma unroll
    for (int r = 0; r < TN; ++r) {
        const int n = perm[slot0 + r];
        if (n < 0) continue;
        const int d = BITS == 1 ? K - 2 * acc[0][r] : 2 * (acc[0][r] + 2 * acc[BITS - 1][r]) - cs;
        if (INT_ONLY) {
            if (col_ok) D[(size_t)n * M + m] = d;
            continue;
        }
        double a = alpha * (double)d;
        const int q1 = row_ptr[n + 1];
        for (int q = row_ptr[n]; q < q1; ++q) {
            const int c = col_idx[q];
            const double v = (double)val[q];
            const size_t off = (size_t)(c >> 5) * Mp;
            const int bit = c & 31;
            int code;
            if (BITS == 1) {
                code = 2 * (int)((xp[off] >> bit) & 1u) - 1;
            } else {
                code = (int)((xp[off] >> bit) & 1u) + 2 * (int)((xp[plane_stride + off] >> bit) & 1u);
            }
            a = fma(v, (double)code, a);
        }
        if (col_ok) Y[(size_t)n * M + m] = (float)(a * step);
    }
}

}  // namespace

int launch_forward(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, int M, int bits, float step,
                   float* Y, int32_t* D, hipStream_t s) {
    const int Mp = kWave * ((M + kWave - 1) / kWave);
    const int row_tiles = L.Np / kRowTile;
    const long long tasks = (long long)row_tiles * (Mp / kWave);
    const long long blocks = (tasks + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > 0x7fffffffLL) return APB_ERR_SHAPE;
    const dim3 grid((unsigned)blocks), block(kBlock);
    const double a = (double)L.alpha, st = (double)step;
#define APB_FWD(B, I)                                                                                          \
    hipLaunchKernelGGL((k_forward_valu<B, I>), grid, block, 0, s, L.signT, L.Np, L.Kw, L.K, planes, colsum, Mp, \
                       M, L.perm, L.row_ptr, L.col_idx, L.val, a, st, row_tiles, tasks, Y, D)
    if (D != nullptr) {
        if (bits == 1) APB_FWD(1, true); else APB_FWD(2, true);
    } else {
        if (bits == 1) APB_FWD(1, false); else APB_FWD(2, false);
    }
#undef APB_FWD
    APB_HIP(hipGetLastError());
    return APB_OK;
}

}  // namespace apb
