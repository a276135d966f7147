// Host side of the stand-alone matrix-core product (the integer part D of a binary layer, and the 2/2
// routine of Sec. IV): fills the kernel parameters and hands them to the instantiation for the operand
// format.  The kernel itself is in apb_binary_mfma_kernel.h.
#include "apb_binary_mfma_kernel.h"

namespace apb {

using mfma_detail::MfmaParams;

// The float accumulators of the matrix instruction hold P / 4 exactly only while P, the largest possible
// sum of products (weight value times activation code, in units of the operand encodings), stays below
// 2^24.  Longer K is refused rather than computed inexactly.
bool mfma_sum_exact(int K, int max_weight, int max_code) {
    return (long long)K * max_weight * max_code < (1LL << 24);
}

// Binary layer: the integer part D into `out` (N*M int32).
int launch_binary_mfma(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, int M, int bits,
                       int32_t* out, hipStream_t s) {
    if (!mfma_sum_exact(L.K, 1, bits == 1 ? 1 : 3)) return APB_ERR_SHAPE;
    MfmaParams p{};
    p.signT = L.signC;                                        // rows in the layer's own order
    p.planes = planes;
    p.colsum = colsum;
    p.rowsum = L.rowsum;
    p.out = out;
    p.Np = L.N;
    p.Kw = L.Kw;
    p.Mp = kWave * ((M + kWave - 1) / kWave);
    p.M = M;
    return bits == 1 ? launch_mfma_d_1bit(p, L.N, s) : launch_mfma_d_2bit(p, L.N, s);
}

// 2/2 routine: D22 (int32) when Y == nullptr, else Y = scale * D22 (float).
int launch_gemm_2_2(const uint32_t* wplanesC, int N, int Kw, const uint32_t* planes, const int32_t* colsum, int M,
                    double scale, int32_t* D, float* Y, hipStream_t s) {
    if (!mfma_sum_exact(32 * Kw, 3, 3)) return APB_ERR_SHAPE;
    MfmaParams p{};
    p.signT = wplanesC;
    p.wplane_stride = (size_t)(2 * ((Kw + 1) / 2)) * N;
    p.planes = planes;
    p.colsum = colsum;
    p.out = Y ? static_cast<void*>(Y) : static_cast<void*>(D);
    p.scale = scale;
    p.Np = N;
    p.Kw = Kw;
    p.Mp = kWave * ((M + kWave - 1) / kWave);
    p.M = M;
    return Y ? launch_mfma_22_float(p, N, s) : launch_mfma_22_int(p, N, s);
}

}  // namespace apb
