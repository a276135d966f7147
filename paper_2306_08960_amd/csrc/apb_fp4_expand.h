// Bit-packed operands -> FP4 (E2M1) operand registers of v_mfma_scale_f32_32x32x64_f8f6f4, shared by
// the matrix-core kernels.  A weight bit becomes the nibble 0b0001 (= 0.5), the two plane bits of an
// activation (or of a 2-bit weight) become the nibble p0 | p1<<1 (= 0.5, 1.0, 1.5 for codes 1, 2,
// 3 -- additive in the planes, so no table).  Products are multiples of 1/4 and every partial sum is far below 2^24 of
// those, so a float accumulator holds P/4 exactly, P = sum_k bit * code.
//   lane l = 32*g + i (i: row of A / column of B, g: lane half) owns word 2*s+g of K step s;
//   nibble t of operand dword d  <->  bit d + 4*t of that word (the same for both operands, which is
//   all the contraction needs).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace apb {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr uint32_t kNib = 0x11111111u;
constexpr int kScaleOne = 0x7f7f7f7f;                          // E8M0 exponent 127 = 1.0 in every byte

template <int RN, int RM>
struct Frag {
    v8i a[RN];
    v8i b[RM];
};

// FP4 uses the low four operand dwords; the upper four are cleared once.
template <int RN, int RM>
__device__ __forceinline__ void clear_upper(Frag<RN, RM>& f) {
#pragma unroll
    for (int t = 0; t < RN; ++t)
#pragma unroll
        for (int d = 4; d < 8; ++d) f.a[t][d] = 0;
#pragma unroll
    for (int u = 0; u < RM; ++u)
#pragma unroll
        for (int d = 4; d < 8; ++d) f.b[u][d] = 0;
}

// One operand register set from the words of NB bit-planes (NB = 1: a bit; NB = 2: a 2-bit code).
template <int NB>
__device__ __forceinline__ void expand_words(uint32_t w0, uint32_t w1, v8i& f) {
    if (NB == 1) {
#pragma unroll
        for (int d = 0; d < 4; ++d) f[d] = (int)((w0 >> d) & kNib);
    } else {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            // the plane-1 bit goes one position up inside the nibble: bit d+4t -> bit 4t+1
            const uint32_t hi = d == 0 ? (w1 << 1) : (w1 >> (d - 1));
            f[d] = (int)((hi & (kNib << 1)) | ((w0 >> d) & kNib));
        }
    }
}

// WBITS weight planes (1: sign bits of a binary layer; 2: level indices of 2-bit weights), BITS
// activation planes.
template <int WBITS, int BITS, int RN, int RM>
__device__ __forceinline__ void expand(const uint32_t (&aw)[WBITS][RN], const uint32_t (&bw)[BITS][RM],
                                       Frag<RN, RM>& f) {
#pragma unroll
    for (int t = 0; t < RN; ++t) expand_words<WBITS>(aw[0][t], aw[WBITS - 1][t], f.a[t]);
#pragma unroll
    for (int u = 0; u < RM; ++u) expand_words<BITS>(bw[0][u], bw[BITS - 1][u], f.b[u]);
}

__device__ __forceinline__ v16f mfma_fp4(const v8i& a, const v8i& b, const v16f& c) {
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 4, 4, 0, kScaleOne, 0, kScaleOne);
}

}  // namespace apb
