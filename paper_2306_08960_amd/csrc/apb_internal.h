// Internal declarations shared by the host entry points and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "apb.h"

namespace apb {

constexpr int kWave = 64;        // CDNA wavefront width
constexpr int kRowTile = 16;     // weight rows one wave keeps in registers in the popcount GEMM
constexpr int kChunkWords = 8;   // K is walked in chunks of 8 words = 256 weights (one LDS code table each)
constexpr int kChunkK = 32 * kChunkWords;
constexpr int kMaxWavesPerBlock = 8;
// ent_val holds residual * 2^895: finite for every float, and large enough that the sparse kernel's
// table codes (code * 2^-1009, see apb_sparse.hip) give products far from underflow.
constexpr int kEntValScaleLog2 = 895;
constexpr int kEntBlockWords = 24;   // one block of 8 residual entries: 8 key words + 8 float64

struct LayerDev {
    int N = 0, K = 0, Kw = 0;    // Kw = ceil(K/32)
    int Np = 0;                  // launch slots: N rounded up to a multiple of kRowTile * waves
    int waves = 2;               // waves per workgroup of the forward kernel (2, 4 or 8)
    int nchunks = 0;             // ceil(Kw / kChunkWords)
    long long nnz = 0;
    float alpha = 0.f;
    uint32_t* sign = nullptr;    // [N][Kw]   canonical sign words
    uint32_t* signT = nullptr;   // [Kw2][Np] sign words, slot-major: word j of launch slot i (padding slots and
                                 //           the extra word row of an odd Kw are zero; Kw2 as for signC)
    uint32_t* signC = nullptr;   // [Kw2][N]  sign words, word-major in the layer's own row order;
                                 //           Kw2 = Kw rounded up to even, the extra word row is zero
    int32_t* perm = nullptr;     // [Np]      row index served by launch slot i, -1 for padding
    int32_t* row_ptr = nullptr;  // [N+1]
    int32_t* col_idx = nullptr;  // [nnz]
    float* val = nullptr;        // [nnz]
    double* vald = nullptr;      // [nnz]     the same residuals widened to float64 (exact), for the kernel
    int32_t* rowsum = nullptr;   // [N]
    int32_t* chunk_ptr = nullptr;  // [nchunks+1][Np]  first residual of slot i with column >= 256*c
    double* slot_valsum = nullptr; // [Np]             sum of the residuals of slot i (float64)
    // Residuals regrouped for the sparse kernel: one flat run per (tile of kRowTile slots, chunk of
    // 256 columns), sorted by row inside the run, in blocks of 8 entries.
    int32_t* seg_ptr = nullptr;    // [Np/kRowTile][nchunks+1]  first block of (tile, chunk)
    uint32_t* ent = nullptr;       // [blocks][24]  8 keys: 2 * row_in_tile | (col - 256*chunk) << 8, then
                                   //               8 float64: residual * 2^kEntValScaleLog2 (0 for padding)
    // Row lists for the rows-in-lanes forward kernel (apb_rows.hip), built for layers with many residuals
    // per row whose K fits the on-chip code table; rows_steps == 0 when not built.  Rows are sorted by
    // residual count and cut into blocks of 64 launch slots; block b walks steps rows_blk[b] .. rows_blk[b+1],
    // and in a step lane l handles one residual of its row (or a padding entry: offset 0, value 0).
    int rows_Nr = 0;               // 64 * blocks
    int rows_Kw4 = 0;              // Kw rounded up to a multiple of 4 (one matrix step = 128 values of k)
    long long rows_steps = 0;
    int32_t* rows_perm = nullptr;  // [Nr]        row served by slot i, -1 for padding
    int32_t* rows_blk = nullptr;   // [Nr/64 + 1]
    uint32_t* rows_ek = nullptr;   // [steps][64] kRowsRowBytes * column: byte offset of the column's row in the code table
    double* rows_ev = nullptr;     // [steps][64] residual * 2^kEntValScaleLog2
    uint32_t* rows_sign = nullptr; // [Kw4][Nr]   sign words of the slots (pad rows and slots zero); inside a block of 64
                                   //             slots, slot 16 * t + i sits at position 4 * i + t (the order the matrix tiles take them)
    double* rows_valsum = nullptr; // [Nr]        sum of the residuals of the slot's row (float64, CSR order)
    // The same lists with the rows sorted by residual count only inside groups of kRowsGroupRows consecutive rows
    // (whole 32-row words of a packed output): a workgroup of the packed-output epilogue that takes one such group
    // owns its output words -- plain stores, nothing to clear, no atomics.  Built for layers of more than one
    // group (otherwise the lists above already are of this kind); rowsw_steps == 0 when not built.
    long long rowsw_steps = 0;
    int32_t* rowsw_perm = nullptr;
    int32_t* rowsw_blk = nullptr;
    uint32_t* rowsw_ek = nullptr;
    double* rowsw_ev = nullptr;
    uint32_t* rowsw_sign = nullptr;
    double* rowsw_valsum = nullptr;
};

constexpr int kRowsCols = 16;            // output columns one workgroup of the rows-in-lanes kernel covers
constexpr int kRowsGroupRows = 256;      // rows of one group of the word-aligned lists: 4 blocks of 64, 8 output words
constexpr int kRowsRowBytes = 8;         // bytes of its code table per value of k (two dwords of 8 columns x 2 bits)
constexpr int kRowsStageBytesPerK = 8;   // LDS per value of k of its staged activation operand (16 columns x FP4)
constexpr int kRowsMaxTableBytes = 144 * 1024;   // the staged operand of all of K, and the table after it, have to fit on chip

void set_last_hip_error(hipError_t e);

// Shapes of an activation matrix the entry points refuse (APB_ERR_SHAPE).
inline bool bad_shape_acts(int K, int M) {
    if (K <= 0 || M <= 0) return true;
    if ((long long)K * 3 >= (1LL << 31)) return true;
    if ((long long)M + kWave >= (1LL << 31)) return true;
    return false;
}

// The 2-bit activation quantizer (Sec. IV "1/2"): p = clamp(rint(x / s), 0, 3) with one float
// multiply by the precomputed 1/s, ties to even; NaN -> 0.
__device__ __forceinline__ uint32_t code2(float x, float inv_step) {
    return (uint32_t)(int)fminf(3.0f, fmaxf(0.0f, rintf(x * inv_step)));
}
// The same code as the two low bits of the result (the bits above are not zero): clamping first and rounding
// second gives the same p (rounding is monotone and 0, 3 are integers), and adding 2^23 to a float in [0, 3]
// IS the rounding to the nearest integer, ties to even, with p left in the low mantissa bits -- four vector
// instructions instead of five, and no conversion.
__device__ __forceinline__ uint32_t code2_low_bits(float x, float inv_step) {
    return __float_as_uint(fminf(3.0f, fmaxf(0.0f, x * inv_step)) + 8388608.0f);
}
// Shift a word right by one and put bit 0 of `bits` on top: after 32 calls the first bit sits at position 0.
__device__ __forceinline__ uint32_t push_bit(uint32_t word, uint32_t bits) { return __builtin_amdgcn_alignbit(bits, word, 1); }

#define APB_HIP(expr)                                 \
    do {                                              \
        hipError_t e_ = (expr);                       \
        if (e_ != hipSuccess) {                       \
            ::apb::set_last_hip_error(e_);            \
            return APB_ERR_HIP;                       \
        }                                             \
    } while (0)

// ---- kernel launchers (each returns an apb_status) ------------------------------------------

// compress
int launch_inlier_abs_sum(const float* W, long long count, float delta, double* part_sum, long long* part_cnt,
                          int parts, hipStream_t s);
int launch_sign_pack_count(const float* W, int N, int K, int Kw, float delta, uint32_t* sign, int32_t* counts,
                           int32_t* rowsum, hipStream_t s);
int launch_scatter_csr(const float* W, int N, int K, float delta, float alpha, const int32_t* row_ptr,
                       int32_t* col_idx, float* val, double* vald, hipStream_t s);
int launch_slot_major_signs(const uint32_t* sign, const int32_t* perm, int Np, int Kw, int rows_out,
                            uint32_t* signT, hipStream_t s);
int launch_slot_tables(const int32_t* perm, const int32_t* row_ptr, const int32_t* col_idx, const float* val, int Np,
                       int nchunks, int32_t* chunk_ptr, double* slot_valsum, hipStream_t s);

// activations.  colsum == nullptr: the planes only (for a consumer that adds the code sums up from the words itself)
int launch_quantize(const float* X, int K, int M, int bits, float inv_step, uint32_t* planes, int32_t* colsum,
                    hipStream_t s);
int launch_zero_words(uint32_t* p, size_t count, hipStream_t s);

// forward
// the popcount formulation on the vector ALU (Y, or D alone when D != nullptr)
int launch_forward_popcount(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, int M, int bits,
                            float step, float* Y, int32_t* D, hipStream_t s);
// the forward kernel: binary part on the matrix cores, residual part and epilogue, one launch.
// conv == nullptr: `planes` is the packed K x M matrix; otherwise a packed feature map of conv->C channels
// (L.K = 9 * C, C a multiple of 32) of images of H x W pixels, read through an implicit im2col (3 x 3,
// padding 1, the given stride), and M = B * Ho * Wo output pixels.
struct ConvShape {
    int C, H, W;
    int stride, Ho, Wo;            // Ho = (H - 1) / stride + 1, Wo likewise
    int Pp_in;                     // B * H * W rounded up to a multiple of 64: columns of the packed input map
};
int launch_forward(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, int M, int bits, float step,
                   const ConvShape* conv, float* Y, hipStream_t s);
// the packed patch matrix of a convolution (9 * C x M, as apb_quantize_acts lays a matrix out) written into `out`
// (and, on the side, `clear_words` words at `clear` set to zero)
int launch_pack_patches(const LayerDev& L, const uint32_t* planes, const int32_t* pixsum, int M, int bits,
                        const ConvShape& conv, uint32_t* out, uint32_t* clear, size_t clear_words, hipStream_t s);
const char* forward_kernel_name(const LayerDev& L, int M, int bits);
// quantize + forward in one kernel, from the float matrix X (K x M): same Y, bit for bit, as launch_quantize +
// launch_forward; only where forward_float_applies says so (APB_ERR_SHAPE otherwise)
bool forward_float_applies(const LayerDev& L, int M, int bits);
int launch_forward_float(const LayerDev& L, const float* X, int M, int bits, float step, float* Y, hipStream_t s);
// the same with the next layer's quantizer applied to scale[n] * Y + shift[n] (scale, shift nullable) and
// the codes packed into `packed_out` (K = L.N, same M), fully overwritten
int launch_forward_requant(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, int M, int bits, float step,
                           const ConvShape* conv, const float* scale, const float* shift, int bits_out,
                           float inv_step_out, uint32_t* packed_out, hipStream_t s, bool out_cleared = false);
// (out_cleared: packed_out is known to be all zero already -- only the kernels that OR into it care)

// true while K * max_weight * max_code < 2^24: the float accumulators of the matrix instruction then hold
// every partial sum exactly (launchers return APB_ERR_SHAPE otherwise)
bool mfma_sum_exact(int K, int max_weight, int max_code);

// the rows-in-lanes forward kernel (apb_rows.hip): same Y as launch_forward for a plain K x M matrix;
// forward_rows_applies says whether the layer has row lists and the launch is worth it
bool forward_rows_applies(const LayerDev& L, int M, int bits);
const char* forward_rows_kernel_name(const LayerDev& L, int M, int bits);
// colsum == nullptr: the kernel adds the code sums of its columns up from the packed words
int launch_forward_rows(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, int M, int bits, float step,
                        float* Y, hipStream_t s);
// the rows-in-lanes kernel ending in the next layer's quantizer (what launch_forward_requant does on a plain matrix)
bool forward_rows_requant_applies(const LayerDev& L, const uint32_t* planes, int M, int bits);
int launch_forward_rows_requant(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, int M, int bits,
                                float step, const float* scale, const float* shift, int bits_out, float inv_step_out,
                                uint32_t* packed_out, hipStream_t s, bool out_cleared = false);
// launch_quantize + launch_forward_best through the scratch buffer planes / colsum (the step of layers that do
// not run as one kernel); what `colsum` holds afterwards is unspecified
int launch_quantize_then_forward(const LayerDev& L, const float* X, int M, int bits, float step, uint32_t* planes,
                                 int32_t* colsum, float* Y, hipStream_t s);
// apb_forward's choice between the two forward kernels for a plain K x M matrix and a float output
int launch_forward_best(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, int M, int bits, float step,
                        float* Y, hipStream_t s);

// binary part alone on the matrix cores: the integer part D
int launch_binary_mfma(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, int M, int bits,
                       int32_t* out, hipStream_t s);

// 2/2 routine: quantize + pack 2-bit weights (canonical [2][N][Kw] and word-major [2][Kw2][N], Kw2 =
// Kw rounded up to even with a zero pad row), and the product itself (D22 when Y == nullptr)
int launch_w2_pack(const float* W, int N, int K, float inv_step, uint32_t* planes, uint32_t* planesC, hipStream_t s);
int launch_gemm_2_2(const uint32_t* wplanesC, int N, int Kw, const uint32_t* planes, const int32_t* colsum, int M,
                    double scale, int32_t* D, float* Y, hipStream_t s);

}  // namespace apb

struct apb_layer {
    apb::LayerDev d;
};

struct apb_w2 {
    int N = 0, K = 0, Kw = 0;
    float step_w = 0.f;
    uint32_t* planes = nullptr;    // [2][N][Kw]   canonical bit-planes of the level indices
    uint32_t* planesC = nullptr;   // [2][Kw2][N]  the same, word-major, for the matrix-core kernel
};
