/* apb.h -- C ABI of the MI355X (gfx950) library for the forward pass of an
 * Automatic Prune Binarization (APB) layer, arXiv 2306.08960.
 *
 * The layer computes (Sec. III, "Inference Considerations", Eqs. 11-13)
 *
 *      Y = A^bin * X^ + A^full * X^ ,
 *
 * where A^bin = alpha * sign(W) holds ONE BIT FOR EVERY weight (the binary
 * matrix is fully represented, Sec. III "Memory Impact"), A^full is the sparse
 * matrix of the residuals w - alpha*sign(w) of the few weights whose magnitude
 * lies outside the binarization interval (Eq. 3), and X^ are the activations
 * quantized to 1 bit (+-beta, Sec. IV "1/1") or 2 bits (p*s, p in 0..3,
 * Sec. IV "1/2").  Both operands of the binary product stay bit-packed in memory;
 * it is computed exactly in integers, by default on the matrix cores (each lane
 * spreads the bits it owns into 4-bit operand slots; the algebra is that of the
 * paper's and/xor + popcount forms, Eqs. 16, 18, 19, which are kept as the
 * *_popcount entry points for comparison).  The sparse product reads the same
 * packed activations.
 *
 * Shapes and names: W is N x K row-major (N output channels, K = C_in*kh*kw),
 * X is K x M row-major (column m = one im2col patch), Y is N x M row-major.
 *
 * Conventions
 *  - Every function returns APB_OK (0) or a negative apb_status; nothing throws
 *    and nothing aborts.  apb_strerror() names a code; after APB_ERR_HIP,
 *    apb_last_hip_error() returns the hipError_t of the calling thread.
 *  - "DEVICE" pointers are HIP device memory of the current device and must be
 *    4-byte aligned; the caller owns them.  The library owns only what lives
 *    inside an apb_layer.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    apb_quantize_acts, the apb_forward* family and apb_gemm_2_2* only enqueue work and return
 *    (none of them allocates, and none records a memset: a caller may capture them in a HIP
 *    graph); apb_compress, apb_layer_export and apb_w2_export synchronize the stream.
 *  - A packed activation buffer is plain, untyped device memory: it carries no record of the
 *    K, M and bits it was written with, and the entry points that read one cannot check them
 *    (a check would need either a device-to-host read on the hot path or a host-side table of
 *    pointers that a plain copy of the buffer would leave stale).  Passing K, M or bits other
 *    than the writer's reads a different layout: unspecified numbers, never out of bounds as
 *    long as the buffer has apb_acts_bytes(K, M, bits) bytes for the values passed.
 *  - K limits: 3*K < 2^31 everywhere; the matrix-core entry points additionally need every
 *    partial sum of the binary product exact in a float accumulator: K < 2^24 for 1-bit
 *    activations, 3*K < 2^24 for 2-bit ones, 9*K < 2^24 for the 2/2 routine (APB_ERR_SHAPE
 *    beyond; the *_popcount entry points have no such limit).
 *  - Non-finite values in W or X give unspecified numbers but never touch
 *    memory out of bounds (a NaN activation quantizes to code 0 / sign -).
 *  - Distinct layers and buffers may be used from distinct host threads.
 */
#ifndef APB_H_
#define APB_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum apb_status {
    APB_OK = 0,
    APB_ERR_NULL = -1,     /* a required pointer is NULL                                   */
    APB_ERR_SHAPE = -2,    /* N, K or M <= 0, or too large (N*K >= 2^31, 3*K >= 2^31, ...)  */
    APB_ERR_BITS = -3,     /* bits is not 1 or 2                                           */
    APB_ERR_VALUE = -4,    /* delta is NaN; alpha negative or infinite; step not finite or <= 0 */
    APB_ERR_NOMEM = -5,    /* host or device allocation failed                             */
    APB_ERR_HIP = -6,      /* a HIP call failed; see apb_last_hip_error()                  */
    APB_ERR_SCRATCH = -7   /* apb_quantize_forward_static: sizes beyond the static scratch array */
} apb_status;

/* Opaque compressed layer.  Holds, in device memory: the sign words, the CSR of
 * residuals, per-row sign sums and a launch-order row permutation. */
typedef struct apb_layer apb_layer;

/* Sec. III Eq. 1 (sign(0) = +), Eq. 3 (partition), Eqs. 11-12 (A^bin, A^full).
 *   W      DEVICE, N*K floats, row-major, read-only.
 *   delta  half-width of the binarization interval: weight w is binarized iff
 *          |w| <= delta (exact float compare).  This is the paper's alpha + delta.
 *          +inf keeps no residuals; a negative value makes every weight a residual.
 *   alpha  the layer scale.  A finite value >= 0 is used as given (a learned
 *          scale); NaN asks for the default: the mean of |w| over the binarized
 *          set (float64 sum, rounded to float), 0 if that set is empty.
 *   out    receives a new layer on APB_OK (free with apb_layer_free), NULL otherwise.
 * Per weight: sign bit = (w >= 0).  Per residual: val = w - (bit ? alpha : -alpha),
 * a single float subtraction.  Synchronizes `stream`. */
int apb_compress(const float* W, int N, int K, float delta, float alpha, void* stream, apb_layer** out);

/* Sizes and scalars of a layer; any output pointer may be NULL.
 *   mem_bits  Sec. III Eq. 10 in its fully represented form, N*K + nnz*(32 + b_p),
 *             with b_p = floor(log2(N*K - 1)) + 1 (bits of a flat index; 1 if N*K <= 2). */
int apb_layer_info(const apb_layer* layer, int* N, int* K, float* alpha, long long* nnz, long long* mem_bits);

/* Copy the canonical representation out (each destination may be NULL to skip it;
 * destinations may be device or host memory):
 *   sign_words  N * ceil(K/32) uint32, row-major; bit i of word j of row n is 1 iff
 *               W[n, 32*j+i] >= 0; bits beyond K are 0.
 *   row_ptr     N+1 int32;  col_idx  nnz int32, ascending inside a row;  val  nnz floats.
 *   rowsum      N int32, sum over k of (+1 | -1) of row n (the weight-only term of the
 *               zero-centred form, Sec. IV "1/2").
 * Synchronizes `stream`. */
int apb_layer_export(const apb_layer* layer, uint32_t* sign_words, int32_t* row_ptr, int32_t* col_idx,
                     float* val, int32_t* rowsum, void* stream);

/* NULL-safe.  The caller makes sure no enqueued work still uses the layer. */
void apb_layer_free(apb_layer* layer);

/* Size in bytes of the packed activation buffer for a K x M matrix; 0 on bad arguments.
 * Layout, with Kw = ceil(K/32) and Mp = 64*ceil(M/64):
 *   uint32 planes[bits][Kw][Mp]   bit i of planes[b][j][m] = bit b of the code of X[32*j+i, m]
 *   int32  colsum[Mp]             sum over k of code[k, m]
 * Codes: 1-bit, code = (x >= 0) and the value is (2*code-1)*step; 2-bit, code = the
 * level index p and the value is p*step.  Columns m >= M and bits k >= K are zero. */
size_t apb_acts_bytes(int K, int M, int bits);

/* Sec. IV: quantize and pack the activations.
 *   X       DEVICE, K*M floats row-major, read-only.
 *   bits    1: sign, sign(0) = +.   2: p = clamp(rint(x * (1/step)), 0, 3), float
 *           arithmetic, round-half-to-even, 1/step computed once in float.
 *   step    beta (1 bit) or s (2 bits); finite and > 0.
 *   packed  DEVICE, apb_acts_bytes(K, M, bits) bytes, fully overwritten.
 * Asynchronous on `stream`. */
int apb_quantize_acts(const float* X, int K, int M, int bits, float step, void* packed, void* stream);

/* Sec. III Eq. 13 with the scalar multipliers of Sec. IV:
 *      Y[n,m] = alpha*step * D[n,m] + sum_{j in row n} val_j * step * c[col_j, m]
 * where c is the integer activation value (+-1 or p) and D = sum_k sign(W[n,k]) * c[k,m]
 * is computed exactly in integers from the packed words.  The sparse sum and the
 * combination are accumulated in float64 and rounded once to float.
 *   packed  DEVICE buffer written by apb_quantize_acts with the SAME K (the layer's), M, bits.
 *   Y       DEVICE, N*M floats row-major, fully overwritten.
 * Asynchronous on `stream`. */
int apb_forward(const apb_layer* layer, const void* packed, int M, int bits, float step, float* Y, void* stream);

/* The kernel apb_forward launches for this layer, M and bits, by the name a profiler shows for it
 * (a static string; "" on bad arguments).  For matching benchmark figures with profiler output. */
const char* apb_forward_kernel_name(const apb_layer* layer, int M, int bits);

/* apb_quantize_acts followed by apb_forward as ONE call, with the same Y bit for bit.  For layers of at
 * most 128 rows (one workgroup then holds every row, so no strip of X is quantized twice) whose K fits
 * the on-chip memory, a single kernel reads X, keeps the packed codes of its 64 columns on chip and
 * writes Y: the packed activations never travel to HBM and the memory-bound quantize phase of one
 * workgroup overlaps the arithmetic of the others.  Other layers run the two kernels one after the
 * other through `packed`.
 *   X       DEVICE, K*M floats row-major, read-only.
 *   packed  DEVICE, apb_acts_bytes(K, M, bits) bytes of scratch; contents unspecified afterwards.
 *   Y       DEVICE, N*M floats, fully overwritten.
 * Asynchronous on `stream`. */
int apb_quantize_forward(const apb_layer* layer, const float* X, int M, int bits, float step, void* packed, float* Y,
                         void* stream);
/* 1 if apb_quantize_forward runs as the single kernel for this layer, M and bits, else 0 (also on bad arguments). */
int apb_quantize_forward_is_one_kernel(const apb_layer* layer, int M, int bits);

/* For callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and the same Y,
 * bit for bit, as apb_quantize_forward, without its `packed` workspace: the packed activations
 * pass through a static array in device memory that belongs to the library
 * (APB_STATIC_SCRATCH_BYTES bytes on every GPU the library is used on, held until the process
 * ends).  The call allocates nothing, frees nothing and records no memset.
 *   - APB_ERR_SCRATCH, and nothing enqueued, if apb_acts_bytes(K, M, bits) exceeds
 *     APB_STATIC_SCRATCH_BYTES (also for layers that would run as the single kernel).
 *   - Every call on one GPU uses that GPU's one array: two calls whose work overlaps in time
 *     on the same GPU (different streams, different host threads) race on it.  Calls on one stream
 *     are ordered and safe; the array keeps the last call's contents, which the next call
 *     overwrites or clears as far as it reads them.
 * Asynchronous on `stream`. */
#define APB_STATIC_SCRATCH_BYTES (32u << 20)
int apb_quantize_forward_static(const apb_layer* layer, const float* X, int M, int bits, float step, float* Y,
                                void* stream);

/* Two layers in a row without the float round trip: Eq. 13 of this layer followed directly by the
 * activation quantizer (Sec. IV) of the layer it feeds, whose K is this layer's N.  The result is
 * the packed buffer that apb_quantize_acts(Z, N, M, bits_out, step_out) would write for
 *      Z[n,m] = scale[n] * Y[n,m] + shift[n]          (a folded batch normalization; Z = Y without)
 * with Y as apb_forward computes it; Z is formed in float64 from the float64 Y and rounded once to
 * float, then quantized exactly as apb_quantize_acts does (for bits_out = 2 the clamp at 0 is the
 * ReLU).  Neither Y nor Z is written to memory.
 *   scale, shift  DEVICE, N floats each, read-only; both NULL for Z = Y (one NULL: APB_ERR_NULL).
 *   bits_out, step_out  the next layer's activation format (as `bits`, `step` of apb_quantize_acts).
 *   packed_out    DEVICE, apb_acts_bytes(N, M, bits_out) bytes, fully overwritten; must not overlap `packed`.
 * Asynchronous on `stream`. */
int apb_forward_requant(const apb_layer* layer, const void* packed, int M, int bits, float step,
                        const float* scale, const float* shift, int bits_out, float step_out, void* packed_out,
                        void* stream);

/* A 3 x 3 convolution (padding 1, stride 1 or 2) as Eq. 13 on the im2col matrix (Sec. III, footnote on
 * convolutions), without building that matrix: the activations are a packed FEATURE MAP and the
 * kernel reads the nine shifted views of it.
 *   layer   compressed from W [N][K = 9*C]: N output channels, k = tap*C + c with tap = 3*ky + kx
 *           (ky, kx in 0..2) and c the input channel; C must be a multiple of 32.
 *   fmap    DEVICE, the packed buffer of the C x P code matrix of the input map (row = channel,
 *           column p = (b*H + y)*W + x, P = B*H*W): exactly what apb_quantize_acts writes for a
 *           C x P float matrix, or apb_forward_requant / apb_forward_conv3x3_requant of the layer
 *           before; apb_acts_bytes(C, P, bits) bytes.
 *   stride  1 or 2.  The output map has Ho = (H - 1) / stride + 1 rows and Wo = (W - 1) / stride + 1 columns;
 *           output pixel (b, yo, xo) sees the inputs (b, stride*yo + ky - 1, stride*xo + kx - 1).
 *   padding pixels outside the image have code 0: the value 0 for 2-bit activations, -step for 1-bit.
 *   workspace, workspace_bytes  optional DEVICE scratch (NULL, 0: none), 16-byte aligned.  With at least
 *           apb_acts_bytes(9*C, Po, bits) bytes, layers with many residuals per row (those apb_forward runs
 *           with its lanes along the rows) first write the packed patch matrix there -- bit words, 1/16 or
 *           1/32 of the float im2col matrix -- and multiply it as a plain matrix, which is faster for them
 *           than gathering inside the kernel; other layers, and calls without a workspace, gather.  Contents
 *           unspecified afterwards; must not overlap fmap, Y or fmap_out.  Same results either way (to the
 *           rounding of the float64 sums).
 *   Y       DEVICE, N*Po floats (Po = B*Ho*Wo), channel-major like the input map, fully overwritten.
 * The _requant form ends with the next layer's quantizer as apb_forward_requant does and writes the
 * packed output map (apb_acts_bytes(N, Po, bits_out) bytes), which a following 3 x 3 layer with C = N and
 * images of Ho x Wo pixels takes as its fmap.  APB_ERR_SHAPE if K is not 9*C with C % 32 == 0 and C <= 16384,
 * if stride is neither 1 nor 2, if B*H*W >= 2^28 or if one bit-plane of the map reaches 2^31 bytes.
 * Asynchronous on `stream`. */
int apb_forward_conv3x3(const apb_layer* layer, const void* fmap, int B, int H, int W, int stride, int bits, float step,
                        void* workspace, size_t workspace_bytes, float* Y, void* stream);
int apb_forward_conv3x3_requant(const apb_layer* layer, const void* fmap, int B, int H, int W, int stride, int bits,
                                float step, const float* scale, const float* shift, int bits_out, float step_out,
                                void* workspace, size_t workspace_bytes, void* fmap_out, void* stream);

/* Test hook: the integer part D (N*M int32, row-major, DEVICE) alone, computed by the stand-alone
 * matrix-core kernel (the same bit expansion and matrix instruction as apb_forward's first
 * phase). Asynchronous on `stream`. */
int apb_forward_int(const apb_layer* layer, const void* packed, int M, int bits, int32_t* D, void* stream);

/* The same D through the paper's own formulation: xor/and + popcount over packed words
 * (Sec. IV Eq. 16 and Eqs. 18-19) on the vector ALU.  Kept as the measured comparison for the
 * matrix-core kernel and as a second, independent route to D in the tests. */
int apb_forward_int_popcount(const apb_layer* layer, const void* packed, int M, int bits, int32_t* D,
                             void* stream);

/* apb_forward with the binary part computed by the popcount formulation above, fused with the
 * sparse part in one vector-ALU kernel.  Same arguments, same result as apb_forward; exists so
 * that the two formulations can be timed against each other. */
int apb_forward_popcount(const apb_layer* layer, const void* packed, int M, int bits, float step, float* Y,
                         void* stream);

/* ---- Sec. IV "2/2": 2-bit weights times 2-bit activations ----------------------------------
 *
 * Both operands are 2-bit uniformly quantized; the weights take the zero-centred levels
 * (q - 3/2) * step_w, q in 0..3, the activations the levels p * step_a, p in 0..3 (the packed
 * buffer of apb_quantize_acts with bits = 2).  The paper decomposes both into three binary
 * vectors and applies its 1/2 routine twice (four masked binary products, cost 8x the 1/1
 * routine); here the two bit-planes of q and of p feed the same matrix-core kernel as the binary
 * layer, which yields sum_k q*p exactly, and the zero-centring of the weights is applied with
 * the per-column sums of p:
 *      D22[n,m] = sum_k (2*q[n,k] - 3) * p[k,m] = 2 * sum_k q*p - 3 * colsum[m],
 *      Y[n,m]   = (step_w * step_a / 2) * D22[n,m]        (float64 product, rounded once).
 * The paper takes the quantized weights as given; apb_w2_pack uses the uniform mid-rise
 * quantizer q = clamp(floor(w * (1/step_w)) + 2, 0, 3) in float arithmetic (NaN -> 0). */
typedef struct apb_w2 apb_w2;   /* opaque; owns the packed weight planes in device memory */

/*   W       DEVICE, N*K floats, row-major, read-only.     step_w  finite and > 0.
 *   out     receives a new handle on APB_OK (free with apb_w2_free), NULL otherwise.
 * Asynchronous on `stream` except for the allocations. */
int apb_w2_pack(const float* W, int N, int K, float step_w, void* stream, apb_w2** out);

/* Copy the canonical planes out: 2 * N * ceil(K/32) uint32 (device or host), plane b first;
 * bit i of word j of row n of plane b = bit b of q[n, 32*j+i]; bits beyond K are 0.
 * Synchronizes `stream`. */
int apb_w2_export(const apb_w2* w2, uint32_t* planes, void* stream);

/* NULL-safe.  The caller makes sure no enqueued work still uses the handle. */
void apb_w2_free(apb_w2* w2);

/*   packed  DEVICE buffer written by apb_quantize_acts with the same K, M and bits = 2.
 *   D / Y   DEVICE, N*M int32 / floats, row-major, fully overwritten.
 * Asynchronous on `stream`. */
int apb_gemm_2_2_int(const apb_w2* w2, const void* packed, int M, int32_t* D, void* stream);
int apb_gemm_2_2(const apb_w2* w2, const void* packed, int M, float step_a, float* Y, void* stream);

/* ---- Sec. III Eqs. 3-9: the training-side operators of one layer ---------------------------------
 *
 * During training the layer keeps full-precision latent weights and two learned scalars: alpha, the
 * scale of the binarized weights, and delta, how far the binarization interval reaches beyond alpha
 * (the interval is |w| <= alpha + delta; apb_compress takes that sum as its `delta` argument).
 *
 * apb_train_forward: Eq. 3 element-wise on the latent weights,
 *      out[i] = sign(W[i]) * alpha  if |W[i]| <= alpha + delta (float compare against the float sum),
 *               W[i]                otherwise;       sign(0) = + (Eq. 1).
 * apb_train_backward: given the upstream gradient G (dL/dAPB(w), what backpropagation delivers),
 *      grad_w[i]   = G[i]                                  Eq. 4 with the identity as surrogate: the
 *                                                          straight-through gradient of the latent weight
 *      dL/dw_hat_i = delta * sign(W[i]) * G[i]             Eq. 9 solved for dL/dw_hat
 *      chi_B,i     = 1 if |W[i]| <= alpha + delta else 0   Eq. 6
 *      grad_alpha  = -1 / (delta * n)   * sum_i dL/dw_hat_i * chi_B,i                    Eq. 8
 *      grad_delta  =  1 / (delta^2 * n) * sum_i dL/dw_hat_i * (alpha - |W[i]|) * chi_B,i Eq. 7
 *   with n the number of weights.  Terms and sums are float64; the sums are deterministic (fixed
 *   partition, fixed order), so two calls on the same inputs give the same bits.
 *   W, G              DEVICE, n floats each, read-only.      n in 1 .. 2^40 - 1.
 *   alpha, delta      finite, alpha >= 0; delta >= 0 (forward), delta > 0 (backward).
 *   out / grad_w      DEVICE, n floats, fully overwritten; grad_w may be NULL (the latent gradient is G
 *                     itself) and may alias G.
 *   grad_alpha_delta  DEVICE, 2 doubles: [0] = grad_alpha, [1] = grad_delta.
 *   n_binarized       DEVICE, 1 int64 (the size of the binarized set), or NULL.
 *   workspace         DEVICE, apb_train_workspace_bytes() bytes of scratch, 8-byte aligned.
 * Asynchronous on `stream`; no allocation, no memset. */
size_t apb_train_workspace_bytes(void);
int apb_train_forward(const float* W, long long n, float alpha, float delta, float* out, void* stream);
int apb_train_backward(const float* W, const float* G, long long n, float alpha, float delta, float* grad_w,
                       double* grad_alpha_delta, long long* n_binarized, void* workspace, void* stream);

/* ---- Measurement support: instruction-rate probes ---------------------------------------------
 *
 * The roofs this library's kernels are priced against (Sec. IV derives the paper's own "theoretical
 * peak performance" from the instruction mix of its routines; this is the same exercise for this
 * chip) come from the data sheet and, beside it, from what the chip sustains for each mix in a
 * register-only loop.  apb_probe_rate launches one such loop: 2048 workgroups of 256 lanes, `iters`
 * passes, no memory traffic but one word per lane at the end.
 *   kind             which mix (below); APB_ERR_VALUE for another value.
 *   iters            1 .. 2^20 loop passes per lane.
 *   out              DEVICE, apb_probe_out_bytes() bytes of scratch, overwritten.
 *   work_per_launch  HOST, receives the work of one launch in the unit of the mix: multiply-add
 *                    flops (2 per product) for the two matrix probes, lane operations for the
 *                    vector and LDS probes.
 * Asynchronous on `stream`. */
enum {
    APB_PROBE_MFMA_FP4 = 0,   /* v_mfma_scale_f32_32x32x64_f8f6f4 with FP4 operands                    */
    APB_PROBE_MFMA_I8 = 1,    /* v_mfma_i32_32x32x32_i8                                               */
    APB_PROBE_AND_BCNT = 2,   /* v_and_b32 + v_bcnt_u32_b32: the popcount formulation's pair           */
    APB_PROBE_FMA_F64 = 3,    /* v_fma_f64: the residual part's multiply-add                          */
    APB_PROBE_LDS_U8 = 4,     /* ds_read_u8 from a 260-byte-pitch table, one column for all lanes      */
    APB_PROBE_LDS_B128 = 5,   /* four 16-byte LDS reads per lane and pass (work = bytes)               */
    APB_PROBE_MFMA_FP4_LDS = 6,               /* ... feeding four FP4 matrix instructions              */
    APB_PROBE_MFMA_FP4_LDS_BARRIER = 7,       /* ... plus an LDS write and a workgroup barrier per pass */
    APB_PROBE_MFMA_FP4_LDS_BARRIER_VALU = 8   /* ... plus 32 vector-ALU instructions per pass          */
};
size_t apb_probe_out_bytes(void);
int apb_probe_rate(int kind, int iters, void* out, double* work_per_launch, void* stream);

const char* apb_strerror(int code);
int apb_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* APB_H_ */
