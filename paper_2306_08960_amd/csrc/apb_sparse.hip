// The forward kernel of apb_forward (Sec. III Eqs. 12-13):
//     Y[n,m] = s * ( alpha * D[n,m] + sum_{j in row n} val_j * c[col_j, m] )
// A workgroup (2, 4 or 8 waves) first computes the binary product of its tile on the matrix cores
// (binary_tile_to_lds below), starts its float64 row sums at alpha * D, adds the residual part and
// writes its outputs: nothing else goes to HBM.  The outputs are Y, or -- for a layer that feeds
// another one -- the packed codes of the next layer's quantizer applied to Y (see write_rows).
//
// Mapping of the residual part: lanes run along m, so residual columns and values are wave-uniform
// and arrive through the scalar path.  A workgroup (up to 8 waves, each owning a tile of 16 weight
// rows in launch-slot order) shares one strip of 64 output columns and walks K in chunks of 256:
//   1. the waves expand the chunk's activation bit-planes into a byte-per-activation code table in
//      LDS (row = output column, 256 bytes + 4 pad bytes, so the 64 lanes of a wave hit distinct
//      banks when they read the same k);
//   2. after a barrier each wave streams the residuals of its 16 rows that fall in the chunk.  They
//      were laid out at compress time as ONE flat run per (tile, chunk), padded to whole blocks of
//      8, so the loop has no per-row work at all.  The 16 float64 row sums of a lane live in 32
//      consecutive vector registers, and the multiply-add of a residual addresses its row's pair
//      through the register-index mode: one scalar instruction (index <- low byte of the entry
//      key = 2*row) and one v_fma_f64.  With the address add (column taken straight from byte 1 of
//      the key) and a ds_read_u8_d16_hi whose result is the float64 multiplicand as it stands
//      (see kCodeBytes), that is four instructions per residual and wave, and no branch.
// Tiles are filled by dealing rows in order of residual count (see balanced_slots), so the skewed
// rows of pruned layers are spread over the waves instead of serialising one of them.
#include <atomic>

#include "apb_fp4_expand.h"
#include "apb_internal.h"

namespace apb {

namespace {

constexpr int TN = kRowTile;
constexpr int kMaxDevices = 64;                                // devices of one process the launchers keep state for
constexpr int kTablePitch = kChunkK + 4;                       // bytes per column row of the code table
constexpr int kTableBytes = kWave * kTablePitch;               // one table (see table_buffers for how many a workgroup keeps)

typedef __attribute__((address_space(3))) uint8_t lds_u8;

// Fourth word of a raw buffer descriptor on gfx9-family parts: 32-bit data format, no swizzle.
constexpr int kBufferFlags = 0x00020000;

// 8-wave workgroups alternate between two tables (one barrier per chunk); smaller ones keep one, so
// that twice as many fit a CU, and pay a second barrier per chunk.
__host__ __device__ constexpr int table_buffers(int wpw) { return wpw == 1 ? 2 : 1; }

struct SparseParams {
    double alpha, step;
    int Np, Kw, Mp, M, nchunks;
    int row_groups;                          // Np / (TN * waves)
    int blocks;                              // row_groups * strips
    int out_bits;                            // 0: float Y;  1 or 2: packed codes of the next layer
    int out_exclusive;                       // packed output: the workgroup holds ALL rows of its columns
    int out_Kw;                              // ceil(N / 32), words per column of a packed output plane
    float out_inv_step;                      // 1 / step of the 2-bit output quantizer
    // Implicit im2col (CONV kernels): the activations are a packed feature map [bits][Cw][conv_Mp] (+ per-pixel
    // code sums) of B images of H x W pixels; a column m is the OUTPUT pixel (b, yo, xo) = (m / (Ho*Wo),
    // (m / Wo) % Ho, m % Wo), its window is centred on the input pixel (b, stride*yo, stride*xo), and word row
    // j = tap * Cw + cw of the patch matrix is word row cw of the map at that pixel shifted by tap
    // (dy, dx) = (tap / 3 - 1, tap % 3 - 1), or zero outside the image.
    int conv_Cw, conv_H, conv_W, conv_Ho, conv_Wo, conv_stride;
    int conv_Mp;                             // columns of the input map, padded as its packed buffer is
    float conv_inv_Cw;
    // Float activations (FX kernels): K rows of X and 1 / step of the input quantizer.
    int K;
    float in_inv_step;
};

// Output column m of a convolution: returns the tap mask (bit t: tap t of its window lies inside the image;
// none for columns >= M) and sets `pin`, the column of the window's centre in the input map.
__device__ __forceinline__ uint32_t conv_pixel(int m, const SparseParams& p, int& pin) {
    const int xo = m % p.conv_Wo, rest = m / p.conv_Wo;
    const int yo = rest % p.conv_Ho, img = rest / p.conv_Ho;
    const int x = p.conv_stride * xo, y = p.conv_stride * yo;
    pin = m < p.M ? (img * p.conv_H + y) * p.conv_W + x : 0;
    uint32_t vm = 0;
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        const int yy = y + t / 3 - 1, xx = x + t % 3 - 1;
        if (m < p.M && yy >= 0 && yy < p.conv_H && xx >= 0 && xx < p.conv_W) vm |= 1u << t;
    }
    return vm;
}

// Tap of word row j (exact for j * Cw < 2^22) and the pixel shift of a tap.
__device__ __forceinline__ int tap_of_row(int j, const SparseParams& p) { return (int)(((float)j + 0.5f) * p.conv_inv_Cw); }
__device__ __forceinline__ int tap_shift(int tap, int W) {
    const int t3 = (tap * 11) >> 5;                              // tap / 3 for tap < 12
    return (t3 - 1) * W + (tap - 3 * t3 - 1);
}

// A lane's byte offset into the map for tap `tap`: the word at `at` (row base + centre pixel) shifted by the
// tap, or an offset beyond any buffer range (a buffer load out of range returns zero: that is the zero
// padding).  Ranges stay below 2^31 bytes (checked by the entry points).
__device__ __forceinline__ int tap_offset(uint32_t vm, int tap, int at, int shift) {
    return ((vm >> tap) & 1u) ? (at + shift) * 4 : (int)0x80000000u;
}

// Spread the 4 low bits of `nib` to the least significant bits of the 4 bytes of a word.
__device__ __forceinline__ uint32_t spread4(uint32_t nib) { return (nib * 0x00204081u) & 0x01010101u; }

// A table byte is bits 55..48 of a float64 whose other bits are zero: exponent field in the high
// nibble, top of the mantissa in the low one.  Codes 0,1,2,3 map to 0x00, 0xE0, 0xF0, 0xF8, i.e. to
// the (normal) numbers code * 2^-1009, so a byte loaded into the upper half of the high register of
// a zeroed pair IS the multiplicand -- no integer-to-float conversion per residual.  The residuals
// are stored times 2^895 (finite for every float) and the row sums are multiplied by 2^114 at the
// end; powers of two commute with rounding, so the sums are those of the unscaled arithmetic.
constexpr uint32_t kCodeBytes = 0xF8F0E000u;
static_assert(kEntValScaleLog2 == 895, "kSumUnscale undoes 2^895 * 2^-1009");
constexpr double kSumUnscale = 0x1p114;

template <int BITS>
__device__ __forceinline__ void expand_word(uint32_t x0, uint32_t x1, uint8_t* dst_bytes) {
    uint32_t* dst = reinterpret_cast<uint32_t*>(dst_bytes);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint32_t t = spread4((x0 >> (4 * i)) & 0xFu);
        if (BITS == 2) t |= spread4((x1 >> (4 * i)) & 0xFu) << 1;
        // bytes of t: codes of k = 32*j + 4*i + 0..3; each selects its byte of kCodeBytes
        dst[i] = __builtin_amdgcn_perm(0u, kCodeBytes, t);
    }
}

typedef double v16d __attribute__((ext_vector_type(TN)));
typedef double v8d __attribute__((ext_vector_type(8)));

// Eight residuals: acc[key_i.byte0 / 2] += v_i * table[key_i.byte1].
// `acc` is pinned to v[0:31] and `pairs` (eight zeroed register pairs) to v[32:47].  Per entry: the
// byte address (table row of this lane + byte 1 of the key), a byte read into bits 31..16 of the
// pair's high register (the low halves stay zero), and, once the reads have landed, one v_fma_f64
// whose destination and addend are v[0:1] displaced by M0[7:0] = low byte of the key = 2*row.  Only
// the multiply-adds sit inside the indexed region; the mode is off again when the statement ends.
// The wait is for everything (lgkmcnt(0)): scalar loads in flight share the counter and may return
// out of order, so no smaller count would prove that the table reads are back.
// The statement names physical registers (v[0:31], v[32:47], v33 ... v47) under a budget of 64: that holds only
// as long as the compiler keeps nothing else live there, which the parity tests establish for one compiler.
// Validated with AMD clang 22.0 (ROCm 7.2); another major version has to re-run the GPU parity tests before
// this check is moved.
#if !defined(__clang_major__) || __clang_major__ != 22
#error "accumulate8 pins vector registers by name and was validated with AMD clang 22 (ROCm 7.2) only: re-run the GPU parity tests with this compiler, then update this check"
#endif
// The index mode rewrites M0, so M0 is on the clobber list: the compiler then keeps no M0-dependent
// sequence of its own alive across the statement (it warns that M0 is a reserved register, which is the
// point).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void accumulate8(v16d& acc, v8d& pairs, const uint32_t* k, const double* v,
                                            uint32_t table_off) {
    uint32_t t0, t1;
#define APB_SDWA " dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_1 src1_sel:DWORD\n\t"
    asm volatile(
        "v_add_u32_sdwa %2, %4, %20" APB_SDWA "ds_read_u8_d16_hi v33, %2\n\t"
        "v_add_u32_sdwa %3, %5, %20" APB_SDWA "ds_read_u8_d16_hi v35, %3\n\t"
        "v_add_u32_sdwa %2, %6, %20" APB_SDWA "ds_read_u8_d16_hi v37, %2\n\t"
        "v_add_u32_sdwa %3, %7, %20" APB_SDWA "ds_read_u8_d16_hi v39, %3\n\t"
        "v_add_u32_sdwa %2, %8, %20" APB_SDWA "ds_read_u8_d16_hi v41, %2\n\t"
        "v_add_u32_sdwa %3, %9, %20" APB_SDWA "ds_read_u8_d16_hi v43, %3\n\t"
        "v_add_u32_sdwa %2, %10, %20" APB_SDWA "ds_read_u8_d16_hi v45, %2\n\t"
        "v_add_u32_sdwa %3, %11, %20" APB_SDWA "ds_read_u8_d16_hi v47, %3\n\t"
        "s_waitcnt lgkmcnt(0)\n\t"
        "s_set_gpr_idx_on %4, gpr_idx(SRC2,DST)\n\t"
        "v_fma_f64 v[0:1], %12, v[32:33], v[0:1]\n\t"
        "s_set_gpr_idx_idx %5\n\t"
        "v_fma_f64 v[0:1], %13, v[34:35], v[0:1]\n\t"
        "s_set_gpr_idx_idx %6\n\t"
        "v_fma_f64 v[0:1], %14, v[36:37], v[0:1]\n\t"
        "s_set_gpr_idx_idx %7\n\t"
        "v_fma_f64 v[0:1], %15, v[38:39], v[0:1]\n\t"
        "s_set_gpr_idx_idx %8\n\t"
        "v_fma_f64 v[0:1], %16, v[40:41], v[0:1]\n\t"
        "s_set_gpr_idx_idx %9\n\t"
        "v_fma_f64 v[0:1], %17, v[42:43], v[0:1]\n\t"
        "s_set_gpr_idx_idx %10\n\t"
        "v_fma_f64 v[0:1], %18, v[44:45], v[0:1]\n\t"
        "s_set_gpr_idx_idx %11\n\t"
        "v_fma_f64 v[0:1], %19, v[46:47], v[0:1]\n\t"
        "s_set_gpr_idx_off"
        : "+{v[0:31]}"(acc), "+{v[32:47]}"(pairs), "=&v"(t0), "=&v"(t1)
        : "s"(k[0]), "s"(k[1]), "s"(k[2]), "s"(k[3]), "s"(k[4]), "s"(k[5]), "s"(k[6]), "s"(k[7]),
          "s"(v[0]), "s"(v[1]), "s"(v[2]), "s"(v[3]), "s"(v[4]), "s"(v[5]), "s"(v[6]), "s"(v[7]),
          "v"(table_off)
        : "memory", "m0");
#undef APB_SDWA
}
#pragma clang diagnostic pop

// NB (1 to 3) blocks of 8 entries starting at block b.  Keys and values of a block sit side by side,
// so all the scalar loads of a batch leave together and cost one round trip.
template <int NB>
__device__ __forceinline__ void batch(v16d& acc, v8d& pairs, const uint32_t* __restrict__ ent, int b,
                                      uint32_t table_off) {
    uint32_t k[NB][8];
    double v[NB][8];
    const uint32_t* blk = ent + (size_t)b * kEntBlockWords;
#pragma unroll
    for (int h = 0; h < NB; ++h) {
#pragma unroll
        for (int i = 0; i < 8; ++i) k[h][i] = blk[h * kEntBlockWords + i];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[h][i] = reinterpret_cast<const double*>(blk + h * kEntBlockWords + 8)[i];
    }
#pragma unroll
    for (int h = 0; h < NB; ++h) accumulate8(acc, pairs, k[h], v[h], table_off);
}

// Fused mode, first phase: the raw binary product P = sum_k bit * code of a workgroup's rows x 64
// columns on the matrix cores, left in LDS as int32 [rows][64].  A wave computes the 32 x 32 tile
// (tn, tm) over the K steps [s_begin, s_end) (a step is 64 values of k) with one FP4 MFMA per step
// (see apb_fp4_expand.h); rows are launch slots, read from the slot-major sign words (padding slots and
// the pad word row past an odd Kw are zero).  The upper lane half of the last step of an odd Kw
// reads one activation row past its plane -- still inside the packed buffer (the next plane, or the
// column sums) and multiplied by zero weights.  Words are fetched four steps ahead.
// CONV: the activation words come from a packed feature map through the implicit im2col (see
// SparseParams); vm and pin are the tap mask and the input-map column of this lane's column
// m_base + 32*tm + (lane & 31).  The two word rows of a step may belong to different taps (odd Cw).
// FX: the activation words of the workgroup's 64 columns sit in LDS (`lplanes`, [BITS][Kw rounded up to
// even][64], written by quantize_strip).
template <int BITS, bool CONV, bool FX = false>
__device__ __forceinline__ void binary_tile_to_lds(const uint32_t* __restrict__ signT,
                                                   const uint32_t* __restrict__ planes, int Np, int Kw, int Mp,
                                                   int slot_base, int m_base, int tn, int tm, int s_begin, int s_end,
                                                   int lane, int32_t* tile, const SparseParams& p, uint32_t vm, int pin,
                                                   const uint32_t* lplanes = nullptr) {
    const int i = lane & 31, g = lane >> 5;
    const unsigned aoff = (unsigned)(g * Np + slot_base + 32 * tn + i);
    const unsigned boff = (unsigned)(g * Mp + m_base + 32 * tm + i);
    const size_t plane_stride = CONV ? (size_t)p.conv_Cw * p.conv_Mp : (size_t)Kw * Mp;
    // running (tap, word row of the map) of the first word row of the next step to be loaded
    int ld_tap = 0, ld_cw = 0;
    if (CONV) {
        ld_tap = tap_of_row(2 * s_begin, p);
        ld_cw = 2 * s_begin - ld_tap * p.conv_Cw;
    }
    const int steps = (Kw + 1) / 2;
    constexpr int kRing = 4;
    uint32_t aw[kRing][1][1], bw[kRing][BITS][1];
    Frag<1, 1> f[2];
    clear_upper(f[0]);
    clear_upper(f[1]);
    auto load_words = [&](int st, uint32_t (&a)[1][1], uint32_t (&b)[BITS][1]) {
        const int ss = min(st, steps - 1);                      // past the end: harmless re-read, never used
        a[0][0] = (signT + (size_t)(2 * ss) * Np)[aoff];
        if (FX) {
            const int Kw2 = 2 * ((Kw + 1) / 2);
#pragma unroll
            for (int pl = 0; pl < BITS; ++pl) b[pl][0] = lplanes[(pl * Kw2 + 2 * ss + g) * kWave + 32 * tm + i];
        } else if (!CONV) {
#pragma unroll
            for (int pl = 0; pl < BITS; ++pl) b[pl][0] = (planes + pl * plane_stride + (size_t)(2 * ss) * Mp)[boff];
        } else {
            // word row ld_cw of the map under tap ld_tap (lower lane half) and the word row after it (upper half:
            // the next tap's first row where ld_cw is the last of an odd Cw), each shifted by its tap; past the
            // last step the tap runs past 8, whose mask bits are clear: zeros, never used
            const bool wrap = ld_cw + 1 >= p.conv_Cw;
            const int my_tap = g ? ld_tap + (wrap ? 1 : 0) : ld_tap;
            const int my_cw = g ? (wrap ? 0 : ld_cw + 1) : ld_cw;
            const int off = tap_offset(vm, my_tap, my_cw * p.conv_Mp + pin, tap_shift(my_tap, p.conv_W));
#pragma unroll
            for (int pl = 0; pl < BITS; ++pl) {
                const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
                    const_cast<uint32_t*>(planes + pl * plane_stride), 0, p.conv_Cw * p.conv_Mp * 4, kBufferFlags);
                b[pl][0] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, off, 0, 0);
            }
            ld_cw += 2;
            while (ld_cw >= p.conv_Cw) {                        // (twice for Cw = 1)
                ld_cw -= p.conv_Cw;
                ++ld_tap;
            }
        }
    };
    v16f c;
#pragma unroll
    for (int r = 0; r < 16; ++r) c[r] = 0.0f;
#pragma unroll
    for (int q = 0; q < kRing; ++q) load_words(s_begin + q, aw[q], bw[q]);
    expand<1, BITS, 1, 1>(aw[0], bw[0], f[0]);
    auto one_step = [&](int st, int q) {
        const Frag<1, 1>& cur = f[q & 1];
        load_words(st + kRing, aw[q], bw[q]);
        expand<1, BITS, 1, 1>(aw[(q + 1) % kRing], bw[(q + 1) % kRing], f[(q + 1) & 1]);
        c = mfma_fp4(cur.a[0], cur.b[0], c);
    };
    int s0 = s_begin;
    for (; s0 + kRing <= s_end; s0 += kRing) {
#pragma unroll
        for (int q = 0; q < kRing; ++q) one_step(s0 + q, q);
    }
#pragma unroll
    for (int q = 0; q < kRing - 1; ++q)
        if (s0 + q < s_end) one_step(s0 + q, q);
    // C layout of the 32x32 tile: lane (i, g), register r  ->  row 8*(r/4) + 4*g + (r%4), column i.
#pragma unroll
    for (int r = 0; r < 16; ++r)
        tile[(32 * tn + 8 * (r / 4) + 4 * g + (r % 4)) * kWave + 32 * tm + i] = (int)(c[r] * 4.0f);
}

// Epilogue of both kernels: a lane holds, for its column m, the 16 scaled float64 sums of the tile's
// rows (alpha * D included).
//   out_bits == 0: Y[n, m] = float(sum * step).
//   otherwise `out` is the packed activation buffer of the NEXT layer, whose K is this layer's N
//   (planes [out_bits][out_Kw][Mp], then colsum [Mp]; zero-filled before the launch): the value
//   z = scale[n] * y + shift[n] (float64, rounded once to float; z = y without scale) is quantized
//   exactly as apb_quantize_acts does and its code bits are OR-ed into word n / 32 of column m.  The
//   rows of a tile are ascending, so the bits of rows that share a word are gathered in registers
//   and leave as one atomic; rows of other tiles and workgroups add theirs to the same words, in any
//   order (integer OR and add commute).
//   out_exclusive (layers of at most 128 rows in the plain kernel: one workgroup holds every row of its
//   64 columns): the waves meet in LDS instead (`gather`, at most 2 * 4 + 1 rows of 64 words; every wave
//   of the workgroup must make this call) and the finished words and column sums leave as plain,
//   coalesced stores, so the buffer needs no zero fill.
template <int BITS>
__device__ __forceinline__ void write_rows(const v16d& acc, int slot0, int m, const int32_t* __restrict__ perm,
                                           const double* __restrict__ slot_valsum, const float* __restrict__ scale,
                                           const float* __restrict__ shift, float* out, const SparseParams& p,
                                           uint32_t* gather = nullptr) {
    const bool col_ok = m < p.M;
    int n[TN];
    double y[TN];
#pragma unroll
    for (int r = 0; r < TN; ++r) n[r] = perm[slot0 + r];
#pragma unroll
    for (int r = 0; r < TN; ++r) {
        // 1-bit activations: the table holds (c+1)/2 in {0,1}: sum val*c = 2*sum val*code - sum val.
        const double sum = acc[r] * kSumUnscale;
        y[r] = (BITS == 1 ? 2.0 * sum - slot_valsum[slot0 + r] : sum) * p.step;
    }
    if (p.out_bits == 0) {
#pragma unroll
        for (int r = 0; r < TN; ++r)
            if (col_ok && n[r] >= 0) out[(size_t)n[r] * p.M + m] = (float)y[r];
        return;
    }
    uint32_t* words = reinterpret_cast<uint32_t*>(out);
    const size_t plane = (size_t)p.out_Kw * p.Mp;
    const bool excl = gather != nullptr && p.out_exclusive;
    const int lane = m & (kWave - 1);
    const int gather_rows = p.out_bits * p.out_Kw + 1;          // word rows of both planes, then the column sums
    if (excl) {
        __syncthreads();                                        // every wave is done with the code tables
        for (int i = threadIdx.x; i < gather_rows * kWave; i += blockDim.x) gather[i] = 0u;
        __syncthreads();
    }
    uint32_t w0 = 0, w1 = 0;
    int total = 0;
#pragma unroll
    for (int r = 0; r < TN; ++r) {
        if (n[r] < 0) continue;                                 // padding slot (wave-uniform)
        double z = y[r];
        if (scale) z = fma((double)scale[n[r]], z, (double)shift[n[r]]);
        const float zf = (float)z;
        uint32_t code = p.out_bits == 1 ? (zf >= 0.0f ? 1u : 0u) : code2(zf, p.out_inv_step);
        if (!col_ok) code = 0;
        w0 |= (code & 1u) << (n[r] & 31);
        w1 |= (code >> 1) << (n[r] & 31);
        total += (int)code;
        const bool last_of_word = r == TN - 1 || n[r + 1] < 0 || (n[r + 1] >> 5) != (n[r] >> 5);
        if (last_of_word) {
            if (excl) {
                uint32_t* at = gather + (n[r] >> 5) * kWave + lane;
                if (w0) __hip_atomic_fetch_or(at, w0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                if (w1) __hip_atomic_fetch_or(at + p.out_Kw * kWave, w1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            } else {
                const size_t at = (size_t)(n[r] >> 5) * p.Mp + m;
                if (w0) __hip_atomic_fetch_or(words + at, w0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (w1) __hip_atomic_fetch_or(words + plane + at, w1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            w0 = w1 = 0;
        }
    }
    if (!excl) {
        if (total)
            __hip_atomic_fetch_add(reinterpret_cast<int32_t*>(words + p.out_bits * plane) + m, total, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    if (total)
        __hip_atomic_fetch_add(gather + (gather_rows - 1) * kWave + lane, (uint32_t)total, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_WORKGROUP);
    __syncthreads();
    // row i of `gather` is word row i of the packed output (planes one after the other, then the sums),
    // columns of this workgroup's strip
    const int m0 = m - lane;
    for (int i = threadIdx.x; i < gather_rows * kWave; i += blockDim.x)
        words[(size_t)(i / kWave) * p.Mp + m0 + (i & (kWave - 1))] = gather[i];
}

// Sum of the codes of column m: read as it stands, or (CONV) added up over the taps of the patch from
// the per-pixel sums of the feature map.
template <bool CONV>
__device__ __forceinline__ int column_code_sum(const int32_t* __restrict__ colsum, int m, uint32_t vm, int pin,
                                               const SparseParams& p) {
    if (!CONV) return colsum[m];
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t*>(colsum), 0, p.conv_Mp * 4, kBufferFlags);
    int cs = 0;
#pragma unroll
    for (int t = 0; t < 9; ++t)
        cs += (int)__builtin_amdgcn_raw_buffer_load_b32(rsrc, tap_offset(vm, t, pin, tap_shift(t, p.conv_W)), 0, 0);
    return cs;
}

// Word row j of the activations for this lane's column (byte offset m_off = 4 * m), plane b: a buffer
// load whose descriptor carries the wave-uniform row (range = one row of Mp words) and to which the
// lane adds its 32-bit offset.  Rows past Kw re-read the last row (plain matrix) or return zero
// (CONV: their tap has no mask bit); they are never expanded.  The load is unconditional and unmasked
// so that the wait for it can sit at the next chunk.
template <bool CONV>
__device__ __forceinline__ uint32_t load_act_word(const uint32_t* __restrict__ planes, size_t plane_stride, int b, int j,
                                                  int m_off, uint32_t vm, int pin, const SparseParams& p) {
    if (!CONV) {
        const uint32_t* row = planes + (b * plane_stride + (size_t)min(j, p.Kw - 1) * p.Mp);
        const __amdgpu_buffer_rsrc_t rsrc =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(row), 0, p.Mp * 4, kBufferFlags);
        return __builtin_amdgcn_raw_buffer_load_b32(rsrc, m_off, 0, 0);
    }
    const int tap = tap_of_row(j, p);
    const int cw = j - tap * p.conv_Cw;
    const uint32_t* row = planes + (b * plane_stride + (size_t)cw * p.conv_Mp);
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(row), 0, p.conv_Mp * 4, kBufferFlags);
    return __builtin_amdgcn_raw_buffer_load_b32(rsrc, tap_offset(vm, tap, pin, tap_shift(tap, p.conv_W)), 0, 0);
}

// FX kernels, phase 0: quantize the workgroup's strip of 64 columns of the float matrix X (K x M,
// row-major) and leave its packed words in LDS -- lplanes[BITS][Kw2][64] (Kw2 = Kw rounded up to even,
// the extra row zero) and the column sums lcol[64] -- instead of HBM.  The arithmetic is that of
// apb_quantize_acts, bit for bit (same code2, same masks).  Waves take the words of K round-robin; a
// wave's load of one row of X is one contiguous 256-byte segment, 32 of them in flight.
template <int BITS>
__device__ __forceinline__ void quantize_strip(const float* __restrict__ X, const SparseParams& p, int m, int wave,
                                               int waves, int lane, uint32_t* lplanes, int32_t* lcol) {
    const int Kw2 = 2 * ((p.Kw + 1) / 2);
    if (wave == 0) lcol[lane] = 0;
    __syncthreads();
    const bool col_ok = m < p.M;
    const unsigned mc = (unsigned)min(m, p.M - 1);
    int sum = 0;
    for (int j = wave; j < Kw2; j += waves) {
        uint32_t w0 = 0, w1 = 0;
        if (j < p.Kw) {
            const int k0 = 32 * j;
            float xv[32];                                       // one word of K: 32 independent loads in flight
#pragma unroll
            for (int i = 0; i < 32; ++i)
                xv[i] = __builtin_nontemporal_load((X + (size_t)min(k0 + i, p.K - 1) * p.M) + mc);
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                if (BITS == 1) {
                    w0 |= (xv[i] >= 0.0f ? 1u : 0u) << i;
                } else {
                    const uint32_t c = code2_low_bits(xv[i], p.in_inv_step);
                    w0 = push_bit(w0, c);
                    w1 = push_bit(w1, c >> 1);
                }
            }
            const int valid = p.K - k0;
            const uint32_t keep = !col_ok ? 0u : (valid >= 32 ? 0xffffffffu : ((1u << valid) - 1u));
            w0 &= keep;
            w1 &= keep;
            sum += __builtin_popcount(w0) + 2 * __builtin_popcount(w1);
        }
        lplanes[j * kWave + lane] = w0;
        if (BITS == 2) lplanes[(Kw2 + j) * kWave + lane] = w1;
    }
    if (sum) __hip_atomic_fetch_add(lcol + lane, sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __syncthreads();
}

// WPW = words of a chunk each wave expands = 8 / waves per workgroup.
// CONV: 3x3 convolution over a packed feature map (implicit im2col, see SparseParams).
// FX: `planes` is the float matrix X itself; the workgroup quantizes its strip into LDS first (only for
// layers whose rows all sit in one workgroup, so that no strip is quantized twice).
template <int BITS, int WPW, bool CONV, bool FX = false>
__global__ __launch_bounds__(kWave* kChunkWords / WPW) __attribute__((amdgpu_waves_per_eu(WPW <= 2 ? 8 : 4, 8))) void k_sparse_epilogue(
    // Separate restrict-qualified arguments (not struct members) so that the compiler knows the
    // read-only arrays cannot alias Y and keeps the wave-uniform loads on the scalar path.
    const uint32_t* __restrict__ planes, const int32_t* __restrict__ colsum, const int32_t* __restrict__ rowsum,
    const int32_t* __restrict__ perm,
    const int32_t* __restrict__ seg_ptr,     // [tiles][nchunks+1] first entry block of (tile, chunk)
    const uint32_t* __restrict__ ent,        // blocks of 8 keys + 8 scaled residuals
    const double* __restrict__ slot_valsum,
    const uint32_t* __restrict__ signT,      // [Kw rounded up to even][Np] slot-major sign words
    const float* __restrict__ scale, const float* __restrict__ shift,   // [N] each or both null (packed output)
    float* __restrict__ out,                 // Y, or the packed buffer of the next layer (see write_rows)
    const SparseParams p) {
    extern __shared__ __align__(16) uint8_t lds[];
    constexpr int waves = kChunkWords / WPW;
    constexpr int kBufs = table_buffers(WPW);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of tasks so
    // that the row groups sharing one activation strip also share one L2.
    int task = blockIdx.x;
    if ((p.blocks & 7) == 0) task = (blockIdx.x & 7) * (p.blocks >> 3) + (blockIdx.x >> 3);
    const int rg = task % p.row_groups;
    const int strip = task / p.row_groups;
    const int tile = rg * waves + wave;
    const int slot0 = tile * TN;
    const int m = strip * kWave + lane;                         // < Mp: the strips tile Mp exactly
    const int m_off = m * 4;                                    // the launcher keeps 4 * Mp below 2^31

    static_assert(TN == 16, "row field of an entry key addresses 16 register pairs");
    static_assert(!(CONV && FX), "float input goes with the plain matrix form");
    int pin = 0;                                                // CONV: the lane's column in the input map
    const uint32_t vm = CONV ? conv_pixel(m, p, pin) : 0u;
    uint32_t* lplanes = reinterpret_cast<uint32_t*>(lds + kBufs * kTableBytes);      // FX only
    int32_t* lcol = reinterpret_cast<int32_t*>(lplanes + BITS * (2 * ((p.Kw + 1) / 2)) * kWave);
    if (FX) quantize_strip<BITS>(reinterpret_cast<const float*>(planes), p, m, wave, waves, lane, lplanes, lcol);
    v16d acc;
    {
        // Binary part first; every lane then picks up the 16 products of its column and starts its
        // float64 sums at alpha * D (in the scaled domain of the residual products, and halved for
        // 1-bit activations, whose sum is doubled at the end).  The tile shares LDS with the code
        // tables, hence the second barrier.
        int32_t* tile_lds = reinterpret_cast<int32_t*>(lds);
        // (the binary tile's column of a lane is column 32 * (wave & 1) + (lane & 31) of the strip: its mask
        // is that lane's)
        const uint32_t vm_tile = CONV ? (uint32_t)__shfl((int)vm, 32 * (wave & 1) + (lane & 31)) : 0u;
        const int pin_tile = CONV ? __shfl(pin, 32 * (wave & 1) + (lane & 31)) : 0;
        binary_tile_to_lds<BITS, CONV, FX>(signT, planes, p.Np, p.Kw, p.Mp, rg * waves * TN, strip * kWave, wave >> 1,
                                           wave & 1, 0, (p.Kw + 1) / 2, lane, tile_lds, p, vm_tile, pin_tile, lplanes);
        __syncthreads();
        int P[TN];
#pragma unroll
        for (int r = 0; r < TN; ++r) P[r] = tile_lds[(wave * TN + r) * kWave + lane];
        __syncthreads();
        const int cs = FX ? lcol[lane] : column_code_sum<CONV>(colsum, m, vm, pin, p);
        const double a0 = p.alpha * (BITS == 1 ? 0.5 : 1.0) * (1.0 / kSumUnscale);
#pragma unroll
        for (int r = 0; r < TN; ++r) {
            const int nr = perm[slot0 + r];
            const int d = BITS == 1 ? 4 * P[r] - rowsum[max(nr, 0)] - 2 * cs : 2 * P[r] - cs;
            acc[r] = a0 * (double)d;
        }
    }
    v8d pairs;
#pragma unroll
    for (int r = 0; r < 8; ++r) pairs[r] = 0.0;

    const size_t plane_stride = CONV ? (size_t)p.conv_Cw * p.conv_Mp : (size_t)p.Kw * p.Mp;
    uint8_t* my_row = lds + lane * kTablePitch;
    const uint32_t my_row_off = (uint32_t)(uintptr_t)(lds_u8*)my_row;   // the same row as an LDS byte address
    const int32_t* seg = seg_ptr + (size_t)tile * (p.nchunks + 1);

    // Words this wave expands in a chunk: jj = wave, wave + waves, ...  They are fetched one chunk
    // ahead so that their latency hides behind the residual loop of the chunk before.
    uint32_t xw[BITS][WPW];
    auto fetch = [&](int c) {
#pragma unroll
        for (int i = 0; i < WPW; ++i) {
            const int j = c * kChunkWords + wave + i * waves;
#pragma unroll
            for (int b = 0; b < BITS; ++b)
                xw[b][i] = FX ? lplanes[(b * (2 * ((p.Kw + 1) / 2)) + min(j, p.Kw - 1)) * kWave + lane]
                              : load_act_word<CONV>(planes, plane_stride, b, j, m_off, vm, pin, p);
        }
    };
    fetch(0);
    int e1 = seg[0];

    for (int c = 0; c < p.nchunks; ++c) {
        // Large workgroups alternate between two table buffers (one barrier per chunk); small ones keep
        // one buffer, so that twice as many of them fit a CU, and pay a second barrier.
        const int buf = kBufs == 2 ? (c & 1) * kTableBytes : 0;
        if (kBufs == 1 && c > 0) __syncthreads();               // every wave has finished reading the table
#pragma unroll
        for (int i = 0; i < WPW; ++i) {
            const int jj = wave + i * waves;
            if (c * kChunkWords + jj < p.Kw)                    // no residual refers to columns >= K
                expand_word<BITS>(xw[0][i], xw[BITS - 1][i], my_row + buf + 32 * jj);
        }
        if (c + 1 < p.nchunks) fetch(c + 1);
        int e = e1;
        e1 = seg[c + 1];
        __syncthreads();                                        // the chunk's code table is complete

        // Two blocks (16 entries) per scalar-load round trip while they last, then at most one block.
        // A large batch is what amortises the scalar-cache latency.
        const uint32_t table_off = my_row_off + buf;
        for (; e + 2 <= e1; e += 2) batch<2>(acc, pairs, ent, e, table_off);
        if (e < e1) batch<1>(acc, pairs, ent, e, table_off);
        // With two buffers the next chunk writes the other one; this one is rewritten two chunks from
        // now, after every wave has passed the next barrier, i.e. has finished reading it.
    }

    // (The column is recomputed from the lane number here rather than kept in a register -- or
    // spilled -- through the loops above.)
    const int m_e = strip * kWave + (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    write_rows<BITS>(acc, slot0, m_e, perm, slot_valsum, scale, shift, out, p, reinterpret_cast<uint32_t*>(lds));
}

// The same forward for launches that would leave most of the chip idle (few column strips, few row
// groups): the 8 waves of a workgroup are KS parts of K times 8/KS tiles, so a workgroup covers fewer
// rows and there are KS times as many waves, each with 1/KS of the chunks of its tile.  Part kp of
// K = chunks [kp*H, (kp+1)*H), H = ceil(nchunks / KS), and the K steps [kp*SP, (kp+1)*SP) of the
// binary product.  Every part has its own code table (KS buffers, rebuilt together once per round by
// all 8 waves: wave w expands word w of each), the partial binary products meet in LDS before the
// residual loop (part 0 starts its sums at alpha*D, the others at zero) and the partial float64 sums
// meet in LDS after it, added in a fixed order by part 0, which writes Y.  All waves run the same
// number of barriers whatever their run lengths.
template <int BITS, int KS, bool CONV>
__global__ __launch_bounds__(kWave* kChunkWords) __attribute__((amdgpu_waves_per_eu(4, 8))) void k_forward_ksplit(
    const uint32_t* __restrict__ planes, const int32_t* __restrict__ colsum, const int32_t* __restrict__ rowsum,
    const int32_t* __restrict__ perm, const int32_t* __restrict__ seg_ptr, const uint32_t* __restrict__ ent,
    const double* __restrict__ slot_valsum, const uint32_t* __restrict__ signT, const float* __restrict__ scale,
    const float* __restrict__ shift, float* __restrict__ out, const SparseParams p) {
    extern __shared__ __align__(16) uint8_t lds[];
    constexpr int TW = kChunkWords / KS;                         // tiles (of 16 rows) per workgroup
    static_assert(KS == 2 || KS == 4, "two or four parts of K");
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    int task = blockIdx.x;
    if ((p.blocks & 7) == 0) task = (blockIdx.x & 7) * (p.blocks >> 3) + (blockIdx.x >> 3);
    const int rg = task % p.row_groups;                          // row group of TW tiles
    const int strip = task / p.row_groups;
    const int tl = wave % TW, kp = wave / TW;
    const int tile = rg * TW + tl;
    const int slot0 = tile * TN;
    const int m = strip * kWave + lane;
    const int m_off = m * 4;
    const int H = (p.nchunks + KS - 1) / KS;
    int pin = 0;                                                // CONV: the lane's column in the input map
    const uint32_t vm = CONV ? conv_pixel(m, p, pin) : 0u;

    // binary part: wave (tl, kp) computes 32 x 32 tile tl of the workgroup's 16*TW x 64 block over
    // its share of the K steps
    int32_t* part_lds = reinterpret_cast<int32_t*>(lds);        // [KS][16 * TW][64]
    {
        const int steps = (p.Kw + 1) / 2;
        const int SP = (steps + KS - 1) / KS;
        const int s_begin = min(steps, kp * SP), s_end = min(steps, s_begin + SP);
        const uint32_t vm_tile = CONV ? (uint32_t)__shfl((int)vm, 32 * (tl & 1) + (lane & 31)) : 0u;
        const int pin_tile = CONV ? __shfl(pin, 32 * (tl & 1) + (lane & 31)) : 0;
        binary_tile_to_lds<BITS, CONV>(signT, planes, p.Np, p.Kw, p.Mp, rg * TW * TN, strip * kWave, tl >> 1, tl & 1,
                                       s_begin, s_end, lane, part_lds + kp * (TN * TW * kWave), p, vm_tile, pin_tile);
    }
    __syncthreads();
    v16d acc;
    if (kp == 0) {
        int P[TN];
#pragma unroll
        for (int r = 0; r < TN; ++r) {
            P[r] = 0;
#pragma unroll
            for (int q = 0; q < KS; ++q) P[r] += part_lds[q * (TN * TW * kWave) + (tl * TN + r) * kWave + lane];
        }
        const int cs = column_code_sum<CONV>(colsum, m, vm, pin, p);
        const double a0 = p.alpha * (BITS == 1 ? 0.5 : 1.0) * (1.0 / kSumUnscale);
#pragma unroll
        for (int r = 0; r < TN; ++r) {
            const int nr = perm[slot0 + r];
            const int d = BITS == 1 ? 4 * P[r] - rowsum[max(nr, 0)] - 2 * cs : 2 * P[r] - cs;
            acc[r] = a0 * (double)d;
        }
    } else {
#pragma unroll
        for (int r = 0; r < TN; ++r) acc[r] = 0.0;
    }
    v8d pairs;
#pragma unroll
    for (int r = 0; r < 8; ++r) pairs[r] = 0.0;
    __syncthreads();                                            // the partial products are read; tables may overwrite them

    const size_t plane_stride = CONV ? (size_t)p.conv_Cw * p.conv_Mp : (size_t)p.Kw * p.Mp;
    uint8_t* my_row = lds + lane * kTablePitch;
    const uint32_t my_row_off = (uint32_t)(uintptr_t)(lds_u8*)my_row;
    const int32_t* seg = seg_ptr + (size_t)tile * (p.nchunks + 1);

    // word `wave` of chunk q*H + i for every part q, fetched one round ahead
    uint32_t xw[BITS][KS];
    auto fetch = [&](int i) {
#pragma unroll
        for (int q = 0; q < KS; ++q) {
            const int j = (q * H + i) * kChunkWords + wave;
#pragma unroll
            for (int b = 0; b < BITS; ++b) xw[b][q] = load_act_word<CONV>(planes, plane_stride, b, j, m_off, vm, pin, p);
        }
    };
    fetch(0);
    for (int i = 0; i < H; ++i) {
        if (i > 0) __syncthreads();                             // every wave has finished reading the tables
#pragma unroll
        for (int q = 0; q < KS; ++q) {
            const int c = q * H + i;
            if (c < p.nchunks && c * kChunkWords + wave < p.Kw)
                expand_word<BITS>(xw[0][q], xw[BITS - 1][q], my_row + q * kTableBytes + 32 * wave);
        }
        if (i + 1 < H) fetch(i + 1);
        const int c = min(kp * H + i, p.nchunks);               // past the end: an empty run
        int e = seg[c];
        const int e1 = seg[min(c + 1, p.nchunks)];
        __syncthreads();                                        // the tables of this round are complete
        const uint32_t table_off = my_row_off + kp * kTableBytes;
        // (three blocks per scalar round trip: at this occupancy the scalar registers are there)
        for (; e + 3 <= e1; e += 3) batch<3>(acc, pairs, ent, e, table_off);
        if (e + 2 <= e1) {
            batch<2>(acc, pairs, ent, e, table_off);
            e += 2;
        }
        if (e < e1) batch<1>(acc, pairs, ent, e, table_off);
    }

    // the partial sums of parts 1.. go through LDS to part 0
    __syncthreads();                                            // every wave is done with the tables
    double* red = reinterpret_cast<double*>(lds);               // [KS - 1][TW][16][64]
    if (kp > 0) {
#pragma unroll
        for (int r = 0; r < TN; ++r) red[(((kp - 1) * TW + tl) * TN + r) * kWave + lane] = acc[r];
    }
    __syncthreads();
    if (kp > 0) return;
#pragma unroll
    for (int q = 1; q < KS; ++q)
#pragma unroll
        for (int r = 0; r < TN; ++r) acc[r] += red[(((q - 1) * TW + tl) * TN + r) * kWave + lane];

    write_rows<BITS>(acc, slot0, m, perm, slot_valsum, scale, shift, out, p);
}


// The packed patch matrix of a convolution written out: word row tap * Cw + cw of column m (an output pixel) is
// word row cw of the map at the pixel shifted by the tap, or zero outside the image; the column sum is the sum
// of the per-pixel sums over the valid taps.  Bit words only -- 1/16 (2-bit) or 1/32 (1-bit) of the float im2col
// matrix.  For layers that run faster on the plain-matrix kernel with the lanes along the rows (apb_rows.hip) than
// on the implicit gather.  Thread = one column of one tap and a slab of kPatchRows word rows of the map.
constexpr int kPatchRows = 8;

template <int BITS>
__global__ __launch_bounds__(128) void k_pack_patches(const uint32_t* __restrict__ planes, const int32_t* __restrict__ pixsum,
                                                     uint32_t* __restrict__ out, int32_t* __restrict__ out_colsum,
                                                     uint32_t* __restrict__ clear, size_t clear_words, const SparseParams p) {
    // On the side: clear `clear_words` words at `clear` (the packed output buffer of a kernel that ORs into it --
    // one launch less than a fill kernel of its own).
    {
        const size_t threads = (size_t)gridDim.x * gridDim.y * gridDim.z * 128;
        const size_t me = (((size_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * 128 + threadIdx.x;
        for (size_t i = me; i < clear_words; i += threads) clear[i] = 0u;
    }
    // blockIdx.y = tap, blockIdx.z = slab of kPatchRows word rows of the map: validity and shift are computed once
    const int m = blockIdx.x * 128 + threadIdx.x;               // < Mp: the grid tiles Mp (a multiple of 64) in 128s
    if (m >= p.Mp) return;
    int pin = 0;
    const uint32_t vm = conv_pixel(m, p, pin);
    const int tap = blockIdx.y;
    const bool ok = (vm >> tap) & 1u;
    const size_t in_stride = (size_t)p.conv_Cw * p.conv_Mp, out_stride = (size_t)p.Kw * p.Mp;
    const int cw0 = blockIdx.z * kPatchRows, cw1 = min(p.conv_Cw, cw0 + kPatchRows);
    const uint32_t* src = planes + (ok ? (size_t)(pin + tap_shift(tap, p.conv_W)) : 0);
    uint32_t* dst = out + (size_t)tap * p.conv_Cw * p.Mp + m;
    uint32_t w[kPatchRows][BITS];                               // all loads of the slab in flight, then the stores
#pragma unroll
    for (int i = 0; i < kPatchRows; ++i)
#pragma unroll
        for (int pl = 0; pl < BITS; ++pl)
            w[i][pl] = ok ? src[pl * in_stride + (size_t)min(cw0 + i, cw1 - 1) * p.conv_Mp] : 0u;
#pragma unroll
    for (int i = 0; i < kPatchRows; ++i)
        if (cw0 + i < cw1) {
#pragma unroll
            for (int pl = 0; pl < BITS; ++pl) dst[pl * out_stride + (size_t)(cw0 + i) * p.Mp] = w[i][pl];
        }
    if (tap == 0 && blockIdx.z == 0) {
        int cs = 0;
#pragma unroll
        for (int t = 0; t < 9; ++t)
            if ((vm >> t) & 1u) cs += pixsum[pin + tap_shift(t, p.conv_W)];
        out_colsum[m] = cs;
    }
}

template <int KS>
constexpr int ksplit_lds_bytes() {
    constexpr int tables = KS * kTableBytes;
    constexpr int partial_products = KS * TN * (kChunkWords / KS) * kWave * 4;
    constexpr int partial_sums = (KS - 1) * (kChunkWords / KS) * TN * kWave * 8;
    return tables > partial_products ? (tables > partial_sums ? tables : partial_sums)
                                     : (partial_products > partial_sums ? partial_products : partial_sums);
}

struct OutArgs {
    const float* scale;
    const float* shift;
    float* out;
};

template <int BITS, int KS, bool CONV>
int launch_ksplit(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, const OutArgs& o, SparseParams p,
                  hipStream_t s) {
    constexpr int TW = kChunkWords / KS;
    constexpr int kLds = ksplit_lds_bytes<KS>();
    p.row_groups = L.Np / (TN * TW);
    const long long blocks = (long long)p.row_groups * (p.Mp / kWave);
    if (blocks > 0x7fffffffLL) return APB_ERR_SHAPE;
    p.blocks = (int)blocks;
    if (kLds > 64 * 1024) {                                     // more LDS than a launch gets without asking:
        static std::atomic<bool> asked[kMaxDevices];            // asked for once per device, not per launch
        int dev = 0;
        APB_HIP(hipGetDevice(&dev));
        if (dev < 0 || dev >= kMaxDevices) return APB_ERR_SHAPE;
        if (!asked[dev].load(std::memory_order_acquire)) {
            APB_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_forward_ksplit<BITS, KS, CONV>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, kLds));
            asked[dev].store(true, std::memory_order_release);
        }
    }
    hipLaunchKernelGGL((k_forward_ksplit<BITS, KS, CONV>), dim3((unsigned)p.blocks), dim3(kWave * kChunkWords), kLds, s,
                       planes, colsum, L.rowsum, L.perm, L.seg_ptr, L.ent, L.slot_valsum, L.signT, o.scale, o.shift, o.out,
                       p);
    return APB_OK;
}

template <int BITS, int WPW, bool CONV>
void launch_one(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, const OutArgs& o, const SparseParams& p,
                hipStream_t s) {
    hipLaunchKernelGGL((k_sparse_epilogue<BITS, WPW, CONV>), dim3((unsigned)p.blocks), dim3(kWave * kChunkWords / WPW),
                       table_buffers(WPW) * kTableBytes, s, planes, colsum, L.rowsum, L.perm, L.seg_ptr, L.ent,
                       L.slot_valsum, L.signT, o.scale, o.shift, o.out, p);
}

// LDS of a float-input launch: the code tables, then the strip's packed words and column sums.
int float_input_lds_bytes(const LayerDev& L, int bits) {
    const int wpw = kChunkWords / L.waves;
    return table_buffers(wpw) * kTableBytes + bits * (2 * ((L.Kw + 1) / 2)) * kWave * 4 + kWave * 4;
}

template <int BITS, int WPW>
void launch_one_float(const LayerDev& L, const float* X, const OutArgs& o, const SparseParams& p, hipStream_t s) {
    hipLaunchKernelGGL((k_sparse_epilogue<BITS, WPW, false, true>), dim3((unsigned)p.blocks),
                       dim3(kWave * kChunkWords / WPW), float_input_lds_bytes(L, BITS), s,
                       reinterpret_cast<const uint32_t*>(X), static_cast<const int32_t*>(nullptr), L.rowsum, L.perm,
                       L.seg_ptr, L.ent, L.slot_valsum, L.signT, o.scale, o.shift, o.out, p);
}

template <int BITS>
int launch_bits_float(const LayerDev& L, const float* X, const OutArgs& o, const SparseParams& p, hipStream_t s) {
    switch (L.waves) {
        case 8: launch_one_float<BITS, 1>(L, X, o, p, s); break;
        case 4: launch_one_float<BITS, 2>(L, X, o, p, s); break;
        case 2: launch_one_float<BITS, 4>(L, X, o, p, s); break;
        default: return APB_ERR_SHAPE;
    }
    return APB_OK;
}

template <int BITS, bool CONV>
int launch_bits(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, const OutArgs& o, const SparseParams& p,
                int ks, hipStream_t s) {
    if (ks == 2) return launch_ksplit<BITS, 2, CONV>(L, planes, colsum, o, p, s);
    if (ks == 4) return launch_ksplit<BITS, 4, CONV>(L, planes, colsum, o, p, s);
    switch (L.waves) {
        case 8: launch_one<BITS, 1, CONV>(L, planes, colsum, o, p, s); break;
        case 4: launch_one<BITS, 2, CONV>(L, planes, colsum, o, p, s); break;
        case 2: launch_one<BITS, 4, CONV>(L, planes, colsum, o, p, s); break;
        default: return APB_ERR_SHAPE;
    }
    return APB_OK;
}

// Launches of 8-wave workgroups that would put fewer than ~3000 waves on the chip split K two or four
// ways inside the workgroup instead (see k_forward_ksplit).
int ksplit_parts(const LayerDev& L, long long blocks) {
    int ks = 1;
    if (L.waves == 8) {
        if (blocks * 8 < 3000 && L.nchunks >= 2) ks = 2;
        if (blocks * 16 < 3000 && L.nchunks >= 4) ks = 4;
    }
    return ks;
}

// X != nullptr: float activations, quantized inside the kernel (see forward_float_applies).
int launch_any(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, int M, int bits, float step,
               const ConvShape* conv, const OutArgs& o, int out_bits, float out_inv_step, hipStream_t s,
               const float* X = nullptr) {
    if (!mfma_sum_exact(L.K, 1, bits == 1 ? 1 : 3)) return APB_ERR_SHAPE;
    const int Mp = kWave * ((M + kWave - 1) / kWave);
    SparseParams p;
    p.alpha = (double)L.alpha;
    p.step = (double)step;
    p.Np = L.Np;
    p.Kw = L.Kw;
    p.Mp = Mp;
    p.M = M;
    p.nchunks = L.nchunks;
    p.out_bits = out_bits;
    p.out_exclusive = 0;
    p.out_Kw = (L.N + 31) / 32;
    p.out_inv_step = out_inv_step;
    p.conv_Cw = conv ? conv->C / 32 : 0;
    p.conv_H = conv ? conv->H : 0;
    p.conv_W = conv ? conv->W : 0;
    p.conv_Ho = conv ? conv->Ho : 1;
    p.conv_Wo = conv ? conv->Wo : 1;
    p.conv_stride = conv ? conv->stride : 1;
    p.conv_Mp = conv ? conv->Pp_in : 0;
    p.conv_inv_Cw = conv ? 1.0f / (float)(conv->C / 32) : 0.0f;
    p.K = L.K;
    p.in_inv_step = 1.0f / step;
    p.row_groups = L.Np / (TN * L.waves);
    const long long blocks = (long long)p.row_groups * (Mp / kWave);
    if (blocks > 0x7fffffffLL || (long long)Mp * 8 >= (1LL << 31)) return APB_ERR_SHAPE;
    p.blocks = (int)blocks;
    const int ks = X ? 1 : ksplit_parts(L, blocks);
    int rc;
    if (out_bits != 0) {
        // One workgroup holds every row of its columns: it stores whole words, nothing to clear.  Otherwise
        // the workgroups OR their bits into a buffer cleared here (a fill kernel, not a memset node: the
        // call may be recorded into a graph).
        p.out_exclusive = p.row_groups == 1 && ks == 1;
        if (!p.out_exclusive) {
            rc = launch_zero_words(reinterpret_cast<uint32_t*>(o.out), ((size_t)out_bits * p.out_Kw + 1) * Mp, s);
            if (rc != APB_OK) return rc;
        }
    }
    if (X) rc = bits == 1 ? launch_bits_float<1>(L, X, o, p, s) : launch_bits_float<2>(L, X, o, p, s);
    else if (conv) rc = bits == 1 ? launch_bits<1, true>(L, planes, colsum, o, p, ks, s) : launch_bits<2, true>(L, planes, colsum, o, p, ks, s);
    else rc = bits == 1 ? launch_bits<1, false>(L, planes, colsum, o, p, ks, s) : launch_bits<2, false>(L, planes, colsum, o, p, ks, s);
    if (rc != APB_OK) return rc;
    APB_HIP(hipGetLastError());
    return APB_OK;
}

}  // namespace

// conv == nullptr: `planes` is the packed K x M matrix.  Otherwise it is a packed feature map of conv->C
// channels (L.K = 9 * C, C a multiple of 32) and M = B * Ho * Wo output pixels, read through the implicit im2col.
int launch_forward(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, int M, int bits, float step,
                   const ConvShape* conv, float* Y, hipStream_t s) {
    return launch_any(L, planes, colsum, M, bits, step, conv, OutArgs{nullptr, nullptr, Y}, 0, 0.0f, s);
}

// conv -> the packed K x M patch matrix in `out` (planes, then column sums: apb_acts_bytes(9 * C, M, bits) bytes);
// clears `clear_words` words at `clear` as well (nullptr, 0: nothing)
int launch_pack_patches(const LayerDev& L, const uint32_t* planes, const int32_t* pixsum, int M, int bits,
                        const ConvShape& conv, uint32_t* out, uint32_t* clear, size_t clear_words, hipStream_t s) {
    const int Mp = kWave * ((M + kWave - 1) / kWave);
    SparseParams p{};
    p.Kw = L.Kw;
    p.Mp = Mp;
    p.M = M;
    p.conv_Cw = conv.C / 32;
    p.conv_H = conv.H;
    p.conv_W = conv.W;
    p.conv_Ho = conv.Ho;
    p.conv_Wo = conv.Wo;
    p.conv_stride = conv.stride;
    p.conv_Mp = conv.Pp_in;
    p.conv_inv_Cw = 1.0f / (float)(conv.C / 32);
    int32_t* out_colsum = reinterpret_cast<int32_t*>(out + (size_t)bits * L.Kw * Mp);
    const dim3 grid((unsigned)((Mp + 127) / 128), 9u, (unsigned)((p.conv_Cw + kPatchRows - 1) / kPatchRows));
    if (bits == 1)
        hipLaunchKernelGGL(k_pack_patches<1>, grid, dim3(128), 0, s, planes, pixsum, out, out_colsum, clear, clear_words, p);
    else
        hipLaunchKernelGGL(k_pack_patches<2>, grid, dim3(128), 0, s, planes, pixsum, out, out_colsum, clear, clear_words, p);
    APB_HIP(hipGetLastError());
    return APB_OK;
}

// Quantize + forward in one kernel applies when one workgroup holds every row of the layer (so that no
// strip of X is quantized twice), the launch fills the chip without splitting K, and the strip's packed
// words fit the LDS a launch gets without asking.
bool forward_float_applies(const LayerDev& L, int M, int bits) {
    const long long Mp = (long long)kWave * ((M + kWave - 1) / kWave);
    if (L.Np != TN * L.waves) return false;
    if (ksplit_parts(L, Mp / kWave) != 1) return false;
    return float_input_lds_bytes(L, bits) <= 64 * 1024;
}

int launch_forward_float(const LayerDev& L, const float* X, int M, int bits, float step, float* Y, hipStream_t s) {
    if (!forward_float_applies(L, M, bits)) return APB_ERR_SHAPE;
    return launch_any(L, nullptr, nullptr, M, bits, step, nullptr, OutArgs{nullptr, nullptr, Y}, 0, 0.0f, s, X);
}

// Name of the kernel launch_forward picks for this layer, M and bits, as a profiler prints it (template
// arguments: bits; words per wave or parts of K; implicit im2col; float input).
const char* forward_kernel_name(const LayerDev& L, int M, int bits) {
    const long long Mp = (long long)kWave * ((M + kWave - 1) / kWave);
    const int ks = ksplit_parts(L, (long long)(L.Np / (TN * L.waves)) * (Mp / kWave));
    if (ks == 4) return bits == 1 ? "k_forward_ksplit<1, 4, false>" : "k_forward_ksplit<2, 4, false>";
    if (ks == 2) return bits == 1 ? "k_forward_ksplit<1, 2, false>" : "k_forward_ksplit<2, 2, false>";
    switch (L.waves) {
        case 8: return bits == 1 ? "k_sparse_epilogue<1, 1, false, false>" : "k_sparse_epilogue<2, 1, false, false>";
        case 4: return bits == 1 ? "k_sparse_epilogue<1, 2, false, false>" : "k_sparse_epilogue<2, 2, false, false>";
        default: return bits == 1 ? "k_sparse_epilogue<1, 4, false, false>" : "k_sparse_epilogue<2, 4, false, false>";
    }
}

// packed_out: the next layer's packed activation buffer (K = L.N), fully overwritten.
int launch_forward_requant(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, int M, int bits, float step,
                           const ConvShape* conv, const float* scale, const float* shift, int bits_out,
                           float inv_step_out, uint32_t* packed_out, hipStream_t s, bool out_cleared) {
    if (!conv && forward_rows_requant_applies(L, planes, M, bits))
        return launch_forward_rows_requant(L, planes, colsum, M, bits, step, scale, shift, bits_out, inv_step_out, packed_out,
                                           s, out_cleared);
    return launch_any(L, planes, colsum, M, bits, step, conv, OutArgs{scale, shift, reinterpret_cast<float*>(packed_out)},
                      bits_out, inv_step_out, s);
}

}  // namespace apb
