// The forward kernel for layers with many residuals per row (Sec. III Eqs. 12-13):
//     Y[n,m] = s * ( alpha * D[n,m] + sum_{j in row n} val_j * c[col_j, m] )
// with the LANES ALONG THE ROWS n.  (The other forward kernel, apb_sparse.hip, runs its lanes along the
// columns m; per residual and 64 outputs it needs one LDS read, and the LDS accepts one wave-wide read every
// two cycles per compute unit -- measured, that read rate is what bounds it on layers like a 512 x 4608
// convolution with 3 % residuals.)  Here a lane owns one row of the sparse matrix and kRowsCols = 16 output
// columns:
//   * a workgroup (up to 8 waves = 512 rows) takes one group of 16 columns and keeps the code table of those
//     columns for ALL of K in LDS, two bits per activation in 8 bytes per value of k -- built once, shared by
//     every row, no walk over chunks of K and no barrier inside the residual loop;
//   * a step of the residual loop: the lane loads its next residual (table offset of its column, value) from
//     the row lists laid out at compress time ([step][lane], so the loads are contiguous), reads the 16 codes
//     of that column with ONE 8-byte LDS read and does 16 x (field mask + float64 multiply-add) into 16
//     accumulators it keeps in registers.  Nothing is wave-uniform, so there is no scalar traffic, no index
//     register and no out-of-order counter shared between entry loads and table reads: the entry loads are
//     vector loads (in-order counter), fetched several steps ahead.
// Per residual and output that is 2 vector-ALU instructions and 1/16 of an LDS read.
// The binary part runs first on the matrix cores exactly as in the other kernels (apb_fp4_expand.h), here
// with the 16x16x128 FP4 instruction: a wave computes its 64 rows x 16 columns as four tiles.
// A table row is two dwords: the 16 codes of one k, two bits each, eight to a dword (its low half).  A code becomes
// a float64 multiplicand by masking its two bits in place inside the high half of a register pair (a subnormal
// number; see col_bit); the residuals are stored times 2^895 so that the products are ordinary numbers, and all
// scales are powers of two.
#include <algorithm>
#include <atomic>

#include "apb_fp4_expand.h"
#include "apb_internal.h"

namespace apb {

namespace {

constexpr int T = kRowsCols;
constexpr int kMaxDevices = 64;
constexpr int kBufferFlags = 0x00020000;                        // fourth word of a raw buffer descriptor: 32-bit data, no swizzle
constexpr int kRowBytes = kRowsRowBytes;                        // table bytes per value of k: two dwords of 8 columns x 2 bits

// Column c of a table row sits in dword c / 8 at bits 2 * (c % 8) and the bit above.  Its multiplicand is that
// field left where it is in an otherwise zero high half of a float64 -- a subnormal number, code * 2^(P - 1042)
// with P the bit position; all eight fields of a dword lie in the mantissa part (bits 0..19) of that half, so a
// multiplicand costs one AND: no shift, no conversion.  Every column thus carries its own power-of-two scale,
// which commutes with rounding and is taken out at the end.
__host__ __device__ constexpr int col_bit(int c) { return 2 * (c & 7); }
static_assert(kEntValScaleLog2 == 895, "col_unscale undoes 2^895 * 2^(P - 1042)");
// 2^(147 - col_bit(c)) and its inverse, by column (literals: nothing to evaluate at run time, and no function
// call in device code).
__device__ __forceinline__ double col_unscale(int c) {
    constexpr double t[8] = {0x1p147, 0x1p145, 0x1p143, 0x1p141, 0x1p139, 0x1p137, 0x1p135, 0x1p133};
    return t[c & 7];
}
__device__ __forceinline__ double col_scale(int c) {
    constexpr double t[8] = {0x1p-147, 0x1p-145, 0x1p-143, 0x1p-141, 0x1p-139, 0x1p-137, 0x1p-135, 0x1p-133};
    return t[c & 7];
}
static_assert(col_bit(0) == 0 && col_bit(4) == 8 && col_bit(7) == 14 && col_bit(8) == 0 && col_bit(15) == 14,
              "the literals above are 2^(147 - col_bit)");
static_assert(T == 16, "a table row holds 16 columns");

typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v2u __attribute__((ext_vector_type(2)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));

struct RowsParams {
    double alpha, step;
    int N, Nr, Kw, Kw4, Mp, M;
    int nblocks;                                                 // row blocks of 64 slots
    int row_groups;                                              // ceil(nblocks / waves per workgroup)
    int tasks;                                                   // row_groups * column groups
    int split;                                                   // waves that share one block of 64 rows (1, 2 or 4): the SPLIT of the kernel launched
    int tail_tasks, tail_cg0;                                    // k_forward_rows_tailed: tasks of the finer-grained tail, its first column group
    int exclusive;                                               // REQ: one workgroup holds every row of its columns (plain stores)
    int aligned_lists;                                           // host side: launch with the word-aligned lists
    int lds_main_bytes;                                          // LDS up to the waves' partial column sums
    // REQ kernels: the output is the packed activation buffer of the next layer (its K = this layer's N)
    int out_bits, out_Kw;                                        // 1 or 2; ceil(N / 32)
    float out_inv_step;
};

__device__ __forceinline__ uint32_t spread4(uint32_t nib) { return (nib * 0x00204081u) & 0x01010101u; }

// Codes of the 4 activations k = 32*j + 4*d + 0..3 of one column, one per byte, from the plane words of word row j.
template <int BITS>
__device__ __forceinline__ uint32_t codes4(uint32_t x0, uint32_t x1, int d) {
    uint32_t t = spread4((x0 >> (4 * d)) & 0xFu);
    if (BITS == 2) t |= spread4((x1 >> (4 * d)) & 0xFu) << 1;
    return t;
}

// Operands of this kernel's matrix steps.  A sign word is expanded once per wave, tile and step, the activation
// words once per workgroup and step, so the weight side gets the cheap form: dword d of the weight operand is the
// word masked IN PLACE -- bit d of every nibble, i.e. the FP4 numbers 0.5 (d = 0), 1 (d = 1), 2 (d = 2); only
// d = 3, whose bit would be the sign, is shifted first (to bit 2: the number 2) -- five instructions a word instead
// of seven.  The activation side makes up for the scales: its dword d holds code * 2 (d = 0: the FP4 numbers 2,
// 4, 6), code (d = 1: 1, 2, 3) or code / 2 (d = 2, 3: 0.5, 1, 1.5), so that every product is bit * code and the
// float accumulator holds P = sum_k bit * code itself (exact below 2^24).  Nibble t of dword d <-> bit d + 4t of
// the word on both sides, as in apb_fp4_expand.h.
__device__ __forceinline__ void expand_signs_scaled(uint32_t w, v8i& f) {
    f[0] = (int)(w & kNib);
    f[1] = (int)(w & (kNib << 1));
    f[2] = (int)(w & (kNib << 2));
    f[3] = (int)((w >> 1) & (kNib << 2));
}
template <int BITS>
__device__ __forceinline__ void expand_acts_scaled(uint32_t w0, uint32_t w1, v8i& f) {
    if (BITS == 1) {                                             // code = bit: 2, 1, 0.5, 0.5
        f[0] = (int)((w0 << 2) & (kNib << 2));
        f[1] = (int)(w0 & (kNib << 1));
        f[2] = (int)((w0 >> 2) & kNib);
        f[3] = (int)((w0 >> 3) & kNib);
    } else {
        // x0, x1: the plane bits of dword d at the bottom of every nibble
        {   // d = 0: code * 2 = 0b0100, 0b0110, 0b0111 for codes 1, 2, 3: bit 2 = x0 | x1, bit 1 = x1, bit 0 = x0 & x1
            const uint32_t x0 = w0 & kNib, x1 = w1 & kNib;
            f[0] = (int)(((x0 | x1) << 2) | (x1 << 1) | (x0 & x1));
        }
        {   // d = 1: code = 0b0010, 0b0100, 0b0101: bit 2 = x1, bit 1 = x0 & ~x1, bit 0 = x0 & x1
            const uint32_t x0 = (w0 >> 1) & kNib, x1 = (w1 >> 1) & kNib, both = x0 & x1;
            f[1] = (int)((x1 << 2) | ((x0 ^ both) << 1) | both);
        }
#pragma unroll
        for (int d = 2; d < 4; ++d)                              // code / 2: bit 1 = x1, bit 0 = x0
            f[d] = (int)(((w1 >> (d - 1)) & (kNib << 1)) | ((w0 >> d) & kNib));
    }
}

__device__ __forceinline__ v4f mfma_fp4_16(const v8i& a, const v8i& b, const v4f& c) {
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 4, 4, 0, kScaleOne, 0, kScaleOne);
}

// The code table starts at LDS address 0 (the kernels here have no static LDS, which the launchers check), so a
// list entry -- the byte offset of its table row -- IS the address: read through a pointer made from the number,
// the read needs no address arithmetic at all (through the kernel's shared array the compiler adds the array's
// link-time base, one vector instruction per step).
typedef __attribute__((address_space(3))) const v2u lds_table_row;
__device__ __forceinline__ v2u table_row(uint32_t offset) { return *reinterpret_cast<lds_table_row*>(offset); }

// acc[c] += v * code(column c of the table row q) * 2^(col_bit(c) - 1042), c = 0..15.  `m` is a register pair whose
// low half stays zero: the masked two-bit field in its high half makes it the float64 multiplicand.
__device__ __forceinline__ void accumulate16(double (&acc)[T], v2i& m, const v2u& q, double v) {
#pragma unroll
    for (int c = 0; c < T; ++c) {
        m.y = (int)(q[c >> 3] & (0x3u << col_bit(c)));
        acc[c] = fma(v, __builtin_bit_cast(double, m), acc[c]);
    }
}

// REQ: instead of Y the kernel writes the packed codes of the next layer's quantizer applied to
// scale[n] * Y + shift[n] (see the epilogue); Y then points to that buffer, zero-filled before the launch.
// The work of one workgroup: task `task` of a range of column groups that starts at cg0 and has `row_groups` row
// groups per column group (waves / SPLIT blocks of 64 rows each).
template <int BITS, bool REQ, int SPLIT>
__device__ __forceinline__ void rows_task(
    const uint32_t* __restrict__ planes, const int32_t* __restrict__ colsum, const int32_t* __restrict__ rowsum,
    const int32_t* __restrict__ rperm, const int32_t* __restrict__ blk, const uint32_t* __restrict__ ek,
    const double* __restrict__ ev, const uint32_t* __restrict__ signR, const double* __restrict__ valsumR,
    const float* __restrict__ scale, const float* __restrict__ shift, float* __restrict__ Y, const RowsParams& p,
    uint8_t* lds, int task, int row_groups, int cg0, int exclusive) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int waves = blockDim.x / kWave;
    const int rg = task % row_groups;
    const int cg = cg0 + task / row_groups;
    // Launches with few tasks (few columns) let p.split waves share a block of 64 rows: each takes a contiguous
    // part of the block's matrix steps and of its residual steps, and part 0 adds the partial results up in a
    // fixed order (integers for the binary part, float64 sums in the order of the parts).
    constexpr int split = SPLIT;                                 // (1: every wave has a block of its own)
    const int part = wave % split;
    const int b = rg * (waves / split) + wave / split;           // this wave's block of 64 rows
    const bool active = b < p.nblocks;                           // (the last row group may have idle waves)
    const int m0 = cg * T;
    const int slot = b * kWave + lane;

    // ---- binary part: P = sum_k bit * code for 64 rows x 16 columns, four 16 x 16 tiles over K in steps of 128.
    // Lane (i, g), i = lane & 15, g = lane >> 4, owns word 4*s + g of step s for row / column i of a tile.
    // The activation operand is the same for every wave of the workgroup: it is expanded once, by all threads
    // together, into LDS (16 bytes per step and lane -- as many bytes as the code table that later takes the
    // same place) and the waves read it back with one 16-byte LDS read per step.
    const int steps = p.Kw4 / 4;
    // Without a colsum array the code sums of the 16 columns are added up here, from the same words: a thread
    // stages words of one column only (lane & 15: the workgroup size is a multiple of 64), the four lanes of a
    // wave that share a column add theirs up, and the waves' partial sums wait in LDS behind the table.
    int32_t* cs_part = reinterpret_cast<int32_t*>(lds + p.lds_main_bytes);        // [waves][16]
    {
        const size_t plane_stride = (size_t)p.Kw * p.Mp;
        v4u* stage = reinterpret_cast<v4u*>(lds);
        int my_cs = 0;
        // kBatch items per thread at a time: all their loads leave together (one round trip per batch, not per item)
        constexpr int kBatch = 8;
        const int items = steps * kWave;
        for (int it0 = threadIdx.x; it0 < items; it0 += kBatch * blockDim.x) {
            uint32_t w0[kBatch], w1[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int it = min(it0 + u * (int)blockDim.x, items - 1);        // (past the end: re-read, unused)
                const int l = it & (kWave - 1), s = it >> 6;
                const uint32_t* brow = planes + (size_t)min(4 * s + (l >> 4), p.Kw - 1) * p.Mp + m0 + (l & 15);
                w0[u] = brow[0];
                w1[u] = BITS == 2 ? brow[plane_stride] : 0u;
            }
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int it = it0 + u * (int)blockDim.x;
                if (it < items) {
                    const int row = 4 * (it >> 6) + ((it & (kWave - 1)) >> 4);
                    if (row < p.Kw) my_cs += __builtin_popcount(w0[u]) + 2 * __builtin_popcount(w1[u]);
                    v8i fb;
                    expand_acts_scaled<BITS>(w0[u], w1[u], fb);
                    stage[it] = v4u{(uint32_t)fb[0], (uint32_t)fb[1], (uint32_t)fb[2], (uint32_t)fb[3]};
                }
            }
        }
        if (colsum == nullptr) {
            my_cs += __shfl_xor(my_cs, 16);
            my_cs += __shfl_xor(my_cs, 32);
            if (lane < T) cs_part[wave * T + lane] = my_cs;
        }
    }
    __syncthreads();
    if (colsum == nullptr && wave == 0 && lane < T) {            // the waves' partial sums become one sum per column,
        int tot = 0;                                             // read below after two more barriers
        for (int w = 0; w < waves; ++w) tot += cs_part[w * T + lane];
        cs_part[lane] = tot;
    }
    double acc[T];
    {
        const int i = lane & 15, g = lane >> 4;
        v4f c[4];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) c[t][r] = 0.0f;
        if (active) {
            v8i fa, fb;
#pragma unroll
            for (int d = 4; d < 8; ++d) fa[d] = fb[d] = 0;
            // Sign words are fetched kRing steps ahead (a ring of register sets indexed by step % kRing), so that
            // the expansion and the matrix instructions of a step never wait for that step's own loads.
            // (the four tiles' words of this lane's rows lie side by side: see the layout of rows_sign)
            const uint32_t* arow = signR + (size_t)g * p.Nr + (size_t)b * kWave + 4 * i;
            const v4u* stage = reinterpret_cast<const v4u*>(lds) + lane;
            constexpr int kRing = 4;
            uint32_t aw[kRing][4];
            auto load_words = [&](int s, uint32_t (&a)[4]) {
                const int ss = min(s, steps - 1);                // past the end: a harmless re-read, never used
                const v4u w = *reinterpret_cast<const v4u*>(arow + (size_t)(4 * ss) * p.Nr);
#pragma unroll
                for (int t = 0; t < 4; ++t) a[t] = w[t];
            };
            auto one_step = [&](int s, int q) {
                uint32_t a[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) a[t] = aw[q][t];
                load_words(s + kRing, aw[q]);
                const v4u bq = stage[(size_t)s * kWave];
#pragma unroll
                for (int d = 0; d < 4; ++d) fb[d] = (int)bq[d];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    expand_signs_scaled(a[t], fa);
                    c[t] = mfma_fp4_16(fa, fb, c[t]);
                }
            };
            const int steps_per_part = (steps + split - 1) / split;
            const int s_begin = min(steps, part * steps_per_part), s_end = min(steps, s_begin + steps_per_part);
#pragma unroll
            for (int q = 0; q < kRing; ++q) load_words(s_begin + q, aw[q]);
            int s0 = s_begin;
            for (; s0 + kRing <= s_end; s0 += kRing) {
#pragma unroll
                for (int q = 0; q < kRing; ++q) one_step(s0 + q, q);
            }
#pragma unroll
            for (int q = 0; q < kRing - 1; ++q)
                if (s0 + q < s_end) one_step(s0 + q, q);
        }
        __syncthreads();                                         // every wave is done with the staged operands
        // C layout of a 16 x 16 tile: lane (i, g), register r -> row 4*g + r, column i.  Through LDS, so that
        // every lane gets the 16 products of ITS row.
        int32_t* tile = reinterpret_cast<int32_t*>(lds) + wave * (kWave * T);
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) tile[(16 * t + 4 * g + r) * T + i] = (int)c[t][r];
        __syncthreads();
        const int n = active ? rperm[slot] : -1;
        const int rs = BITS == 1 && n >= 0 ? rowsum[n] : 0;
        const double a0 = part == 0 ? p.alpha * (BITS == 1 ? 0.5 : 1.0) : 0.0;     // (the other parts start at zero)
        const int32_t* tiles_of_block = reinterpret_cast<const int32_t*>(lds) + (wave - part) * (kWave * T);
#pragma unroll
        for (int cc = 0; cc < T; ++cc) {
            int P = 0;
            for (int pp = 0; pp < split; ++pp) P += tiles_of_block[pp * (kWave * T) + lane * T + cc];
            const int cs = colsum ? colsum[m0 + cc] : cs_part[cc];          // m0 + 15 < Mp: Mp is a multiple of 64
            const int d = BITS == 1 ? 4 * P - rs - 2 * cs : 2 * P - cs;
            acc[cc] = a0 * (double)d * col_scale(cc);  // in the scaled domain of column cc's products
        }
        __syncthreads();                                         // the tiles are read; the table may overwrite them
    }

    // ---- code table of the 16 columns for all of K: table[k] = two dwords, column c in dword c / 8 at bits
    // 2 * (c % 8).  Thread -> (word row j, quad d of its 32 values of k): it reads the 16 columns' words of row j
    // (64 contiguous bytes per plane), takes nibble d of each and writes the four finished table rows
    // k = 32*j + 4*d + 0..3 -- 32 contiguous bytes -- with two 16-byte stores.
    {
        const int items = p.Kw * 8;
        const size_t plane_stride = (size_t)p.Kw * p.Mp;
        for (int it = threadIdx.x; it < items; it += blockDim.x) {
            const int d = it & 7, j = it >> 3;
            const v4u* src0 = reinterpret_cast<const v4u*>(planes + (size_t)j * p.Mp + m0);
            const v4u* src1 = reinterpret_cast<const v4u*>(planes + plane_stride + (size_t)j * p.Mp + m0);
            // u[g], g = 0..3: byte q of u[g] holds the codes of columns 4g .. 4g+3 for k = 32*j + 4*d + q,
            // i.e. byte g % 2 of dword g / 2 of table row q
            uint32_t u[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const v4u x0 = src0[g];
                const v4u x1 = BITS == 2 ? src1[g] : v4u{0, 0, 0, 0};
                u[g] = codes4<BITS>(x0[0], x1[0], d) | (codes4<BITS>(x0[1], x1[1], d) << 2) |
                       (codes4<BITS>(x0[2], x1[2], d) << 4) | (codes4<BITS>(x0[3], x1[3], d) << 6);
            }
            // table row q = { u[0].q | u[1].q << 8, u[2].q | u[3].q << 8 } (selector byte 0x0c: zero)
            v4u* dst = reinterpret_cast<v4u*>(lds + (size_t)(32 * j + 4 * d) * kRowBytes);
            dst[0] = v4u{__builtin_amdgcn_perm(u[1], u[0], 0x0c0c0400u), __builtin_amdgcn_perm(u[3], u[2], 0x0c0c0400u),
                         __builtin_amdgcn_perm(u[1], u[0], 0x0c0c0501u), __builtin_amdgcn_perm(u[3], u[2], 0x0c0c0501u)};
            dst[1] = v4u{__builtin_amdgcn_perm(u[1], u[0], 0x0c0c0602u), __builtin_amdgcn_perm(u[3], u[2], 0x0c0c0602u),
                         __builtin_amdgcn_perm(u[1], u[0], 0x0c0c0703u), __builtin_amdgcn_perm(u[3], u[2], 0x0c0c0703u)};
        }
    }
    __syncthreads();
    if (!REQ && split == 1 && !active) return;                   // (otherwise every wave meets again below)

    // ---- residual part: steps e0 .. e1 of this block; entries fetched kAhead steps ahead, the table row of
    // the next step read while the multiply-adds of this one issue.
    if (active) {
        const int steps_of_block = blk[b + 1] - blk[b], steps_per_part = (steps_of_block + split - 1) / split;
        const int e0 = blk[b] + min(steps_of_block, part * steps_per_part);
        const int e1 = min(blk[b + 1], e0 + steps_per_part);
        const int n_steps = e1 - e0;
        // Entry loads are buffer loads: descriptor = this block's part of the lists, the step in the scalar
        // offset, the lane in a constant vector offset -- no address arithmetic on the vector ALU.
        const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint32_t*>(ek + (size_t)e0 * kWave), 0, max(n_steps, 1) * kWave * 4, kBufferFlags);
        const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<double*>(ev + (size_t)e0 * kWave), 0, max(n_steps, 1) * kWave * 8, kBufferFlags);
        const int lane4 = lane * 4, lane8 = lane * 8;
        auto load_k = [&](int jj) { return (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rk, lane4, jj * (kWave * 4), 0); };
        auto load_v = [&](int jj) {
            const v2u r = __builtin_amdgcn_raw_buffer_load_b64(rv, lane8, jj * (kWave * 8), 0);
            return __builtin_bit_cast(double, r);
        };
        constexpr int kAhead = 4;
        // The offsets wait in kAhead registers (a slot is free once its table row has been read, one step before its
        // value is used); the values in twice as many, used as two halves in turn, so that the load for step
        // j + kAhead never lands in the register the multiply-adds of step j still read -- no copies.
        uint32_t kq[kAhead];
        double vq[2 * kAhead];
#pragma unroll
        for (int a = 0; a < kAhead; ++a) {
            const int j = min(a, max(n_steps - 1, 0));
            kq[a] = n_steps > 0 ? load_k(j) : 0u;
            vq[a] = n_steps > 0 ? load_v(j) : 0.0;
        }
        v2i m = v2i{0, 0};
        // kq[a], vq[half * kAhead + a]: the entry of step j + a; q: the table row of the step about to be processed
        v2u q = table_row(kq[0]);                               // (offset 0 for an empty list: in bounds)
        int j = 0;
        // kAhead steps on one half of vq, refilling the other (the slots are refilled before the multiply-adds:
        // measured faster than after, the loads get a full kAhead steps of lead)
        auto four_steps = [&](int half) {
#pragma unroll
            for (int a = 0; a < kAhead; ++a) {
                const v2u qc = q;
                q = table_row(kq[(a + 1) % kAhead]);
                const int jn = min(j + a + kAhead, n_steps - 1); // past the end: the last entry again, never used
                kq[a] = load_k(jn);
                if (half == 0) vq[kAhead + a] = load_v(jn); else vq[a] = load_v(jn);
                accumulate16(acc, m, qc, half == 0 ? vq[a] : vq[kAhead + a]);
            }
            j += kAhead;
        };
        while (j + 2 * kAhead <= n_steps) {
            four_steps(0);
            four_steps(1);
        }
        // fewer than 2 kAhead steps left: kAhead more if there are, then what waits in the queue
        if (j + kAhead <= n_steps) {
            four_steps(0);
            for (int a = 0; j < n_steps; ++j, ++a) {
                const v2u qc = a == 0 ? q : table_row(kq[a]);
                accumulate16(acc, m, qc, vq[kAhead + a]);
            }
        } else {
            for (int a = 0; j < n_steps; ++j, ++a) {
                const v2u qc = a == 0 ? q : table_row(kq[a]);
                accumulate16(acc, m, qc, vq[a]);
            }
        }
    }

    // ---- several waves per block: the partial sums of parts 1.. go through LDS (where the table was) to part 0,
    // which adds them in the order of the parts
    const bool owner = active && part == 0;
    if (split > 1) {
        __syncthreads();                                         // every wave is done with the table
        double* red = reinterpret_cast<double*>(lds);            // [blocks of the workgroup][split - 1][16][64]
        const int bw = wave / split;
        if (part > 0) {
#pragma unroll
            for (int cc = 0; cc < T; ++cc) red[((size_t)(bw * (split - 1) + part - 1) * T + cc) * kWave + lane] = acc[cc];
        }
        __syncthreads();
        if (part == 0) {
            for (int pp = 1; pp < split; ++pp)
#pragma unroll
                for (int cc = 0; cc < T; ++cc) acc[cc] += red[((size_t)(bw * (split - 1) + pp - 1) * T + cc) * kWave + lane];
        }
        if (!REQ && !owner) return;
    }

    // ---- epilogue.  REQ: z = scale[n] * y + shift[n] (float64, rounded once to float; z = y without scale) is
    // quantized exactly as apb_quantize_acts does and its code bits go into word n / 32 of column m of the next
    // layer's buffer (planes [out_bits][out_Kw][Mp], then the column sums [Mp]).  The rows of a workgroup are
    // scattered over all of N (the lists are sorted by length), so its bits first meet in LDS -- where the table
    // was: [out_bits][out_Kw][16] words and 16 partial column sums -- and then leave as one atomic OR per
    // non-zero word and one atomic add per column; integer OR and add commute, so the order between
    // workgroups does not matter.
    if (REQ && exclusive != 0) {
        // The workgroup holds whole words of the output: all rows (exclusive 1: at most kRowsGroupRows of them) or,
        // with the word-aligned lists, the kRowsGroupRows rows of row group rg (exclusive 2).  Every lane packs the
        // codes of its row -- two bits per column -- into one word and leaves it in LDS at the row's place in the
        // group; read back in row order, a wave holds the 64 rows of two output words, and the ballot over bit b of
        // those code words IS the pair of output words of column b / 2, plane b % 2.  No atomics on the way.
        const int w_lo = exclusive == 2 ? rg * (kRowsGroupRows / 32) : 0;
        uint32_t* codes = reinterpret_cast<uint32_t*>(lds);      // [kRowsGroupRows] code words, then 16 column sums
        __syncthreads();                                         // every wave is done with the table
        for (int i = threadIdx.x; i < kRowsGroupRows + T; i += blockDim.x) codes[i] = 0u;
        __syncthreads();
        const int n = owner ? rperm[slot] : -1;
        const double vs = BITS == 1 && n >= 0 ? valsumR[slot] : 0.0;
        const double sc = scale && n >= 0 ? (double)scale[n] : 1.0, sh = scale && n >= 0 ? (double)shift[n] : 0.0;
        uint32_t cw = 0;
#pragma unroll
        for (int cc = 0; cc < T; ++cc) {
            const double sum = acc[cc] * col_unscale(cc);
            double z = (BITS == 1 ? 2.0 * sum - vs : sum) * p.step;
            if (scale) z = fma(sc, z, sh);
            const float zf = (float)z;
            const uint32_t code = p.out_bits == 1 ? (zf >= 0.0f ? 1u : 0u) : code2(zf, p.out_inv_step);
            if (m0 + cc < p.M) cw |= code << (2 * cc);           // (the columns behind M keep their zeros)
        }
        if (n >= 0) codes[n - 32 * w_lo] = cw;
        __syncthreads();
        uint32_t* words = reinterpret_cast<uint32_t*>(Y);
        for (int t0 = threadIdx.x; t0 < kRowsGroupRows; t0 += blockDim.x) {      // (whole waves: 64 divides both)
            const uint32_t mine = codes[t0];
            uint32_t wa = 0, wb = 0;                             // lane b: output words 2 * (t0 / 64) and + 1 of bit b
#pragma unroll
            for (int bb = 0; bb < 32; ++bb) {
                const unsigned long long mask = __ballot(((mine >> bb) & 1u) != 0);
                if (lane == bb) {
                    wa = (uint32_t)mask;
                    wb = (uint32_t)(mask >> 32);
                }
            }
            const int col = lane >> 1, plane = lane & 1, wr = w_lo + 2 * (t0 / kWave);
            if (lane < 32 && plane < p.out_bits) {
                uint32_t* at = words + ((size_t)plane * p.out_Kw + wr) * p.Mp + m0 + col;
                if (wr < p.out_Kw) at[0] = wa;
                if (wr + 1 < p.out_Kw) at[p.Mp] = wb;
                const uint32_t cnt = (uint32_t)(__builtin_popcount(wa) + __builtin_popcount(wb)) << plane;
                if (cnt) __hip_atomic_fetch_add(codes + kRowsGroupRows + col, cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        }
        __syncthreads();
        // column sums: stored by the one row group, added up over several (cleared before the launch)
        if (threadIdx.x < T) {
            const uint32_t tot = codes[kRowsGroupRows + threadIdx.x];
            uint32_t* at = words + (size_t)p.out_bits * p.out_Kw * p.Mp + m0 + threadIdx.x;
            if (exclusive == 1) *at = tot;
            else if (tot) __hip_atomic_fetch_add(at, tot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        return;
    }
    if (REQ) {
        // exclusive 0: every word of the columns may hold rows of this workgroup and of others; 1: one row group,
        // the workgroup holds all rows; 2: word-aligned lists, the rows of row group rg are those of
        // kRowsGroupRows / 32 words
        const int w_lo = exclusive == 2 ? rg * (kRowsGroupRows / 32) : 0;
        const int nW = exclusive == 2 ? min(p.out_Kw - w_lo, kRowsGroupRows / 32) : p.out_Kw;
        uint32_t* merged = reinterpret_cast<uint32_t*>(lds);     // [out_bits][nW][16] words, then 16 column sums
        const int nwords = p.out_bits * nW * T;
        __syncthreads();                                         // every wave is done with the table
        for (int i = threadIdx.x; i < nwords + T; i += blockDim.x) merged[i] = 0u;
        __syncthreads();
        const int n = owner ? rperm[slot] : -1;
        const double vs = BITS == 1 && n >= 0 ? valsumR[slot] : 0.0;
        const double sc = scale && n >= 0 ? (double)scale[n] : 1.0, sh = scale && n >= 0 ? (double)shift[n] : 0.0;
        const uint32_t bit = 1u << (n & 31);
        uint32_t* w0_at = merged + (size_t)max((n >> 5) - w_lo, 0) * T;
        uint32_t* w1_at = w0_at + (size_t)nW * T;
#pragma unroll
        for (int cc = 0; cc < T; ++cc) {
            const double sum = acc[cc] * col_unscale(cc);
            double z = (BITS == 1 ? 2.0 * sum - vs : sum) * p.step;
            if (scale) z = fma(sc, z, sh);
            const float zf = (float)z;
            uint32_t code = p.out_bits == 1 ? (zf >= 0.0f ? 1u : 0u) : code2(zf, p.out_inv_step);
            if (n < 0 || m0 + cc >= p.M) code = 0;
            if (code & 1u) __hip_atomic_fetch_or(w0_at + cc, bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (code >> 1) __hip_atomic_fetch_or(w1_at + cc, bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            // the wave's share of the column sum: two ballots instead of 64 additions to one address
            const int tot = __builtin_popcountll(__ballot((code & 1u) != 0)) + 2 * __builtin_popcountll(__ballot((code >> 1) != 0));
            if (lane == 0 && tot)
                __hip_atomic_fetch_add(merged + nwords + cc, (uint32_t)tot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        __syncthreads();
        uint32_t* words = reinterpret_cast<uint32_t*>(Y);
        // merged word i: plane i / (nW * 16), word row w_lo + (i / 16) % nW, column i % 16.  Where the workgroup
        // owns its words (exclusive 1 and 2) it stores every one of them plainly, zero or not: nothing to clear
        // beforehand, no atomics.
        for (int i = threadIdx.x; i < nwords; i += blockDim.x) {
            const uint32_t w = merged[i];
            const int plane = i / (nW * T), r = i - plane * (nW * T);
            uint32_t* at = words + ((size_t)plane * p.out_Kw + w_lo + r / T) * p.Mp + m0 + (r % T);
            if (exclusive != 0) *at = w;
            else if (w) __hip_atomic_fetch_or(at, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        // column sums: stored by the one row group, added up over several (cleared before the launch)
        if (threadIdx.x < T) {
            const uint32_t tot = merged[nwords + threadIdx.x];
            uint32_t* at = words + (size_t)p.out_bits * p.out_Kw * p.Mp + m0 + threadIdx.x;
            if (exclusive == 1) *at = tot;
            else if (tot) __hip_atomic_fetch_add(at, tot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        return;
    }
    // 16 consecutive floats of row n.
    const int n = rperm[slot];
    const double vs = BITS == 1 && n >= 0 ? valsumR[slot] : 0.0;
    float y[T];
#pragma unroll
    for (int cc = 0; cc < T; ++cc) {
        const double sum = acc[cc] * col_unscale(cc);
        y[cc] = (float)((BITS == 1 ? 2.0 * sum - vs : sum) * p.step);
    }
    if (m0 + T <= p.M && (p.M & 3) == 0 && (reinterpret_cast<uintptr_t>(Y) & 15u) == 0) {
        // A lane storing its own 64 bytes takes four store instructions that each touch 64 rows, 16 bytes in each
        // (measured alone: 2.0 TB/s).  Instead the four lanes of a quad transpose their 4 x 4 blocks of 16 bytes
        // (two butterfly steps over the lane bits, through the data-parallel lane swizzle), after which lane q of
        // a quad holds bytes 16q .. 16q+15 of the quad's four rows and a store instruction writes 16 rows, 64
        // contiguous bytes in each (4.5 TB/s).  Every lane of the wave takes part; lanes without a row store nothing.
        const bool q0 = (lane & 1) != 0, q1 = (lane & 2) != 0;
#pragma unroll
        for (int k = 0; k < 4; k += 2)                           // lane bit 0: blocks k and k + 1 with lane ^ 1
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float send = q0 ? y[4 * k + e] : y[4 * (k + 1) + e];
                const float recv = __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, send), 0xB1, 0xF, 0xF, true));
                if (q0) y[4 * k + e] = recv; else y[4 * (k + 1) + e] = recv;
            }
#pragma unroll
        for (int k = 0; k < 2; ++k)                              // lane bit 1: blocks k and k + 2 with lane ^ 2
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float send = q1 ? y[4 * k + e] : y[4 * (k + 2) + e];
                const float recv = __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, send), 0x4E, 0xF, 0xF, true));
                if (q1) y[4 * k + e] = recv; else y[4 * (k + 2) + e] = recv;
            }
        // block j now belongs to the row of lane j of the quad
        const int n_of[4] = {__builtin_amdgcn_mov_dpp(n, 0x00, 0xF, 0xF, true), __builtin_amdgcn_mov_dpp(n, 0x55, 0xF, 0xF, true),
                             __builtin_amdgcn_mov_dpp(n, 0xAA, 0xF, 0xF, true), __builtin_amdgcn_mov_dpp(n, 0xFF, 0xF, 0xF, true)};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int nj = n_of[j];
            if (nj >= 0)
                *reinterpret_cast<v4f*>(Y + (size_t)nj * p.M + m0 + 4 * (lane & 3)) = v4f{y[4 * j], y[4 * j + 1], y[4 * j + 2], y[4 * j + 3]};
        }
    } else if (n >= 0) {
        float* out = Y + (size_t)n * p.M + m0;
#pragma unroll
        for (int cc = 0; cc < T; ++cc)
            if (m0 + cc < p.M) out[cc] = y[cc];
    }
}

// Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of tasks so that the row
// groups of one column group share an L2.
__device__ __forceinline__ int xcd_contiguous(int block, int tasks) {
    return (tasks & 7) == 0 ? (block & 7) * (tasks >> 3) + (block >> 3) : block;
}

template <int BITS, bool REQ, int SPLIT>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 4))) void k_forward_rows(
    const uint32_t* __restrict__ planes, const int32_t* __restrict__ colsum, const int32_t* __restrict__ rowsum,
    const int32_t* __restrict__ rperm, const int32_t* __restrict__ blk, const uint32_t* __restrict__ ek,
    const double* __restrict__ ev, const uint32_t* __restrict__ signR, const double* __restrict__ valsumR,
    const float* __restrict__ scale, const float* __restrict__ shift, float* __restrict__ Y, const RowsParams p) {
    extern __shared__ __align__(16) uint8_t lds[];
    rows_task<BITS, REQ, SPLIT>(planes, colsum, rowsum, rperm, blk, ek, ev, signR, valsumR, scale, shift, Y, p, lds,
                                xcd_contiguous(blockIdx.x, p.tasks), p.row_groups, 0, p.exclusive);
}

// The same with a finer-grained TAIL.  A launch whose tasks are a little more than a whole number per compute unit
// ends with a few compute units running one more workgroup, alone and therefore slowly, while the others idle
// (measured on 512 x 4608: 1536 tasks 92 us, 1568 tasks 103 us).  Here the column groups of that remainder are
// cut into four times as many tasks -- one block of 64 rows each, shared by the four waves as in the SPLIT = 4
// kernel -- which come last in the grid and spread over four times as many compute units.
template <int BITS, bool REQ>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 4))) void k_forward_rows_tailed(
    const uint32_t* __restrict__ planes, const int32_t* __restrict__ colsum, const int32_t* __restrict__ rowsum,
    const int32_t* __restrict__ rperm, const int32_t* __restrict__ blk, const uint32_t* __restrict__ ek,
    const double* __restrict__ ev, const uint32_t* __restrict__ signR, const double* __restrict__ valsumR,
    const float* __restrict__ scale, const float* __restrict__ shift, float* __restrict__ Y, const RowsParams p) {
    extern __shared__ __align__(16) uint8_t lds[];
    if ((int)blockIdx.x < p.tasks)
        rows_task<BITS, REQ, 1>(planes, colsum, rowsum, rperm, blk, ek, ev, signR, valsumR, scale, shift, Y, p, lds,
                                xcd_contiguous(blockIdx.x, p.tasks), p.row_groups, 0, p.exclusive);
    else                                                         // (a tail task holds one block of rows: it shares its words)
        rows_task<BITS, REQ, 4>(planes, colsum, rowsum, rperm, blk, ek, ev, signR, valsumR, scale, shift, Y, p, lds,
                                (int)blockIdx.x - p.tasks, p.nblocks, p.tail_cg0, 0);
}

// Clears columns c0 .. Mp of `rows` rows of Mp words and all of the row after them (the column sums).
__global__ __launch_bounds__(256) void k_zero_columns(uint32_t* __restrict__ words, size_t rows, int Mp, int c0) {
    for (size_t r = blockIdx.x; r <= rows; r += gridDim.x)
        for (int c = (r < rows ? c0 : 0) + (int)threadIdx.x; c < Mp; c += 256) words[r * Mp + c] = 0u;
}

int rows_waves(const LayerDev& L) {
    const int nb = L.rows_Nr / kWave;
    return nb >= 4 ? 4 : (nb >= 2 ? 2 : 1);
}

constexpr int kComputeUnits = 256;                             // of the MI355X
constexpr size_t kColsumBytes = 8 * T * sizeof(int32_t);      // partial column sums of up to 8 waves
// the largest table, the staged operands of a K rounded up to whole steps, the partial sums
constexpr int kMaxLdsBytes = kRowsMaxTableBytes + 1024 + (int)kColsumBytes;
static_assert(kMaxLdsBytes <= 160 * 1024, "LDS of one compute unit");

size_t rows_lds_bytes(const LayerDev& L, int waves, int split) {
    // the code table; before it, in the same place, the staged activation operands (16 bytes per step and lane)
    // and the tiles of the binary product
    const size_t table = (size_t)32 * L.Kw * kRowBytes, stage = (size_t)(L.rows_Kw4 / 4) * kWave * 16;
    const size_t tiles = (size_t)waves * kWave * T * 4;
    // (and the partial float64 sums of waves that share a block)
    const size_t partial = (size_t)(waves / split) * (split - 1) * kWave * T * 8;
    return (std::max(std::max(table, partial), std::max(stage, tiles)) + 15) & ~(size_t)15;
}

// bytes of LDS the packed-output epilogue needs for a layer of N rows (both planes) -- it reuses the table's place
size_t rows_merge_bytes(int N) { return ((size_t)2 * ((N + 31) / 32) * T + T) * sizeof(uint32_t); }

// The kernels address their code table from LDS address 0 (table_row): true while they have no static LDS in
// front of the dynamic array.  Checked once per kernel and process, from the kernel's own attributes.
int check_no_static_lds(const void* kernel, std::atomic<int>& state) {
    int st = state.load(std::memory_order_acquire);
    if (st == 0) {
        hipFuncAttributes attr;
        APB_HIP(hipFuncGetAttributes(&attr, kernel));
        st = attr.sharedSizeBytes == 0 ? 1 : -1;
        state.store(st, std::memory_order_release);
    }
    return st == 1 ? APB_OK : APB_ERR_SHAPE;
}

template <int BITS, bool REQ, int SPLIT>
int launch_rows_split(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, const float* scale, const float* shift,
                      float* Y, const RowsParams& p, int waves, hipStream_t s) {
    size_t lds = rows_lds_bytes(L, waves, SPLIT) + kColsumBytes;
    if (REQ) lds = std::max(lds, rows_merge_bytes(L.N));
    if (lds > (size_t)kMaxLdsBytes) return APB_ERR_SHAPE;
    static std::atomic<int> no_static_lds{0};
    if (const int rc = check_no_static_lds(reinterpret_cast<const void*>(&k_forward_rows<BITS, REQ, SPLIT>), no_static_lds)) return rc;
    if (lds > 64 * 1024) {                                      // more LDS than a launch gets without asking
        static std::atomic<size_t> asked[kMaxDevices];          // largest size asked for, per device and kernel
        int dev = 0;
        APB_HIP(hipGetDevice(&dev));
        if (dev < 0 || dev >= kMaxDevices) return APB_ERR_SHAPE;
        if (asked[dev].load(std::memory_order_acquire) < lds) {
            APB_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_forward_rows<BITS, REQ, SPLIT>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes));
            asked[dev].store((size_t)kMaxLdsBytes, std::memory_order_release);
        }
    }
    const bool w = p.aligned_lists != 0;
    hipLaunchKernelGGL((k_forward_rows<BITS, REQ, SPLIT>), dim3((unsigned)p.tasks), dim3(kWave * waves), lds, s, planes, colsum,
                       L.rowsum, w ? L.rowsw_perm : L.rows_perm, w ? L.rowsw_blk : L.rows_blk, w ? L.rowsw_ek : L.rows_ek,
                       w ? L.rowsw_ev : L.rows_ev, w ? L.rowsw_sign : L.rows_sign, w ? L.rowsw_valsum : L.rows_valsum, scale,
                       shift, Y, p);
    APB_HIP(hipGetLastError());
    return APB_OK;
}

template <int BITS, bool REQ>
int launch_rows_tailed(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, const float* scale,
                       const float* shift, float* Y, const RowsParams& p, hipStream_t s) {
    size_t lds = p.lds_main_bytes + kColsumBytes;               // (rows_params sized it for both task shapes)
    if (REQ) lds = std::max(lds, rows_merge_bytes(L.N));
    if (lds > (size_t)kMaxLdsBytes) return APB_ERR_SHAPE;
    static std::atomic<int> no_static_lds{0};
    if (const int rc = check_no_static_lds(reinterpret_cast<const void*>(&k_forward_rows_tailed<BITS, REQ>), no_static_lds)) return rc;
    if (lds > 64 * 1024) {
        static std::atomic<size_t> asked[kMaxDevices];
        int dev = 0;
        APB_HIP(hipGetDevice(&dev));
        if (dev < 0 || dev >= kMaxDevices) return APB_ERR_SHAPE;
        if (asked[dev].load(std::memory_order_acquire) < lds) {
            APB_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_forward_rows_tailed<BITS, REQ>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes));
            asked[dev].store((size_t)kMaxLdsBytes, std::memory_order_release);
        }
    }
    const bool w = p.aligned_lists != 0;
    hipLaunchKernelGGL((k_forward_rows_tailed<BITS, REQ>), dim3((unsigned)(p.tasks + p.tail_tasks)), dim3(kWave * 4), lds, s,
                       planes, colsum, L.rowsum, w ? L.rowsw_perm : L.rows_perm, w ? L.rowsw_blk : L.rows_blk,
                       w ? L.rowsw_ek : L.rows_ek, w ? L.rowsw_ev : L.rows_ev, w ? L.rowsw_sign : L.rows_sign,
                       w ? L.rowsw_valsum : L.rows_valsum, scale, shift, Y, p);
    APB_HIP(hipGetLastError());
    return APB_OK;
}

template <int BITS, bool REQ>
int launch_rows(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, const float* scale, const float* shift,
                float* Y, const RowsParams& p, int waves, hipStream_t s) {
    if (p.tail_tasks > 0) return launch_rows_tailed<BITS, REQ>(L, planes, colsum, scale, shift, Y, p, s);
    switch (p.split) {
        case 1: return launch_rows_split<BITS, REQ, 1>(L, planes, colsum, scale, shift, Y, p, waves, s);
        case 2: return launch_rows_split<BITS, REQ, 2>(L, planes, colsum, scale, shift, Y, p, waves, s);
        case 4: return launch_rows_split<BITS, REQ, 4>(L, planes, colsum, scale, shift, Y, p, waves, s);
        default: return APB_ERR_SHAPE;
    }
}

// Fills the launch parameters; APB_ERR_SHAPE where the kernel does not apply.
int rows_params(const LayerDev& L, const uint32_t* planes, int M, int bits, float step, RowsParams& p, int& waves) {
    if (L.rows_steps == 0 || (reinterpret_cast<uintptr_t>(planes) & 15u) != 0) return APB_ERR_SHAPE;
    if (!mfma_sum_exact(L.K, 1, bits == 1 ? 1 : 3)) return APB_ERR_SHAPE;
    const int Mp = kWave * ((M + kWave - 1) / kWave);
    waves = rows_waves(L);
    p.alpha = (double)L.alpha;
    p.step = (double)step;
    p.N = L.N;
    p.Nr = L.rows_Nr;
    p.Kw = L.Kw;
    p.Kw4 = L.rows_Kw4;
    p.Mp = Mp;
    p.M = M;
    p.nblocks = L.rows_Nr / kWave;
    // Few columns (at most 32 groups of 16: fully connected layers at small batch) and fewer workgroups than
    // compute units: let 2 or 4 waves share a block of rows until every compute unit has one.  Long rows
    // (K >= 4096) in at most 16 column groups pay for one doubling more -- in 8-wave workgroups, one per unit with
    // one table for four blocks, where that fills the units evenly; else two 4-wave ones per unit.
    // (Measured, same box each: 1024 x 4096 x 64 a third faster than unshared; 4096 x 4096 x 128 25 -> 21 us and
    // 2048 x 4096 x 256 22 -> 19 us against sharing up to two workgroups per unit; the doubling more: K = 4096
    // 2-8 % faster, K = 9216 7 %, K = 2048 5 % slower, K = 1024 15 %, 25 column groups 6 % slower; 8 waves:
    // 4096 x 4096 x 256 27.8 -> 26.4 us, 4096 x 9216 x 256 51 -> 45, but 6144 x 4096 x 256 -- one and a half
    // workgroups per unit -- 35 -> 38.  On shapes with more columns sharing loses, 5-15 %.)
    const long long col_groups = (M + T - 1) / T;
    const long long blocks_total = (long long)p.nblocks * col_groups;
    p.split = 1;
    while (col_groups <= 32 && p.split < waves && blocks_total * p.split < 4 * kComputeUnits) p.split *= 2;
    if (col_groups <= 16 && p.split == 1 && waves == 4 && L.K >= 4096 && blocks_total < 8 * kComputeUnits) {
        p.split = 2;
        if (p.nblocks % 4 == 0 && (blocks_total / 4) % kComputeUnits == 0) waves = 8;
    }
    const int blocks_per_group = waves / p.split;
    p.row_groups = (p.nblocks + blocks_per_group - 1) / blocks_per_group;
    const long long tasks = (long long)p.row_groups * col_groups;
    if (tasks > 0x7fffffffLL || (long long)Mp * 8 >= (1LL << 31)) return APB_ERR_SHAPE;
    p.tasks = (int)tasks;
    p.lds_main_bytes = (int)rows_lds_bytes(L, waves, p.split);
    p.tail_tasks = 0;
    p.tail_cg0 = 0;
    p.exclusive = 0;
    p.aligned_lists = 0;
    // A remainder of at most half a task per compute unit after one whole one or more: the column groups of the
    // remainder become the finer tail of k_forward_rows_tailed (4-wave workgroups only).  (Measured on 512 x 4608:
    // 288 tasks 39 -> 31 us, 544 tasks 51 -> 44 us, 784 tasks 63 -> 54 us, 1568 tasks 110 -> 104 us.)
    if (waves == 4 && p.split == 1) {
        const long long whole = tasks / kComputeUnits, rest = tasks % kComputeUnits;
        if (whole >= 1 && rest > 0 && rest <= kComputeUnits / 2) {
            const long long tail_groups = std::min<long long>(col_groups, (rest + p.row_groups - 1) / p.row_groups);
            p.tail_cg0 = (int)(col_groups - tail_groups);
            p.tasks = (int)((long long)p.row_groups * p.tail_cg0);
            p.tail_tasks = (int)(tail_groups * p.nblocks);
            p.lds_main_bytes = (int)std::max(rows_lds_bytes(L, waves, 1), rows_lds_bytes(L, waves, 4));
        }
    }
    p.out_bits = 0;
    p.out_Kw = 0;
    p.out_inv_step = 0.0f;
    return APB_OK;
}

}  // namespace

// The rows-in-lanes kernel pays for a code table of all of K per 16 columns and for lists padded to the
// longest row of each block; it wins where the residual multiply-adds dominate.
bool forward_rows_applies(const LayerDev& L, int M, int bits) {
    // Measured on the benchmark layers: ahead of the columns-in-lanes kernel from 0.5 % residuals upwards on
    // layers of 256 rows and more; with fewer than four blocks of 64 rows a workgroup has too few waves.
    return L.rows_steps > 0 && M > 0 && L.rows_Nr >= 4 * kWave;
}

// The name a profiler shows for the kernel launch_forward_rows launches (float output).
const char* forward_rows_kernel_name(const LayerDev& L, int M, int bits) {
    RowsParams p;
    int waves;
    if (rows_params(L, reinterpret_cast<const uint32_t*>(uintptr_t{16}), M, bits, 1.0f, p, waves) != APB_OK) return "";
    if (p.tail_tasks > 0) return bits == 1 ? "k_forward_rows_tailed<1, false>" : "k_forward_rows_tailed<2, false>";
    switch (p.split) {
        case 1: return bits == 1 ? "k_forward_rows<1, false, 1>" : "k_forward_rows<2, false, 1>";
        case 2: return bits == 1 ? "k_forward_rows<1, false, 2>" : "k_forward_rows<2, false, 2>";
        default: return bits == 1 ? "k_forward_rows<1, false, 4>" : "k_forward_rows<2, false, 4>";
    }
}

int launch_forward_rows(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, int M, int bits, float step,
                        float* Y, hipStream_t s) {
    RowsParams p;
    int waves;
    const int rc = rows_params(L, planes, M, bits, step, p, waves);
    if (rc != APB_OK) return rc;
    return bits == 1 ? launch_rows<1, false>(L, planes, colsum, nullptr, nullptr, Y, p, waves, s)
                     : launch_rows<2, false>(L, planes, colsum, nullptr, nullptr, Y, p, waves, s);
}

// The same kernel ending in the next layer's quantizer (packed output): where the float-output form applies and
// the bits of all N rows of 16 columns fit the LDS of a workgroup.
bool forward_rows_requant_applies(const LayerDev& L, const uint32_t* planes, int M, int bits) {
    return forward_rows_applies(L, M, bits) && (reinterpret_cast<uintptr_t>(planes) & 15u) == 0 &&
           rows_merge_bytes(L.N) <= (size_t)kMaxLdsBytes;
}

int launch_forward_rows_requant(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, int M, int bits,
                                float step, const float* scale, const float* shift, int bits_out, float inv_step_out,
                                uint32_t* packed_out, hipStream_t s, bool out_cleared) {
    RowsParams p;
    int waves;
    int rc = rows_params(L, planes, M, bits, step, p, waves);
    if (rc != APB_OK) return rc;
    p.out_bits = bits_out;
    p.out_Kw = (L.N + 31) / 32;
    p.out_inv_step = inv_step_out;
    // One row group, or row groups that are whole words of the output (the word-aligned lists, four blocks of rows
    // to a workgroup): the workgroups own their words and store them plainly, nothing clears those beforehand.
    const bool aligned = p.row_groups > 1 && L.rowsw_steps > 0 && waves / p.split == kRowsGroupRows / kWave;
    const size_t plane_rows = (size_t)bits_out * p.out_Kw;
    if (p.row_groups == 1) {
        // (the column groups cover the padding columns up to Mp as well -- their codes are zero -- and there is no
        // finer tail: its tasks would share words)
        p.tasks = p.Mp / T;
        p.tail_tasks = 0;
        p.lds_main_bytes = (int)rows_lds_bytes(L, waves, p.split);
        p.exclusive = 1;
    } else if (aligned) {
        p.exclusive = 2;
        p.aligned_lists = 1;
        // The column groups of a finer tail, whose tasks hold one block of rows each, still OR their bits into the
        // buffer: those columns -- and the padding columns behind them -- are cleared, and so are the column sums,
        // which the row groups add up (a fill kernel, not a memset node: the call may be recorded into a graph).
        const int c0 = p.tail_tasks > 0 ? p.tail_cg0 * T : (int)(((long long)M + T - 1) / T) * T;
        if (!out_cleared) {
            hipLaunchKernelGGL(k_zero_columns, dim3((unsigned)std::min<size_t>(plane_rows + 1, 65535)), dim3(256), 0, s,
                               packed_out, plane_rows, p.Mp, c0);
            APB_HIP(hipGetLastError());
        }
    } else if (!out_cleared) {
        // several row groups OR their bits into the buffer and add their column sums up in it
        rc = launch_zero_words(packed_out, (plane_rows + 1) * p.Mp, s);
        if (rc != APB_OK) return rc;
    }
    float* out = reinterpret_cast<float*>(packed_out);
    return bits == 1 ? launch_rows<1, true>(L, planes, colsum, scale, shift, out, p, waves, s)
                     : launch_rows<2, true>(L, planes, colsum, scale, shift, out, p, waves, s);
}

int launch_forward_best(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, int M, int bits, float step,
                        float* Y, hipStream_t s) {
    // (the rows-in-lanes kernel reads the packed words 16 bytes at a time)
    if (forward_rows_applies(L, M, bits) && (reinterpret_cast<uintptr_t>(planes) & 15u) == 0)
        return launch_forward_rows(L, planes, colsum, M, bits, step, Y, s);
    return launch_forward(L, planes, colsum, M, bits, step, nullptr, Y, s);
}

int launch_quantize_then_forward(const LayerDev& L, const float* X, int M, int bits, float step, uint32_t* planes,
                                 int32_t* colsum, float* Y, hipStream_t s) {
    // The rows-in-lanes kernel reads every word of its columns anyway and adds their code sums up itself: the
    // quantize kernel then writes the planes only -- no sums in LDS, and where it splits K no fill launch and
    // no atomics.
    const bool rows = forward_rows_applies(L, M, bits) && (reinterpret_cast<uintptr_t>(planes) & 15u) == 0;
    const int rc = launch_quantize(X, L.K, M, bits, 1.0f / step, planes, rows ? nullptr : colsum, s);
    if (rc != APB_OK) return rc;
    if (rows) return launch_forward_rows(L, planes, nullptr, M, bits, step, Y, s);
    return launch_forward(L, planes, colsum, M, bits, step, nullptr, Y, s);
}

}  // namespace apb
