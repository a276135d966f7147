// Vector-ALU comparison kernels of apb_forward:  Y = s * (alpha*D + sum_j val_j * c[col_j, :])
// (Sec. III Eq. 13).  They serve apb_forward_popcount / apb_forward_int_popcount -- the measured
// alternative to the matrix-core path and a second route to D in the tests -- not apb_forward.
//
// One kernel template, two uses:
//   kFusedPopcount   the paper's own formulation end to end on the vector ALU: xor/and + popcount
//                    for D (Sec. IV Eq. 16; for 2-bit activations the two stored bit-planes P0, P1
//                    of the level index stand in for the (t, h, m) vectors of Eqs. 18-19:
//                    D = 2 * sum_b 2^b * popcount(w & P_b) - colsum), fused with the sparse part.
//   kIntPopcount     D alone by popcount (test / measurement hook).
//
// Mapping: lanes run along m (one output column per lane), so a wave's activation word load is one
// contiguous 256-byte segment of a plane row, and everything that depends only on the weight row --
// sign words, residual columns and values -- is wave-uniform and travels through the scalar path.
// In the popcount loop the sign words feed v_and/v_xor as SGPR operands: per 32 binary
// multiply-adds one logic op and one v_bcnt_u32_b32 (popcount with accumulate), the CDNA counterpart
// of the paper's xor/popcount/add port analysis.
//
// Sparse part: a workgroup (up to 8 waves = 128 weight rows in launch-slot order, one 64-column
// strip) walks K in chunks of 256.  The waves expand the chunk's plane words into a byte-per-
// activation code table in LDS (row = output column, 256 codes + pad; the 260-byte row pitch keeps
// the 64 lanes of a wave on distinct banks).  After a barrier every wave adds the residuals of its
// rows whose column falls in the chunk: one ds_read_u8, one convert and one float64 fused
// multiply-add per residual and lane, found through per-(row, chunk) offsets prepared at compress
// time.  Rows are dealt to waves by residual count (see balanced_slots), which is what keeps the
// skewed rows of pruned layers from serialising one wave.
#include "apb_internal.h"

namespace apb {

namespace {

constexpr int TN = kRowTile;
constexpr int kTablePitch = kChunkK + 4;                       // bytes per column row of the code table
constexpr int kTableBytes = kWave * kTablePitch;               // one buffer; two are used alternately

enum FwdMode { kFusedPopcount = 0, kIntPopcount = 1 };

struct FwdParams {
    const uint32_t* __restrict__ signT;
    const uint32_t* __restrict__ planes;
    const int32_t* __restrict__ colsum;
    const int32_t* __restrict__ rowsum;
    const int32_t* __restrict__ perm;
    const int32_t* __restrict__ chunk_ptr;
    const int32_t* __restrict__ col_idx;
    const double* __restrict__ vald;
    const double* __restrict__ slot_valsum;
    float* Y;
    int32_t* __restrict__ D;
    double alpha, step;
    int Np, Kw, K, Mp, M, nchunks;
    int row_groups;              // Np / (TN * waves)
    int blocks;                  // row_groups * strips
};

// Spread the 4 low bits of `nib` to the least significant bits of the 4 bytes of a word.
__device__ __forceinline__ uint32_t spread4(uint32_t nib) { return (nib * 0x00204081u) & 0x01010101u; }

template <int BITS>
__device__ __forceinline__ void expand_word(uint32_t x0, uint32_t x1, uint8_t* dst_bytes) {
    uint32_t* dst = reinterpret_cast<uint32_t*>(dst_bytes);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint32_t t = spread4((x0 >> (4 * i)) & 0xFu);
        if (BITS == 2) t |= spread4((x1 >> (4 * i)) & 0xFu) << 1;
        dst[i] = t;                                             // bytes: codes of k = 32*j + 4*i + 0..3
    }
}

template <int BITS, int MODE>
__global__ __launch_bounds__(kWave* kMaxWavesPerBlock) void k_forward_valu(const FwdParams p) {
    extern __shared__ __align__(16) uint8_t lds[];
    constexpr bool kSparse = MODE != kIntPopcount;              // sparse part present
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int waves = blockDim.x / kWave;

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of tasks so
    // that the row groups sharing one activation strip also share one L2.
    int task = blockIdx.x;
    if ((p.blocks & 7) == 0) task = (blockIdx.x & 7) * (p.blocks >> 3) + (blockIdx.x >> 3);
    const int rg = task % p.row_groups;
    const int strip = task / p.row_groups;
    const int slot0 = (rg * waves + wave) * TN;
    const int m = strip * kWave + lane;

    int acc[BITS][TN];
    double accd[TN];
#pragma unroll
    for (int r = 0; r < TN; ++r) {
        acc[0][r] = 0;
        acc[BITS - 1][r] = 0;
        accd[r] = 0.0;
    }

    const uint32_t* wp = p.signT + slot0;
    const uint32_t* xp = p.planes + m;
    const size_t plane_stride = (size_t)p.Kw * p.Mp;
    uint8_t* my_row = lds + lane * kTablePitch;

    // The activation words of one whole chunk live in registers and are fetched one
    // chunk ahead; the weight words (scalar loads) one word ahead.
    uint32_t xcur[BITS][kChunkWords], xnext[BITS][kChunkWords];
    uint32_t wnext[TN];
#pragma unroll
    for (int jj = 0; jj < kChunkWords; ++jj)
#pragma unroll
        for (int b = 0; b < BITS; ++b) xnext[b][jj] = jj < p.Kw ? xp[b * plane_stride + (size_t)jj * p.Mp] : 0u;
#pragma unroll
    for (int r = 0; r < TN; ++r) wnext[r] = wp[r];

    for (int c = 0; c < p.nchunks; ++c) {
        const int j0 = c * kChunkWords;
        uint8_t* table_row = my_row + (c & 1) * kTableBytes;
#pragma unroll
        for (int jj = 0; jj < kChunkWords; ++jj)
#pragma unroll
            for (int b = 0; b < BITS; ++b) {
                xcur[b][jj] = xnext[b][jj];
                const int jn = j0 + kChunkWords + jj;           // words past the end read as zero
                xnext[b][jj] = jn < p.Kw ? xp[b * plane_stride + (size_t)jn * p.Mp] : 0u;
            }
#pragma unroll
        for (int jj = 0; jj < kChunkWords; ++jj) {
            const int j = j0 + jj;
            if (j >= p.Kw) break;
            uint32_t wcur[TN];
#pragma unroll
            for (int r = 0; r < TN; ++r) wcur[r] = wnext[r];
            if (j + 1 < p.Kw) {
                const uint32_t* w = wp + (size_t)(j + 1) * p.Np;
#pragma unroll
                for (int r = 0; r < TN; ++r) wnext[r] = w[r];
            }
            const uint32_t x0 = xcur[0][jj];
            const uint32_t x1 = xcur[BITS - 1][jj];
#pragma unroll
            for (int r = 0; r < TN; ++r) {
                if (BITS == 1) {
                    acc[0][r] += __builtin_popcount(wcur[r] ^ x0);
                } else {
                    acc[0][r] += __builtin_popcount(wcur[r] & x0);
                    acc[1][r] += __builtin_popcount(wcur[r] & x1);
                }
            }
            if (kSparse && (jj % waves) == wave) expand_word<BITS>(x0, x1, table_row + 32 * jj);
        }
        if (!kSparse) continue;
        __syncthreads();                                        // the chunk's code table is complete
        const int kbase = c * kChunkK;
        const int32_t* cur_ptr = p.chunk_ptr + (size_t)c * p.Np + slot0;
        const int32_t* next_ptr = cur_ptr + p.Np;
#pragma unroll
        for (int r = 0; r < TN; ++r) {
            int q = cur_ptr[r];
            const int q1 = next_ptr[r];
            double a = accd[r];
            for (; q + 4 <= q1; q += 4) {
                const int c0 = p.col_idx[q] - kbase, c1 = p.col_idx[q + 1] - kbase;
                const int c2 = p.col_idx[q + 2] - kbase, c3 = p.col_idx[q + 3] - kbase;
                const double v0 = p.vald[q], v1 = p.vald[q + 1], v2 = p.vald[q + 2], v3 = p.vald[q + 3];
                const uint32_t e0 = table_row[c0], e1 = table_row[c1], e2 = table_row[c2], e3 = table_row[c3];
                a = fma(v0, (double)e0, a);
                a = fma(v1, (double)e1, a);
                a = fma(v2, (double)e2, a);
                a = fma(v3, (double)e3, a);
            }
            for (; q < q1; ++q) {
                const uint32_t e = table_row[p.col_idx[q] - kbase];
                a = fma(p.vald[q], (double)e, a);
            }
            accd[r] = a;
        }
        // The next chunk writes the other buffer; this one is rewritten two chunks from now, after
        // every wave has passed the next barrier, i.e. has finished reading it.
    }

    const int cs = p.colsum[m];
    const bool col_ok = m < p.M;
#pragma unroll
    for (int r = 0; r < TN; ++r) {
        const int n = p.perm[slot0 + r];
        if (n < 0) continue;
        const int d = BITS == 1 ? p.K - 2 * acc[0][r] : 2 * (acc[0][r] + 2 * acc[BITS - 1][r]) - cs;
        if (MODE == kIntPopcount) {
            if (col_ok) p.D[(size_t)n * p.M + m] = d;
            continue;
        }
        // 1-bit activations: the table holds (c+1)/2 in {0,1}, so sum val*c = 2*sum val*code - sum val.
        const double sparse = BITS == 1 ? 2.0 * accd[r] - p.slot_valsum[slot0 + r] : accd[r];
        const double y = fma(p.alpha, (double)d, sparse) * p.step;
        if (col_ok) p.Y[(size_t)n * p.M + m] = (float)y;
    }
}

int launch_mode(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, int M, int bits, float step,
                float* Y, int32_t* D, int mode, hipStream_t s) {
    const int Mp = kWave * ((M + kWave - 1) / kWave);
    FwdParams p;
    p.signT = L.signT;
    p.planes = planes;
    p.colsum = colsum;
    p.rowsum = L.rowsum;
    p.perm = L.perm;
    p.chunk_ptr = L.chunk_ptr;
    p.col_idx = L.col_idx;
    p.vald = L.vald;
    p.slot_valsum = L.slot_valsum;
    p.Y = Y;
    p.D = D;
    p.alpha = (double)L.alpha;
    p.step = (double)step;
    p.Np = L.Np;
    p.Kw = L.Kw;
    p.K = L.K;
    p.Mp = Mp;
    p.M = M;
    p.nchunks = L.nchunks;
    p.row_groups = L.Np / (TN * L.waves);
    const long long blocks = (long long)p.row_groups * (Mp / kWave);
    if (blocks > 0x7fffffffLL) return APB_ERR_SHAPE;
    p.blocks = (int)blocks;
    const dim3 grid((unsigned)blocks), block(kWave * L.waves);
    const size_t lds_bytes = mode == kIntPopcount ? 0 : 2 * kTableBytes;
#define APB_FWD(B, MD) hipLaunchKernelGGL((k_forward_valu<B, MD>), grid, block, lds_bytes, s, p)
    if (mode == kFusedPopcount) {
        if (bits == 1) APB_FWD(1, kFusedPopcount); else APB_FWD(2, kFusedPopcount);
    } else {
        if (bits == 1) APB_FWD(1, kIntPopcount); else APB_FWD(2, kIntPopcount);
    }
#undef APB_FWD
    APB_HIP(hipGetLastError());
    return APB_OK;
}

}  // namespace

int launch_forward_popcount(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, int M, int bits,
                            float step, float* Y, int32_t* D, hipStream_t s) {
    return launch_mode(L, planes, colsum, M, bits, step, Y, D, D ? kIntPopcount : kFusedPopcount, s);
}

}  // namespace apb
