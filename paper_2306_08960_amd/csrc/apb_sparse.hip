// Sparse part and epilogue of apb_forward (Sec. III Eqs. 12-13):
//     Y[n,m] = s * ( alpha * D[n,m] + sum_{j in row n} val_j * c[col_j, m] )
// The matrix-core kernel has left the raw binary product P in the output buffer; this kernel turns
// it into D, adds the residual part in float64 and overwrites the same elements with Y (every lane
// reads and writes only its own outputs, so the pass is in place).
//
// Mapping: lanes run along m (64 output columns per wave), so residual columns and values are
// wave-uniform and arrive through the scalar path.  A workgroup (up to 8 waves, each owning a tile
// of 16 weight rows in launch-slot order) shares one 64-column strip and walks K in chunks of 256:
//   1. the waves expand the chunk's activation bit-planes into a byte-per-activation code table in
//      LDS (row = output column, 256 codes + 4 pad bytes, so the 64 lanes of a wave hit distinct
//      banks when they read the same k);
//   2. after a barrier each wave streams the residuals of its 16 rows that fall in the chunk.  They
//      were laid out at compress time as ONE flat run per (tile, chunk), sorted by row, so the loop
//      has no per-row prologue (runs are padded to whole batches of 8): per residual and lane one address add, one ds_read_u8, one convert
//      and one float64 fused multiply-add, plus a register flush when the run moves to the next row.
// Tiles are filled by dealing rows in order of residual count (see balanced_slots), so the skewed
// rows of pruned layers are spread over the waves instead of serialising one of them.
#include "apb_internal.h"

namespace apb {

namespace {

constexpr int TN = kRowTile;
constexpr int kTablePitch = kChunkK + 4;                       // bytes per column row of the code table
constexpr int kTableBytes = kWave * kTablePitch;               // one buffer; two are used alternately
constexpr int kMaxWordsPerWave = kChunkWords;                  // a lone wave expands all 8 words of a chunk

struct SparseParams {
    double alpha, step;
    int Np, Kw, Mp, M, nchunks;
    int row_groups;                          // Np / (TN * waves)
    int blocks;                              // row_groups * strips
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

typedef double v16d __attribute__((ext_vector_type(TN)));

// acc[row] += a for a wave-uniform row; `a` restarts at zero.  The accumulators are one register
// vector indexed through the scalar GPR-index mode (two moves in, one add, two moves out).  The
// empty asm keeps this a real (uniform) branch: folded into selects it would touch all 16 rows.
#define APB_FLUSH(KEY)                                   \
    if ((KEY) & 0x1000u) {                               \
        asm volatile("" ::: "memory");                   \
        acc[((KEY) >> 8) & 15] += a;                     \
        a = 0.0;                                         \
    }

template <int BITS>
__global__ __launch_bounds__(kWave* kMaxWavesPerBlock) void k_sparse_epilogue(
    // Separate restrict-qualified arguments (not struct members) so that the compiler knows the
    // read-only arrays cannot alias Y and keeps the wave-uniform loads on the scalar path.
    const uint32_t* __restrict__ planes, const int32_t* __restrict__ colsum, const int32_t* __restrict__ rowsum,
    const int32_t* __restrict__ perm,
    const int32_t* __restrict__ seg_ptr,     // [tiles][nchunks+1] first entry of (tile, chunk)
    const uint32_t* __restrict__ ent_key,    // col_local | row_in_tile << 8 | last_of_row_run << 12
    const double* __restrict__ ent_val, const double* __restrict__ slot_valsum,
    float* Y,                                // holds P (int32 bits) on entry, Y on exit
    const SparseParams p) {
    extern __shared__ __align__(16) uint8_t lds[];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int waves = blockDim.x / kWave;

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of tasks so
    // that the row groups sharing one activation strip also share one L2.
    int task = blockIdx.x;
    if ((p.blocks & 7) == 0) task = (blockIdx.x & 7) * (p.blocks >> 3) + (blockIdx.x >> 3);
    const int rg = task % p.row_groups;
    const int strip = task / p.row_groups;
    const int tile = rg * waves + wave;
    const int slot0 = tile * TN;
    const int m = strip * kWave + lane;

    static_assert(TN == 16, "row field of an entry key is 4 bits");
    v16d acc;
#pragma unroll
    for (int r = 0; r < TN; ++r) acc[r] = 0.0;

    const uint32_t* xp = planes + m;
    const size_t plane_stride = (size_t)p.Kw * p.Mp;
    uint8_t* my_row = lds + lane * kTablePitch;
    const int32_t* seg = seg_ptr + (size_t)tile * (p.nchunks + 1);

    // Words this wave expands in a chunk: jj = wave, wave + waves, ...  They are fetched one chunk
    // ahead so that their latency hides behind the residual loop of the chunk before.
    uint32_t xw[BITS][kMaxWordsPerWave];
    auto fetch = [&](int c) {
#pragma unroll
        for (int i = 0; i < kMaxWordsPerWave; ++i) {
            const int jj = wave + i * waves;
            const int j = c * kChunkWords + jj;
            const bool ok = jj < kChunkWords && j < p.Kw;
#pragma unroll
            for (int b = 0; b < BITS; ++b) xw[b][i] = ok ? xp[b * plane_stride + (size_t)j * p.Mp] : 0u;
        }
    };
    fetch(0);
    int e1 = seg[0];

    for (int c = 0; c < p.nchunks; ++c) {
        uint8_t* table_row = my_row + (c & 1) * kTableBytes;
#pragma unroll
        for (int i = 0; i < kMaxWordsPerWave; ++i) {
            const int jj = wave + i * waves;
            if (jj < kChunkWords) expand_word<BITS>(xw[0][i], xw[BITS - 1][i], table_row + 32 * jj);
        }
        if (c + 1 < p.nchunks) fetch(c + 1);
        int e = e1;
        e1 = seg[c + 1];
        __syncthreads();                                        // the chunk's code table is complete

        double a = 0.0;                                         // partial sum of the current row run
        // Runs are padded to a multiple of 8 entries (key 0, value 0.0) at compress time, so the loop
        // works in whole batches: 16 entries per scalar-load round trip while they last, then at most
        // one batch of 8.  A large batch is what amortises the scalar-cache latency.
        for (; e + 16 <= e1; e += 16) {
            uint32_t k[16];
            double v[16];
            uint32_t cc[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                k[i] = ent_key[e + i];
                v[i] = ent_val[e + i];
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) cc[i] = table_row[k[i] & 255u];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                a = fma(v[i], (double)cc[i], a);
                APB_FLUSH(k[i])
            }
        }
        if (e < e1) {
            uint32_t k[8];
            double v[8];
            uint32_t cc[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                k[i] = ent_key[e + i];
                v[i] = ent_val[e + i];
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) cc[i] = table_row[k[i] & 255u];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                a = fma(v[i], (double)cc[i], a);
                APB_FLUSH(k[i])
            }
        }
        // Every run ends with a flagged entry, so `a` is zero here.  The next chunk writes the other
        // table buffer; this one is rewritten two chunks from now, after every wave has passed the
        // next barrier, i.e. has finished reading it.
    }

    const int cs = colsum[m];
    const bool col_ok = m < p.M;
#pragma unroll
    for (int r = 0; r < TN; ++r) {
        const int n = perm[slot0 + r];
        if (n < 0) continue;
        // raw matrix-core product P = sum_k b*code  ->  D (b = sign bit, code = stored code)
        const int P = col_ok ? reinterpret_cast<const int32_t*>(Y)[(size_t)n * p.M + m] : 0;
        const int d = BITS == 1 ? 4 * P - rowsum[n] - 2 * cs : 2 * P - cs;
        // 1-bit activations: the table holds (c+1)/2 in {0,1}, so sum val*c = 2*sum val*code - sum val.
        const double sparse = BITS == 1 ? 2.0 * acc[r] - slot_valsum[slot0 + r] : acc[r];
        const double y = fma(p.alpha, (double)d, sparse) * p.step;
        if (col_ok) Y[(size_t)n * p.M + m] = (float)y;
    }
}

}  // namespace

int launch_sparse_epilogue(const LayerDev& L, const uint32_t* planes, const int32_t* colsum, int M, int bits,
                           float step, float* Y, hipStream_t s) {
    const int Mp = kWave * ((M + kWave - 1) / kWave);
    SparseParams p;
    p.alpha = (double)L.alpha;
    p.step = (double)step;
    p.Np = L.Np;
    p.Kw = L.Kw;
    p.Mp = Mp;
    p.M = M;
    p.nchunks = L.nchunks;
    p.row_groups = L.Np / (TN * L.waves);
    const long long blocks = (long long)p.row_groups * (Mp / kWave);
    if (blocks > 0x7fffffffLL) return APB_ERR_SHAPE;
    p.blocks = (int)blocks;
    const dim3 grid((unsigned)blocks), block(kWave * L.waves);
#define APB_SPARSE(B)                                                                                       \
    hipLaunchKernelGGL(k_sparse_epilogue<B>, grid, block, 2 * kTableBytes, s, planes, colsum, L.rowsum, L.perm, \
                       L.seg_ptr, L.ent_key, L.ent_val, L.slot_valsum, Y, p)
    if (bits == 1) APB_SPARSE(1); else APB_SPARSE(2);
#undef APB_SPARSE
    APB_HIP(hipGetLastError());
    return APB_OK;
}

}  // namespace apb
