// apb_quantize_acts: quantize K x M float activations to 1 or 2 bits (Sec. IV, "1/1": +-beta;
// "1/2": a_p = p*s, p in 0..3) and pack them K-wise into bit-planes [bits][Kw][Mp], plus the
// per-column code sums (the Theta(n^2) term hoisted out of the product, Sec. IV "1/2").
//
// HBM-bound: reads 4*K*M bytes once, writes bits*K*M/8.  Lanes run along m; a lane owns CPL (4, 2
// or 1) adjacent columns, so a load is a 16-, 8- or 4-byte vector and a wave's load covers one
// contiguous piece of a row of X.  A lane builds, for 32 consecutive k, CPL words per plane and
// stores them as one vector.  One workgroup owns a strip of 64*CPL columns for ALL of K: its waves
// take the words of K round-robin, add their per-column code sums up in LDS at the end and write
// them with a plain store -- no zero-fill launch, no atomics.  CPL and the number of waves are
// picked per shape: wide strips for wide M (long bursts), narrow strips and many waves when M alone
// cannot fill the chip, and a wave count that divides the words of K evenly.  Only when M is so
// small that even 64-column strips leave most CUs idle is K also split across workgroups, whose
// (integer, hence order-independent) sums then meet in a zero-filled colsum through atomics.
#include "apb_internal.h"

namespace apb {

namespace {

constexpr int kMaxWaves = 16;

__global__ __launch_bounds__(256) void k_zero_words(uint32_t* __restrict__ p, size_t count) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (size_t)gridDim.x * 256) p[i] = 0u;
}

template <int CPL>
struct Vec;
template <>
struct Vec<4> {
    typedef float F __attribute__((ext_vector_type(4)));
    typedef uint4 U;
};
template <>
struct Vec<2> {
    typedef float F __attribute__((ext_vector_type(2)));
    typedef uint2 U;
};
template <>
struct Vec<1> {
    typedef float F;
    typedef uint32_t U;
};

// CPL > 1 needs M % CPL == 0 and 16-byte (CPL 4) / 8-byte (CPL 2) aligned X and planes.
template <int BITS, int CPL>
__global__ __launch_bounds__(kWave* kMaxWaves) void k_quantize_pack(const float* __restrict__ X, int K, int M, int Kw,
                                                                    int Mp, float inv_step, int words_per_slab,
                                                                    uint32_t* __restrict__ planes,
                                                                    int32_t* __restrict__ colsum) {
    typedef typename Vec<CPL>::F FV;
    typedef typename Vec<CPL>::U UV;
    constexpr int kStrip = kWave * CPL;                             // columns per workgroup
    extern __shared__ int s_sum[];                                  // [waves][kStrip]
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int waves = blockDim.x / kWave;
    const int m0 = blockIdx.x * kStrip + lane * CPL;                // first of this lane's columns
    const bool col_ok = m0 < M;                                     // M % CPL == 0: all of them or none
    int sum[CPL];
#pragma unroll
    for (int q = 0; q < CPL; ++q) sum[q] = 0;

    // Loads are unconditional (addresses clamped into the matrix, results masked afterwards): a
    // branch around each load would make every load wait for the one before.  They carry the
    // non-temporal hint: X is read exactly once, and streaming it through L2 as ordinary data would
    // evict what the forward kernel is about to read (the planes written here, the layer).
    const float* src = X + min(m0, M - CPL);
    const int j_begin = blockIdx.y * words_per_slab;
    const int j_end = min(Kw, j_begin + words_per_slab);
    for (int j = j_begin + wave; j < j_end; j += waves) {
        uint32_t w0[CPL], w1[CPL];
#pragma unroll
        for (int q = 0; q < CPL; ++q) w0[q] = w1[q] = 0;
        const int k0 = j * 32;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            FV xv[16];                                              // 16 independent loads in flight
#pragma unroll
            for (int i = 0; i < 16; ++i)
                xv[i] = __builtin_nontemporal_load(reinterpret_cast<const FV*>(src + (size_t)min(k0 + 16 * half + i, K - 1) * M));
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float xs[CPL];
                __builtin_memcpy(xs, &xv[i], sizeof(xs));
                const int bit = 16 * half + i;
#pragma unroll
                for (int q = 0; q < CPL; ++q) {
                    if (BITS == 1) {
                        w0[q] |= (xs[q] >= 0.0f ? 1u : 0u) << bit;
                    } else {
                        // (the values of k arrive in order: each pushes its two bits on top of the words)
                        const uint32_t p = code2_low_bits(xs[q], inv_step);
                        w0[q] = push_bit(w0[q], p);
                        w1[q] = push_bit(w1[q], p >> 1);
                    }
                }
            }
        }
        // Bits of k >= K (last word) and of columns >= M are cleared here, in one go; the code sums
        // come from popcounts of the finished words.
        const int valid = K - k0;
        const uint32_t keep = !col_ok ? 0u : (valid >= 32 ? 0xffffffffu : ((1u << valid) - 1u));
#pragma unroll
        for (int q = 0; q < CPL; ++q) {
            w0[q] &= keep;
            w1[q] &= keep;
            sum[q] += __builtin_popcount(w0[q]) + 2 * __builtin_popcount(w1[q]);
        }
        if (m0 < Mp) {
            UV o0, o1;
            __builtin_memcpy(&o0, w0, sizeof(o0));
            __builtin_memcpy(&o1, w1, sizeof(o1));
            *reinterpret_cast<UV*>(planes + (size_t)j * Mp + m0) = o0;
            if (BITS == 2) *reinterpret_cast<UV*>(planes + ((size_t)Kw + j) * Mp + m0) = o1;
        }
    }
    if (colsum == nullptr) return;                                  // the caller takes the code sums from the words
#pragma unroll
    for (int q = 0; q < CPL; ++q) s_sum[wave * kStrip + lane * CPL + q] = sum[q];
    __syncthreads();
    for (int c = threadIdx.x; c < kStrip; c += blockDim.x) {        // one column per thread now
        const int m = blockIdx.x * kStrip + c;
        if (m < Mp) {
            int total = 0;
            for (int w = 0; w < waves; ++w) total += s_sum[w * kStrip + c];
            if (gridDim.y == 1) colsum[m] = total;
            else if (total != 0) atomicAdd(&colsum[m], total);
        }
    }
}

template <int BITS, int CPL>
void launch_pack(const float* X, int K, int M, int Kw, int Mp, float inv_step, uint32_t* planes, int32_t* colsum,
                 int strips, int slabs, int words_per_slab, int waves, hipStream_t s) {
    hipLaunchKernelGGL((k_quantize_pack<BITS, CPL>), dim3(strips, slabs), dim3(kWave * waves),
                       (size_t)waves * kWave * CPL * sizeof(int), s, X, K, M, Kw, Mp, inv_step, words_per_slab, planes,
                       colsum);
}

}  // namespace

// A fill kernel rather than a memset node: the launch may be recorded into a graph.
int launch_zero_words(uint32_t* p, size_t count, hipStream_t s) {
    if (count == 0) return APB_OK;
    const size_t blocks = (count + 255) / 256;
    hipLaunchKernelGGL(k_zero_words, dim3((unsigned)(blocks < 65536 ? blocks : 65536)), dim3(256), 0, s, p, count);
    APB_HIP(hipGetLastError());
    return APB_OK;
}

int launch_quantize(const float* X, int K, int M, int bits, float inv_step, uint32_t* planes, int32_t* colsum,
                    hipStream_t s) {
    const int Kw = (K + 31) / 32;
    const int Mp = kWave * ((M + kWave - 1) / kWave);
    const uintptr_t addr = reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(planes);
    // Widest strip (16-byte loads per lane: measured 5.6 against 5.0 TB/s with 4-byte ones on M = 12544) that still
    // leaves 32 strips or more; K is split below where that is too few workgroups.
    int cpl = 1;
    if (M % 4 == 0 && (addr & 15u) == 0 && (long long)((Mp + 255) / 256) * kMaxWaves >= 512) cpl = 4;
    else if (M % 2 == 0 && (addr & 7u) == 0 && (long long)((Mp + 127) / 128) * kMaxWaves >= 1024) cpl = 2;
    const int strip = kWave * cpl;
    const int strips = (Mp + strip - 1) / strip;
    // Few strips: split K into slabs as well, until three quarters of the 256 compute units have a workgroup
    // (and there are 1024 waves) or a slab is down to 4 words.  (Measured: 128 strips -> 2 slabs gains a fifth;
    // splitting 196 strips further loses -- with column sums to the extra fill launch and the atomics, and
    // without them (colsum == nullptr) 384 or 768 workgroups were still 3 % slower than 196.)
    const long long min_groups = 192;
    int slabs = 1;
    while (((long long)strips * slabs < min_groups || (long long)strips * kMaxWaves * slabs < 1024) &&
           (Kw + 2 * slabs - 1) / (2 * slabs) >= 4)
        slabs *= 2;
    const int words_per_slab = (Kw + slabs - 1) / slabs;
    slabs = (Kw + words_per_slab - 1) / words_per_slab;
    // Waves per workgroup: at least what it takes to put 2048 waves on the chip (16 at most), and among
    // those the count that wastes the fewest word slots (a wave takes ceil(words / waves) words).
    int lo = 1;
    while (lo < kMaxWaves && (long long)strips * slabs * lo < 2048) ++lo;
    int waves = lo;
    long long best = -1;
    for (int w = lo; w <= kMaxWaves; ++w) {
        const long long slots = (long long)((words_per_slab + w - 1) / w) * w;
        if (best < 0 || slots < best || (slots == best && w <= words_per_slab)) {
            best = slots;
            waves = w;
        }
    }
    if (slabs > 1 && colsum) {
        const int rc = launch_zero_words(reinterpret_cast<uint32_t*>(colsum), (size_t)Mp, s);
        if (rc != APB_OK) return rc;
    }
#define APB_PACK(B, C) launch_pack<B, C>(X, K, M, Kw, Mp, inv_step, planes, colsum, strips, slabs, words_per_slab, waves, s)
    if (bits == 1) {
        if (cpl == 4) APB_PACK(1, 4); else if (cpl == 2) APB_PACK(1, 2); else APB_PACK(1, 1);
    } else {
        if (cpl == 4) APB_PACK(2, 4); else if (cpl == 2) APB_PACK(2, 2); else APB_PACK(2, 1);
    }
#undef APB_PACK
    APB_HIP(hipGetLastError());
    return APB_OK;
}

}  // namespace apb
