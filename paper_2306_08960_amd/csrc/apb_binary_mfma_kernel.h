// Binary part on the matrix cores (kernel template and tile choice; instantiated by the
// apb_binary_mfma_*.hip files, one operand format each, so that they compile in parallel):
// P[n,m] = sum_k b[n,k] * code[k,m] with b = sign bit in {0,1} and
// code = stored activation code (0..3 for 2-bit, 0/1 for 1-bit), from which
//   2-bit:  D = sum_k sigma*p       = 2*P - colsum[m]
//   1-bit:  D = sum_k sigma*(2c-1)  = 4*P - rowsum[n] - 2*colsum[m]
// (sigma = 2b-1; the same algebra that turns Sec. IV Eq. 16 / Eqs. 18-19 into and+popcount forms).
//
// The operands stay packed (one bit per weight, one bit per activation plane) all the way into
// registers.  There each lane spreads the 32 bits it owns into the 32 four-bit operand slots of one
// v_mfma_scale_f32_32x32x64_f8f6f4 in FP4 (E2M1) format with shift+and: a weight bit becomes the
// nibble 0b0001 (= 0.5), the two plane bits of an activation become the nibble p0 | p1<<1
// (= 0.5, 1.0, 1.5 for codes 1, 2, 3 -- the encoding is additive in the planes, so no table is
// needed).  Products are multiples of 1/4 and every partial sum is far below 2^24 of those, so the
// float accumulators hold P/4 exactly; the result is converted back to int32.  HBM, L2 and the load
// path only ever carry bits.  The k-slot a bit lands in is the same function of (lane half, dword,
// nibble) for both operands, which is all the contraction needs:
//   lane l = 32*g + i (i: row of A / column of B, g: lane half) owns word 2*s+g of K step s;
//   nibble t of operand dword d  <->  bit d + 4*t of that word.
//
// The same kernel serves the 2/2 routine of Sec. IV (2-bit weights x 2-bit activations): the
// weight operand is then expanded from two bit-planes exactly like the activations, P = sum_k q*p,
// and the epilogue applies the zero-centring of the weights, D22 = sum_k (2q-3)*p = 2*P - 3*colsum[m]
// (written as int32, or scaled to Y = (s_w*s_a/2) * D22).
//
// The K loop is software-pipelined by hand: words are fetched four steps ahead into a ring of
// register sets, and the expansion of step s+1 is interleaved with the MFMAs of step s so that the
// vector ALU works in the shadow of the matrix pipe.
#pragma once

#include "apb_fp4_expand.h"
#include "apb_internal.h"

namespace apb {
namespace mfma_detail {

enum Epilogue { kInt22 = 1, kFloat22 = 2, kIntD = 3 };   // kIntD: D of the binary layer

struct MfmaParams {
    const uint32_t* __restrict__ signT;   // [wbits][Kw2][Np]  word j of row n, rows in the layer's own order
    const uint32_t* __restrict__ planes;  // [bits][Kw][Mp]
    const int32_t* __restrict__ colsum;   // [Mp]
    const int32_t* __restrict__ rowsum;   // [N]    (kIntD with 1-bit activations)
    void* __restrict__ out;               // [N][M] int32 (kIntD, kInt22) or float (kFloat22)
    double scale;                         // kFloat22: s_w * s_a / 2
    size_t wplane_stride;                 // words between the weight planes
    int Np, Kw, Mp, M;
    int tiles_m;                          // workgroup tiles along m
    int waves_m;                          // waves of a workgroup laid along m (2 or 4); the rest along n
};

// Workgroup = 4 waves; each wave owns RN x RM MFMA tiles of 32 x 32 and walks K in steps of 64.
template <int WBITS, int BITS, int RN, int RM, int EPI>
__global__ __launch_bounds__(256) void k_binary_mfma(const MfmaParams p) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i = lane & 31, g = lane >> 5;
    const int tile_m = blockIdx.x % p.tiles_m;
    const int tile_n = blockIdx.x / p.tiles_m;
    const int waves_n = 4 / p.waves_m;
    const int slot_base = (tile_n * waves_n + wave / p.waves_m) * (32 * RN);
    const int m_base = (tile_m * p.waves_m + wave % p.waves_m) * (32 * RM);
    if (slot_base >= p.Np || m_base >= p.Mp) return;          // wave-uniform: a tile fully outside

    // Row/column this lane feeds in each tile, clamped so that loads stay inside the arrays (tiles
    // may hang over Np / Mp; results of the overhang are never stored).  The lane half g selects the
    // odd word of a step, which is a constant per-lane offset on top of a wave-uniform row pointer.
    unsigned aoff[RN], boff[RM];
#pragma unroll
    for (int t = 0; t < RN; ++t) aoff[t] = (unsigned)(g * p.Np + min(slot_base + 32 * t + i, p.Np - 1));
#pragma unroll
    for (int u = 0; u < RM; ++u) boff[u] = (unsigned)(g * p.Mp + min(m_base + 32 * u + i, p.Mp - 1));
    const size_t plane_stride = (size_t)p.Kw * p.Mp;
    const int steps = (p.Kw + 1) / 2;

    v16f acc[RN][RM];
#pragma unroll
    for (int t = 0; t < RN; ++t)
#pragma unroll
        for (int u = 0; u < RM; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][u][r] = 0.0f;

    auto load_words = [&](int s, uint32_t (&a)[WBITS][RN], uint32_t (&b)[BITS][RM]) {
        // Branch-free on purpose (a branch here would make every step wait for its own loads).
        // Odd word count: the weight array carries one extra all-zero word row, so the upper lane
        // half of the last step multiplies by zero; its activation load then reads one row past
        // the plane, which is still inside the packed buffer (the next plane, or the Mp column
        // sums that follow the last plane) and, being FP4, cannot be a NaN or an infinity.
        const int ss = min(s, steps - 1);                     // past the end: harmless re-read, never used
#pragma unroll
        for (int pl = 0; pl < WBITS; ++pl) {
            const uint32_t* arow = p.signT + pl * p.wplane_stride + (size_t)(2 * ss) * p.Np;
#pragma unroll
            for (int t = 0; t < RN; ++t) a[pl][t] = arow[aoff[t]];
        }
#pragma unroll
        for (int pl = 0; pl < BITS; ++pl) {
            const uint32_t* brow = p.planes + pl * plane_stride + (size_t)(2 * ss) * p.Mp;
#pragma unroll
            for (int u = 0; u < RM; ++u) b[pl][u] = brow[boff[u]];
        }
    };

    // A ring of kRing word sets (set s % kRing holds the words of step s) and two operand sets used
    // alternately: the loads of step s+kRing are issued during step s and first touched in step
    // s+kRing-1, so kRing-1 whole steps of work cover their latency.  No register copies.
    constexpr int kRing = (WBITS * RN + BITS * RM) <= 4 ? 16 : 8;    // ~1.5 us of HBM latency to cover
    uint32_t aw[kRing][WBITS][RN], bw[kRing][BITS][RM];
    Frag<RN, RM> f[2];
    clear_upper(f[0]);
    clear_upper(f[1]);
#pragma unroll
    for (int q = 0; q < kRing; ++q) load_words(q, aw[q], bw[q]);
    expand<WBITS, BITS, RN, RM>(aw[0], bw[0], f[0]);

    constexpr int kValuPerMfma = ((WBITS == 2 ? 15 : 7) * RN + (BITS == 2 ? 15 : 7) * RM + RN * RM - 1) / (RN * RM);
    // The main loop runs whole groups of kRing steps as straight-line code (no branch between a
    // load and its use); the remainder (at most kRing-1 steps) is finished below.
    auto one_step = [&](int s, int q) {
        const Frag<RN, RM>& cur = f[q & 1];
        load_words(s + kRing, aw[q], bw[q]);                                      // words of step s+kRing
        expand<WBITS, BITS, RN, RM>(aw[(q + 1) % kRing], bw[(q + 1) % kRing], f[(q + 1) & 1]);   // operands of step s+1
#pragma unroll
        for (int t = 0; t < RN; ++t)
#pragma unroll
            for (int u = 0; u < RM; ++u)
                acc[t][u] = mfma_fp4(cur.a[t], cur.b[u], acc[t][u]);
        // Ask the scheduler to alternate: one MFMA, then a slice of the expansion ALU work.
#pragma unroll
        for (int e = 0; e < RN * RM; ++e) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                     // 1 MFMA
            __builtin_amdgcn_sched_group_barrier(0x002, kValuPerMfma, 0);          // VALU
        }
    };
    int s0 = 0;
    for (; s0 + kRing <= steps; s0 += kRing) {
#pragma unroll
        for (int q = 0; q < kRing; ++q) one_step(s0 + q, q);
    }
#pragma unroll
    for (int q = 0; q < kRing - 1; ++q)
        if (s0 + q < steps) one_step(s0 + q, q);

    // C layout of the 32x32 tile: lane (i, g), register r  ->  row 8*(r/4) + 4*g + (r%4), column i.
    // Rows are in the layer's own order here (the dense part needs no load balancing), so the
    // epilogue is straight-line: no index loads between the stores.
    const size_t out0 = (size_t)(slot_base + 4 * g) * p.M + m_base + i;
    int cs[RM];
#pragma unroll
    for (int u = 0; u < RM; ++u) cs[u] = p.colsum[min(m_base + 32 * u + i, p.Mp - 1)];
#pragma unroll
    for (int t = 0; t < RN; ++t) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = 32 * t + 8 * (r / 4) + (r % 4);          // + slot_base + 4*g
            if (slot_base + 4 * g + row >= p.Np) continue;
#pragma unroll
            for (int u = 0; u < RM; ++u) {
                if (m_base + 32 * u + i >= p.M) continue;
                const size_t at = out0 + (size_t)row * p.M + 32 * u;
                const int P = (int)(acc[t][u][r] * 4.0f);
                if (EPI == kIntD)
                    static_cast<int32_t*>(p.out)[at] =
                        BITS == 2 ? 2 * P - cs[u] : 4 * P - p.rowsum[slot_base + 4 * g + row] - 2 * cs[u];
                else if (EPI == kInt22) static_cast<int32_t*>(p.out)[at] = 2 * P - 3 * cs[u];
                else static_cast<float*>(p.out)[at] = (float)(p.scale * (double)(2 * P - 3 * cs[u]));
            }
        }
    }
}


// The same product with the activation operand SHARED by the four waves of a workgroup through LDS.
// The waves are stacked along n (wave w: rows [32*RN*w, 32*RN*(w+1)) of the workgroup's 128*RN rows) and
// all multiply by the same 128 columns.  Wave w fetches and expands the activation words of columns
// [32*w, 32*w + 32) only and leaves the operand (16 bytes per lane) in LDS; after a barrier every wave
// reads the four operands back.  Against k_binary_mfma with the same wave tile that is a quarter of the
// activation words through L2 and a quarter of their expansion work per wave (the weight operands stay in
// registers: nothing to share along n).  Three LDS buffers rotate, one barrier per K step (see the pipeline
// in the kernel).
// No wave leaves early (the barriers, and its share of the activation operand): rows and columns outside
// the matrices are clamped for the loads and skipped by the stores.
template <int WBITS, int BITS, int RN, int EPI>
__global__ __launch_bounds__(256) void k_binary_mfma_shared(const MfmaParams p) {
    constexpr int RM = 4;
    typedef uint32_t v4u __attribute__((ext_vector_type(4)));
    __shared__ v4u bstage[3][RM][64];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i = lane & 31, g = lane >> 5;
    const int tile_m = blockIdx.x % p.tiles_m;
    const int tile_n = blockIdx.x / p.tiles_m;
    const int slot_base = (tile_n * 4 + wave) * (32 * RN);
    const int m_base = tile_m * (32 * RM);

    unsigned aoff[RN];
#pragma unroll
    for (int t = 0; t < RN; ++t) aoff[t] = (unsigned)(g * p.Np + min(slot_base + 32 * t + i, p.Np - 1));
    const unsigned boff = (unsigned)(g * p.Mp + min(m_base + 32 * wave + i, p.Mp - 1));   // this wave's share
    const size_t plane_stride = (size_t)p.Kw * p.Mp;
    const int steps = (p.Kw + 1) / 2;

    v16f acc[RN][RM];
#pragma unroll
    for (int t = 0; t < RN; ++t)
#pragma unroll
        for (int u = 0; u < RM; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][u][r] = 0.0f;

    auto load_words = [&](int s, uint32_t (&a)[WBITS][RN], uint32_t (&b)[BITS][1]) {
        const int ss = min(s, steps - 1);                     // past the end: harmless re-read, never used
#pragma unroll
        for (int pl = 0; pl < WBITS; ++pl) {
            const uint32_t* arow = p.signT + pl * p.wplane_stride + (size_t)(2 * ss) * p.Np;
#pragma unroll
            for (int t = 0; t < RN; ++t) a[pl][t] = arow[aoff[t]];
        }
#pragma unroll
        for (int pl = 0; pl < BITS; ++pl) b[pl][0] = (p.planes + pl * plane_stride + (size_t)(2 * ss) * p.Mp)[boff];
    };

    // Pipeline over the K steps (s % kRing, s % 3 and s % 2 are compile-time constants inside the unrolled loop):
    //   words:    fetched kRing steps ahead into a ring of register sets;
    //   step s:   reads the shared operands of step s+1 from LDS buffer (s+1) % 3 (written during step s-1, visible
    //             since the barrier that ended it), expands its weight words of step s+1 into the other register set
    //             and its share of the activation words of step s+2 into buffer (s+2) % 3 (last read during step
    //             s-2, whose data every wave has waited for before the barrier of step s-1), and runs the matrix
    //             instructions of step s on operands it read one step earlier -- no LDS latency in front of them.
    constexpr int kRing = 6;                                  // (12 measured the same)
    static_assert(kRing % 6 == 0, "s % 3 and s % 2 from s % kRing");
    uint32_t aw[kRing][WBITS][RN], bw[kRing][BITS][1];
    v8i fa[2][RN], fb[2][RM];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int t = 0; t < RN; ++t)
#pragma unroll
            for (int d = 4; d < 8; ++d) fa[h][t][d] = 0;
#pragma unroll
        for (int u = 0; u < RM; ++u)
#pragma unroll
            for (int d = 4; d < 8; ++d) fb[h][u][d] = 0;
    }
    auto expand_a = [&](const uint32_t (&a)[WBITS][RN], int set) {
#pragma unroll
        for (int t = 0; t < RN; ++t) expand_words<WBITS>(a[0][t], a[WBITS - 1][t], fa[set][t]);
    };
    auto expand_b = [&](const uint32_t (&b)[BITS][1], int buf) {
        v8i f;
        expand_words<BITS>(b[0][0], b[BITS - 1][0], f);
        bstage[buf][wave][lane] = v4u{(uint32_t)f[0], (uint32_t)f[1], (uint32_t)f[2], (uint32_t)f[3]};
    };
    auto read_b = [&](int buf, int set) {
#pragma unroll
        for (int u = 0; u < RM; ++u) {
            const v4u b = bstage[buf][u][lane];
#pragma unroll
            for (int d = 0; d < 4; ++d) fb[set][u][d] = (int)b[d];
        }
    };
#pragma unroll
    for (int q = 0; q < kRing; ++q) load_words(q, aw[q], bw[q]);
    expand_a(aw[0], 0);
    expand_b(bw[0], 0);
    expand_b(bw[1], 1);
    __syncthreads();
    read_b(0, 0);

    constexpr int kValuPerMfma = ((WBITS == 2 ? 15 : 7) * RN + (BITS == 2 ? 15 : 7) + RN * RM - 1) / (RN * RM);
    auto one_step = [&](int s, int q) {
        read_b((q + 1) % 3, (q + 1) & 1);                                         // operands of step s+1
        // (the words of steps s+1 and s+2 are taken out of the ring before slot q is refilled below; past the
        //  last step they are clamped re-reads, expanded and never used)
        expand_a(aw[(q + 1) % kRing], (q + 1) & 1);
        expand_b(bw[(q + 2) % kRing], (q + 2) % 3);
        load_words(s + kRing, aw[q], bw[q]);
#pragma unroll
        for (int t = 0; t < RN; ++t)
#pragma unroll
            for (int u = 0; u < RM; ++u) acc[t][u] = mfma_fp4(fa[q & 1][t], fb[q & 1][u], acc[t][u]);
        // Ask the scheduler to alternate: one matrix instruction, then a slice of the expansion work, which
        // issues in its shadow.  (Pinning the whole step -- LDS reads first, nothing across the barrier --
        // measured 5 % slower than what the scheduler makes of it.)
#pragma unroll
        for (int e = 0; e < RN * RM; ++e) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                     // 1 MFMA
            __builtin_amdgcn_sched_group_barrier(0x002, kValuPerMfma, 0);          // VALU
        }
        __syncthreads();
    };
    int s0 = 0;
    for (; s0 + kRing <= steps; s0 += kRing) {
#pragma unroll
        for (int q = 0; q < kRing; ++q) one_step(s0 + q, q);
    }
#pragma unroll
    for (int q = 0; q < kRing - 1; ++q)
        if (s0 + q < steps) one_step(s0 + q, q);              // (steps is the same for every wave: so are the barriers)

    if (slot_base >= p.Np) return;
    const size_t out0 = (size_t)(slot_base + 4 * g) * p.M + m_base + i;
    int cs[RM];
#pragma unroll
    for (int u = 0; u < RM; ++u) cs[u] = p.colsum[min(m_base + 32 * u + i, p.Mp - 1)];
#pragma unroll
    for (int t = 0; t < RN; ++t) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = 32 * t + 8 * (r / 4) + (r % 4);          // + slot_base + 4*g
            if (slot_base + 4 * g + row >= p.Np) continue;
#pragma unroll
            for (int u = 0; u < RM; ++u) {
                if (m_base + 32 * u + i >= p.M) continue;
                const size_t at = out0 + (size_t)row * p.M + 32 * u;
                const int P = (int)(acc[t][u][r] * 4.0f);
                if (EPI == kIntD)
                    static_cast<int32_t*>(p.out)[at] =
                        BITS == 2 ? 2 * P - cs[u] : 4 * P - p.rowsum[slot_base + 4 * g + row] - 2 * cs[u];
                else if (EPI == kInt22) static_cast<int32_t*>(p.out)[at] = 2 * P - 3 * cs[u];
                else static_cast<float*>(p.out)[at] = (float)(p.scale * (double)(2 * P - 3 * cs[u]));
            }
        }
    }
}

template <int WBITS, int BITS, int RN, int EPI>
void launch_shared(MfmaParams p, hipStream_t s) {
    p.waves_m = 1;
    p.tiles_m = (p.Mp + 127) / 128;
    const int tiles_n = (p.Np + 128 * RN - 1) / (128 * RN);
    hipLaunchKernelGGL((k_binary_mfma_shared<WBITS, BITS, RN, EPI>), dim3((unsigned)(p.tiles_m * tiles_n)), dim3(256), 0, s, p);
}

template <int WBITS, int BITS, int RN, int RM, int EPI>
void launch_shape(MfmaParams p, int waves_m, hipStream_t s) {
    const int waves_n = 4 / waves_m;
    p.waves_m = waves_m;
    p.tiles_m = (p.Mp + 32 * RM * waves_m - 1) / (32 * RM * waves_m);
    const int tiles_n = (p.Np + 32 * RN * waves_n - 1) / (32 * RN * waves_n);
    hipLaunchKernelGGL((k_binary_mfma<WBITS, BITS, RN, RM, EPI>), dim3((unsigned)(p.tiles_m * tiles_n)), dim3(256), 0, s,
                       p);
}

// Wave tile.  Small tiles put more waves on the chip (a lone wave per SIMD keeps neither the matrix
// pipe nor the store path busy) but re-read the packed operands from L2 more often: a wave fetches
// 256 * (WBITS*rn + BITS*rm) bytes per K step.  Measured on the benchmark shapes, the kernel slows
// down once that re-read traffic passes roughly 200 MB (about 30 us at the L2
// rate it sustains here), so: the smallest tile that stays under it, else the one that reads least.
template <int WBITS, int BITS, int EPI>
int launch_best_tile(MfmaParams p, int N, hipStream_t s) {
    if ((long long)2 * N >= (1LL << 30) || (long long)2 * p.Mp >= (1LL << 30)) return APB_ERR_SHAPE;
    // Enough workgroups of 128 rows x 128 columns for one and a half per compute unit: the kernel that shares the
    // activation operand through LDS (measured ahead of the one below from there on: 2/2 on 512 x 4608 x 12544
    // 36 -> 30 us, squares of 4096 and 8192 a quarter faster; behind it on shapes with fewer workgroups, where
    // the small wave tiles of the menu put more waves on the chip).
    if (N >= 128 && (long long)((N + 127) / 128) * ((p.Mp + 127) / 128) >= 384) {
        launch_shared<WBITS, BITS, 1, EPI>(p, s);
        APB_HIP(hipGetLastError());
        return APB_OK;
    }
    static const int menu[5][2] = {{1, 1}, {2, 1}, {2, 2}, {2, 4}, {4, 2}};    // smallest first
    constexpr double kL2Budget = 200e6;
    const double steps = (p.Kw + 1) / 2;
    int best = 0;
    double best_bytes = 1e300;
    for (int c = 0; c < 5; ++c) {
        const double waves = (double)((N + 32 * menu[c][0] - 1) / (32 * menu[c][0])) *
                             ((p.Mp + 32 * menu[c][1] - 1) / (32 * menu[c][1]));
        const double bytes = waves * steps * 256.0 * (WBITS * menu[c][0] + BITS * menu[c][1]);
        if (bytes <= kL2Budget) {
            best = c;
            break;
        }
        if (bytes < best_bytes) {
            best_bytes = bytes;
            best = c;
        }
    }
    const int rn = menu[best][0], rm = menu[best][1];
    // Waves of a workgroup: two along n when the layer has the rows for them, the rest along m.
    const int waves_n = 32 * rn * 2 <= N ? 2 : 1;
    const int waves_m = 4 / waves_n;
#define APB_SHAPE(RN, RM) \
    if (rn == RN && rm == RM) launch_shape<WBITS, BITS, RN, RM, EPI>(p, waves_m, s);
    APB_SHAPE(4, 2)
    APB_SHAPE(2, 4)
    APB_SHAPE(2, 2)
    APB_SHAPE(2, 1)
    APB_SHAPE(1, 1)
#undef APB_SHAPE
    APB_HIP(hipGetLastError());
    return APB_OK;
}


}  // namespace mfma_detail

// One operand format per translation unit (see the files of the same names).
int launch_mfma_d_1bit(const mfma_detail::MfmaParams& p, int N, hipStream_t s);      // binary layer, 1-bit activations: D
int launch_mfma_d_2bit(const mfma_detail::MfmaParams& p, int N, hipStream_t s);      // binary layer, 2-bit activations: D
int launch_mfma_22_int(const mfma_detail::MfmaParams& p, int N, hipStream_t s);      // 2/2 routine: D22
int launch_mfma_22_float(const mfma_detail::MfmaParams& p, int N, hipStream_t s);    // 2/2 routine: Y

}  // namespace apb
