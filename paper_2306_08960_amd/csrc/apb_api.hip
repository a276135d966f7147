// Host side of the C ABI: argument checks, layer ownership, launch-order row binning.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <numeric>
#include <vector>

#include "apb_internal.h"

namespace apb {

static thread_local int g_last_hip_error = 0;
void set_last_hip_error(hipError_t e) { g_last_hip_error = (int)e; }

namespace {

hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

void free_layer_buffers(LayerDev& d) {
    void* ptrs[] = {d.sign, d.signT, d.perm, d.row_ptr, d.col_idx, d.val, d.rowsum, d.chunk_ptr, d.slot_valsum, d.vald, d.signC,
                    d.seg_ptr, d.ent, d.rows_perm, d.rows_blk, d.rows_ek, d.rows_ev, d.rows_sign, d.rows_valsum,
                    d.rowsw_perm, d.rowsw_blk, d.rowsw_ek, d.rowsw_ev, d.rowsw_sign, d.rowsw_valsum};
    for (void* p : ptrs)
        if (p) (void)hipFree(p);
    d = LayerDev{};
}

template <typename T>
int dev_alloc(T** p, size_t count) {
    *p = nullptr;
    if (count == 0) count = 1;                       // keep pointers non-null for empty CSR
    hipError_t e = hipMalloc(reinterpret_cast<void**>(p), count * sizeof(T));
    if (e == hipErrorOutOfMemory) return APB_ERR_NOMEM;
    if (e != hipSuccess) {
        set_last_hip_error(e);
        return APB_ERR_HIP;
    }
    return APB_OK;
}

// Launch-order row binning for the skewed residual counts: rows sorted by decreasing residual
// count are dealt to the row tiles like cards, forwards then backwards (a "snake"), so every
// tile of kRowTile rows carries about the same number of residuals.
std::vector<int32_t> balanced_slots(const std::vector<int32_t>& counts, int Np) {
    const int N = (int)counts.size();
    const int tiles = Np / kRowTile;
    std::vector<int32_t> order(N);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return counts[a] > counts[b]; });
    std::vector<int32_t> perm(Np, -1);
    std::vector<int> fill(tiles, 0);
    for (int i = 0; i < N; ++i) {
        const int round = i / tiles, pos = i % tiles;
        const int t = (round & 1) ? tiles - 1 - pos : pos;
        perm[t * kRowTile + fill[t]++] = order[i];
    }
    // Inside a tile the order of the rows is free: ascending, so that rows sharing a 32-row word of
    // a packed output sit next to each other.
    for (int t = 0; t < tiles; ++t) std::sort(perm.begin() + t * kRowTile, perm.begin() + t * kRowTile + fill[t]);
    return perm;
}

// Regroup the CSR for the sparse kernel: for every tile of kRowTile launch slots and every chunk of
// kChunkK columns one flat run of entries, sorted by (row in tile, column) and padded to whole
// blocks of 8.  A block is 24 words: 8 keys (2*row | column_in_chunk << 8), then the 8 residuals as
// float64 times 2^kEntValScaleLog2; padding entries have key 0 and value 0.  seg_ptr counts blocks.
void build_tile_runs(const std::vector<int32_t>& perm, const std::vector<int32_t>& row_ptr,
                     const std::vector<int32_t>& col, const std::vector<float>& val, int nchunks,
                     std::vector<int32_t>& seg_ptr, std::vector<uint32_t>& ent) {
    const int tiles = (int)perm.size() / kRowTile;
    seg_ptr.assign((size_t)tiles * (nchunks + 1), 0);
    ent.clear();
    ent.reserve(col.size() * 3 + 24);
    std::vector<int32_t> cursor(kRowTile);
    std::vector<uint32_t> key;
    std::vector<double> dval;
    for (int t = 0; t < tiles; ++t) {
        for (int r = 0; r < kRowTile; ++r) {
            const int n = perm[(size_t)t * kRowTile + r];
            cursor[r] = n >= 0 ? row_ptr[n] : 0;
        }
        for (int c = 0; c < nchunks; ++c) {
            seg_ptr[(size_t)t * (nchunks + 1) + c] = (int32_t)(ent.size() / kEntBlockWords);
            const int hi = (c + 1) * kChunkK;
            key.clear();
            dval.clear();
            for (int r = 0; r < kRowTile; ++r) {
                const int n = perm[(size_t)t * kRowTile + r];
                if (n < 0) continue;
                const int end = row_ptr[n + 1];
                while (cursor[r] < end && col[cursor[r]] < hi) {
                    key.push_back((uint32_t)(2 * r) | ((uint32_t)(col[cursor[r]] - c * kChunkK) << 8));
                    dval.push_back(std::ldexp((double)val[cursor[r]], kEntValScaleLog2));
                    ++cursor[r];
                }
            }
            while (key.size() % 8 != 0) {
                key.push_back(0u);
                dval.push_back(0.0);
            }
            for (size_t b = 0; b < key.size(); b += 8) {
                const size_t at = ent.size();
                ent.resize(at + kEntBlockWords);
                std::memcpy(&ent[at], &key[b], 8 * sizeof(uint32_t));
                std::memcpy(&ent[at + 8], &dval[b], 8 * sizeof(double));
            }
        }
        seg_ptr[(size_t)t * (nchunks + 1) + nchunks] = (int32_t)(ent.size() / kEntBlockWords);
    }
}

// Row lists for the rows-in-lanes kernel (see LayerDev): rows in order of decreasing residual count, so
// that the 64 rows of a block have nearly the same number of steps; a block takes as many steps as its
// longest row, shorter rows are padded with (offset 0, value 0).
void build_row_lists(const std::vector<int32_t>& row_ptr, const std::vector<int32_t>& col, const std::vector<float>& val,
                     std::vector<int32_t>& perm, std::vector<int32_t>& blk, std::vector<uint32_t>& ek,
                     std::vector<double>& ev, std::vector<double>& valsum, int group_rows) {
    // group_rows: rows are sorted by length inside groups of that many consecutive rows (a multiple of 64; every
    // group but the last fills whole blocks), or over the whole layer (0)
    const int N = (int)row_ptr.size() - 1;
    const int nb = (N + kWave - 1) / kWave, Nr = nb * kWave;
    const int G = group_rows > 0 ? group_rows : std::max(N, 1);
    perm.assign(Nr, -1);
    for (int g0 = 0; g0 < N; g0 += G) {
        const int g1 = std::min(N, g0 + G);
        std::iota(perm.begin() + g0, perm.begin() + g1, g0);
        std::stable_sort(perm.begin() + g0, perm.begin() + g1, [&](int a, int b) {
            return row_ptr[a + 1] - row_ptr[a] > row_ptr[b + 1] - row_ptr[b];
        });
    }
    blk.assign(nb + 1, 0);
    for (int b = 0; b < nb; ++b) {
        const int n0 = perm[(size_t)b * kWave];                    // longest row of the block (its first slot is a row)
        blk[b + 1] = blk[b] + (row_ptr[n0 + 1] - row_ptr[n0]);
    }
    ek.assign((size_t)blk[nb] * kWave, 0u);
    ev.assign((size_t)blk[nb] * kWave, 0.0);
    valsum.assign(Nr, 0.0);
    for (int i = 0; i < Nr; ++i) {
        const int n = perm[i];
        if (n < 0) continue;
        const int b = i / kWave, lane = i % kWave;
        double sum = 0.0;
        for (int e = row_ptr[n]; e < row_ptr[n + 1]; ++e) {
            const size_t at = ((size_t)blk[b] + (e - row_ptr[n])) * kWave + lane;
            ek[at] = (uint32_t)col[e] * kRowsRowBytes;
            ev[at] = std::ldexp((double)val[e], kEntValScaleLog2);
            sum += (double)val[e];
        }
        valsum[i] = sum;
    }
}

int compress_impl(const float* W, int N, int K, float delta, float alpha, hipStream_t s, LayerDev& d) {
    d.N = N;
    d.K = K;
    d.Kw = (K + 31) / 32;
    d.waves = 2;                                       // workgroup = 2, 4 or 8 waves of kRowTile rows each
    while (d.waves < kMaxWavesPerBlock && d.waves * kRowTile < N) d.waves *= 2;
    const int rows_per_block = kRowTile * d.waves;
    d.Np = rows_per_block * ((N + rows_per_block - 1) / rows_per_block);
    d.nchunks = (d.Kw + kChunkWords - 1) / kChunkWords;
    int rc;

    if (std::isnan(alpha)) {                          // default scale: mean |w| over the binarized set
        constexpr int kParts = 1024;
        double* part_sum = nullptr;
        long long* part_cnt = nullptr;
        if ((rc = dev_alloc(&part_sum, kParts)) != APB_OK) return rc;
        if ((rc = dev_alloc(&part_cnt, kParts)) != APB_OK) {
            (void)hipFree(part_sum);
            return rc;
        }
        std::vector<double> hs(kParts);
        std::vector<long long> hc(kParts);
        rc = launch_inlier_abs_sum(W, (long long)N * K, delta, part_sum, part_cnt, kParts, s);
        hipError_t e = hipSuccess;
        if (rc == APB_OK) e = hipMemcpyAsync(hs.data(), part_sum, kParts * sizeof(double), hipMemcpyDeviceToHost, s);
        if (rc == APB_OK && e == hipSuccess)
            e = hipMemcpyAsync(hc.data(), part_cnt, kParts * sizeof(long long), hipMemcpyDeviceToHost, s);
        if (rc == APB_OK && e == hipSuccess) e = hipStreamSynchronize(s);
        (void)hipFree(part_sum);
        (void)hipFree(part_cnt);
        if (rc != APB_OK) return rc;
        APB_HIP(e);
        double total = 0.0;
        long long cnt = 0;
        for (int i = 0; i < kParts; ++i) {
            total += hs[i];
            cnt += hc[i];
        }
        alpha = cnt > 0 ? (float)(total / (double)cnt) : 0.0f;
    }
    d.alpha = alpha;

    int32_t* counts = nullptr;
    if ((rc = dev_alloc(&d.sign, (size_t)N * d.Kw)) != APB_OK) return rc;
    if ((rc = dev_alloc(&d.rowsum, (size_t)N)) != APB_OK) return rc;
    if ((rc = dev_alloc(&d.row_ptr, (size_t)N + 1)) != APB_OK) return rc;
    if ((rc = dev_alloc(&d.perm, (size_t)d.Np)) != APB_OK) return rc;
    if ((rc = dev_alloc(&d.signT, (size_t)d.Np * (2 * ((d.Kw + 1) / 2)))) != APB_OK) return rc;
    if ((rc = dev_alloc(&d.signC, (size_t)N * (2 * ((d.Kw + 1) / 2)))) != APB_OK) return rc;
    if ((rc = dev_alloc(&d.chunk_ptr, (size_t)d.Np * (d.nchunks + 1))) != APB_OK) return rc;
    if ((rc = dev_alloc(&d.slot_valsum, (size_t)d.Np)) != APB_OK) return rc;
    if ((rc = dev_alloc(&counts, (size_t)N)) != APB_OK) return rc;

    std::vector<int32_t> hcounts(N);
    rc = launch_sign_pack_count(W, N, K, d.Kw, delta, d.sign, counts, d.rowsum, s);
    hipError_t e = hipSuccess;
    if (rc == APB_OK) e = hipMemcpyAsync(hcounts.data(), counts, (size_t)N * sizeof(int32_t), hipMemcpyDeviceToHost, s);
    if (rc == APB_OK && e == hipSuccess) e = hipStreamSynchronize(s);
    (void)hipFree(counts);
    if (rc != APB_OK) return rc;
    APB_HIP(e);

    std::vector<int32_t> hrow_ptr((size_t)N + 1, 0);
    long long nnz = 0;
    for (int n = 0; n < N; ++n) {
        nnz += hcounts[n];
        hrow_ptr[n + 1] = (int32_t)nnz;
    }
    d.nnz = nnz;
    const std::vector<int32_t> hperm = balanced_slots(hcounts, d.Np);

    if ((rc = dev_alloc(&d.col_idx, (size_t)nnz)) != APB_OK) return rc;
    if ((rc = dev_alloc(&d.val, (size_t)nnz)) != APB_OK) return rc;
    if ((rc = dev_alloc(&d.vald, (size_t)nnz)) != APB_OK) return rc;
    APB_HIP(hipMemcpyAsync(d.row_ptr, hrow_ptr.data(), ((size_t)N + 1) * sizeof(int32_t), hipMemcpyHostToDevice, s));
    APB_HIP(hipMemcpyAsync(d.perm, hperm.data(), (size_t)d.Np * sizeof(int32_t), hipMemcpyHostToDevice, s));
    if (nnz > 0 && (rc = launch_scatter_csr(W, N, K, delta, alpha, d.row_ptr, d.col_idx, d.val, d.vald, s)) != APB_OK) return rc;
    if ((rc = launch_slot_major_signs(d.sign, d.perm, d.Np, d.Kw, 2 * ((d.Kw + 1) / 2), d.signT, s)) != APB_OK) return rc;
    if ((rc = launch_slot_major_signs(d.sign, nullptr, N, d.Kw, 2 * ((d.Kw + 1) / 2), d.signC, s)) != APB_OK) return rc;
    if ((rc = launch_slot_tables(d.perm, d.row_ptr, d.col_idx, d.val, d.Np, d.nchunks, d.chunk_ptr, d.slot_valsum,
                                 s)) != APB_OK)
        return rc;
    // Tile runs for the sparse kernel: built on the host from the CSR just written (offline work).
    std::vector<int32_t> hcol((size_t)nnz);
    std::vector<float> hval((size_t)nnz);
    if (nnz > 0) {
        APB_HIP(hipMemcpyAsync(hcol.data(), d.col_idx, (size_t)nnz * sizeof(int32_t), hipMemcpyDeviceToHost, s));
        APB_HIP(hipMemcpyAsync(hval.data(), d.val, (size_t)nnz * sizeof(float), hipMemcpyDeviceToHost, s));
    }
    APB_HIP(hipStreamSynchronize(s));
    std::vector<int32_t> hseg;
    std::vector<uint32_t> hent;
    build_tile_runs(hperm, hrow_ptr, hcol, hval, d.nchunks, hseg, hent);
    if ((rc = dev_alloc(&d.seg_ptr, hseg.size())) != APB_OK) return rc;
    if ((rc = dev_alloc(&d.ent, hent.size())) != APB_OK) return rc;
    APB_HIP(hipMemcpyAsync(d.seg_ptr, hseg.data(), hseg.size() * sizeof(int32_t), hipMemcpyHostToDevice, s));
    if (!hent.empty())
        APB_HIP(hipMemcpyAsync(d.ent, hent.data(), hent.size() * sizeof(uint32_t), hipMemcpyHostToDevice, s));
    // Row lists for the rows-in-lanes kernel: only where K fits its on-chip code table and rows carry
    // enough residuals for the padding of the lists (to the longest row of each block of 64) to stay small.
    std::vector<int32_t> rperm, rblk;
    // The sign words of a block of 64 slots are stored in the order the matrix tiles take them: the kernel's lane
    // i (of 16) owns slots i, 16 + i, 32 + i, 48 + i of the block -- row i of its four tiles -- and finds their
    // words of one word row side by side, position 4 * i + t: one 16-byte load.
    auto signs_in_tile_order = [&](const std::vector<int32_t>& slot_rows, uint32_t* out) -> int {
        std::vector<int32_t> order(slot_rows.size());
        for (size_t s0 = 0; s0 < slot_rows.size(); s0 += kWave)
            for (int i = 0; i < 16; ++i)
                for (int t = 0; t < 4; ++t) order[s0 + 4 * i + t] = slot_rows[s0 + 16 * t + i];
        int32_t* tmp = nullptr;
        int rc2 = dev_alloc(&tmp, order.size());
        if (rc2 != APB_OK) return rc2;
        hipError_t e = hipMemcpyAsync(tmp, order.data(), order.size() * sizeof(int32_t), hipMemcpyHostToDevice, s);
        if (e == hipSuccess) rc2 = launch_slot_major_signs(d.sign, tmp, d.rows_Nr, d.Kw, d.rows_Kw4, out, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);        // `order` and `tmp` are released below
        (void)hipFree(tmp);
        if (rc2 != APB_OK) return rc2;
        APB_HIP(e);
        return APB_OK;
    };
    std::vector<uint32_t> rek;
    std::vector<double> rev, rvalsum;
    if ((long long)32 * d.Kw * kRowsStageBytesPerK <= kRowsMaxTableBytes && nnz >= (long long)4 * N) {
        build_row_lists(hrow_ptr, hcol, hval, rperm, rblk, rek, rev, rvalsum, 0);
        const long long steps = rblk.back();
        if (steps * kWave <= 2 * nnz) {                   // at most half of the list entries are padding
            d.rows_Nr = (int)rperm.size();
            d.rows_Kw4 = 4 * ((d.Kw + 3) / 4);
            d.rows_steps = steps;
            if ((rc = dev_alloc(&d.rows_perm, rperm.size())) != APB_OK) return rc;
            if ((rc = dev_alloc(&d.rows_blk, rblk.size())) != APB_OK) return rc;
            if ((rc = dev_alloc(&d.rows_ek, rek.size())) != APB_OK) return rc;
            if ((rc = dev_alloc(&d.rows_ev, rev.size())) != APB_OK) return rc;
            if ((rc = dev_alloc(&d.rows_valsum, rvalsum.size())) != APB_OK) return rc;
            if ((rc = dev_alloc(&d.rows_sign, (size_t)d.rows_Kw4 * d.rows_Nr)) != APB_OK) return rc;
            APB_HIP(hipMemcpyAsync(d.rows_perm, rperm.data(), rperm.size() * sizeof(int32_t), hipMemcpyHostToDevice, s));
            APB_HIP(hipMemcpyAsync(d.rows_blk, rblk.data(), rblk.size() * sizeof(int32_t), hipMemcpyHostToDevice, s));
            APB_HIP(hipMemcpyAsync(d.rows_ek, rek.data(), rek.size() * sizeof(uint32_t), hipMemcpyHostToDevice, s));
            APB_HIP(hipMemcpyAsync(d.rows_ev, rev.data(), rev.size() * sizeof(double), hipMemcpyHostToDevice, s));
            APB_HIP(hipMemcpyAsync(d.rows_valsum, rvalsum.data(), rvalsum.size() * sizeof(double), hipMemcpyHostToDevice, s));
            if ((rc = signs_in_tile_order(rperm, d.rows_sign)) != APB_OK) return rc;
            // the word-aligned lists beside them (more than one group of rows; the same padding rule)
            if (N > kRowsGroupRows) {
                APB_HIP(hipStreamSynchronize(s));              // the staging vectors above are reused
                build_row_lists(hrow_ptr, hcol, hval, rperm, rblk, rek, rev, rvalsum, kRowsGroupRows);
                const long long wsteps = rblk.back();
                if (wsteps * kWave <= 2 * nnz) {
                    d.rowsw_steps = wsteps;
                    if ((rc = dev_alloc(&d.rowsw_perm, rperm.size())) != APB_OK) return rc;
                    if ((rc = dev_alloc(&d.rowsw_blk, rblk.size())) != APB_OK) return rc;
                    if ((rc = dev_alloc(&d.rowsw_ek, rek.size())) != APB_OK) return rc;
                    if ((rc = dev_alloc(&d.rowsw_ev, rev.size())) != APB_OK) return rc;
                    if ((rc = dev_alloc(&d.rowsw_valsum, rvalsum.size())) != APB_OK) return rc;
                    if ((rc = dev_alloc(&d.rowsw_sign, (size_t)d.rows_Kw4 * d.rows_Nr)) != APB_OK) return rc;
                    APB_HIP(hipMemcpyAsync(d.rowsw_perm, rperm.data(), rperm.size() * sizeof(int32_t), hipMemcpyHostToDevice, s));
                    APB_HIP(hipMemcpyAsync(d.rowsw_blk, rblk.data(), rblk.size() * sizeof(int32_t), hipMemcpyHostToDevice, s));
                    APB_HIP(hipMemcpyAsync(d.rowsw_ek, rek.data(), rek.size() * sizeof(uint32_t), hipMemcpyHostToDevice, s));
                    APB_HIP(hipMemcpyAsync(d.rowsw_ev, rev.data(), rev.size() * sizeof(double), hipMemcpyHostToDevice, s));
                    APB_HIP(hipMemcpyAsync(d.rowsw_valsum, rvalsum.data(), rvalsum.size() * sizeof(double), hipMemcpyHostToDevice, s));
                    if ((rc = signs_in_tile_order(rperm, d.rowsw_sign)) != APB_OK) return rc;
                }
            }
        }
    }
    APB_HIP(hipStreamSynchronize(s));                 // host staging vectors go out of scope after this
    return APB_OK;
}

int position_bits(long long n) {
    if (n <= 2) return 1;
    int b = 0;
    for (long long v = n - 1; v > 0; v >>= 1) ++b;
    return b;
}

}  // namespace
}  // namespace apb

using namespace apb;

extern "C" {

int apb_compress(const float* W, int N, int K, float delta, float alpha, void* stream, apb_layer** out) {
    if (out) *out = nullptr;
    if (!W || !out) return APB_ERR_NULL;
    if (N <= 0 || K <= 0 || (long long)N * K >= (1LL << 31) || (long long)K * 3 >= (1LL << 31)) return APB_ERR_SHAPE;
    if (std::isnan(delta)) return APB_ERR_VALUE;
    if (!std::isnan(alpha) && (alpha < 0.0f || std::isinf(alpha))) return APB_ERR_VALUE;
    apb_layer* L = new (std::nothrow) apb_layer();
    if (!L) return APB_ERR_NOMEM;
    int rc;
    try {
        rc = compress_impl(W, N, K, delta, alpha, as_stream(stream), L->d);
    } catch (const std::bad_alloc&) {
        rc = APB_ERR_NOMEM;
    }
    if (rc != APB_OK) {
        free_layer_buffers(L->d);
        delete L;
        return rc;
    }
    *out = L;
    return APB_OK;
}

int apb_layer_info(const apb_layer* layer, int* N, int* K, float* alpha, long long* nnz, long long* mem_bits) {
    if (!layer) return APB_ERR_NULL;
    const LayerDev& d = layer->d;
    if (N) *N = d.N;
    if (K) *K = d.K;
    if (alpha) *alpha = d.alpha;
    if (nnz) *nnz = d.nnz;
    if (mem_bits) {
        const long long n = (long long)d.N * d.K;
        *mem_bits = n + d.nnz * (32 + position_bits(n));
    }
    return APB_OK;
}

int apb_layer_export(const apb_layer* layer, uint32_t* sign_words, int32_t* row_ptr, int32_t* col_idx, float* val,
                     int32_t* rowsum, void* stream) {
    if (!layer) return APB_ERR_NULL;
    const LayerDev& d = layer->d;
    hipStream_t s = as_stream(stream);
    if (sign_words)
        APB_HIP(hipMemcpyAsync(sign_words, d.sign, (size_t)d.N * d.Kw * sizeof(uint32_t), hipMemcpyDefault, s));
    if (row_ptr) APB_HIP(hipMemcpyAsync(row_ptr, d.row_ptr, ((size_t)d.N + 1) * sizeof(int32_t), hipMemcpyDefault, s));
    if (col_idx && d.nnz > 0)
        APB_HIP(hipMemcpyAsync(col_idx, d.col_idx, (size_t)d.nnz * sizeof(int32_t), hipMemcpyDefault, s));
    if (val && d.nnz > 0) APB_HIP(hipMemcpyAsync(val, d.val, (size_t)d.nnz * sizeof(float), hipMemcpyDefault, s));
    if (rowsum) APB_HIP(hipMemcpyAsync(rowsum, d.rowsum, (size_t)d.N * sizeof(int32_t), hipMemcpyDefault, s));
    APB_HIP(hipStreamSynchronize(s));
    return APB_OK;
}

void apb_layer_free(apb_layer* layer) {
    if (!layer) return;
    free_layer_buffers(layer->d);
    delete layer;
}

size_t apb_acts_bytes(int K, int M, int bits) {
    if (bad_shape_acts(K, M) || (bits != 1 && bits != 2)) return 0;
    const size_t Kw = ((size_t)K + 31) / 32;
    const size_t Mp = (size_t)kWave * (((size_t)M + kWave - 1) / kWave);
    return sizeof(uint32_t) * Mp * ((size_t)bits * Kw + 1);
}

int apb_quantize_acts(const float* X, int K, int M, int bits, float step, void* packed, void* stream) {
    if (!X || !packed) return APB_ERR_NULL;
    if (bad_shape_acts(K, M)) return APB_ERR_SHAPE;
    if (bits != 1 && bits != 2) return APB_ERR_BITS;
    if (!std::isfinite(step) || !(step > 0.0f)) return APB_ERR_VALUE;
    const size_t Kw = ((size_t)K + 31) / 32;
    const size_t Mp = (size_t)kWave * (((size_t)M + kWave - 1) / kWave);
    uint32_t* planes = static_cast<uint32_t*>(packed);
    int32_t* colsum = reinterpret_cast<int32_t*>(planes + (size_t)bits * Kw * Mp);
    const float inv_step = 1.0f / step;
    return launch_quantize(X, K, M, bits, inv_step, planes, colsum, as_stream(stream));
}

enum FwdKind { kFwdFull, kFwdFullPopcount, kFwdIntPopcount, kFwdIntMfma };

static int forward_common(const apb_layer* layer, const void* packed, int M, int bits, float step, float* Y,
                          int32_t* D, void* stream, FwdKind kind) {
    if (!layer || !packed || (!Y && !D)) return APB_ERR_NULL;
    const LayerDev& d = layer->d;
    if (bad_shape_acts(d.K, M) || (long long)d.N * M >= (1LL << 40)) return APB_ERR_SHAPE;
    if (bits != 1 && bits != 2) return APB_ERR_BITS;
    if (Y && (!std::isfinite(step) || !(step > 0.0f))) return APB_ERR_VALUE;
    const size_t Mp = (size_t)kWave * (((size_t)M + kWave - 1) / kWave);
    const uint32_t* planes = static_cast<const uint32_t*>(packed);
    const int32_t* colsum = reinterpret_cast<const int32_t*>(planes + (size_t)bits * d.Kw * Mp);
    hipStream_t s = as_stream(stream);
    if (kind == kFwdIntMfma) {
        return launch_binary_mfma(d, planes, colsum, M, bits, D, s);
    }
    if (kind == kFwdFull) {
        return launch_forward_best(d, planes, colsum, M, bits, step, Y, s);
    }
    return launch_forward_popcount(d, planes, colsum, M, bits, step, Y, D, s);
}

int apb_forward(const apb_layer* layer, const void* packed, int M, int bits, float step, float* Y, void* stream) {
    if (!Y) return APB_ERR_NULL;
    return forward_common(layer, packed, M, bits, step, Y, nullptr, stream, kFwdFull);
}

int apb_forward_requant(const apb_layer* layer, const void* packed, int M, int bits, float step, const float* scale,
                        const float* shift, int bits_out, float step_out, void* packed_out, void* stream) {
    if (!layer || !packed || !packed_out || (scale == nullptr) != (shift == nullptr)) return APB_ERR_NULL;
    const LayerDev& d = layer->d;
    if (bad_shape_acts(d.K, M) || bad_shape_acts(d.N, M) || (long long)d.N * M >= (1LL << 40)) return APB_ERR_SHAPE;
    if ((bits != 1 && bits != 2) || (bits_out != 1 && bits_out != 2)) return APB_ERR_BITS;
    if (!std::isfinite(step) || !(step > 0.0f) || !std::isfinite(step_out) || !(step_out > 0.0f)) return APB_ERR_VALUE;
    const size_t Mp = (size_t)kWave * (((size_t)M + kWave - 1) / kWave);
    const uint32_t* planes = static_cast<const uint32_t*>(packed);
    const int32_t* colsum = reinterpret_cast<const int32_t*>(planes + (size_t)bits * d.Kw * Mp);
    hipStream_t s = as_stream(stream);
    uint32_t* out = static_cast<uint32_t*>(packed_out);
    return launch_forward_requant(d, planes, colsum, M, bits, step, nullptr, scale, shift, bits_out, 1.0f / step_out, out, s);
}

const char* apb_forward_kernel_name(const apb_layer* layer, int M, int bits) {
    if (!layer || M <= 0 || (bits != 1 && bits != 2)) return "";
    if (forward_rows_applies(layer->d, M, bits)) return forward_rows_kernel_name(layer->d, M, bits);
    return forward_kernel_name(layer->d, M, bits);
}

int apb_quantize_forward_is_one_kernel(const apb_layer* layer, int M, int bits) {
    if (!layer || M <= 0 || (bits != 1 && bits != 2)) return 0;
    return forward_float_applies(layer->d, M, bits) ? 1 : 0;
}

int apb_quantize_forward(const apb_layer* layer, const float* X, int M, int bits, float step, void* packed, float* Y,
                         void* stream) {
    if (!layer || !X || !packed || !Y) return APB_ERR_NULL;
    const LayerDev& d = layer->d;
    if (bad_shape_acts(d.K, M) || (long long)d.N * M >= (1LL << 40)) return APB_ERR_SHAPE;
    if (bits != 1 && bits != 2) return APB_ERR_BITS;
    if (!std::isfinite(step) || !(step > 0.0f)) return APB_ERR_VALUE;
    hipStream_t s = as_stream(stream);
    if (forward_float_applies(d, M, bits)) return launch_forward_float(d, X, M, bits, step, Y, s);
    uint32_t* planes = static_cast<uint32_t*>(packed);
    int32_t* colsum = reinterpret_cast<int32_t*>(planes + (size_t)bits * d.Kw * ((size_t)kWave * (((size_t)M + kWave - 1) / kWave)));
    return launch_quantize_then_forward(d, X, M, bits, step, planes, colsum, Y, s);
}

// Shape checks shared by the two convolution entry points; fills `conv` and the output pixel count.
static int conv_shape(const LayerDev& d, int B, int H, int W, int stride, ConvShape& conv, int& P_out) {
    if (B <= 0 || H <= 0 || W <= 0 || (stride != 1 && stride != 2)) return APB_ERR_SHAPE;
    if (d.K % 9 != 0 || (d.K / 9) % 32 != 0) return APB_ERR_SHAPE;
    if (d.K / 9 > 16384) return APB_ERR_SHAPE;                 // the kernels' row -> tap arithmetic is exact up to here
    const long long pixels = (long long)B * H * W;
    if (pixels >= (1LL << 28)) return APB_ERR_SHAPE;
    const long long Pp_in = kWave * ((pixels + kWave - 1) / kWave);
    // a plane of the map is one buffer range of the kernels' loads: below 2^31 bytes
    if ((long long)(d.K / 9 / 32) * Pp_in * 4 >= (1LL << 31)) return APB_ERR_SHAPE;
    const int Ho = (H - 1) / stride + 1, Wo = (W - 1) / stride + 1;
    const long long out_pixels = (long long)B * Ho * Wo;
    if ((long long)d.N * out_pixels >= (1LL << 40)) return APB_ERR_SHAPE;
    conv = ConvShape{d.K / 9, H, W, stride, Ho, Wo, (int)Pp_in};
    P_out = (int)out_pixels;
    return APB_OK;
}

// With a workspace, layers on which the rows-in-lanes kernel applies write the packed patch matrix there first and
// run the plain-matrix kernels on it; `patches` is null otherwise.
static int conv_patches(const LayerDev& d, const uint32_t* planes, const int32_t* pixsum, int P, int bits,
                        const ConvShape& conv, void* workspace, size_t workspace_bytes, uint32_t* clear, size_t clear_words,
                        hipStream_t s, const uint32_t** patches, const int32_t** colsum) {
    *patches = nullptr;
    *colsum = nullptr;
    const size_t Pp = (size_t)kWave * (((size_t)P + kWave - 1) / kWave);
    const size_t need = sizeof(uint32_t) * Pp * ((size_t)bits * d.Kw + 1);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 15u) != 0) return APB_OK;
    if (!forward_rows_applies(d, P, bits)) return APB_OK;
    uint32_t* out = static_cast<uint32_t*>(workspace);
    const int rc = launch_pack_patches(d, planes, pixsum, P, bits, conv, out, clear, clear_words, s);
    if (rc != APB_OK) return rc;
    *patches = out;
    *colsum = reinterpret_cast<const int32_t*>(out + (size_t)bits * d.Kw * Pp);
    return APB_OK;
}

int apb_forward_conv3x3(const apb_layer* layer, const void* fmap, int B, int H, int W, int stride, int bits, float step,
                        void* workspace, size_t workspace_bytes, float* Y, void* stream) {
    if (!layer || !fmap || !Y) return APB_ERR_NULL;
    const LayerDev& d = layer->d;
    ConvShape conv;
    int P;
    int rc = conv_shape(d, B, H, W, stride, conv, P);
    if (rc != APB_OK) return rc;
    if (bits != 1 && bits != 2) return APB_ERR_BITS;
    if (!std::isfinite(step) || !(step > 0.0f)) return APB_ERR_VALUE;
    hipStream_t s = as_stream(stream);
    const uint32_t* planes = static_cast<const uint32_t*>(fmap);
    const int32_t* pixsum = reinterpret_cast<const int32_t*>(planes + (size_t)bits * (conv.C / 32) * conv.Pp_in);
    const uint32_t* patches;
    const int32_t* colsum;
    if ((rc = conv_patches(d, planes, pixsum, P, bits, conv, workspace, workspace_bytes, nullptr, 0, s, &patches, &colsum)) != APB_OK)
        return rc;
    if (patches) return launch_forward_best(d, patches, colsum, P, bits, step, Y, s);
    return launch_forward(d, planes, pixsum, P, bits, step, &conv, Y, s);
}

int apb_forward_conv3x3_requant(const apb_layer* layer, const void* fmap, int B, int H, int W, int stride, int bits,
                                float step, const float* scale, const float* shift, int bits_out, float step_out,
                                void* workspace, size_t workspace_bytes, void* fmap_out, void* stream) {
    if (!layer || !fmap || !fmap_out || (scale == nullptr) != (shift == nullptr)) return APB_ERR_NULL;
    const LayerDev& d = layer->d;
    ConvShape conv;
    int P;
    int rc = conv_shape(d, B, H, W, stride, conv, P);
    if (rc != APB_OK) return rc;
    if ((bits != 1 && bits != 2) || (bits_out != 1 && bits_out != 2)) return APB_ERR_BITS;
    if (!std::isfinite(step) || !(step > 0.0f) || !std::isfinite(step_out) || !(step_out > 0.0f)) return APB_ERR_VALUE;
    const uint32_t* planes = static_cast<const uint32_t*>(fmap);
    const int32_t* pixsum = reinterpret_cast<const int32_t*>(planes + (size_t)bits * (conv.C / 32) * conv.Pp_in);
    hipStream_t s = as_stream(stream);
    uint32_t* out = static_cast<uint32_t*>(fmap_out);
    const uint32_t* patches;
    const int32_t* colsum;
    // (the kernel that follows the packed patch matrix ORs its bits into the output: cleared by the same launch)
    const size_t Pp = (size_t)kWave * (((size_t)P + kWave - 1) / kWave);
    const size_t out_words = ((size_t)bits_out * ((d.N + 31) / 32) + 1) * Pp;
    if ((rc = conv_patches(d, planes, pixsum, P, bits, conv, workspace, workspace_bytes, out, out_words, s, &patches, &colsum)) != APB_OK)
        return rc;
    if (patches)
        return launch_forward_requant(d, patches, colsum, P, bits, step, nullptr, scale, shift, bits_out, 1.0f / step_out, out, s,
                                      true);
    return launch_forward_requant(d, planes, pixsum, P, bits, step, &conv, scale, shift, bits_out, 1.0f / step_out, out, s);
}

int apb_forward_popcount(const apb_layer* layer, const void* packed, int M, int bits, float step, float* Y,
                         void* stream) {
    if (!Y) return APB_ERR_NULL;
    return forward_common(layer, packed, M, bits, step, Y, nullptr, stream, kFwdFullPopcount);
}

int apb_forward_int(const apb_layer* layer, const void* packed, int M, int bits, int32_t* D, void* stream) {
    if (!D) return APB_ERR_NULL;
    return forward_common(layer, packed, M, bits, 1.0f, nullptr, D, stream, kFwdIntMfma);
}

int apb_forward_int_popcount(const apb_layer* layer, const void* packed, int M, int bits, int32_t* D, void* stream) {
    if (!D) return APB_ERR_NULL;
    return forward_common(layer, packed, M, bits, 1.0f, nullptr, D, stream, kFwdIntPopcount);
}

int apb_w2_pack(const float* W, int N, int K, float step_w, void* stream, apb_w2** out) {
    if (out) *out = nullptr;
    if (!W || !out) return APB_ERR_NULL;
    if (N <= 0 || K <= 0 || (long long)N * K >= (1LL << 31) || (long long)K * 3 >= (1LL << 31)) return APB_ERR_SHAPE;
    if (!std::isfinite(step_w) || !(step_w > 0.0f)) return APB_ERR_VALUE;
    apb_w2* w = new (std::nothrow) apb_w2();
    if (!w) return APB_ERR_NOMEM;
    w->N = N;
    w->K = K;
    w->Kw = (K + 31) / 32;
    w->step_w = step_w;
    const size_t Kw2 = 2 * (((size_t)w->Kw + 1) / 2);
    int rc = dev_alloc(&w->planes, (size_t)2 * N * w->Kw);
    if (rc == APB_OK) rc = dev_alloc(&w->planesC, (size_t)2 * Kw2 * N);
    if (rc == APB_OK) rc = launch_w2_pack(W, N, K, 1.0f / step_w, w->planes, w->planesC, as_stream(stream));
    if (rc != APB_OK) {
        apb_w2_free(w);
        return rc;
    }
    *out = w;
    return APB_OK;
}

int apb_w2_export(const apb_w2* w2, uint32_t* planes, void* stream) {
    if (!w2 || !planes) return APB_ERR_NULL;
    hipStream_t s = as_stream(stream);
    APB_HIP(hipMemcpyAsync(planes, w2->planes, (size_t)2 * w2->N * w2->Kw * sizeof(uint32_t), hipMemcpyDefault, s));
    APB_HIP(hipStreamSynchronize(s));
    return APB_OK;
}

void apb_w2_free(apb_w2* w2) {
    if (!w2) return;
    if (w2->planes) (void)hipFree(w2->planes);
    if (w2->planesC) (void)hipFree(w2->planesC);
    delete w2;
}

static int gemm_2_2_common(const apb_w2* w2, const void* packed, int M, float step_a, int32_t* D, float* Y,
                           void* stream) {
    if (!w2 || !packed || (!D && !Y)) return APB_ERR_NULL;
    if (bad_shape_acts(w2->K, M) || (long long)w2->N * M >= (1LL << 40)) return APB_ERR_SHAPE;
    if (Y && (!std::isfinite(step_a) || !(step_a > 0.0f))) return APB_ERR_VALUE;
    const size_t Mp = (size_t)kWave * (((size_t)M + kWave - 1) / kWave);
    const uint32_t* planes = static_cast<const uint32_t*>(packed);
    const int32_t* colsum = reinterpret_cast<const int32_t*>(planes + (size_t)2 * w2->Kw * Mp);
    const double scale = 0.5 * (double)w2->step_w * (double)step_a;
    return launch_gemm_2_2(w2->planesC, w2->N, w2->Kw, planes, colsum, M, scale, D, Y, as_stream(stream));
}

int apb_gemm_2_2_int(const apb_w2* w2, const void* packed, int M, int32_t* D, void* stream) {
    if (!D) return APB_ERR_NULL;
    return gemm_2_2_common(w2, packed, M, 1.0f, D, nullptr, stream);
}

int apb_gemm_2_2(const apb_w2* w2, const void* packed, int M, float step_a, float* Y, void* stream) {
    if (!Y) return APB_ERR_NULL;
    return gemm_2_2_common(w2, packed, M, step_a, nullptr, Y, stream);
}

const char* apb_strerror(int code) {
    switch (code) {
        case APB_OK: return "ok";
        case APB_ERR_NULL: return "a required pointer is NULL";
        case APB_ERR_SHAPE: return "bad shape (non-positive or too large)";
        case APB_ERR_BITS: return "activation bits must be 1 or 2";
        case APB_ERR_VALUE: return "bad scalar (delta NaN, alpha negative/infinite, or step not finite and > 0)";
        case APB_ERR_NOMEM: return "out of memory";
        case APB_ERR_HIP: return "a HIP call failed (see apb_last_hip_error)";
        case APB_ERR_SCRATCH: return "the packed activations of this K, M and bits do not fit the library's static scratch array";
        default: return "unknown apb status";
    }
}

int apb_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
