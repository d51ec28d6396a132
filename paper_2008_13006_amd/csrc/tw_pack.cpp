// Host-side packer for the tile-wise (TW) format: tiling analysis, compaction, schedule.
// Paper: Sec. IV-A (pattern, column pruning first, re-grouping), Sec. VI "Tiling" (pruned rows and
// columns of B are removed offline; per-tile mask vectors tell the kernel what to skip) and
// "Load Imbalance Mitigation" (tiles differ in work; here they are ordered by kept rows).
#include "../../include/tw.h"
#include "tw_format.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>
#include <vector>

namespace {

struct Tiling {
    std::vector<int32_t> col_idx;
    std::vector<int32_t> tile_col_ptr;  // T+1
    std::vector<int32_t> tile_row_ptr;  // T+1
    std::vector<int32_t> row_idx;
    std::vector<int32_t> tile_span;     // T+1
    int T = 0;
    int64_t nnz = 0;
};

struct Layout {
    int k_chunk = 0, n_chunks = 0, ncb = 0;
    std::vector<int32_t> step_ptr;    // [T][n_chunks+1], tile-local step numbers
    std::vector<int32_t> first_step;  // [T] global step index
    int64_t total_steps = 0;
    uint64_t off_col_idx, off_tile_col_ptr, off_tile_row_ptr, off_row_idx, off_tile_span,
        off_sched_order, off_tile_desc, off_step_ptr, off_goff, off_dpos, off_bvals, off_sched_desc, off_zero_ptr,
        off_zero_cols, off_zero_xc, off_urow, off_ucnt, off_ew_ptr, off_ew_goff, off_ew_b, off_ew_mask, off_xm_ptr, off_xm_goff, off_xm_b, off_xc_col, off_xc_ptr, off_xc_k, off_xc_v, off_xc_tile_ptr, off_xc_rank, bytes;
    int64_t ew_nnz = 0;
    std::vector<int32_t> ew_ptr;   // residual steps per (tile, chunk), prefix sums
    // residual weights in columns without tile-wise weights, by column
    std::vector<int32_t> xc_col, xc_ptr, xc_k, xc_tile_ptr, xc_rank;
    std::vector<int32_t> xm_ptr;   // K resident: steps of every tile's first TW_XC_INLINE such columns, prefix sums
    int32_t xc_overflow = 0;
};

inline uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

bool supported_g(int G) { return G == 32 || G == 64 || G == 128; }

// Sweep of the surviving columns (see tw.h, tw_pack_size).
int analyse(const uint8_t* mask, int K, int N, int G, Tiling& tl) {
    std::vector<uint8_t> alive(N, 0);
    for (int k = 0; k < K; ++k) {
        const uint8_t* r = mask + (size_t)k * N;
        for (int n = 0; n < N; ++n) alive[n] |= (r[n] != 0);
    }
    for (int n = 0; n < N; ++n)
        if (alive[n]) tl.col_idx.push_back(n);
    const int nk = (int)tl.col_idx.size();
    const int max_tiles = 2 * ((N + G - 1) / G);
    std::vector<uint8_t> pat(K), cur(K);
    tl.tile_col_ptr.push_back(0);
    tl.tile_row_ptr.push_back(0);
    int i = 0;
    while (i < nk) {
        const int c0 = tl.col_idx[i];
        for (int k = 0; k < K; ++k) pat[k] = mask[(size_t)k * N + c0] != 0;
        int j = i + 1;
        while (j < nk && j - i < G) {
            const int c = tl.col_idx[j];
            bool same = true;
            for (int k = 0; k < K; ++k)
                if ((mask[(size_t)k * N + c] != 0) != (pat[k] != 0)) { same = false; break; }
            if (!same) break;
            ++j;
        }
        for (int k = 0; k < K; ++k)
            if (pat[k]) tl.row_idx.push_back(k);
        tl.tile_col_ptr.push_back(j);
        tl.tile_row_ptr.push_back((int32_t)tl.row_idx.size());
        if ((int)tl.tile_col_ptr.size() - 1 > max_tiles) return TW_ERR_NOT_TILEWISE;
        i = j;
    }
    tl.T = (int)tl.tile_col_ptr.size() - 1;
    tl.tile_span.assign(tl.T + 1, 0);
    for (int t = 1; t < tl.T; ++t) tl.tile_span[t] = tl.col_idx[tl.tile_col_ptr[t]];
    tl.tile_span[tl.T] = tl.T > 0 ? N : 0;
    tl.nnz = 0;
    for (int t = 0; t < tl.T; ++t)
        tl.nnz += (int64_t)(tl.tile_col_ptr[t + 1] - tl.tile_col_ptr[t]) *
                  (tl.tile_row_ptr[t + 1] - tl.tile_row_ptr[t]);
    return TW_OK;
}

// K rows of [k0, k1) in which one of the packed columns [c_lo, c_hi) of the tiling has a residual weight (kept by
// `ew`, not by the tile-wise mask), ascending; returns the number of such weights.
int64_t residual_rows(const Tiling& tl, const uint8_t* mask, const uint8_t* ew, int N, int c_lo, int c_hi, int k0,
                      int k1, std::vector<int32_t>& rows) {
    rows.clear();
    int64_t cnt = 0;
    for (int k = k0; k < k1; ++k) {
        int here = 0;
        for (int c = c_lo; c < c_hi; ++c) {
            const size_t i = (size_t)k * N + tl.col_idx[c];
            here += ew[i] != 0 && mask[i] == 0;
        }
        if (here) rows.push_back(k);
        cnt += here;
    }
    return cnt;
}

// Order of a column block's residual rows inside its steps.  A transposing LDS read of the kernel serves four
// contraction slots (4*i .. 4*i+3 of a step) per 32 lanes, 64 bytes of each row; rows of the LDS copy of A are
// 8 bytes more than a multiple of 128 bytes apart, so the four pieces cover the 64 banks once exactly when the four
// K rows agree modulo 8 and differ in (k / 8) modulo 4.  Rows are dealt out in such fours as far as they go; the
// rest follows in ascending order.  `base` is the first row of the chunk (LDS rows are chunk-local).
void order_residual_rows(std::vector<int32_t>& rows, int base) {
    std::vector<int32_t> bucket[32], out, rest;
    for (int32_t k : rows) bucket[(k - base) & 31].push_back(k);
    for (int c = 0; c < 8; ++c) {
        size_t n = rows.size();
        for (int i = 0; i < 4; ++i) n = std::min(n, bucket[c + 8 * i].size());
        for (size_t j = 0; j < n; ++j)
            for (int i = 0; i < 4; ++i) out.push_back(bucket[c + 8 * i][j]);
        for (int i = 0; i < 4; ++i) rest.insert(rest.end(), bucket[c + 8 * i].begin() + n, bucket[c + 8 * i].end());
    }
    std::sort(rest.begin(), rest.end());
    out.insert(out.end(), rest.begin(), rest.end());
    rows.swap(out);
}

// K rows of [k0, k1) in which one of the first TW_XC_INLINE residual-only columns of tile t has a weight, in the
// order of order_residual_rows.
void inline_xc_rows(const Layout& lo, int t, int k0, int k1, std::vector<int32_t>& rows) {
    rows.clear();
    const int x0 = lo.xc_tile_ptr[t], x1 = std::min(lo.xc_tile_ptr[t + 1], x0 + TW_XC_INLINE);
    for (int j = x0; j < x1; ++j)
        for (int32_t q = lo.xc_ptr[j]; q < lo.xc_ptr[j + 1]; ++q)
            if (lo.xc_k[q] >= k0 && lo.xc_k[q] < k1) rows.push_back(lo.xc_k[q]);
    std::sort(rows.begin(), rows.end());
    rows.erase(std::unique(rows.begin(), rows.end()), rows.end());
    order_residual_rows(rows, k0);
}

void plan(const Tiling& tl, int K, int G, Layout& lo, const uint8_t* mask = nullptr, const uint8_t* ew = nullptr, int N = 0) {
    const int T = tl.T;
    if (K <= TW_K_RESIDENT_MAX) {
        lo.k_chunk = (K + 7) / 8 * 8;
        lo.n_chunks = 1;
    } else {
        lo.k_chunk = TW_K_STREAM_CHUNK;
        lo.n_chunks = (K + lo.k_chunk - 1) / lo.k_chunk;
    }
    lo.ncb = G / TW_COLBLK;
    lo.step_ptr.assign((size_t)T * (lo.n_chunks + 1), 0);
    lo.first_step.assign(T, 0);
    int64_t total = 0;
    for (int t = 0; t < T; ++t) {
        lo.first_step[t] = (int32_t)total;
        int32_t* sp = &lo.step_ptr[(size_t)t * (lo.n_chunks + 1)];
        const int32_t* r = tl.row_idx.data() + tl.tile_row_ptr[t];
        const int kt = tl.tile_row_ptr[t + 1] - tl.tile_row_ptr[t];
        int p = 0, steps = 0;
        for (int c = 0; c < lo.n_chunks; ++c) {
            sp[c] = steps;
            int cnt = 0;
            const int hi = (c + 1) * lo.k_chunk;
            while (p < kt && r[p] < hi) { ++p; ++cnt; }
            steps += (cnt + TW_KSTEP - 1) / TW_KSTEP;
        }
        sp[lo.n_chunks] = steps;
        total += steps;
    }
    lo.total_steps = total;
    uint64_t o = sizeof(TwHeader);
    auto take = [&](uint64_t bytes, uint64_t al) { o = align_up(o, al); uint64_t r = o; o += bytes; return r; };
    const size_t nk = tl.col_idx.size();
    lo.off_col_idx = take(4 * nk, 16);
    lo.off_tile_col_ptr = take(4 * (size_t)(T + 1), 16);
    lo.off_tile_row_ptr = take(4 * (size_t)(T + 1), 16);
    lo.off_row_idx = take(4 * tl.row_idx.size(), 16);
    lo.off_tile_span = take(4 * (size_t)(T + 1), 16);
    lo.off_sched_order = take(4 * (size_t)T, 16);
    lo.off_tile_desc = take(sizeof(TwTileDesc) * (size_t)T, 64);
    lo.off_sched_desc = take(sizeof(TwSchedDesc) * (size_t)T, 64);
    lo.off_step_ptr = take(4 * lo.step_ptr.size(), 16);
    {
        size_t n_zero = 0;   // pruned columns inside spans = N - kept columns (every column lies in one span)
        if (T > 0) n_zero = (size_t)tl.tile_span[T] - tl.col_idx.size();
        lo.off_zero_ptr = take(4 * (size_t)(T + 1), 16);
        lo.off_zero_cols = take(4 * (n_zero + 1), 16);
        lo.off_zero_xc = take(n_zero + 1, 16);
    }
    {
        const size_t n_sets = lo.n_chunks > 1 && T > 0 ? (size_t)(T + TW_SET_TILES(T) - 1) / TW_SET_TILES(T) : 0;
        lo.off_ucnt = take(4 * (n_sets * lo.n_chunks + 1), 16);
        lo.off_urow = take(2 * (n_sets * lo.n_chunks * (size_t)lo.k_chunk + 1), 16);
    }
    {
        // residual steps per (tile, chunk): what the column block with the most residual rows in the chunk needs
        const int nc = lo.n_chunks;
        lo.ew_ptr.assign((size_t)T * nc + 1, 0);
        lo.ew_nnz = 0;
        if (ew) {
            std::vector<int32_t> rows;
            for (int t = 0; t < T; ++t)
                for (int ch = 0; ch < nc; ++ch) {
                    const int k0 = ch * lo.k_chunk, k1 = std::min(K, k0 + lo.k_chunk);
                    int smax = 0;
                    for (int c = tl.tile_col_ptr[t]; c < tl.tile_col_ptr[t + 1]; c += TW_COLBLK) {
                        lo.ew_nnz += residual_rows(tl, mask, ew, N, c, std::min(c + TW_COLBLK, tl.tile_col_ptr[t + 1]), k0, k1, rows);
                        smax = std::max(smax, ((int)rows.size() + TW_KSTEP - 1) / TW_KSTEP);
                    }
                    lo.ew_ptr[(size_t)t * nc + ch + 1] = lo.ew_ptr[(size_t)t * nc + ch] + smax;
                }
        }
        const size_t rsteps = (size_t)lo.ew_ptr[(size_t)T * nc];
        lo.off_ew_ptr = take(4 * ((size_t)T * nc + 1), 16);
        lo.off_ew_goff = take(2 * 16 * (rsteps * lo.ncb + 1), 256);
        lo.off_ew_b = take(2 * 512 * (rsteps * lo.ncb) + 16, 256);
        lo.off_ew_mask = take(4 * 16 * (rsteps * lo.ncb) + 16, 16);
        // residual weights in columns that keep no tile-wise weight
        lo.xc_ptr.assign(1, 0);
        if (ew) {
            std::vector<uint8_t> alive(N, 0);
            for (int32_t n : tl.col_idx) alive[n] = 1;
            for (int n = 0; n < N; ++n) {
                if (alive[n]) continue;
                const size_t before = lo.xc_k.size();
                for (int k = 0; k < K; ++k)
                    if (ew[(size_t)k * N + n] != 0) lo.xc_k.push_back(k);
                if (lo.xc_k.size() != before) {
                    lo.xc_col.push_back(n);
                    lo.xc_ptr.push_back((int32_t)lo.xc_k.size());
                }
            }
            lo.ew_nnz += (int64_t)lo.xc_k.size();
        }
        // which tile's span holds each of these columns, and its position among that tile's
        lo.xc_tile_ptr.assign((size_t)T + 1, 0);
        lo.xc_rank.assign(lo.xc_col.size(), 0);
        {
            size_t j = 0;
            for (int t = 0; t < T; ++t) {
                lo.xc_tile_ptr[t] = (int32_t)j;
                while (j < lo.xc_col.size() && lo.xc_col[j] < tl.tile_span[t + 1]) {
                    lo.xc_rank[j] = (int32_t)j - lo.xc_tile_ptr[t];
                    if (lo.xc_rank[j] >= TW_XC_INLINE) ++lo.xc_overflow;
                    ++j;
                }
            }
            lo.xc_tile_ptr[T] = (int32_t)j;
            if (T == 0) lo.xc_overflow = (int32_t)lo.xc_col.size();
        }
        lo.xm_ptr.assign((size_t)T * lo.n_chunks + 1, 0);
        {
            std::vector<int32_t> rows;
            for (int t = 0; t < T; ++t)
                for (int ch = 0; ch < lo.n_chunks; ++ch) {
                    inline_xc_rows(lo, t, ch * lo.k_chunk, std::min(K, (ch + 1) * lo.k_chunk), rows);
                    const size_t i = (size_t)t * lo.n_chunks + ch;
                    lo.xm_ptr[i + 1] = lo.xm_ptr[i] + ((int32_t)rows.size() + TW_KSTEP - 1) / TW_KSTEP;
                }
        }
        lo.off_xm_ptr = take(4 * lo.xm_ptr.size(), 16);
        lo.off_xm_goff = take(2 * 16 * ((size_t)lo.xm_ptr.back() + 1), 256);
        lo.off_xm_b = take(2 * 512 * (size_t)lo.xm_ptr.back() + 16, 256);
        lo.off_xc_tile_ptr = take(4 * ((size_t)T + 1), 16);
        lo.off_xc_rank = take(4 * (lo.xc_rank.size() + 1), 16);
        lo.off_xc_col = take(4 * (lo.xc_col.size() + 1), 16);
        lo.off_xc_ptr = take(4 * lo.xc_ptr.size(), 16);
        lo.off_xc_k = take(4 * (lo.xc_k.size() + 1), 16);
        lo.off_xc_v = take(2 * (lo.xc_k.size() + 1), 16);
    }
    lo.off_goff = take(2 * 16 * (uint64_t)total, 256);
    lo.off_dpos = take(4 * (uint64_t)T * 32 * lo.ncb, 256);
    lo.off_bvals = take(2 * (uint64_t)total * lo.ncb * 64 * 8, 256);
    lo.bytes = align_up(o, 256);
}

int check_common(const uint8_t* mask, int K, int N, int G, int dt) {
    if (!mask || K <= 0 || N <= 0) return TW_ERR_ARG;
    if (dt != TW_F16 && dt != TW_BF16) return TW_ERR_ARG;
    if (G <= 0) return TW_ERR_ARG;
    if (!supported_g(G)) return TW_ERR_UNSUPPORTED;
    return TW_OK;
}

const TwHeader* header_of(const void* blob) {
    if (!blob) return nullptr;
    const TwHeader* h = (const TwHeader*)blob;
    if (h->magic != TW_MAGIC || h->version != TW_FORMAT_VERSION) return nullptr;
    return h;
}

}  // namespace

extern "C" int tw_pack_size(const uint8_t* mask, int K, int N, int G, tw_dtype dt, size_t* blob_bytes) {
    return tw_pack_tew_size(mask, nullptr, K, N, G, dt, blob_bytes);
}

extern "C" int tw_pack_tew_size(const uint8_t* mask, const uint8_t* ew_mask, int K, int N, int G, tw_dtype dt,
                                size_t* blob_bytes) {
    if (!blob_bytes) return TW_ERR_ARG;
    int rc = check_common(mask, K, N, G, (int)dt);
    if (rc) return rc;
    Tiling tl;
    rc = analyse(mask, K, N, G, tl);
    if (rc) return rc;
    Layout lo;
    plan(tl, K, G, lo, mask, ew_mask, N);
    if (lo.xc_col.size() >= (1u << 26)) return TW_ERR_UNSUPPORTED;   // TwSchedDesc::xc holds 26 bits of the list position
    *blob_bytes = (size_t)lo.bytes;
    return TW_OK;
}

extern "C" int tw_pack(const void* B, int ldb, const uint8_t* mask, int K, int N, int G, tw_dtype dt,
                       void* blob, size_t blob_bytes) {
    return tw_pack_tew(B, ldb, mask, nullptr, K, N, G, dt, blob, blob_bytes);
}

extern "C" int tw_pack_tew(const void* B, int ldb, const uint8_t* mask, const uint8_t* ew_mask, int K, int N, int G,
                           tw_dtype dt, void* blob, size_t blob_bytes) {
    if (!B || !blob) return TW_ERR_ARG;
    int rc = check_common(mask, K, N, G, (int)dt);
    if (rc) return rc;
    if (ldb < N) return TW_ERR_ARG;
    if (((uintptr_t)blob & 15) != 0) return TW_ERR_ALIGN;
    Tiling tl;
    rc = analyse(mask, K, N, G, tl);
    if (rc) return rc;
    Layout lo;
    plan(tl, K, G, lo, mask, ew_mask, N);
    if (lo.xc_col.size() >= (1u << 26)) return TW_ERR_UNSUPPORTED;
    if (blob_bytes < lo.bytes) return TW_ERR_BUF;

    uint8_t* base = (uint8_t*)blob;
    std::memset(base, 0, (size_t)lo.bytes);
    TwHeader* h = (TwHeader*)base;
    h->magic = TW_MAGIC;
    h->version = TW_FORMAT_VERSION;
    h->dtype = (int)dt; h->K = K; h->N = N; h->G = G; h->T = tl.T;
    h->n_kept_cols = (int32_t)tl.col_idx.size();
    h->nnz = tl.nnz;
    h->blob_bytes = lo.bytes;
    h->k_chunk = lo.k_chunk; h->n_chunks = lo.n_chunks; h->ncb = lo.ncb;
    h->total_steps = lo.total_steps;
    h->off_col_idx = lo.off_col_idx; h->off_tile_col_ptr = lo.off_tile_col_ptr;
    h->off_tile_row_ptr = lo.off_tile_row_ptr; h->off_row_idx = lo.off_row_idx;
    h->off_tile_span = lo.off_tile_span; h->off_sched_order = lo.off_sched_order;
    h->off_tile_desc = lo.off_tile_desc; h->off_step_ptr = lo.off_step_ptr;
    h->off_goff = lo.off_goff; h->off_dpos = lo.off_dpos; h->off_bvals = lo.off_bvals;
    h->off_sched_desc = lo.off_sched_desc;
    h->off_zero_ptr = lo.off_zero_ptr; h->off_zero_cols = lo.off_zero_cols; h->off_zero_xc = lo.off_zero_xc;
    h->off_urow = lo.off_urow; h->off_ucnt = lo.off_ucnt;
    h->ew_nnz = lo.ew_nnz; h->off_ew_ptr = lo.off_ew_ptr; h->off_ew_goff = lo.off_ew_goff; h->off_ew_b = lo.off_ew_b;
    h->off_ew_mask = lo.off_ew_mask;
    h->off_xm_ptr = lo.off_xm_ptr; h->off_xm_goff = lo.off_xm_goff; h->off_xm_b = lo.off_xm_b;
    h->xc_n = (int32_t)lo.xc_col.size();
    h->off_xc_col = lo.off_xc_col; h->off_xc_ptr = lo.off_xc_ptr; h->off_xc_k = lo.off_xc_k; h->off_xc_v = lo.off_xc_v;
    h->off_xc_tile_ptr = lo.off_xc_tile_ptr; h->off_xc_rank = lo.off_xc_rank; h->xc_overflow = lo.xc_overflow;

    auto put = [&](uint64_t off, const std::vector<int32_t>& v) {
        if (!v.empty()) std::memcpy(base + off, v.data(), 4 * v.size());
    };
    put(lo.off_col_idx, tl.col_idx);
    put(lo.off_tile_col_ptr, tl.tile_col_ptr);
    put(lo.off_tile_row_ptr, tl.tile_row_ptr);
    put(lo.off_row_idx, tl.row_idx);
    put(lo.off_tile_span, tl.tile_span);
    put(lo.off_step_ptr, lo.step_ptr);

    // element-wise residual in the tiles' kept columns: steps of 16 rows per column block
    put(lo.off_ew_ptr, lo.ew_ptr);
    if (ew_mask && lo.ew_ptr[(size_t)tl.T * lo.n_chunks] > 0) {
        uint16_t* eg = (uint16_t*)(base + lo.off_ew_goff);
        uint16_t* eb = (uint16_t*)(base + lo.off_ew_b);
        uint32_t* em = (uint32_t*)(base + lo.off_ew_mask);
        const uint16_t* Bw = (const uint16_t*)B;
        const int nc = lo.n_chunks, ncb = lo.ncb;
        const size_t minis = (size_t)lo.ew_ptr[(size_t)tl.T * nc] * ncb;
        for (size_t i = 0; i < minis * 16; ++i) eg[i] = (uint16_t)lo.k_chunk;   // weights and mask words are zero already
        std::vector<int32_t> rows;
        for (int t = 0; t < tl.T; ++t) {
            const int c0 = tl.tile_col_ptr[t], c1 = tl.tile_col_ptr[t + 1];
            for (int ch = 0; ch < nc; ++ch) {
                const int k0 = ch * lo.k_chunk, k1 = std::min(K, k0 + lo.k_chunk);
                const size_t rs0 = (size_t)lo.ew_ptr[(size_t)t * nc + ch];
                for (int cb = 0; c0 + cb * TW_COLBLK < c1; ++cb) {
                    const int cl = c0 + cb * TW_COLBLK, chi = std::min(cl + TW_COLBLK, c1);
                    residual_rows(tl, mask, ew_mask, N, cl, chi, k0, k1, rows);
                    order_residual_rows(rows, k0);
                    for (size_t j = 0; j < rows.size(); ++j) {
                        const int k = rows[j];
                        const size_t rs = rs0 + j / 16;
                        const int kl = (int)(j % 16), half = kl / 8, e = kl % 8;
                        eg[((rs * 8 + half * 4 + (e & 3)) * ncb + cb) * 2 + (e >> 2)] = (uint16_t)(k - k0);
                        for (int c = cl; c < chi; ++c) {
                            const size_t i = (size_t)k * N + tl.col_idx[c];
                            if (ew_mask[i] == 0 || mask[i] != 0) continue;
                            const int n = c - cl;
                            eb[((rs * ncb + cb) * 64 + 32 * half + n) * 8 + e] = Bw[(size_t)k * ldb + tl.col_idx[c]];
                            em[(rs * ncb + cb) * 16 + kl] |= 1u << n;
                        }
                    }
                }
            }
        }
    }

    // the residual's columns without tile-wise weights
    put(lo.off_xc_col, lo.xc_col);
    put(lo.off_xc_ptr, lo.xc_ptr);
    put(lo.off_xc_k, lo.xc_k);
    put(lo.off_xc_tile_ptr, lo.xc_tile_ptr);
    put(lo.off_xc_rank, lo.xc_rank);
    {
        uint16_t* xv = (uint16_t*)(base + lo.off_xc_v);
        const uint16_t* Bw = (const uint16_t*)B;
        for (size_t j = 0; j < lo.xc_col.size(); ++j)
            for (int32_t e = lo.xc_ptr[j]; e < lo.xc_ptr[j + 1]; ++e)
                xv[e] = Bw[(size_t)lo.xc_k[e] * ldb + lo.xc_col[j]];
    }

    // the tiles' first residual-only columns as a column block for the matrix cores, chunk by chunk
    put(lo.off_xm_ptr, lo.xm_ptr);
    if (lo.xm_ptr.back() > 0) {
        uint16_t* xg = (uint16_t*)(base + lo.off_xm_goff);
        uint16_t* xb = (uint16_t*)(base + lo.off_xm_b);
        const uint16_t* Bw = (const uint16_t*)B;
        for (size_t i = 0; i < (size_t)lo.xm_ptr.back() * 16; ++i) xg[i] = (uint16_t)lo.k_chunk;
        std::vector<int32_t> rows, slot_of(K, -1);
        for (int t = 0; t < tl.T; ++t)
            for (int ch = 0; ch < lo.n_chunks; ++ch) {
                const int k0 = ch * lo.k_chunk, k1 = std::min(K, k0 + lo.k_chunk);
                const size_t first = (size_t)lo.xm_ptr[(size_t)t * lo.n_chunks + ch];
                inline_xc_rows(lo, t, k0, k1, rows);
                for (size_t j = 0; j < rows.size(); ++j) {
                    slot_of[rows[j]] = (int32_t)j;
                    const size_t st = first + j / 16;
                    const int kl = (int)(j % 16), half = kl / 8, e = kl % 8;
                    xg[st * 16 + (half * 4 + (e & 3)) * 2 + (e >> 2)] = (uint16_t)(rows[j] - k0);
                }
                const int x0 = lo.xc_tile_ptr[t], x1 = std::min(lo.xc_tile_ptr[t + 1], x0 + TW_XC_INLINE);
                for (int c = x0; c < x1; ++c)
                    for (int32_t q = lo.xc_ptr[c]; q < lo.xc_ptr[c + 1]; ++q) {
                        const int k = lo.xc_k[q];
                        if (k < k0 || k >= k1) continue;
                        const int j = slot_of[k];
                        const size_t st = first + j / 16;
                        const int kl = j % 16, half = kl / 8, e = kl % 8;
                        xb[(st * 64 + 32 * half + (c - x0)) * 8 + e] = Bw[(size_t)k * ldb + lo.xc_col[c]];
                    }
            }
    }

    // pruned columns inside every span
    {
        std::vector<int32_t> zptr(tl.T + 1, 0), zcols;
        for (int t = 0; t < tl.T; ++t) {
            int c = tl.tile_col_ptr[t];
            for (int n = tl.tile_span[t]; n < tl.tile_span[t + 1]; ++n) {
                if (c < tl.tile_col_ptr[t + 1] && tl.col_idx[c] == n) ++c;
                else zcols.push_back(n);
            }
            zptr[t + 1] = (int32_t)zcols.size();
        }
        put(lo.off_zero_ptr, zptr);
        put(lo.off_zero_cols, zcols);
        // which of them hold residual weights that the owning tile adds itself (both lists ascend)
        int8_t* zx = (int8_t*)(base + lo.off_zero_xc);
        for (int t = 0; t < tl.T; ++t) {
            int x = lo.xc_tile_ptr[t];
            for (int32_t j = zptr[t]; j < zptr[t + 1]; ++j) {
                zx[j] = -1;
                if (x < lo.xc_tile_ptr[t + 1] && lo.xc_col[x] == zcols[j]) {
                    if (x - lo.xc_tile_ptr[t] < TW_XC_INLINE) zx[j] = (int8_t)(x - lo.xc_tile_ptr[t]);
                    ++x;
                }
            }
        }
    }

    // schedule: heaviest tile (most kept rows) first, ties keep tile order
    std::vector<int32_t> order(tl.T);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
        return (tl.tile_row_ptr[a + 1] - tl.tile_row_ptr[a]) > (tl.tile_row_ptr[b + 1] - tl.tile_row_ptr[b]);
    });
    put(lo.off_sched_order, order);

    const uint16_t* Bv = (const uint16_t*)B;
    const uint16_t pad_k = (uint16_t)lo.k_chunk;
    TwTileDesc* desc = (TwTileDesc*)(base + lo.off_tile_desc);
    uint16_t* goff = (uint16_t*)(base + lo.off_goff);
    uint32_t* dpos_all = (uint32_t*)(base + lo.off_dpos);
    uint16_t* bvals = (uint16_t*)(base + lo.off_bvals);
    const int ncb = lo.ncb;

    for (int t = 0; t < tl.T; ++t) {
        const int c0 = tl.tile_col_ptr[t], w = tl.tile_col_ptr[t + 1] - c0;
        const int r0 = tl.tile_row_ptr[t], kt = tl.tile_row_ptr[t + 1] - r0;
        const int32_t* sp = &lo.step_ptr[(size_t)t * (lo.n_chunks + 1)];
        const int nsteps = sp[lo.n_chunks];
        TwTileDesc& d = desc[t];
        d.w = w; d.k = kt;
        d.span_start = tl.tile_span[t];
        d.span_w = tl.tile_span[t + 1] - tl.tile_span[t];
        d.nsteps = nsteps;
        d.step_ptr = t * (lo.n_chunks + 1);
        d.first_step = lo.first_step[t];
        d.bvals_off = lo.off_bvals + 2 * (uint64_t)lo.first_step[t] * ncb * 64 * 8;
        bool nogap = true;
        for (int c = 0; c < w; ++c)
            if (tl.col_idx[c0 + c] != d.span_start + c) { nogap = false; break; }
        d.flags = nogap ? TW_TILE_NOGAP : 0;

        // destination columns, counted from the aligned column at or below the span start
        {
            uint32_t* dp = dpos_all + (size_t)t * 32 * ncb;
            const int origin = d.span_start / 8 * 8;
            for (int n = 0; n < 32; ++n)
                for (int cb = 0; cb < ncb; ++cb) {
                    const int c = 32 * cb + n;
                    dp[n * ncb + cb] = c < w ? (uint32_t)(tl.col_idx[c0 + c] - origin) : 0xFFFFFFFFu;
                }
        }

        // gather offsets and packed values, chunk by chunk
        uint16_t* tg = goff + (size_t)lo.first_step[t] * 16;
        for (int s = 0; s < nsteps * 16; ++s) tg[s] = pad_k;
        uint16_t* tb = bvals + (size_t)lo.first_step[t] * ncb * 64 * 8;
        int p = 0;
        for (int c = 0; c < lo.n_chunks; ++c) {
            const int hi = (c + 1) * lo.k_chunk, kbase = c * lo.k_chunk;
            int slot = sp[c] * 16;
            while (p < kt && tl.row_idx[r0 + p] < hi) {
                const int k = tl.row_idx[r0 + p];
                const int s = slot / 16, kl = slot % 16;       // step, contraction slot in the step
                const int half = kl / 8, e = kl % 8;
                tg[s * 16 + (half * 4 + (e & 3)) * 2 + (e >> 2)] = (uint16_t)(k - kbase);
                for (int cc = 0; cc < w; ++cc) {
                    const int cb = cc / 32, lane = 32 * half + cc % 32;
                    tb[(((size_t)s * ncb + cb) * 64 + lane) * 8 + e] =
                        Bv[(size_t)k * ldb + tl.col_idx[c0 + cc]];
                }
                ++slot; ++p;
            }
        }
    }
    // Dispatch order of the kernel.  With K resident the waves of a workgroup pull tiles one after the
    // other.  Nothing can be stored before the first tiles are finished, and while nothing is stored
    // the memory system idles, so the first TW_WAVES_PER_WG pulls get the lightest tiles (lightest
    // first); the remaining tiles follow heaviest first, which keeps the end of a workgroup balanced.
    // With K streamed the waves of a set advance in lock step, so sets hold tiles of similar weight
    // (plain heaviest-first order).
    std::vector<int32_t> dispatch(order);
    if (lo.n_chunks == 1 && tl.T > TW_WAVES_PER_WG) {
        int n = 0;
        for (int i = 0; i < TW_WAVES_PER_WG; ++i) dispatch[n++] = order[tl.T - 1 - i];
        for (int i = 0; i < tl.T - TW_WAVES_PER_WG; ++i) dispatch[n++] = order[i];
    }
    // streamed K: the K rows every set of tiles needs, chunk by chunk
    if (lo.n_chunks > 1 && tl.T > 0) {
        const int tpw = TW_SET_TILES(tl.T), n_sets = (tl.T + tpw - 1) / tpw;
        uint16_t* urow = (uint16_t*)(base + lo.off_urow);
        int32_t* ucnt = (int32_t*)(base + lo.off_ucnt);
        std::vector<uint8_t> need(K);
        for (int st = 0; st < n_sets; ++st) {
            std::fill(need.begin(), need.end(), 0);
            for (int i = st * tpw; i < std::min(tl.T, (st + 1) * tpw); ++i) {
                const int t = dispatch[i];
                for (int r = tl.tile_row_ptr[t]; r < tl.tile_row_ptr[t + 1]; ++r) need[tl.row_idx[r]] = 1;
                if (ew_mask)   // and the rows of the tile's element-wise residual
                    for (int c = tl.tile_col_ptr[t]; c < tl.tile_col_ptr[t + 1]; ++c) {
                        const int n = tl.col_idx[c];
                        for (int k = 0; k < K; ++k)
                            if (ew_mask[(size_t)k * N + n] != 0) need[k] = 1;
                    }
                // and those of the residual-only columns in its span that the tile adds itself
                for (int x = lo.xc_tile_ptr[t]; x < std::min(lo.xc_tile_ptr[t + 1], lo.xc_tile_ptr[t] + TW_XC_INLINE); ++x)
                    for (int32_t q = lo.xc_ptr[x]; q < lo.xc_ptr[x + 1]; ++q) need[lo.xc_k[q]] = 1;
            }
            for (int c = 0; c < lo.n_chunks; ++c) {
                uint16_t* out = urow + ((size_t)st * lo.n_chunks + c) * lo.k_chunk;
                int n = 0;
                for (int k = c * lo.k_chunk; k < std::min(K, (c + 1) * lo.k_chunk); ++k)
                    if (need[k]) out[n++] = (uint16_t)(k - c * lo.k_chunk);
                ucnt[(size_t)st * lo.n_chunks + c] = n;
                for (int j = n; j < lo.k_chunk; ++j) out[j] = n > 0 ? out[n - 1] : 0;   // padding: a valid row
            }
        }
    }
    TwSchedDesc* sd = (TwSchedDesc*)(base + lo.off_sched_desc);
    for (int i = 0; i < tl.T; ++i) {
        const TwTileDesc& d = desc[dispatch[i]];
        sd[i].w = d.w; sd[i].span_start = d.span_start; sd[i].span_w = d.span_w; sd[i].nsteps = d.nsteps;
        sd[i].tile = dispatch[i]; sd[i].step_ptr = d.step_ptr; sd[i].first_step = d.first_step;
        const int32_t x0 = lo.xc_tile_ptr[dispatch[i]], nx = lo.xc_tile_ptr[dispatch[i] + 1] - x0;
        sd[i].xc = (int32_t)((uint32_t)x0 | (uint32_t)std::min(nx, TW_XC_INLINE) << 26);
    }
    return TW_OK;
}

extern "C" int tw_info(const void* blob, tw_info_t* out) {
    const TwHeader* h = header_of(blob);
    if (!out) return TW_ERR_ARG;
    if (!h) return TW_ERR_BUF;
    out->version = (int32_t)h->version;
    out->dtype = h->dtype; out->K = h->K; out->N = h->N; out->G = h->G; out->T = h->T;
    out->n_kept_cols = h->n_kept_cols;
    out->k_chunk = h->k_chunk;
    out->nnz = h->nnz;
    out->ew_nnz = h->ew_nnz;
    out->padded_macs_per_row = h->total_steps * TW_KSTEP * (int64_t)h->G;
    out->blob_bytes = h->blob_bytes;
    out->off_col_idx = h->off_col_idx; out->off_tile_col_ptr = h->off_tile_col_ptr;
    out->off_tile_row_ptr = h->off_tile_row_ptr; out->off_row_idx = h->off_row_idx;
    out->off_tile_span = h->off_tile_span; out->off_sched_order = h->off_sched_order;
    return TW_OK;
}

extern "C" int tw_unpack(const void* blob, void* B_out, int ldb, uint8_t* mask_out) {
    const TwHeader* h = header_of(blob);
    if (!h) return TW_ERR_BUF;
    if (B_out && ldb < h->N) return TW_ERR_ARG;
    const uint8_t* base = (const uint8_t*)blob;
    const int K = h->K, N = h->N, T = h->T, ncb = h->ncb;
    const int32_t* col_idx = (const int32_t*)(base + h->off_col_idx);
    const int32_t* tcp = (const int32_t*)(base + h->off_tile_col_ptr);
    const int32_t* trp = (const int32_t*)(base + h->off_tile_row_ptr);
    const int32_t* row_idx = (const int32_t*)(base + h->off_row_idx);
    const int32_t* step_ptr = (const int32_t*)(base + h->off_step_ptr);
    const TwTileDesc* desc = (const TwTileDesc*)(base + h->off_tile_desc);
    uint16_t* Bo = (uint16_t*)B_out;
    if (Bo)
        for (int k = 0; k < K; ++k) std::memset(Bo + (size_t)k * ldb, 0, 2 * (size_t)N);
    if (mask_out) std::memset(mask_out, 0, (size_t)K * N);
    for (int t = 0; t < T; ++t) {
        const int c0 = tcp[t], w = tcp[t + 1] - c0, r0 = trp[t], kt = trp[t + 1] - r0;
        const int32_t* sp = step_ptr + desc[t].step_ptr;
        const uint16_t* tb = (const uint16_t*)(base + desc[t].bvals_off);
        int p = 0;
        for (int c = 0; c < h->n_chunks; ++c) {
            const int hi = (c + 1) * h->k_chunk;
            int slot = sp[c] * 16;
            while (p < kt && row_idx[r0 + p] < hi) {
                const int k = row_idx[r0 + p];
                const int s = slot / 16, kl = slot % 16, half = kl / 8, e = kl % 8;
                for (int cc = 0; cc < w; ++cc) {
                    const int n = col_idx[c0 + cc];
                    if (mask_out) mask_out[(size_t)k * N + n] = 1;
                    if (Bo) {
                        const int cb = cc / 32, lane = 32 * half + cc % 32;
                        Bo[(size_t)k * ldb + n] = tb[(((size_t)s * ncb + cb) * 64 + lane) * 8 + e];
                    }
                }
                ++slot; ++p;
            }
        }
    }
    // the element-wise residual: part of the weights the GEMM multiplies by
    if (h->ew_nnz > 0) {
        const int32_t* ep = (const int32_t*)(base + h->off_ew_ptr);
        const uint16_t* eg = (const uint16_t*)(base + h->off_ew_goff);
        const uint16_t* eb = (const uint16_t*)(base + h->off_ew_b);
        const uint32_t* em = (const uint32_t*)(base + h->off_ew_mask);
        const int nc = h->n_chunks, ncb = h->ncb;
        for (int t = 0; t < T; ++t) {
            const int c0 = tcp[t];
            for (int ch = 0; ch < nc; ++ch)
                for (size_t rs = (size_t)ep[(size_t)t * nc + ch]; rs < (size_t)ep[(size_t)t * nc + ch + 1]; ++rs)
                    for (int cb = 0; cb < ncb; ++cb)
                        for (int kl = 0; kl < 16; ++kl) {
                            const uint32_t bits = em[(rs * ncb + cb) * 16 + kl];
                            if (bits == 0) continue;
                            const int half = kl / 8, e = kl % 8;
                            const int k = ch * h->k_chunk + eg[((rs * 8 + half * 4 + (e & 3)) * ncb + cb) * 2 + (e >> 2)];
                            for (int n = 0; n < 32; ++n) {
                                if (!((bits >> n) & 1u)) continue;
                                const int col = col_idx[c0 + cb * TW_COLBLK + n];
                                if (mask_out) mask_out[(size_t)k * N + col] = 1;
                                if (Bo) Bo[(size_t)k * ldb + col] = eb[((rs * ncb + cb) * 64 + 32 * half + n) * 8 + e];
                            }
                        }
        }
        const int32_t* xcol = (const int32_t*)(base + h->off_xc_col);
        const int32_t* xptr = (const int32_t*)(base + h->off_xc_ptr);
        const int32_t* xk = (const int32_t*)(base + h->off_xc_k);
        const uint16_t* xv = (const uint16_t*)(base + h->off_xc_v);
        for (int j = 0; j < h->xc_n; ++j)
            for (int32_t e = xptr[j]; e < xptr[j + 1]; ++e) {
                if (mask_out) mask_out[(size_t)xk[e] * N + xcol[j]] = 1;
                if (Bo) Bo[(size_t)xk[e] * ldb + xcol[j]] = xv[e];
            }
    }
    return TW_OK;
}

// The delta*K*N pruned weights of largest magnitude, wherever they lie (the elements the TEW hybrid puts back,
// Sec. IV-A; magnitude as importance score), ties to the lower (k, n).
extern "C" int tw_restore_ew(const void* B, int ldb, int K, int N, tw_dtype dt, const uint8_t* mask, double delta,
                             uint8_t* ew_mask_out) {
    if (!B || !mask || !ew_mask_out || K <= 0 || N <= 0 || ldb < N) return TW_ERR_ARG;
    if (dt != TW_F16 && dt != TW_BF16) return TW_ERR_ARG;
    if (!(delta >= 0.0 && delta < 1.0)) return TW_ERR_ARG;
    std::memset(ew_mask_out, 0, (size_t)K * N);
    const uint16_t* Bw = (const uint16_t*)B;
    std::vector<std::pair<uint16_t, int64_t>> cand;     // (magnitude bits, position)
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n)
            if (mask[(size_t)k * N + n] == 0)
                cand.emplace_back((uint16_t)(Bw[(size_t)k * ldb + n] & 0x7FFFu), (int64_t)k * N + n);
    int64_t want = (int64_t)std::floor(delta * (double)K * (double)N + 0.5);
    if (want > (int64_t)cand.size()) want = (int64_t)cand.size();
    // for both 16-bit formats the magnitude order of finite values is the order of the bit patterns
    std::stable_sort(cand.begin(), cand.end(),
                     [](const std::pair<uint16_t, int64_t>& a, const std::pair<uint16_t, int64_t>& b) { return a.first > b.first; });
    for (int64_t i = 0; i < want; ++i) ew_mask_out[cand[i].second] = 1;
    return TW_OK;
}

extern "C" const char* tw_strerror(int status) {
    switch (status) {
        case TW_OK: return "ok";
        case TW_ERR_ARG: return "bad argument";
        case TW_ERR_NOT_TILEWISE: return "mask is not tile-wise for this granularity";
        case TW_ERR_BUF: return "buffer too small or not a packed blob";
        case TW_ERR_ALIGN: return "pointer or leading dimension not aligned";
        case TW_ERR_HIP: return "HIP runtime error";
        case TW_ERR_UNSUPPORTED: return "unsupported granularity or shape";
        default: return "unknown status";
    }
}

extern "C" int tw_version(void) { return TW_FORMAT_VERSION; }

// ---- one-shot magnitude pruning into the TW pattern (one stage of Alg. 1 without fine-tuning) ----
namespace {

// 16-bit storage value -> double, exactly
double half_to_double(uint16_t b) {
    const int sign = b >> 15, e = (b >> 10) & 31, m = b & 1023;
    double v;
    if (e == 0) v = std::ldexp((double)m, -24);
    else if (e == 31) v = m ? NAN : INFINITY;
    else v = std::ldexp((double)(m | 1024), e - 25);
    return sign ? -v : v;
}
double bf16_to_double(uint16_t b) {
    const uint32_t u = (uint32_t)b << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return (double)f;
}

}  // namespace

extern "C" int tw_prune(const void* B, int ldb, int K, int N, int G, tw_dtype dt, double col_prune, double sparsity,
                        uint8_t* mask_out) {
    if (!B || !mask_out || K <= 0 || N <= 0 || G <= 0 || ldb < N) return TW_ERR_ARG;
    if (dt != TW_F16 && dt != TW_BF16) return TW_ERR_ARG;
    if (!(col_prune >= 0.0 && col_prune < 1.0) || !(sparsity >= 0.0 && sparsity < 1.0)) return TW_ERR_ARG;
    const uint16_t* Bv = (const uint16_t*)B;
    auto mag = [&](int k, int n) {
        const uint16_t b = Bv[(size_t)k * ldb + n];
        return std::fabs(dt == TW_F16 ? half_to_double(b) : bf16_to_double(b));
    };
    // column stage: importance of a column = sum of its magnitudes (k ascending); the floor(p*N + 0.5)
    // least important go, the lower index first among equals
    std::vector<double> cscore(N, 0.0);
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n) cscore[n] += mag(k, n);
    const int n_prune = (int)std::floor(col_prune * N + 0.5);
    std::vector<int> cord(N);
    std::iota(cord.begin(), cord.end(), 0);
    std::stable_sort(cord.begin(), cord.end(), [&](int a, int b) { return cscore[a] < cscore[b]; });
    std::vector<uint8_t> col_keep(N, 1);
    for (int i = 0; i < n_prune && i < N; ++i) col_keep[cord[i]] = 0;
    std::vector<int> cols;
    for (int n = 0; n < N; ++n)
        if (col_keep[n]) cols.push_back(n);
    const int nk = (int)cols.size();
    std::memset(mask_out, 0, (size_t)K * N);
    if (nk == 0) return TW_OK;
    // row stage: the surviving columns are regrouped G at a time; importance of a row segment = mean
    // magnitude over its columns (columns ascending), compared across ALL tiles, so tiles end up with
    // different numbers of rows
    const int T = (nk + G - 1) / G;
    struct Seg { double score; int t, k, w; };
    std::vector<Seg> segs((size_t)T * K);
    for (int t = 0; t < T; ++t) {
        const int c0 = t * G, w = std::min(G, nk - c0);
        for (int k = 0; k < K; ++k) {
            double acc = 0.0;
            for (int c = 0; c < w; ++c) acc += mag(k, cols[c0 + c]);
            segs[(size_t)t * K + k] = Seg{acc / w, t, k, w};
        }
    }
    std::vector<size_t> sord(segs.size());
    std::iota(sord.begin(), sord.end(), (size_t)0);
    std::stable_sort(sord.begin(), sord.end(), [&](size_t a, size_t b) { return segs[a].score < segs[b].score; });
    // prune segments, least important first, until the zeros reach the target; one row per tile always stays
    const long long total = (long long)K * N;
    const long long want = (long long)std::ceil(sparsity * (double)total);
    long long zeros = (long long)K * (N - nk);
    std::vector<int> left(T, K);
    std::vector<uint8_t> seg_keep(segs.size(), 1);
    for (size_t i = 0; i < sord.size() && zeros < want; ++i) {
        const Seg& sg = segs[sord[i]];
        if (left[sg.t] <= 1) continue;
        seg_keep[sord[i]] = 0;
        --left[sg.t];
        zeros += sg.w;
    }
    for (int t = 0; t < T; ++t) {
        const int c0 = t * G, w = std::min(G, nk - c0);
        for (int k = 0; k < K; ++k)
            if (seg_keep[(size_t)t * K + k])
                for (int c = 0; c < w; ++c) mask_out[(size_t)k * N + cols[c0 + c]] = 1;
    }
    return TW_OK;
}
