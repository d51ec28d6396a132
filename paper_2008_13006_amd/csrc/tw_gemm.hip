// tw_gemm: C = A . (B * mask) for a packed tile-wise weight, one persistent kernel on gfx950.
//
// Paper: Sec. VI.  The kernel in Listing 1 loads A tiles while skipping pruned K positions with a
// per-tile mask vector, multiplies them with pre-processed B tiles on the matrix unit and stores C
// skipping pruned columns; equal-width tiles are batched to share A and batches run concurrently
// to even out the load.  This kernel keeps those ideas and changes the mechanics for CDNA4:
//   * a workgroup stages a block of A rows in LDS ONCE with coalesced 16-byte loads and all the
//     tiles it works on gather their kept K positions from that copy (2-byte LDS reads), so the
//     skipping never touches global memory and A is shared by many tiles (the role of batching);
//   * the compacted tile values are stored offline in MFMA operand order and go from global
//     memory (L2-resident) straight to registers;
//   * workgroups are persistent and pull (row block, tile set) items from an atomic counter;
//     inside a workgroup the waves pull tiles, heaviest first (the role of stream concurrency);
//   * pruned columns inside a tile's span are written as zeros together with the kept ones, in
//     contiguous pieces, through a small per-wave LDS staging area.
#include <hip/hip_runtime.h>

#include "../../include/tw.h"
#include "tw_device.hpp"
#include "tw_format.h"

namespace {

constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
constexpr int kPrefetch = 2;  // B-operand steps in flight per wave

struct TwGemmParams {
    const unsigned char* blob;  // device copy
    const unsigned short* A;
    unsigned short* C;
    int* counters;              // [0] next item, [1] finished workgroups
    long lda, ldc;
    int M, K, N, T;
    int k_chunk, n_chunks;
    int n_mblocks, n_seg, n_items;
    unsigned a_pitch;           // bytes between rows of the LDS copy of A
    unsigned a_buf_bytes;       // one LDS buffer of A
    unsigned stage_off;         // LDS offset of the per-wave staging areas
    unsigned misc_off;          // LDS offset of two ints (item, tile counter)
    uint64_t off_sched_order, off_tile_desc, off_step_ptr, off_goff;
};

__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }

// Wave-uniform copy of the fields of a tile descriptor the kernel steers by (kept in SGPRs).
struct TileU {
    int w, span_start, span_w, nsteps, flags, step_ptr, first_step;
    unsigned dcol_off;
    uint64_t bvals_off;
};
__device__ __forceinline__ TileU load_tile(const TwTileDesc* descs, int t) {
    const TwTileDesc& d = descs[t];
    TileU u;
    u.w = uni(d.w); u.span_start = uni(d.span_start); u.span_w = uni(d.span_w);
    u.nsteps = uni(d.nsteps); u.flags = uni(d.flags); u.step_ptr = uni(d.step_ptr);
    u.first_step = uni(d.first_step); u.dcol_off = (unsigned)uni((int)d.dcol_off);
    const unsigned lo = (unsigned)uni((int)(unsigned)d.bvals_off), hi = (unsigned)uni((int)(unsigned)(d.bvals_off >> 32));
    u.bvals_off = ((uint64_t)hi << 32) | lo;
    return u;
}

// Cooperative load of A[row0 .. row0+32*MS) x [k0, k0+kw) into an LDS buffer (row pitch a_pitch),
// plus the zeroed 8-byte pad behind each row that padded contraction slots read.
template <int MS>
__device__ __forceinline__ void load_a_block(const TwGemmParams& p, unsigned char* buf, int row0, int k0,
                                             int kw, int wave, int lane) {
    constexpr int BM = 32 * MS;
    const int units = (kw + 7) >> 3;  // 16-byte pieces per row
    for (int r = wave; r < BM; r += kWaves) {
        int grow = row0 + r;
        grow = grow < p.M ? grow : p.M - 1;  // rows past M are loaded from the last row, never stored
        const unsigned short* src = p.A + (long)grow * p.lda + k0;
        unsigned char* dst = buf + (unsigned)r * p.a_pitch;
        for (int u = lane; u < units; u += 64) {
            const int k = u * 8;
            tw_u32x4 v;
            if (k0 + k + 8 <= p.K) {
                v = *(const tw_u32x4*)(src + k);
            } else {
                unsigned short e[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) e[i] = (k0 + k + i < p.K) ? src[k + i] : (unsigned short)0;
                v = tw_u32x4{e[0] | ((unsigned)e[1] << 16), e[2] | ((unsigned)e[3] << 16),
                             e[4] | ((unsigned)e[5] << 16), e[6] | ((unsigned)e[7] << 16)};
            }
            *(tw_u32x2*)(dst + u * 16) = tw_u32x2{v.x, v.y};
            *(tw_u32x2*)(dst + u * 16 + 8) = tw_u32x2{v.z, v.w};
        }
        if (lane == 0) *(tw_u32x2*)(dst + 2 * p.k_chunk) = tw_u32x2{0u, 0u};
    }
}

// Steps [s0, s1) of one tile for this wave: gather A from LDS, stream packed B from global, MFMA.
template <int DT, int MS, int NCB>
__device__ __forceinline__ void run_steps(tw_f32x16 (&acc)[MS][NCB], const unsigned char* a_buf, unsigned a_pitch,
                                          const unsigned char* goff_tile, const unsigned char* bvals_tile,
                                          int s0, int s1, int lane) {
    const int h = lane >> 5;
    unsigned rowaddr[MS];
#pragma unroll
    for (int ms = 0; ms < MS; ++ms) rowaddr[ms] = (unsigned)(ms * 32 + (lane & 31)) * a_pitch;

    tw_u16x8 bq[kPrefetch][NCB];
    tw_u16x8 go[kPrefetch];
    auto issue = [&](int slot, int s) {
        go[slot] = *(const tw_u16x8*)(goff_tile + (long)s * 32 + h * 16);
        const unsigned char* b = bvals_tile + ((long)s * NCB) * 1024 + lane * 16;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) bq[slot][cb] = *(const tw_u16x8*)(b + cb * 1024);
    };
#pragma unroll
    for (int i = 0; i < kPrefetch; ++i)
        if (s0 + i < s1) issue(i, s0 + i);

    for (int s = s0; s < s1; s += kPrefetch) {
#pragma unroll
        for (int i = 0; i < kPrefetch; ++i) {
            if (s + i < s1) {
                const tw_u16x8 g = go[i];
                tw_u16x8 a[MS];
#pragma unroll
                for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        a[ms][e] = *(const unsigned short*)(a_buf + rowaddr[ms] + (unsigned)g[e]);
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                    for (int ms = 0; ms < MS; ++ms) acc[ms][cb] = tw_mfma<DT>(bq[i][cb], a[ms], acc[ms][cb]);
                if (s + i + kPrefetch < s1) issue(i, s + i + kPrefetch);
            }
        }
    }
}

template <int DT, int MS, int NCB>
__device__ __forceinline__ void store_tile(const TwGemmParams& p, const TileU& d, tw_f32x16 (&acc)[MS][NCB],
                                           unsigned char* stage, int row0, int lane) {
    const int h = lane >> 5;
    const bool nogap = (d.flags & TW_TILE_NOGAP) != 0;
    // destination columns of this lane's packed columns: [cb][q] -> four 16-bit entries
    tw_u16x4 dc[NCB][4];
    if (!nogap) {
        const tw_u16x4* src = (const tw_u16x4*)(p.blob + d.dcol_off) + h * NCB * 4;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int q = 0; q < 4; ++q) dc[cb][q] = src[cb * 4 + q];
    } else {
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int q = 0; q < 4; ++q) dc[cb][q] = tw_u16x4{0, 0, 0, 0};
    }
#pragma unroll
    for (int ms = 0; ms < MS; ++ms) {
        auto dst = [&](int cb, int q, int e) -> unsigned { return dc[cb][q][e]; };
        tw_store_block<DT, NCB>(acc[ms], dst, nogap, stage, p.C, p.ldc, row0 + 32 * ms, p.M, d.span_start,
                                d.span_w, lane);
    }
}

template <int DT, int MS, int NCB, bool RESIDENT>
__global__ __launch_bounds__(kThreads) void tw_gemm_kernel(const TwGemmParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int BM = 32 * MS;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    unsigned char* stage = smem + p.stage_off + wave * TW_STAGE_BYTES;
    volatile int* misc = (volatile int*)(smem + p.misc_off);
    const int* order = (const int*)(p.blob + p.off_sched_order);
    const TwTileDesc* descs = (const TwTileDesc*)(p.blob + p.off_tile_desc);
    const int* step_ptr = (const int*)(p.blob + p.off_step_ptr);

    for (;;) {
        if (tid == 0) {
            misc[0] = atomicAdd(&p.counters[0], 1);
            misc[1] = 0;
        }
        __syncthreads();
        const int item = misc[0];
        if (item >= p.n_items) break;

        if constexpr (RESIDENT) {
            // the whole K extent of the row block stays in LDS; waves pull tiles of this item's set
            const int mb = item / p.n_seg, seg = item - mb * p.n_seg;
            const int row0 = mb * BM;
            load_a_block<MS>(p, smem, row0, 0, p.K, wave, lane);
            __syncthreads();
            for (;;) {
                int i = 0;
                if (lane == 0) i = atomicAdd((int*)&misc[1], 1);
                i = __builtin_amdgcn_readfirstlane(i);
                const int ti = seg + i * p.n_seg;
                if (ti >= p.T) break;
                const TileU d = load_tile(descs, uni(order[ti]));
                tw_f32x16 acc[MS][NCB];
#pragma unroll
                for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[ms][cb][r] = 0.f;
                run_steps<DT, MS, NCB>(acc, smem, p.a_pitch, p.blob + p.off_goff + (long)d.first_step * 32,
                                       p.blob + d.bvals_off, 0, d.nsteps, lane);
                store_tile<DT, MS, NCB>(p, d, acc, stage, row0, lane);
            }
            __syncthreads();  // everyone is done with the LDS copy of A and with misc[]
        } else {
            // K is streamed in chunks; wave w owns tile (8*set + w) of the kept-K ordering
            const int set = item / p.n_mblocks, mb = item - set * p.n_mblocks;
            const int row0 = mb * BM;
            const int ti = set * kWaves + wave;
            const bool active = ti < p.T;
            const TileU d = load_tile(descs, uni(order[active ? ti : 0]));
            tw_f32x16 acc[MS][NCB];
#pragma unroll
            for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[ms][cb][r] = 0.f;
            const int* sp = step_ptr + d.step_ptr;
            for (int c = 0; c < p.n_chunks; ++c) {
                const int k0 = c * p.k_chunk;
                const int kw = (p.K - k0) < p.k_chunk ? (p.K - k0) : p.k_chunk;
                load_a_block<MS>(p, smem, row0, k0, kw, wave, lane);
                __syncthreads();
                if (active)
                    run_steps<DT, MS, NCB>(acc, smem, p.a_pitch, p.blob + p.off_goff + (long)d.first_step * 32,
                                           p.blob + d.bvals_off, uni(sp[c]), uni(sp[c + 1]), lane);
                __syncthreads();
            }
            if (active) store_tile<DT, MS, NCB>(p, d, acc, stage, row0, lane);
        }
    }
    // the last workgroup to leave puts the counters back to zero for the next call
    if (tid == 0) {
        __threadfence();
        const int done = atomicAdd(&p.counters[1], 1);
        if (done == (int)gridDim.x - 1) {
            atomicExch(&p.counters[0], 0);
            atomicExch(&p.counters[1], 0);
        }
    }
}

// C[0:M, 0:N] = 0 for a weight with no surviving column.
__global__ void tw_zero_kernel(unsigned short* C, long ldc, int M, int N) {
    const long n = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long total = (long)M * N;
    for (long i = n; i < total; i += (long)gridDim.x * blockDim.x) C[(i / N) * ldc + (i % N)] = 0;
}

struct Plan {
    int ms;         // 32-row blocks per workgroup row block (1 or 2)
    int n_mblocks, n_seg, n_items;
    unsigned a_pitch, a_buf_bytes, stage_off, misc_off, lds_bytes;
};

constexpr unsigned kLdsLimit = 160 * 1024;

unsigned lds_need(int ms, int k_chunk) {
    const unsigned pitch = 2u * k_chunk + 8u;
    unsigned a = (32u * ms * pitch + 15u) & ~15u;
    return a + kWaves * TW_STAGE_BYTES + 16u;
}

int make_plan(const TwHeader* h, int M, int n_cu, Plan& pl) {
    if (lds_need(1, h->k_chunk) > kLdsLimit) return TW_ERR_UNSUPPORTED;
    const int T = h->T;
    auto items_for = [&](int ms, int& n_mblocks, int& n_seg) {
        n_mblocks = (M + 32 * ms - 1) / (32 * ms);
        if (h->n_chunks == 1) {
            // split a row block's tiles over several workgroups only when there are too few row blocks
            n_seg = 1;
            if (n_mblocks < n_cu) n_seg = (n_cu + n_mblocks - 1) / n_mblocks;
            if (n_seg > T) n_seg = T;
            if (n_seg < 1) n_seg = 1;
            return (long)n_mblocks * n_seg;
        }
        n_seg = (T + kWaves - 1) / kWaves;
        return (long)n_mblocks * n_seg;
    };
    int ms = 2;
    int nmb, nseg;
    if (lds_need(2, h->k_chunk) > kLdsLimit) ms = 1;
    if (ms == 2) {
        // 64-row blocks halve the traffic of packed B, but only pay when they still fill the GPU
        long it2 = items_for(2, nmb, nseg);
        if (it2 < n_cu) ms = 1;
        (void)it2;
    }
    long items = items_for(ms, nmb, nseg);
    if (items > 0x7fffffffL) return TW_ERR_UNSUPPORTED;
    pl.ms = ms;
    pl.n_mblocks = nmb; pl.n_seg = nseg; pl.n_items = (int)items;
    pl.a_pitch = 2u * h->k_chunk + 8u;
    pl.a_buf_bytes = (32u * ms * pl.a_pitch + 15u) & ~15u;
    pl.stage_off = pl.a_buf_bytes;
    pl.misc_off = pl.stage_off + kWaves * TW_STAGE_BYTES;
    pl.lds_bytes = pl.misc_off + 16u;
    return TW_OK;
}

typedef void (*KernelFn)(const TwGemmParams);

template <int DT, int MS, bool RES>
KernelFn pick_ncb(int ncb) {
    switch (ncb) {
        case 1: return tw_gemm_kernel<DT, MS, 1, RES>;
        case 2: return tw_gemm_kernel<DT, MS, 2, RES>;
        case 4: return tw_gemm_kernel<DT, MS, 4, RES>;
        default: return nullptr;
    }
}

template <int DT>
KernelFn pick_ms(int ms, bool res, int ncb) {
    if (res) return ms == 2 ? pick_ncb<DT, 2, true>(ncb) : pick_ncb<DT, 1, true>(ncb);
    return ms == 2 ? pick_ncb<DT, 2, false>(ncb) : pick_ncb<DT, 1, false>(ncb);
}

KernelFn pick_kernel(int dt, int ms, bool res, int ncb) {
    return dt == TW_F16 ? pick_ms<TW_F16>(ms, res, ncb) : pick_ms<TW_BF16>(ms, res, ncb);
}

int device_cus() {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return -1;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return -1;
    return n;
}

}  // namespace

extern "C" int tw_gemm_workspace(const void* blob_host, int M, size_t* ws_bytes) {
    if (!blob_host || !ws_bytes || M < 0) return TW_ERR_ARG;
    const TwHeader* h = (const TwHeader*)blob_host;
    if (h->magic != TW_MAGIC || h->version != TW_FORMAT_VERSION) return TW_ERR_BUF;
    *ws_bytes = 256;
    return TW_OK;
}

extern "C" int tw_gemm(const void* blob_host, const void* blob_dev, const void* A, int M, int lda, void* C,
                       int ldc, void* workspace, size_t ws_bytes, void* hip_stream) {
    if (!blob_host || !blob_dev || !A || !C || !workspace || M < 0) return TW_ERR_ARG;
    const TwHeader* h = (const TwHeader*)blob_host;
    if (h->magic != TW_MAGIC || h->version != TW_FORMAT_VERSION) return TW_ERR_BUF;
    if (ws_bytes < 256) return TW_ERR_BUF;
    if (lda < h->K || ldc < h->N) return TW_ERR_ARG;
    if ((lda & 7) != 0 || ((uintptr_t)A & 15) != 0 || ((uintptr_t)C & 1) != 0) return TW_ERR_ALIGN;
    if (((uintptr_t)blob_dev & 255) != 0 || ((uintptr_t)workspace & 255) != 0) return TW_ERR_ALIGN;
    if (M == 0) return TW_OK;
    hipStream_t stream = (hipStream_t)hip_stream;

    if (h->T == 0) {
        const long total = (long)M * h->N;
        int blocks = (int)((total + 255) / 256);
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(tw_zero_kernel, dim3(blocks), dim3(256), 0, stream, (unsigned short*)C, (long)ldc, M, h->N);
        return hipGetLastError() == hipSuccess ? TW_OK : TW_ERR_HIP;
    }

    const int n_cu = device_cus();
    if (n_cu <= 0) return TW_ERR_HIP;
    Plan pl;
    int rc = make_plan(h, M, n_cu, pl);
    if (rc) return rc;
    KernelFn fn = pick_kernel(h->dtype, pl.ms, h->n_chunks == 1, h->ncb);
    if (!fn) return TW_ERR_UNSUPPORTED;
    if (hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)pl.lds_bytes) != hipSuccess)
        return TW_ERR_HIP;

    TwGemmParams p;
    p.blob = (const unsigned char*)blob_dev;
    p.A = (const unsigned short*)A;
    p.C = (unsigned short*)C;
    p.counters = (int*)workspace;
    p.lda = lda; p.ldc = ldc;
    p.M = M; p.K = h->K; p.N = h->N; p.T = h->T;
    p.k_chunk = h->k_chunk; p.n_chunks = h->n_chunks;
    p.n_mblocks = pl.n_mblocks; p.n_seg = pl.n_seg; p.n_items = pl.n_items;
    p.a_pitch = pl.a_pitch; p.a_buf_bytes = pl.a_buf_bytes;
    p.stage_off = pl.stage_off; p.misc_off = pl.misc_off;
    p.off_sched_order = h->off_sched_order; p.off_tile_desc = h->off_tile_desc;
    p.off_step_ptr = h->off_step_ptr; p.off_goff = h->off_goff;

    int grid = pl.n_items < n_cu ? pl.n_items : n_cu;
    hipLaunchKernelGGL(fn, dim3(grid), dim3(kThreads), pl.lds_bytes, stream, p);
    return hipGetLastError() == hipSuccess ? TW_OK : TW_ERR_HIP;
}
