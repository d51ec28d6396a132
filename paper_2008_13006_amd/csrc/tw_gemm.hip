// tw_gemm: C = A . (B * mask) for a packed tile-wise weight, one persistent kernel on gfx950.
//
// Paper: Sec. VI.  The kernel in Listing 1 loads A tiles while skipping pruned K positions with a
// per-tile mask vector, multiplies them with pre-processed B tiles on the matrix unit and stores C
// skipping pruned columns; equal-width tiles are batched to share A and batches run concurrently
// to even out the load.  The paper stores A transposed in global memory so that skipping a K
// position skips a whole row.  This kernel keeps those ideas and changes the mechanics for CDNA4:
//   * A stays row-major in HBM.  A workgroup loads a block of A rows ONCE with coalesced 16-byte
//     loads and writes it K-MAJOR into LDS (the transposition happens on chip).  Every tile the
//     workgroup works on then gathers its kept K rows from that copy with transposing LDS reads
//     (ds_read_b64_tr_b16) whose row addresses come from the tile's kept-K list: two reads
//     deliver the eight contraction values of an MFMA operand.  Skipping never touches global
//     memory and A is shared by many tiles (the role of batching).
//   * The compacted tile values are stored offline in MFMA operand order and go from global
//     memory (L2-resident) straight to registers, a few steps ahead of their use.
//   * Workgroups are persistent and pull (row block, tile set) items from an atomic counter;
//     inside a workgroup the waves pull tiles, heaviest first (the role of stream concurrency).
//   * Pruned columns inside a tile's span are written as zeros together with the kept ones, in
//     contiguous pieces, through a small per-wave LDS staging area.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdlib>

#include "../../include/tw.h"
#include "tw_device.hpp"
#include "tw_format.h"

namespace {

constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
constexpr int kPrefetch = 3;  // B-operand steps in flight per wave

typedef short tw_i16x4 __attribute__((ext_vector_type(4)));

struct TwGemmParams {
    const unsigned char* blob;  // device copy
    const unsigned short* A;
    unsigned short* C;
    int* counters;              // [0] next item, [1] finished workgroups
    long lda, ldc;
    int M, K, N, T;
    int k_chunk, n_chunks, G;
    int n_mblocks, n_seg, n_items;
    unsigned at_pitch;          // bytes between K rows of the LDS copy of A (32*MS rows of A wide, padded)
    unsigned stage_off;         // LDS offset of the per-wave staging areas
    unsigned misc_off;          // LDS offset of two ints (item, tile counter)
    uint64_t off_sched_desc, off_step_ptr, off_goff, off_dpos, off_bvals;
#ifdef TW_EXPERIMENT
    int dbg;  // bit0: no A load, bit1: no main loop, bit2: no epilogue
    long long* trace;
#endif
};

__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }
// Returns x, but hides where it came from: values derived from the result are recomputed where they
// are used instead of being hoisted out of the persistent loop and kept (or spilled) across phases.
__device__ __forceinline__ int fresh(int x) {
    asm volatile("" : "+v"(x));
    return x;
}

// Wave-uniform copy of a schedule descriptor, in SGPRs.  The packed weight is read-only for the
// kernel, so descriptors are read through the constant address space: the compiler then uses scalar
// loads, which cost no vector registers and whose wait (lgkmcnt) does not depend on the wave's
// outstanding vector stores.  The compiler places the wait at the first use, so a descriptor requested
// early arrives while other work runs.
struct TileU {
    int w, span_start, span_w, nsteps, tile, step_ptr, first_step;
};
typedef const __attribute__((address_space(4))) int* tw_const_int_ptr;
__device__ __forceinline__ TileU fetch_tile(const TwGemmParams& p, int ti) {
    const uint64_t a = (uint64_t)(p.blob + p.off_sched_desc) + 32ull * (unsigned)ti;
    // the address is wave-uniform; say so to the compiler
    const uint64_t ua = ((uint64_t)(unsigned)uni((int)(a >> 32)) << 32) | (unsigned)uni((int)(unsigned)a);
    tw_const_int_ptr d = (tw_const_int_ptr)ua;
    TileU u;
    u.w = d[0]; u.span_start = d[1]; u.span_w = d[2]; u.nsteps = d[3];
    u.tile = d[4]; u.step_ptr = d[5]; u.first_step = d[6];
    return u;
}

// Cooperative load of A[row0 .. row0+32*MS) x [k0, k0+kw) into LDS, transposed: LDS row k (pitch
// at_pitch bytes) holds the 32*MS values A[row0 .. , k0+k].  A wave instruction reads 8 rows x 128
// contiguous bytes of A (8 lanes x 16 B per row) and scatters them with eight 2-byte LDS writes per
// lane.  Row k_chunk of the LDS copy is kept zero for padded contraction slots.
template <int MS>
__device__ __forceinline__ void load_a_block(const TwGemmParams& p, unsigned char* at, int row0, int k0, int kw,
                                             int wave, int lane_in, int tid_in) {
    const int lane = fresh(lane_in), tid = fresh(tid_in);
    constexpr int BM = 32 * MS;
    constexpr int RG = BM / 8;                 // groups of 8 rows
    const int octets = (kw + 7) >> 3;          // 16-byte pieces per row
    const int og_n = (octets + 7) >> 3;        // groups of 8 pieces
    const int tasks = RG * og_n;
    const int lr = lane >> 3, lo = lane & 7;
    constexpr int BATCH = 4;
    for (int t0 = wave; t0 < tasks; t0 += kWaves * BATCH) {
        tw_u32x4 v[BATCH];
        int oct[BATCH], row[BATCH];
#pragma unroll
        for (int b = 0; b < BATCH; ++b) {
            const int t = t0 + b * kWaves;
            const int rg = t % RG, og = t / RG;
            row[b] = rg * 8 + lr;
            oct[b] = og * 8 + lo;
            v[b] = tw_u32x4{0u, 0u, 0u, 0u};
            if (t < tasks && oct[b] < octets) {
                int grow = row0 + row[b];
                grow = grow < p.M ? grow : p.M - 1;   // rows past M: any valid row, never stored
                const int k = k0 + oct[b] * 8;
                const unsigned short* src = p.A + (long)grow * p.lda + k;
                if (k + 8 <= p.K) {
                    v[b] = *(const tw_u32x4*)src;
                } else {
                    unsigned short e[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) e[i] = (k + i < p.K) ? src[i] : (unsigned short)0;
                    v[b] = tw_u32x4{e[0] | ((unsigned)e[1] << 16), e[2] | ((unsigned)e[3] << 16),
                                    e[4] | ((unsigned)e[5] << 16), e[6] | ((unsigned)e[7] << 16)};
                }
            } else {
                oct[b] = -1;
            }
        }
#pragma unroll
        for (int b = 0; b < BATCH; ++b) {
            if (oct[b] >= 0) {
                unsigned char* dst = at + (unsigned)(oct[b] * 8) * p.at_pitch + row[b] * 2;
                const unsigned w[4] = {v[b].x, v[b].y, v[b].z, v[b].w};
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    *(unsigned short*)(dst + (unsigned)i * p.at_pitch) = (unsigned short)(w[i >> 1] >> (16 * (i & 1)));
            }
        }
    }
    if (tid < BM / 2) *(unsigned*)(at + (unsigned)p.k_chunk * p.at_pitch + tid * 4) = 0u;
}

// Steps [s0, s1) of one tile for this wave: gather A from LDS, stream packed B from global, MFMA.
// The packed B and the K indices of step s+kPrefetch are requested while step s is multiplied, and the
// LDS gather of step s+1 is issued before the MFMAs of step s, so both latencies hide behind MFMAs.
// The loop body has no branches except its exits (requests past the last step are clamped to the last
// step and never used), which keeps the compiler's wait counts exact.
template <int DT, int MS, int NCB>
__device__ __forceinline__ void run_steps(tw_f32x16 (&acc)[MS][NCB], const unsigned char* at, unsigned at_pitch,
                                          const unsigned char* goff_tile, const unsigned char* bvals_tile,
                                          int s0, int s1, int lane_in, int dbg = 0) {
    if (s0 >= s1) return;
    const int lane = fresh(lane_in);
    // lane l: 16-lane block b = l/16 covers rows 16*(b%2).. of the 32-row block, contraction half h = l/32;
    // inside the block, lane j addresses the K row of slot 8h + 4r + j/4 at row quad j%4
    const int h = lane >> 5, j = lane & 15;
    const unsigned lanebase = (unsigned)(((lane >> 4) & 1) * 16 + (j & 3) * 4) * 2;
    const unsigned char* gk = goff_tile + (h * 4 + (j >> 2)) * 4;   // this lane's two K indices of a step
    const unsigned char* bl = bvals_tile + lane * 16;
    const int last = s1 - 1;

    tw_u16x8 bq[kPrefetch][NCB];
    unsigned kk[kPrefetch];
    auto issue = [&](int slot, int s) {
        s = s < last ? s : last;
        kk[slot] = *(const unsigned*)(gk + (long)s * 32);
        const unsigned char* b = bl + ((long)s * NCB) * 1024;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) bq[slot][cb] = *(const tw_u16x8*)(b + cb * 1024);
    };
    auto gather = [&](tw_u16x8 (&a)[MS], unsigned k2) {
        const unsigned a0 = (k2 & 0xFFFFu) * at_pitch + lanebase;
        const unsigned a1 = (k2 >> 16) * at_pitch + lanebase;
#pragma unroll
        for (int ms = 0; ms < MS; ++ms) {
            const tw_i16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) tw_i16x4*)(at + a0 + ms * 64));
            const tw_i16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) tw_i16x4*)(at + a1 + ms * 64));
            a[ms] = tw_u16x8{(unsigned short)lo4[0], (unsigned short)lo4[1], (unsigned short)lo4[2],
                             (unsigned short)lo4[3], (unsigned short)hi4[0], (unsigned short)hi4[1],
                             (unsigned short)hi4[2], (unsigned short)hi4[3]};
        }
    };
#pragma unroll
    for (int i = 0; i < kPrefetch; ++i) issue(i, s0 + i);

    // two gather buffers used alternately (the unrolled body covers an even number of steps)
    tw_u16x8 a[2][MS];
    gather(a[0], kk[0]);
    constexpr int kUnroll = (kPrefetch % 2 == 0) ? kPrefetch : 2 * kPrefetch;
    auto step = [&](int i, int s) {
        const int slot = i % kPrefetch;
        gather(a[(i + 1) & 1], kk[(i + 1) % kPrefetch]);
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int ms = 0; ms < MS; ++ms) acc[ms][cb] = tw_mfma<DT>(a[i & 1][ms], bq[slot][cb], acc[ms][cb]);
#ifdef TW_EXPERIMENT
        if (!(dbg & 64))
#endif
        issue(slot, s + kPrefetch);
    };
    int s = s0;
    for (; s + kUnroll <= s1; s += kUnroll) {      // whole groups: no branch inside
#pragma unroll
        for (int i = 0; i < kUnroll; ++i) step(i, s + i);
    }
    const int rest = s1 - s;                        // 0 .. kUnroll-1 steps left
#pragma unroll
    for (int i = 0; i < kUnroll - 1; ++i)
        if (i < rest) step(i, s + i);
}

// Epilogue of one tile for this wave.  In this kernel the activations are the FIRST MFMA operand, so a
// lane owns one packed column of the tile (n = lane % 32 of every 32-column block) and its registers
// are rows: register r of a 32 x 32 block is row 8*(r/4) + 4*(lane/32) + r%4.  16 rows at a time, every
// lane writes its values into the wave's LDS staging area at the DESTINATION column of its packed
// column (2-byte writes; the staging area was cleared first, so pruned columns inside the span read
// back as zeros).  The staged rows are then read back 16 bytes at a time and stored to C as aligned
// 8-column groups; the two groups at the ragged ends of the span go out as aligned 8/4/2-byte pieces.
// LDS instructions of one wave execute in order, so the wave needs no waits between its own writes
// and reads of the staging area, only compiler barriers.
constexpr int kWinGroups = 18;                    // 8-column groups per staging window (144 columns)
constexpr int kStagePitch = kWinGroups * 16 + 16; // 304 bytes (16-byte aligned rows); the tail takes writes of absent columns
constexpr int kDummyOff = kWinGroups * 16;
constexpr int kReadIters = (kWinGroups + 3) / 4;  // wave instructions that read a window of 16 rows back
static_assert(16 * kStagePitch <= TW_STAGE_BYTES, "staging area too small");

__device__ __forceinline__ void tw_compiler_fence() { asm volatile("" ::: "memory"); }

// rows [16*HP, 16*HP+16) of one 32-row block -> staging rows 0..15
template <int DT, int NCB, int HP>
__device__ __forceinline__ void stage_cols(const tw_f32x16 (&acc)[NCB], unsigned char* wbase, const unsigned (&pos)[NCB]) {
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int rq = 0; rq < 2; ++rq)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                // one conversion per value: a packed conversion of two values followed by 2-byte stores
                // of the two halves was miscompiled by hipcc 7.2 (the low half was stored twice)
                const int r = 8 * HP + 4 * rq + rr;
                *(unsigned short*)(wbase + pos[cb] + (8 * rq + rr) * kStagePitch) = tw_cvt<DT>(acc[cb][r]);
            }
}

// columns [lo, hi) of an aligned group of 8 (16 bytes in v) -> aligned 8/4/2-byte stores
__device__ __forceinline__ void store_ragged(unsigned short* dst, const tw_u32x4& v, int lo, int hi) {
    const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int b = 4 * half;
        if (lo <= b && b + 4 <= hi) {
            *(tw_u32x2_a2*)(dst + b) = tw_u32x2{w[2 * half], w[2 * half + 1]};
        } else {
#pragma unroll
            for (int pr = 0; pr < 2; ++pr) {
                const int e = b + 2 * pr;
                const unsigned x = w[2 * half + pr];
                if (lo <= e && e + 2 <= hi) {
                    *(tw_u32_a2*)(dst + e) = x;
                } else {
                    if (lo <= e && e < hi) dst[e] = (unsigned short)x;
                    if (lo <= e + 1 && e + 1 < hi) dst[e + 1] = (unsigned short)(x >> 16);
                }
            }
        }
    }
}

template <int DT, int NCB, int MSI, int HP>
__device__ __forceinline__ void store_pass(const TwGemmParams& p, const tw_f32x16 (&acc)[NCB], unsigned char* stage,
                                           const unsigned (&pos)[NCB], int row0, int S, int E, int g_first, int ng,
                                           int lane_in, TwTrace& tr) {
    const int lane = fresh(lane_in);
    const int h = lane >> 5, trow = lane & 15, tg = lane >> 4;
    TW_MARK(tr, 100 + 2 * MSI + HP, lane);
    tw_compiler_fence();
    // clear the window, then write this pass's 16 rows
#pragma unroll
    for (int i = 0; i < (16 * kStagePitch + 1023) / 1024; ++i) {
        const int off = i * 1024 + lane * 16;
        if (off < 16 * kStagePitch) *(tw_u32x4*)(stage + off) = tw_u32x4{0u, 0u, 0u, 0u};
    }
    tw_compiler_fence();
    stage_cols<DT, NCB, HP>(acc, stage + 4 * h * kStagePitch, pos);
    tw_compiler_fence();
    TW_MARK(tr, 110, lane);
    const int grow = row0 + 32 * MSI + 16 * HP + trow;
    const unsigned char* rrow = stage + trow * kStagePitch + tg * 16;
    unsigned short* crow = p.C + (long)grow * p.ldc;
    tw_u32x4 v[kReadIters];
#pragma unroll
    for (int it = 0; it < kReadIters; ++it)
        if (4 * it < ng) v[it] = *(const tw_u32x4*)(rrow + it * 64);
#pragma unroll
    for (int it = 0; it < kReadIters; ++it) {
        if (4 * it < ng) {                                   // wave-uniform
            const int g = 4 * it + tg;
            const int col = (g_first + g) * 8;
#ifdef TW_EXPERIMENT
            if (!(p.dbg & 512))
#endif
            if (g < ng && grow < p.M && col >= S && col + 8 <= E) {
#ifdef TW_NT_STORE
                __builtin_nontemporal_store(v[it], (tw_u32x4_a2*)(crow + col));
#else
                *(tw_u32x4_a2*)(crow + col) = v[it];
#endif
            }
        }
    }
    // the ragged ends of the span: only the first and the last group of the whole span can be partial
    {
        const int g = tg == 0 ? 0 : ng - 1;                  // lanes 0-15: first group, 16-31: last group of the window
        const int col = (g_first + g) * 8;
        const bool ragged = (tg == 0 || (tg == 1 && ng > 1)) && (col < S || col + 8 > E);
#ifdef TW_EXPERIMENT
        if (!(p.dbg & 8))
#endif
        if (__builtin_amdgcn_ballot_w64(ragged) != 0ull) {
            if (ragged && grow < p.M) {
                const tw_u32x4 vr = *(const tw_u32x4*)(stage + trow * kStagePitch + g * 16);
                const int lo = S > col ? S - col : 0, hi = (E - col) < 8 ? (E - col) : 8;
                store_ragged(crow + col, vr, lo, hi);
            }
        }
    }
    tw_compiler_fence();
}

// dpos: destination columns of this lane's packed columns (one per 32-column block), counted from the
// aligned column at or below the span start
template <int DT, int MS, int NCB>
__device__ __forceinline__ void store_tile(const TwGemmParams& p, const TileU& d, tw_f32x16 (&acc)[MS][NCB],
                                           unsigned char* stage, const unsigned (&dpos)[NCB], int row0, int lane,
                                           TwTrace& tr) {
    const int S = d.span_start, E = d.span_start + d.span_w;
    const int G0 = S >> 3, G8 = ((E + 7) >> 3) - G0;
    for (int gw = 0; gw < G8; gw += kWinGroups) {            // one window unless the span is very wide
        const int ng = (G8 - gw) < kWinGroups ? (G8 - gw) : kWinGroups;
        unsigned pos[NCB];
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            const unsigned rel = dpos[cb] - (unsigned)(gw * 8);
            pos[cb] = rel < (unsigned)(ng * 8) ? rel * 2u : (unsigned)kDummyOff;
        }
        store_pass<DT, NCB, 0, 0>(p, acc[0], stage, pos, row0, S, E, G0 + gw, ng, lane, tr);
        store_pass<DT, NCB, 0, 1>(p, acc[0], stage, pos, row0, S, E, G0 + gw, ng, lane, tr);
        if constexpr (MS == 2) {
            store_pass<DT, NCB, 1, 0>(p, acc[1], stage, pos, row0, S, E, G0 + gw, ng, lane, tr);
            store_pass<DT, NCB, 1, 1>(p, acc[1], stage, pos, row0, S, E, G0 + gw, ng, lane, tr);
        }
    }
}

template <int MS, int NCB>
__device__ __forceinline__ void zero_acc(tw_f32x16 (&acc)[MS][NCB]) {
#pragma unroll
    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[ms][cb][r] = 0.f;
}

template <int DT, int MS, int NCB, bool RESIDENT>
__global__ __launch_bounds__(kThreads) void tw_gemm_kernel(const TwGemmParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int BM = 32 * MS;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = uni(tid >> 6);
    unsigned char* stage = smem + p.stage_off + wave * TW_STAGE_BYTES;
    volatile int* misc = (volatile int*)(smem + p.misc_off);
    const int* step_ptr = (const int*)(p.blob + p.off_step_ptr);

#ifdef TW_EXPERIMENT
    if (p.dbg & 16) return;
    TwTrace tr{p.trace ? p.trace + ((long)blockIdx.x * kWaves + wave) * 128 : nullptr, 0};
#else
    TwTrace tr{};
#endif
    TW_MARK(tr, 1, lane);
    // the first item of a workgroup is its own index, later ones come from the atomic counter
    for (int turn = 0;; ++turn) {
        if (tid == 0) {
            misc[0] = turn == 0 ? (int)blockIdx.x : (int)gridDim.x + atomicAdd(&p.counters[0], 1);
            misc[1] = 0;
        }
        __syncthreads();
        const int item = misc[0];
        if (item >= p.n_items) break;
        TW_MARK(tr, 2, lane);

        if constexpr (RESIDENT) {
            // the whole K extent of the row block stays in LDS; waves pull tiles of this item's set
            const int mb = item / p.n_seg, seg = item - mb * p.n_seg;
            const int row0 = mb * BM;
            // first tile of this wave: fetch its descriptor while A is being staged
            int i = 0;
            if (lane == 0) i = atomicAdd((int*)&misc[1], 1);
            int ti = seg + uni(i) * p.n_seg;
            TileU next = fetch_tile(p, ti < p.T ? ti : 0);
#ifdef TW_EXPERIMENT
            if (!(p.dbg & 1))
#endif
            load_a_block<MS>(p, smem, row0, 0, p.K, wave, lane, tid);
            TW_MARK(tr, 3, lane);
            __syncthreads();
            TW_MARK(tr, 4, lane);
#ifdef TW_EXPERIMENT
            if (p.dbg & 32) ti = p.T;
#endif
            while (ti < p.T) {
                const TileU d = next;
                TW_MARK(tr, 10, lane);
                // claim the next tile now so that its descriptor arrives during this tile's work
                if (lane == 0) i = atomicAdd((int*)&misc[1], 1);
                ti = seg + uni(i) * p.n_seg;
                next = fetch_tile(p, ti < p.T ? ti : 0);

                // destination columns of this lane's packed columns, needed only in the epilogue: request them now
                unsigned dpos[NCB];
                {
                    const unsigned* dp = (const unsigned*)(p.blob + p.off_dpos) + ((long)d.tile * 32 + (lane & 31)) * NCB;
#pragma unroll
                    for (int cb = 0; cb < NCB; ++cb) dpos[cb] = dp[cb];
                }
                tw_f32x16 acc[MS][NCB];
                zero_acc<MS, NCB>(acc);
#ifdef TW_EXPERIMENT
                if (!(p.dbg & 2))
#endif
                run_steps<DT, MS, NCB>(acc, smem, p.at_pitch, p.blob + p.off_goff + (long)d.first_step * 32,
                                       p.blob + p.off_bvals + (long)d.first_step * NCB * 1024, 0, d.nsteps, lane
#ifdef TW_EXPERIMENT
                                       , p.dbg
#endif
                                       );
                TW_MARK(tr, 20, lane);
#ifdef TW_EXPERIMENT
                if (!(p.dbg & 4))
#endif
                store_tile<DT, MS, NCB>(p, d, acc, stage, dpos, row0, lane, tr);
                TW_MARK(tr, 30, lane);
            }
            TW_MARK(tr, 40, lane);
            __syncthreads();  // everyone is done with the LDS copy of A and with misc[]
            TW_MARK(tr, 41, lane);
        } else {
            // K is streamed in chunks; wave w owns tile (8*set + w) of the kept-K ordering
            const int set = item / p.n_mblocks, mb = item - set * p.n_mblocks;
            const int row0 = mb * BM;
            const int ti = set * kWaves + wave;
            const bool active = ti < p.T;
            const TileU d = fetch_tile(p, active ? ti : 0);
            unsigned dpos[NCB];
            {
                const unsigned* dp = (const unsigned*)(p.blob + p.off_dpos) + ((long)d.tile * 32 + (lane & 31)) * NCB;
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb) dpos[cb] = dp[cb];
            }
            tw_f32x16 acc[MS][NCB];
            zero_acc<MS, NCB>(acc);
            const int* sp = step_ptr + d.step_ptr;
            for (int c = 0; c < p.n_chunks; ++c) {
                const int k0 = c * p.k_chunk;
                const int kw = (p.K - k0) < p.k_chunk ? (p.K - k0) : p.k_chunk;
                load_a_block<MS>(p, smem, row0, k0, kw, wave, lane, tid);
                __syncthreads();
                if (active)
                    run_steps<DT, MS, NCB>(acc, smem, p.at_pitch, p.blob + p.off_goff + (long)d.first_step * 32,
                                           p.blob + p.off_bvals + (long)d.first_step * NCB * 1024, uni(sp[c]),
                                           uni(sp[c + 1]), lane);
                __syncthreads();
            }
            if (active) store_tile<DT, MS, NCB>(p, d, acc, stage, dpos, row0, lane, tr);
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
    unsigned at_pitch, stage_off, misc_off, lds_bytes;
};

constexpr unsigned kLdsLimit = 160 * 1024;

unsigned at_bytes(int ms, int k_chunk) {
    const unsigned pitch = 64u * ms + 8u;
    return ((unsigned)(k_chunk + 1) * pitch + 15u) & ~15u;
}
unsigned lds_need(int ms, int k_chunk) { return at_bytes(ms, k_chunk) + kWaves * TW_STAGE_BYTES + 16u; }

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
        if (items_for(2, nmb, nseg) < n_cu) ms = 1;
    }
    const long items = items_for(ms, nmb, nseg);
    if (items > 0x7fffffffL) return TW_ERR_UNSUPPORTED;
    pl.ms = ms;
    pl.n_mblocks = nmb; pl.n_seg = nseg; pl.n_items = (int)items;
    pl.at_pitch = 64u * ms + 8u;
    pl.stage_off = at_bytes(ms, h->k_chunk);
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

// Per-device facts looked up once (the entries are written with the same value by every thread
// that races to fill them, so no lock is needed).
constexpr int kMaxDevices = 64;
std::atomic<int> g_cus[kMaxDevices];

int current_device() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return -1;
    return dev;
}

int device_cus(int dev) {
    int n = g_cus[dev].load(std::memory_order_relaxed);
    if (n > 0) return n;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return -1;
    g_cus[dev].store(n, std::memory_order_relaxed);
    return n;
}

// The dynamic-LDS limit of a kernel is raised to the hardware maximum once per (device, kernel).
constexpr int kMaxKernels = 24;
std::atomic<unsigned> g_lds_set[kMaxDevices][kMaxKernels];

int ensure_lds(int dev, int kernel_id, const void* fn) {
    if (g_lds_set[dev][kernel_id].load(std::memory_order_acquire)) return TW_OK;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit) != hipSuccess)
        return TW_ERR_HIP;
    g_lds_set[dev][kernel_id].store(1u, std::memory_order_release);
    return TW_OK;
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

    const int dev = current_device();
    if (dev < 0) return TW_ERR_HIP;
    const int n_cu = device_cus(dev);
    if (n_cu <= 0) return TW_ERR_HIP;
    Plan pl;
    int rc = make_plan(h, M, n_cu, pl);
    if (rc) return rc;
    KernelFn fn = pick_kernel(h->dtype, pl.ms, h->n_chunks == 1, h->ncb);
    if (!fn) return TW_ERR_UNSUPPORTED;
    const int kernel_id = (h->dtype == TW_F16 ? 0 : 12) + (pl.ms == 2 ? 0 : 6) + (h->n_chunks == 1 ? 0 : 3) +
                          (h->ncb == 4 ? 0 : h->ncb == 2 ? 1 : 2);
    rc = ensure_lds(dev, kernel_id, (const void*)fn);
    if (rc) return rc;

    TwGemmParams p;
    p.blob = (const unsigned char*)blob_dev;
    p.A = (const unsigned short*)A;
    p.C = (unsigned short*)C;
    p.counters = (int*)workspace;
    p.lda = lda; p.ldc = ldc;
    p.M = M; p.K = h->K; p.N = h->N; p.T = h->T;
    p.k_chunk = h->k_chunk; p.n_chunks = h->n_chunks; p.G = h->G;
    p.n_mblocks = pl.n_mblocks; p.n_seg = pl.n_seg; p.n_items = pl.n_items;
    p.at_pitch = pl.at_pitch;
    p.stage_off = pl.stage_off; p.misc_off = pl.misc_off;
    p.off_sched_desc = h->off_sched_desc; p.off_step_ptr = h->off_step_ptr; p.off_goff = h->off_goff;
    p.off_dpos = h->off_dpos; p.off_bvals = h->off_bvals;
#ifdef TW_EXPERIMENT
    p.dbg = getenv("TW_DBG") ? atoi(getenv("TW_DBG")) : 0;
    p.trace = getenv("TW_TRACE_PTR") ? (long long*)strtoull(getenv("TW_TRACE_PTR"), nullptr, 16) : nullptr;
#endif
    const int grid = pl.n_items < n_cu ? pl.n_items : n_cu;
    hipLaunchKernelGGL(fn, dim3(grid), dim3(kThreads), pl.lds_bytes, stream, p);
    return hipGetLastError() == hipSuccess ? TW_OK : TW_ERR_HIP;
}
