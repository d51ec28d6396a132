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
//   * Workgroups are persistent: one (row block, tile set) item each, further ones from an atomic
//     counter; inside a workgroup the waves pull tiles in the packer's dispatch order (the role of
//     stream concurrency).  When K does not fit in LDS, A is streamed through two LDS buffers.
//   * Pruned columns inside a tile's span are written as zeros together with the kept ones, as whole
//     128-byte lines of C, through a small per-wave LDS staging area.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdlib>
#include <cstring>
#include <type_traits>

#include "../../include/tw.h"
#include "tw_device.hpp"
#include "tw_format.h"

namespace {

constexpr int kWaves = TW_WAVES_PER_WG;
constexpr int kThreads = kWaves * 64;
// staging of A: resident K packs row pairs into 4-byte LDS writes, streamed K writes 2-byte values (see ATask)
constexpr bool kPairResident = true, kPairStream = false;
// B-operand steps in flight per wave: three; six for narrow tiles (at most two column blocks), whose steps
// are too short for three to cover the latency of an L2 hit and whose registers allow it
template <int NCB>
constexpr int prefetch_depth() { return NCB <= 2 ? 6 : 3; }
constexpr int kIdxAhead = 6;  // steps the K indices are requested ahead (they feed the LDS gather, which itself
                              // runs one step ahead of the MFMAs)

typedef short tw_i16x4 __attribute__((ext_vector_type(4)));
typedef float tw_f32x4 __attribute__((ext_vector_type(4)));

struct TwGemmParams {
    const unsigned char* blob;  // device copy
    const unsigned short* A;
    unsigned short* C;
    int* counters;              // [0] next item, [1] finished workgroups
    const unsigned short* bias; // fused epilogue: N values of the storage type, or null
    int act;                    // fused epilogue: tw_act
    long lda, ldc;
    int M, K, N, T;
    int k_chunk, n_chunks, G;
    int n_mblocks, n_seg, n_items;
    int tiles_per_set;          // MODE 2: tiles a workgroup holds (1..4: that many of the multiplying waves have one)
    int row_step;               // rows (tokens) from one row block to the next: 32*MS, or fewer (row-major boundary) so
                                // that the row blocks fill the last round of workgroups; rows past it are not stored
    unsigned at_pitch;          // bytes between K rows of the LDS copy of A (32*MS rows of A wide, padded)
    unsigned abuf_bytes;        // size of one LDS copy of A (streamed K uses two)
    unsigned stage_off;         // LDS offset of the per-wave staging areas
    unsigned misc_off;          // LDS offset of two ints (item, tile counter)
    uint64_t off_sched_desc, off_step_ptr, off_goff, off_dpos, off_bvals, off_zero_ptr, off_zero_cols, off_urow, off_ucnt;
    uint64_t off_ew_ptr, off_ew_goff, off_ew_b, off_xm_ptr, off_xm_goff, off_xm_b, off_zero_xc;
    int has_ew;                 // the blob carries an element-wise residual (TEW)
    uint64_t off_xc_tile_ptr, off_xc_col, off_xc_ptr, off_xc_k, off_xc_v;
    unsigned xbuf_off;          // LDS offset of the per-wave areas for residual-only columns (TEW), 0: the tiles' kernel
                                // leaves those columns to the pass of their own
    int stream_stores;          // rows of the output start on 128-byte boundaries: stores that complete whole lines
                                // may carry the streaming hint
    unsigned urow_off;          // LDS offset of the loading waves' row lists (transposed, streamed K, few tiles), 0: none
    // split K (streamed K, wave per tile, few row blocks): the K chunks are cut into n_parts runs of chunks_per_part
    // and an item is (part, tile set, row block); the tiles' fp32 results go to `partials`
    // ([part][row block][tile in dispatch order][MS][NCB][4 register groups][64 lanes][4]) and
    // tw_splitk_reduce_kernel adds them up in the order of the parts and stores C.  n_parts = 1: no split.
    int n_parts, chunks_per_part;
    float* partials;
};

__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }
// bytes between K rows of the LDS copy of A: 32*MS rows of A wide, padded by 8 (a compile-time value, so that the
// eight K rows a staging request writes to are immediate offsets of its LDS writes, not a multiplication each)
template <int MS> constexpr unsigned at_pitch_of() { return 64u * MS + 8u; }
// one past the last row of the row block that starts at row0
__device__ __forceinline__ int block_end(const TwGemmParams& p, int row0) {
    const int e = row0 + p.row_step;
    return e < p.M ? e : p.M;
}
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
    int w, span_start, span_w, nsteps, tile, step_ptr, first_step, xc;
};
typedef const __attribute__((address_space(4))) int* tw_const_int_ptr;
__device__ __forceinline__ TileU fetch_tile(const TwGemmParams& p, int ti) {
    const uint64_t a = (uint64_t)(p.blob + p.off_sched_desc) + 32ull * (unsigned)ti;
    // the address is wave-uniform; say so to the compiler
    const uint64_t ua = ((uint64_t)(unsigned)uni((int)(a >> 32)) << 32) | (unsigned)uni((int)(unsigned)a);
    tw_const_int_ptr d = (tw_const_int_ptr)ua;
    TileU u;
    u.w = d[0]; u.span_start = d[1]; u.span_w = d[2]; u.nsteps = d[3];
    u.tile = d[4]; u.step_ptr = d[5]; u.first_step = d[6]; u.xc = d[7];
    return u;
}

// Element idx of a read-only int table, wave-uniform, through a scalar load (see fetch_tile).
__device__ __forceinline__ int fetch_int(const int* table, int idx) {
    const uint64_t a = (uint64_t)(table + idx);
    const uint64_t ua = ((uint64_t)(unsigned)uni((int)(a >> 32)) << 32) | (unsigned)uni((int)(unsigned)a);
    return *(tw_const_int_ptr)ua;
}

// Cooperative load of A[row0 .. row0+32*MS) x [k0, k0+kw) into LDS, transposed: LDS row k (pitch
// at_pitch bytes) holds the 32*MS values A[row0 .. , k0+k].  Row k_chunk of the LDS copy is kept zero
// for padded contraction slots; rows k_chunk+1 .. k_chunk+8 take the writes of absent pieces.
// A lane always reads 16-byte pieces (8 columns of one row).  Two ways of cutting the work into tasks:
//   PAIR = false (streamed K): a task is 8 rows x 64 columns; lane l reads piece l%8 of row l/8 (a wave
//     instruction reads 128 contiguous bytes of 8 rows, what streams best from HBM) and scatters its
//     values with eight 2-byte LDS writes.  One request per task.
//   PAIR = true (resident K): a task is 32 rows x 32 columns; lane l reads piece l/16 of the two rows
//     2*(l%16) and 2*(l%16)+1, and the two rows' values of a column go into one 32-bit word: eight
//     4-byte LDS writes per two requests, whose 64 lanes hit 64 different banks (the four pieces lie 16
//     banks apart, the 16 row pairs in consecutive words).  Two requests per task.
// Wave w takes tasks w, w+stride, ...  Neither the loads nor the LDS writes carry branches: a request
// for an absent piece re-reads a valid one and its values go to the spare rows, so all requests of a
// batch are outstanding together.  lda is a multiple of 8 elements, so the bytes past column K-1 of a
// row still belong to that row's pitch; they are dropped at the LDS write (only a width that is not a
// multiple of 8 needs that test).  BATCH counts requests.
template <int BATCH>
struct ARegs {
    tw_u32x4 v[BATCH];
};

// A 16-byte request for activations.  NTA (compile time, one kernel variant each): with the streaming hint when this
// workgroup is the only one that reads these rows (one set of tiles per row block: the rows then do not push the
// packed weights out of the L2; 2 to 6 us on the streamed workloads), plain when the tiles of a row block are split
// into sets whose workgroups read the same rows one after the other (the later ones then hit in the L2; the skewed
// FFN-down of BERT-large: 45 us against 49, transposed 41 against 50).
template <bool NTA>
__device__ __forceinline__ tw_u32x4 load_a16(const unsigned short* src) {
    if constexpr (NTA) return tw_load16_stream(src);
    else return *(const tw_u32x4*)src;
}

template <int MS, bool PAIR>
struct ATask {
    int row, oc;      // (first) row of the lane, 16-byte piece of the row
    bool have;
    __device__ __forceinline__ ATask(int t, int kw, int lane) {
        const int octets = (kw + 7) >> 3;           // 16-byte pieces per row
        if constexpr (PAIR) {
            const int tasks = MS * ((octets + 3) >> 2);
            const int tc = t < tasks ? t : tasks - 1;
            row = (tc % MS) * 32 + 2 * (lane & 15);
            const int o = (tc / MS) * 4 + (lane >> 4);
            have = t < tasks && o < octets;
            oc = o < octets ? o : octets - 1;
        } else {
            constexpr int RG = 4 * MS;              // groups of 8 rows
            const int tasks = RG * ((octets + 7) >> 3);
            const int tc = t < tasks ? t : tasks - 1;
            row = (tc % RG) * 8 + (lane >> 3);
            const int o = (tc / RG) * 8 + (lane & 7);
            have = t < tasks && o < octets;
            oc = o < octets ? o : octets - 1;
        }
    }
};
template <int MS, bool PAIR>
__device__ __forceinline__ int a_tasks(int kw) {
    const int octets = (kw + 7) >> 3;
    return PAIR ? MS * ((octets + 3) >> 2) : 4 * MS * ((octets + 7) >> 3);
}

// requests tasks t0, t0+stride, ... of the block (BATCH requests); stride = number of loading waves
template <int MS, int BATCH, bool PAIR, bool NTA = true>
__device__ __forceinline__ void a_issue(const TwGemmParams& p, ARegs<BATCH>& ar, int row0, int k0, int kw, int t0,
                                        int lane_in, int stride = kWaves) {
    const int lane = fresh(lane_in);
    const int mend = block_end(p, row0);
    if constexpr (PAIR) {
        static_assert(BATCH % 2 == 0, "two requests per task");
#pragma unroll
        for (int b = 0; b < BATCH / 2; ++b) {
            const ATask<MS, true> t(t0 + b * stride, kw, lane);
            int g0 = row0 + t.row, g1 = g0 + 1;
            g0 = g0 < mend ? g0 : mend - 1;           // rows past the block's end: any valid row, never stored
            g1 = g1 < mend ? g1 : mend - 1;
            // (plain loads: with K resident the streaming hint measured 1.5 us slower on the BERT-base shapes;
            // the streamed paths below gain 2 to 6 us from it)
            ar.v[2 * b] = *(const tw_u32x4*)(p.A + (long)g0 * p.lda + (k0 + t.oc * 8));
            ar.v[2 * b + 1] = *(const tw_u32x4*)(p.A + (long)g1 * p.lda + (k0 + t.oc * 8));
        }
    } else {
#pragma unroll
        for (int b = 0; b < BATCH; ++b) {
            const ATask<MS, false> t(t0 + b * stride, kw, lane);
            int grow = row0 + t.row;
            grow = grow < mend ? grow : mend - 1;
            ar.v[b] = load_a16<NTA>(p.A + (long)grow * p.lda + (k0 + t.oc * 8));
        }
    }
}

// writes what a_issue requested into the LDS copy `at`
template <int MS, int BATCH, bool PAIR>
__device__ __forceinline__ void a_commit(const TwGemmParams& p, const ARegs<BATCH>& ar, unsigned char* at, int kw, int t0,
                                         int lane_in, int stride = kWaves) {
    const int lane = fresh(lane_in);
    const int dump = p.k_chunk + 1;
    const bool tail = (kw & 7) != 0;                  // wave-uniform
    if constexpr (PAIR) {
#pragma unroll
        for (int b = 0; b < BATCH / 2; ++b) {
            const ATask<MS, true> t(t0 + b * stride, kw, lane);
            const int kcol = t.have ? t.oc * 8 : dump;
            unsigned char* dst = at + (unsigned)kcol * at_pitch_of<MS>() + t.row * 2;
            const unsigned x[4] = {ar.v[2 * b].x, ar.v[2 * b].y, ar.v[2 * b].z, ar.v[2 * b].w};
            const unsigned y[4] = {ar.v[2 * b + 1].x, ar.v[2 * b + 1].y, ar.v[2 * b + 1].z, ar.v[2 * b + 1].w};
            unsigned w[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                w[i] = (i & 1) ? ((x[i >> 1] >> 16) | (y[i >> 1] & 0xFFFF0000u)) : ((x[i >> 1] & 0xFFFFu) | (y[i >> 1] << 16));
            if (!tail) {
#pragma unroll
                for (int i = 0; i < 8; ++i) *(unsigned*)(dst + (unsigned)i * at_pitch_of<MS>()) = w[i];
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (kcol + i < kw || kcol == dump) *(unsigned*)(dst + (unsigned)i * at_pitch_of<MS>()) = w[i];
            }
        }
    } else {
#pragma unroll
        for (int b = 0; b < BATCH; ++b) {
            const ATask<MS, false> t(t0 + b * stride, kw, lane);
            const int kcol = t.have ? t.oc * 8 : dump;
            unsigned char* dst = at + (unsigned)kcol * at_pitch_of<MS>() + t.row * 2;
            const unsigned w[4] = {ar.v[b].x, ar.v[b].y, ar.v[b].z, ar.v[b].w};
            if (!tail) {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    *(unsigned short*)(dst + (unsigned)i * at_pitch_of<MS>()) = (unsigned short)(w[i >> 1] >> (16 * (i & 1)));
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (kcol + i < kw || kcol == dump)
                        *(unsigned short*)(dst + (unsigned)i * at_pitch_of<MS>()) = (unsigned short)(w[i >> 1] >> (16 * (i & 1)));
            }
        }
    }
}

__device__ __forceinline__ void a_zero_row(const TwGemmParams& p, unsigned char* at, int bm, int tid) {
    if (tid < bm / 2) *(unsigned*)(at + (unsigned)p.k_chunk * p.at_pitch + tid * 4) = 0u;
}

// whole block, BATCH requests per wave in flight at a time (12 cover 64 rows x 768 columns)
template <int MS, int BATCH, bool PAIR, bool NTA = true>
__device__ __forceinline__ void load_a_block(const TwGemmParams& p, unsigned char* at, int row0, int k0, int kw,
                                             int wave, int lane, int tid) {
    const int tasks = a_tasks<MS, PAIR>(kw);
    for (int t0 = wave; t0 < tasks; t0 += kWaves * (PAIR ? BATCH / 2 : BATCH)) {
        ARegs<BATCH> ar;
        a_issue<MS, BATCH, PAIR, NTA>(p, ar, row0, k0, kw, t0, lane);
        a_commit<MS, BATCH, PAIR>(p, ar, at, kw, t0, lane);
    }
    a_zero_row(p, at, 32 * MS, tid);
}

// Operand registers of the main loop: packed B of the next kPrefetch steps, K indices of the next
// kIdxAhead steps.
template <int NCB>
struct StepRegs {
    tw_u16x8 bq[prefetch_depth<NCB>()][NCB];
    unsigned kk[kIdxAhead];
};

// Requests the packed B of step s (clamped to `last`) of a tile into slot `slot`.
template <int NCB>
__device__ __forceinline__ void issue_b(StepRegs<NCB>& rg, int slot, const unsigned char* bl, int s, int last) {
    s = s < last ? s : last;
    const unsigned char* b = bl + ((long)s * NCB) * 1024;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
        rg.bq[slot][cb] = *(const tw_u16x8*)(b + cb * 1024);
    }
}
// Requests this lane's two K indices of step s (clamped to `last`) into slot `slot`.
template <int NCB>
__device__ __forceinline__ void issue_k(StepRegs<NCB>& rg, int slot, const unsigned char* gk, int s, int last) {
    s = s < last ? s : last;
    rg.kk[slot] = *(const unsigned*)(gk + (long)s * 32);
}

// Requests the first steps of a tile; the range [s0, s1) must not be empty.
template <int NCB>
__device__ __forceinline__ void prefetch_first_steps(StepRegs<NCB>& rg, const unsigned char* goff_tile,
                                                     const unsigned char* bvals_tile, int s0, int s1, int lane_in) {
    const int lane = fresh(lane_in);
    const unsigned char* gk = goff_tile + ((lane >> 5) * 4 + ((lane & 15) >> 2)) * 4;
    const unsigned char* bl = bvals_tile + lane * 16;
#pragma unroll
    for (int i = 0; i < kIdxAhead; ++i) issue_k<NCB>(rg, i, gk, s0 + i, s1 - 1);
#pragma unroll
    for (int i = 0; i < prefetch_depth<NCB>(); ++i) issue_b<NCB>(rg, i, bl, s0 + i, s1 - 1);
}

// Steps [s0, s1) (not empty) of one tile for this wave: gather A from LDS, stream packed B from global, MFMA.
// Expects the first steps in `rg` (prefetch_first_steps).  The packed B of step s+kPrefetch and the K
// indices of step s+kIdxAhead are requested while step s is multiplied, and the LDS gather of step s+1
// is issued before the MFMAs of step s, so both latencies hide behind MFMAs.  The loop body has no branches
// except its exits (requests past the last step are clamped to the last step and never used), which
// keeps the compiler's wait counts exact.
template <int DT, int MS, int NCB>
__device__ __forceinline__ void run_steps(tw_f32x16 (&acc)[MS][NCB], StepRegs<NCB>& rg, const unsigned char* at,
                                          unsigned at_pitch, const unsigned char* goff_tile,
                                          const unsigned char* bvals_tile, int s0, int s1, int lane_in) {
    const int lane = fresh(lane_in);
    // lane l: 16-lane block b = l/16 covers rows 16*(b%2).. of the 32-row block, contraction half h = l/32;
    // inside the block, lane j addresses the K row of slot 8h + 4r + j/4 at row quad j%4
    const int h = lane >> 5, j = lane & 15;
    const unsigned lanebase = (unsigned)(((lane >> 4) & 1) * 16 + (j & 3) * 4) * 2;
    const unsigned char* gk = goff_tile + (h * 4 + (j >> 2)) * 4;   // this lane's two K indices of a step
    const unsigned char* bl = bvals_tile + lane * 16;
    const int last = s1 - 1;

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
    // two gather buffers used alternately (the unrolled body covers an even number of steps)
    // (both start defined: an undefined second buffer would be carried around the tile loop as a live value)
    tw_u16x8 a[2][MS];
#pragma unroll
    for (int ms = 0; ms < MS; ++ms) a[1][ms] = tw_u16x8{0, 0, 0, 0, 0, 0, 0, 0};
    gather(a[0], rg.kk[0]);
    constexpr int kPrefetch = prefetch_depth<NCB>();
    constexpr int kUnroll = 6;                      // a multiple of 2, kPrefetch and kIdxAhead
    static_assert(kUnroll % 2 == 0 && kUnroll % kPrefetch == 0 && kUnroll % kIdxAhead == 0, "unroll factor");
    auto step = [&](int i, int s) {
        // the three stages keep this order: left alone, the instruction scheduler sinks the loads of
        // later steps next to their first use and the prefetch distance is lost
        gather(a[(i + 1) & 1], rg.kk[(i + 1) % kIdxAhead]);
        __builtin_amdgcn_sched_barrier(0);
        // the request for a column block of step s+kPrefetch follows the MFMAs that read its registers:
        // the requests reach the memory pipeline spread over the step instead of in a burst
        const int sb = (s + kPrefetch) < last ? (s + kPrefetch) : last;
        const unsigned char* bnext = bl + ((long)sb * NCB) * 1024;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
#pragma unroll
            for (int ms = 0; ms < MS; ++ms)
                acc[ms][cb] = tw_mfma<DT>(a[i & 1][ms], rg.bq[i % kPrefetch][cb], acc[ms][cb]);
            __builtin_amdgcn_sched_barrier(0);
            rg.bq[i % kPrefetch][cb] = *(const tw_u16x8*)(bnext + cb * 1024);
            __builtin_amdgcn_sched_barrier(0);
        }
        issue_k<NCB>(rg, i % kIdxAhead, gk, s + kIdxAhead, last);
        __builtin_amdgcn_sched_barrier(0);
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
// are rows: register r of a 32 x 32 block is row 8*(r/4) + 4*(lane/32) + r%4, i.e. four consecutive
// rows per group of four registers.
//
// What the stores cost is the number of (128-byte line of C, store instruction) pairs, so every store
// instruction should cover whole lines.  The wave's LDS staging window therefore starts at the
// 64-column (128-byte) boundary at or below the tile's span and is up to four lines wide.  It is kept
// COLUMN-major: per destination column the four rows a lane holds are contiguous, so a lane stages
// the four rounded values of a register group with ONE 8-byte LDS write at the destination column of
// its packed column.  Two planes hold rows 0-3 and 4-7 of the eight rows of a pass (the two lane
// halves), each [256 columns][4 rows] followed by one spare slot per lane for absent columns; the
// second plane is skewed by 32 bytes so that reads of both planes use disjoint banks.  The window is
// cleared once per tile: every pass writes the same columns, so the pruned columns inside the span
// keep reading back as zeros.  The read-back uses the transposing LDS read (ds_read_b64_tr_b16):
// within 16 lanes, lane 4e+g supplies the address of column (c_g + e), rows (4 values), and lane
// 4g+x receives row x of columns c_g .. c_g+3.  Two such reads give a lane eight consecutive columns
// of one row (16 bytes), and a store instruction writes one 128-byte line of eight rows.  Groups that
// straddle the ends of the span go out as one 2-byte store per lane, end and pass.
// LDS instructions of one wave execute in order, so the wave needs no waits between its own writes
// and reads of the staging area, only compiler barriers; the writes of pass P+1 are issued behind
// the reads of pass P and ahead of the wait for them.
constexpr int kLineCols = 64;                       // columns in a 128-byte line of C
constexpr int kWinLines = 4;                        // lines per staging window
constexpr int kWinCols = kWinLines * kLineCols;     // 256
constexpr int kSpareOff = kWinCols * 8;             // spare slots behind the window of a plane
constexpr int kPlaneBytes = kWinCols * 8 + 32 * 8 + 32;
constexpr unsigned kStageBytes = 2 * kPlaneBytes;   // per wave
static_assert(kPlaneBytes % 16 == 0 && (kPlaneBytes / 4) % 16 == 8, "plane skew");

__device__ __forceinline__ void tw_compiler_fence() { asm volatile("" ::: "memory"); }

__device__ __forceinline__ tw_i16x4 tw_lds_read_tr(const unsigned char* a) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) tw_i16x4*)a);
}

// dpos: destination columns of this lane's packed columns (one per 32-column block), counted from the
// 8-aligned column at or below the span start.
// Fused epilogue (p.bias and / or p.act): `eb` holds the bias of this lane's packed columns and of the
// four columns lane, lane+64, .. of the first staging window (see fetch_epi_bias).
template <int NCB>
struct EpiBias {
    float col[NCB];
    float fill[kWinLines];
};

// Reads what store_tile needs of the bias.
template <int DT, int NCB>
__device__ __forceinline__ void fetch_epi_bias(const TwGemmParams& p, const TileU& d, const unsigned (&dpos)[NCB],
                                               EpiBias<NCB>& eb, int lane) {
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) eb.col[cb] = 0.f;
#pragma unroll
    for (int l = 0; l < kWinLines; ++l) eb.fill[l] = 0.f;
    if (p.bias != nullptr) {                                // wave-uniform
        const int origin = d.span_start & ~7, E = d.span_start + d.span_w;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
            if (dpos[cb] != 0xFFFFFFFFu) eb.col[cb] = tw_to_f32<DT>(p.bias[origin + (int)dpos[cb]]);
        if (d.span_w != d.w) {                              // pruned columns inside the span: they hold act(bias)
            const int W0 = d.span_start & ~(kLineCols - 1);
#pragma unroll
            for (int l = 0; l < kWinLines; ++l) {
                const int c = W0 + l * kLineCols + lane;
                if (c >= d.span_start && c < E) eb.fill[l] = tw_to_f32<DT>(p.bias[c]);
            }
        }
    }
}

// The fused epilogue's arithmetic, in place on the accumulators and kept apart from the store code, so that
// the plain path's code and registers stay as they are.
template <int MS, int NCB>
__device__ __forceinline__ void apply_bias_act(tw_f32x16 (&acc)[MS][NCB], const EpiBias<NCB>& eb, int act) {
    // The (wave-uniform) choice of the activation is taken once per 32 x 32 block, not once around three loops
    // over all accumulators: with one big three-way branch the register allocator moves accumulators out to
    // scratch memory on every path, the plain bias included.
#pragma unroll
    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            if (act == TW_ACT_GELU) {
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[ms][cb][r] = tw_gelu(acc[ms][cb][r] + eb.col[cb]);
            } else if (act == TW_ACT_RELU) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float x = acc[ms][cb][r] + eb.col[cb];
                    acc[ms][cb][r] = x > 0.f ? x : 0.f;
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[ms][cb][r] += eb.col[cb];
            }
        }
}

// FUSED: the kernel variant with the fused epilogue (a bias and / or an activation); the plain variant
// carries none of its code.
template <int DT, int MS, int NCB, bool FUSED>
__device__ __forceinline__ void store_tile(const TwGemmParams& p, const TileU& d, tw_f32x16 (&acc)[MS][NCB],
                                           unsigned char* stage, const unsigned (&dpos)[NCB], int row0, int lane_in,
                                           unsigned short* xbuf = nullptr,
                                           const int* xcols = nullptr,
                                           int pass0 = 0, int pass1 = 4 * MS) {
    // (pass0, pass1: the passes to run, each eight rows of the block; everything by default.  The second kernel
    // of a split-K product gives a wave one pass of a tile.)
    const int lane = fresh(lane_in);
    constexpr bool fused = FUSED;
    // Residual-only columns of a TEW blob inside this tile's span (Sec. IV-A "Hybrid Pattern": weights restored in a
    // column that the tile-wise pattern pruned altogether).  With K resident the tile that owns the span has computed
    // them (xc_columns) into `xbuf` (16-bit, [column][row % 8][row / 8]); every pass puts its eight rows of them into the staging
    // window, where the pruned columns otherwise read back as zeros - so they leave with the tile's own stores.
    const int nx = xbuf != nullptr ? (int)((unsigned)d.xc >> 26) : 0;   // wave-uniform
    EpiBias<NCB> eb;
    if constexpr (FUSED) {
        fetch_epi_bias<DT, NCB>(p, d, dpos, eb, lane);
        apply_bias_act<MS, NCB>(acc, eb, p.act);
    }
    const int h = lane >> 5, n = lane & 31;
    const int blk = lane >> 4, j = lane & 15;
    // read-back, as the lane that supplies an address: column offset e, group g -> (piece, row quad)
    const int in_piece = 2 * blk + (j & 1), in_rq = (j >> 1) & 1, in_e = j >> 2;
    // read-back, as the lane that receives: group g = j / 4, row x = j % 4 of the quad
    const int piece = 2 * blk + ((j >> 2) & 1), orow = 4 * (j >> 3) + (j & 3);
    const int trow = lane >> 3, tg = lane & 7;              // element-wise stores: row, element of a group
    const int S = d.span_start, E = d.span_start + d.span_w;
    const int W0 = S & ~(kLineCols - 1);
    const unsigned shift = (unsigned)((S & ~7) - W0);       // dpos counts from S & ~7
    constexpr int NP = 4 * MS;
    const int rows_left = block_end(p, row0) - (row0 + orow);   // pass P stores this lane's row iff 8P < rows_left
    for (int win0 = W0; win0 < E; win0 += kWinCols) {       // one window unless the span is very wide
        const int left = E - win0;
        const int nl = left >= kWinCols ? kWinLines : (left + kLineCols - 1) / kLineCols;
        unsigned char* wpos[NCB];
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            const unsigned rel = dpos[cb] + shift - (unsigned)(win0 - W0);   // wraps for columns left of the window
            wpos[cb] = stage + h * kPlaneBytes + (rel < (unsigned)kWinCols ? rel * 8u : (unsigned)(kSpareOff + n * 8));
        }
        const unsigned char* rpos = stage + in_rq * kPlaneBytes + (8 * in_piece + in_e) * 8;
        bool okl[kWinLines], whole[kWinLines];
#pragma unroll
        for (int l = 0; l < kWinLines; ++l) {
            const int col = win0 + l * kLineCols + piece * 8;
            okl[l] = l < nl && col >= S && col + 8 <= E;
            // the span covers this line from end to end (wave-uniform): nobody else writes into it
            whole[l] = p.stream_stores != 0 && win0 + l * kLineCols >= S && win0 + (l + 1) * kLineCols <= E;
        }
        unsigned short* cptr = p.C + (long)(row0 + orow) * p.ldc + (win0 + piece * 8);
        // partial groups at the two ends of the span, if they lie in this window (window-relative index)
        int g_first = -1, g_last = -1;
        if ((S & 7) != 0 && win0 == W0) g_first = (S - win0) >> 3;
        if ((E & 7) != 0 && left <= kWinCols) g_last = (E - 1 - win0) >> 3;
        const int colF = win0 + g_first * 8 + tg, colL = win0 + g_last * 8 + tg;   // this lane's element
        const bool inF = g_first >= 0 && colF >= S && colF < E;
        const bool inL = g_last >= 0 && colL >= S && colL < E;
        const unsigned char* ragbase = stage + (trow >> 2) * kPlaneBytes + (trow & 3) * 2;
        const unsigned char* ragF = ragbase + ((g_first < 0 ? 0 : g_first) * 8 + tg) * 8;
        const unsigned char* ragL = ragbase + ((g_last < 0 ? 0 : g_last) * 8 + tg) * 8;
        unsigned short* rptr = p.C + (long)(row0 + trow) * p.ldc;
        const int rag_left = block_end(p, row0) - (row0 + trow);

        // residual-only columns: lane l handles column l / 8 (and l / 8 + 8) of the tile's list, row l % 8 of a pass
        unsigned char* xpos[TW_XC_INLINE / 8];
#pragma unroll
        for (int g = 0; g < TW_XC_INLINE / 8; ++g) {
            xpos[g] = nullptr;
            const int j = 8 * g + (lane >> 3);
            if (j < nx) {
                const unsigned rel = (unsigned)(xcols[g] - win0);
                if (rel < (unsigned)kWinCols) xpos[g] = stage + ((lane >> 2) & 1) * kPlaneBytes + rel * 8u + (lane & 3) * 2;
            }
        }
        tw_u32x4 xq[TW_XC_INLINE / 8];                       // this lane's row of its columns, all passes
#pragma unroll
        for (int g = 0; g < TW_XC_INLINE / 8; ++g) {
            xq[g] = tw_u32x4{0u, 0u, 0u, 0u};
            if (nx > 0) xq[g] = *(const tw_u32x4*)(xbuf + (8 * g + (lane >> 3)) * 64 + (lane & 7) * 8);
        }
        auto write_pass = [&](int P) {
            const int ms = P >> 2, q = P & 3;
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
                tw_u32x2 v;
                v.x = (unsigned)tw_cvt<DT>(acc[ms][cb][4 * q + 0]) | ((unsigned)tw_cvt<DT>(acc[ms][cb][4 * q + 1]) << 16);
                v.y = (unsigned)tw_cvt<DT>(acc[ms][cb][4 * q + 2]) | ((unsigned)tw_cvt<DT>(acc[ms][cb][4 * q + 3]) << 16);
                *(tw_u32x2*)wpos[cb] = v;
            }
            if (nx > 0) {                                    // wave-uniform
#pragma unroll
                for (int g = 0; g < TW_XC_INLINE / 8; ++g)
                    if (xpos[g] != nullptr)
                        *(unsigned short*)xpos[g] = (unsigned short)(xq[g][P >> 1] >> (16 * (P & 1)));
            }
        };

        // clear both planes once: the passes all write the same columns.  With a fused epilogue a pruned
        // column holds act(bias) in every row instead of zero.
        tw_compiler_fence();
        if (!fused || d.span_w == d.w) {
#pragma unroll
            for (int pl = 0; pl < 2; ++pl)
#pragma unroll
                for (int i = 0; i < kWinCols * 8 / 1024; ++i)
                    *(tw_u32x4*)(stage + pl * kPlaneBytes + i * 1024 + lane * 16) = tw_u32x4{0u, 0u, 0u, 0u};
        } else {
#pragma unroll
            for (int l = 0; l < kWinLines; ++l) {
                const int c = win0 + l * kLineCols + lane;
                float b = eb.fill[l];
                if (win0 != W0) b = (p.bias != nullptr && c >= S && c < E) ? tw_to_f32<DT>(p.bias[c]) : 0.f;   // later windows: read here
                const unsigned hv = (c >= S && c < E) ? (unsigned)tw_cvt<DT>(tw_activate(b, p.act)) : 0u;
                const tw_u32x2 v{hv | (hv << 16), hv | (hv << 16)};
                *(tw_u32x2*)(stage + (l * kLineCols + lane) * 8) = v;
                *(tw_u32x2*)(stage + kPlaneBytes + (l * kLineCols + lane) * 8) = v;
            }
        }
        tw_compiler_fence();
#pragma unroll
        for (int P = 0; P < NP; ++P)
            if (P == pass0) write_pass(P);
        tw_compiler_fence();
#pragma unroll
        for (int P = 0; P < NP; ++P) {
            if (P < pass0 || P >= pass1) continue;               // wave-uniform
            tw_i16x4 lo[kWinLines], hi[kWinLines];
#pragma unroll
            for (int l = 0; l < kWinLines; ++l) {
                lo[l] = tw_lds_read_tr(rpos + l * (kLineCols * 8));
                hi[l] = tw_lds_read_tr(rpos + l * (kLineCols * 8) + 32);
            }
            const unsigned short eF = *(const unsigned short*)ragF;
            const unsigned short eL = *(const unsigned short*)ragL;
            tw_compiler_fence();
            if (P + 1 < NP && P + 1 < pass1) write_pass(P + 1);
            tw_compiler_fence();
#pragma unroll
            for (int l = 0; l < kWinLines; ++l) {
                if (okl[l] && 8 * P < rows_left) {
                    const tw_u32x2 a = __builtin_bit_cast(tw_u32x2, lo[l]), b = __builtin_bit_cast(tw_u32x2, hi[l]);
                    if (whole[l]) tw_store16_stream(cptr + (long)(8 * P) * p.ldc + l * kLineCols, tw_u32x4{a.x, a.y, b.x, b.y});
                    else *(tw_u32x4_a2*)tw_opaque(cptr + (long)(8 * P) * p.ldc + l * kLineCols) = tw_u32x4{a.x, a.y, b.x, b.y};
                }
            }
            if (g_first >= 0) {                              // wave-uniform
                if (inF && 8 * P < rag_left) rptr[(long)(8 * P) * p.ldc + colF] = eF;
            }
            if (g_last >= 0) {
                if (inL && 8 * P < rag_left) rptr[(long)(8 * P) * p.ldc + colL] = eL;
            }
            // At most a few of this wave's stores stay in flight: a long queue of stores in the CU's memory
            // pipeline holds up the loads of the waves that are multiplying (no load of this wave is pending here).
            asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        }
        tw_compiler_fence();
    }
}

// ---- Transposed boundary (TRANS): At is K x M, Ct is N x M (Sec. VI "Memory Accesses Coalescing") ----
// With the activations stored transposed, a K row of the workgroup's block is 128 contiguous bytes in
// global memory and goes to its LDS row as it is: the LDS copy needs no transposition, and skipping a
// pruned K position skips a row, which is what the paper changes the layout for.  A tile's results are
// rows of Ct (one per kept column), each a whole 128-byte line per block of 64 tokens: no line of
// the output is shared between tiles, and pruned columns are whole lines of zeros.

// Staging of At[k0 : k0+kw, m0 : m0 + 32*MS) into LDS (row k - k0 at (k - k0) * at_pitch), cut into tasks
// of 64 / (4*MS) rows: a wave instruction reads whole rows of the block (128 bytes with MS = 2).  Pieces
// past the row's pitch re-read the last piece inside it (they belong to tokens >= M, whose results
// are never stored).  One request per task; absent rows go to the spare rows.
template <int MS>
struct AtTask {
    int krow, pc;     // chunk-local K row, 16-byte piece of the block's row
    bool have;
    __device__ __forceinline__ AtTask(int t, int kw, int lane) {
        constexpr int PPR = 4 * MS, RPI = 64 / PPR;      // pieces per row, rows per instruction
        const int k = t * RPI + lane / PPR;
        have = k < kw;
        krow = have ? k : kw - 1;
        pc = lane % PPR;
    }
};
template <int MS>
__device__ __forceinline__ int at_tasks(int kw) { return (kw + 64 / (4 * MS) - 1) / (64 / (4 * MS)); }

template <int MS, int BATCH, bool NTA = true>
__device__ __forceinline__ void at_issue(const TwGemmParams& p, ARegs<BATCH>& ar, int m0, int k0, int kw, int t0,
                                         int lane_in, int stride = kWaves) {
    const int lane = fresh(lane_in);
    const int pmax = (int)((p.lda - m0) >> 3) - 1;
#pragma unroll
    for (int b = 0; b < BATCH; ++b) {
        const AtTask<MS> t(t0 + b * stride, kw, lane);
        const int pc = t.pc < pmax ? t.pc : pmax;
        ar.v[b] = load_a16<NTA>(p.A + (long)(k0 + t.krow) * p.lda + (m0 + pc * 8));
    }
}

template <int MS, int BATCH>
__device__ __forceinline__ void at_commit(const TwGemmParams& p, const ARegs<BATCH>& ar, unsigned char* at, int kw, int t0,
                                          int lane_in, int stride = kWaves) {
    const int lane = fresh(lane_in);
    constexpr int PPR = 4 * MS;
#pragma unroll
    for (int b = 0; b < BATCH; ++b) {
        const AtTask<MS> t(t0 + b * stride, kw, lane);
        const int krow = t.have ? t.krow : p.k_chunk + 1 + (lane / PPR) % 8;   // absent rows: the spare rows
        unsigned char* dst = at + (unsigned)krow * at_pitch_of<MS>() + t.pc * 16;
        *(tw_u32x2*)dst = tw_u32x2{ar.v[b].x, ar.v[b].y};
        *(tw_u32x2*)(dst + 8) = tw_u32x2{ar.v[b].z, ar.v[b].w};
    }
}

// The same with a row list: request b of the wave, row lane / 8 of it, stages chunk-local K row
// rows[8*b + lane/8] if that entry exists (entry number 8*(t0 + b*stride) + lane/8 below cnt).  K rows
// that no tile of the workgroup's set keeps are never read: with the activations transposed, skipping
// a K position skips a row of At (Sec. VI "Memory Accesses Coalescing").  `rows` is this wave's own
// copy in LDS of its entries of the chunk's list.
template <int BATCH>
__device__ __forceinline__ void at_issue_rows(const TwGemmParams& p, ARegs<BATCH>& ar, int m0, int k0,
                                              const unsigned short* rows, int cnt, int t0, int lane_in, int stride) {
    const int lane = fresh(lane_in);
    const int pmax = (int)((p.lda - m0) >> 3) - 1;
    const int pc = (lane & 7) < pmax ? (lane & 7) : pmax;
#pragma unroll
    for (int b = 0; b < BATCH; ++b) {
        const int j = 8 * (t0 + b * stride) + (lane >> 3);
        const int krow = rows[8 * b + (lane >> 3)];
        ar.v[b] = tw_u32x4{0u, 0u, 0u, 0u};
        if (j < cnt) ar.v[b] = tw_load16_stream(p.A + (long)(k0 + krow) * p.lda + (m0 + pc * 8));
    }
}
template <int BATCH>
__device__ __forceinline__ void at_commit_rows(const TwGemmParams& p, const ARegs<BATCH>& ar, unsigned char* at,
                                               const unsigned short* rows, int cnt, int t0, int lane_in, int stride) {
    const int lane = fresh(lane_in);
#pragma unroll
    for (int b = 0; b < BATCH; ++b) {
        const int j = 8 * (t0 + b * stride) + (lane >> 3);
        const int krow = j < cnt ? (int)rows[8 * b + (lane >> 3)] : p.k_chunk + 1 + (lane >> 3);
        unsigned char* dst = at + (unsigned)krow * at_pitch_of<2>() + (lane & 7) * 16;   // (64 tokens: MS = 2)
        *(tw_u32x2*)dst = tw_u32x2{ar.v[b].x, ar.v[b].y};
        *(tw_u32x2*)(dst + 8) = tw_u32x2{ar.v[b].z, ar.v[b].w};
    }
}

template <int MS, int BATCH, bool NTA = true>
__device__ __forceinline__ void load_at_block(const TwGemmParams& p, unsigned char* at, int m0, int k0, int kw, int wave,
                                              int lane, int tid) {
    const int tasks = at_tasks<MS>(kw);
    for (int t0 = wave; t0 < tasks; t0 += kWaves * BATCH) {
        ARegs<BATCH> ar;
        at_issue<MS, BATCH, NTA>(p, ar, m0, k0, kw, t0, lane);
        at_commit<MS, BATCH>(p, ar, at, kw, t0, lane);
    }
    a_zero_row(p, at, 32 * MS, tid);
}

// The two boundaries behind one name (TRANS: transposed).
// The common case of the streamed row-major staging written out (used where all eight waves stage): a chunk of
// 64 rows whose width is exactly what BATCH requests of STRIDE waves cover (8 * BATCH * STRIDE columns, 384 for
// 6 x 8), wave t0 < STRIDE.
// Same tasks and same LDS layout as a_issue / a_commit without row pairs (task t0 + b * STRIDE: rows
// 8 * (t % 8) .. + 7, columns 64 * (t / 8) .. + 63), but everything that does not depend on the lane is a
// constant here: one or two row pointers per chunk, one LDS address, immediate offsets (the general code
// spends about 75 instructions per request on its bookkeeping): 5 % on the FFN-down of BERT-base.
template <int BATCH, int STRIDE, bool NTA = true>
__device__ __forceinline__ void a_issue_full(const TwGemmParams& p, ARegs<BATCH>& ar, int row0, int k0, int t0, int lane_in) {
    static_assert(STRIDE == 4 || STRIDE == 8, "waves that share a chunk");
    const int lane = fresh(lane_in);
    const int mend = block_end(p, row0);
    constexpr int NRG = 8 / STRIDE;                       // row groups of this wave: t0, t0 + STRIDE, ..
    const unsigned short* rp[NRG];
#pragma unroll
    for (int g = 0; g < NRG; ++g) {
        int grow = row0 + (t0 + g * STRIDE) * 8 + (lane >> 3);
        grow = grow < mend ? grow : mend - 1;             // rows past the block's end: any valid row, never stored
        rp[g] = p.A + (long)grow * p.lda + (k0 + (lane & 7) * 8);
    }
#pragma unroll
    for (int b = 0; b < BATCH; ++b)
        ar.v[b] = load_a16<NTA>(rp[((b * STRIDE) & 7) / STRIDE] + ((b * STRIDE) >> 3) * 64);
}
template <int BATCH, int STRIDE>
__device__ __forceinline__ void a_commit_full(const ARegs<BATCH>& ar, unsigned char* at, int t0, int lane_in) {
    const int lane = fresh(lane_in);
    constexpr unsigned pitch = at_pitch_of<2>();
    unsigned char* base = at + (unsigned)((lane & 7) * 8) * pitch + (lane >> 3) * 2 + t0 * 16;
#pragma unroll
    for (int b = 0; b < BATCH; ++b) {
        unsigned char* dst = base + (unsigned)(((b * STRIDE) >> 3) * 64) * pitch + ((b * STRIDE) & 7) * 16;
        const unsigned w[4] = {ar.v[b].x, ar.v[b].y, ar.v[b].z, ar.v[b].w};
#pragma unroll
        for (int i = 0; i < 8; ++i)
            *(unsigned short*)(dst + (unsigned)i * pitch) = (unsigned short)(w[i >> 1] >> (16 * (i & 1)));
    }
}

template <int MS, int BATCH, bool TRANS, bool NTA = true>
__device__ __forceinline__ void stage_issue(const TwGemmParams& p, ARegs<BATCH>& ar, int r0, int k0, int kw, int t0, int lane,
                                            int stride = kWaves) {
    if constexpr (TRANS) {
        at_issue<MS, BATCH, NTA>(p, ar, r0, k0, kw, t0, lane, stride);
    } else {
        // (with four loading waves the written-out form measured no faster, 1.6 % slower on the conv workload)
        if (MS == 2 && stride == 8 && kw == 64 * BATCH) a_issue_full<BATCH, 8, NTA>(p, ar, r0, k0, t0, lane);
        else a_issue<MS, BATCH, kPairStream, NTA>(p, ar, r0, k0, kw, t0, lane, stride);
    }
}
template <int MS, int BATCH, bool TRANS>
__device__ __forceinline__ void stage_commit(const TwGemmParams& p, const ARegs<BATCH>& ar, unsigned char* at, int kw, int t0,
                                             int lane, int stride = kWaves) {
    if constexpr (TRANS) {
        at_commit<MS, BATCH>(p, ar, at, kw, t0, lane, stride);
    } else {
        if (MS == 2 && stride == 8 && kw == 64 * BATCH) a_commit_full<BATCH, 8>(ar, at, t0, lane);
        else a_commit<MS, BATCH, kPairStream>(p, ar, at, kw, t0, lane, stride);
    }
}

// Epilogue of one tile, transposed output.  Column block by column block, a lane (packed column n, its
// registers hold 4 consecutive tokens per group) writes its rounded values as 8-byte pieces into the
// wave's staging area [32 columns][32*MS tokens]; the rows are read back as 16-byte pieces and a store
// instruction writes whole rows of the block (128-byte lines with MS = 2) of 64 / (4*MS) rows of Ct.
// The destination row of a staged row comes from the lane that owns that packed column
// (ds_bpermute).  The pruned columns inside the tile's span are written as lines of zeros from the
// packer's list.
template <int DT, int MS, int NCB, bool FUSED>
__device__ __forceinline__ void store_tile_t(const TwGemmParams& p, const TileU& d, tw_f32x16 (&acc)[MS][NCB],
                                             unsigned char* stage, const unsigned (&dpos)[NCB], int m0, int lane_in,
                                             int cb0 = 0, int cb1 = NCB, const unsigned short* xbuf = nullptr) {
    // (cb0, cb1: the column blocks to store, all by default; the lines of zeros go with column block 0.  The
    // second kernel of a split-K product gives a wave one column block of a tile.)
    constexpr int PPR = 4 * MS, RPI = 64 / PPR, PITCH = 64 * MS + 8;
    static_assert(32 * PITCH <= (int)kStageBytes, "transposed staging fits the wave's area");
    const int lane = fresh(lane_in);
    if constexpr (FUSED) {   // bias of this lane's packed columns (rows of Ct), activation in place
        EpiBias<NCB> eb;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
            eb.col[cb] = (p.bias != nullptr && dpos[cb] != 0xFFFFFFFFu)
                             ? tw_to_f32<DT>(p.bias[(d.span_start & ~7) + (int)dpos[cb]]) : 0.f;
        apply_bias_act<MS, NCB>(acc, eb, p.act);
    }
    const int n = lane & 31, h = lane >> 5, rr = lane / PPR, pc = lane % PPR;
    const int origin = d.span_start & ~7;
    const int mleft = p.M - m0;                              // tokens of this block that exist
    const bool whole = 8 * pc + 8 <= mleft;                  // this lane's piece lies inside
    // a block of 64 tokens that exists in full is a whole 128-byte line of every row of Ct (wave-uniform)
    const bool stream = p.stream_stores != 0 && MS == 2 && mleft >= 64;
    auto put_piece = [&](long row, tw_u32x4 v) {
        unsigned short* dst = p.C + row * p.ldc + (m0 + 8 * pc);
        if (stream) {
            tw_store16_stream(dst, v);
        } else if (whole) {
            *(tw_u32x4*)tw_opaque(dst) = v;
        } else {
            const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (8 * pc + e < mleft) dst[e] = (unsigned short)(w[e >> 1] >> (16 * (e & 1)));
        }
    };
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
        if (cb < cb0 || cb >= cb1) continue;                     // wave-uniform
        tw_compiler_fence();
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                tw_u32x2 v;
                v.x = (unsigned)tw_cvt<DT>(acc[ms][cb][4 * q + 0]) | ((unsigned)tw_cvt<DT>(acc[ms][cb][4 * q + 1]) << 16);
                v.y = (unsigned)tw_cvt<DT>(acc[ms][cb][4 * q + 2]) | ((unsigned)tw_cvt<DT>(acc[ms][cb][4 * q + 3]) << 16);
                *(tw_u32x2*)(stage + n * PITCH + (32 * ms + 8 * q + 4 * h) * 2) = v;
            }
        tw_compiler_fence();
#pragma unroll
        for (int i = 0; i < 32 / RPI; ++i) {
            const int row = rr + RPI * i;                    // staged row = packed column 32*cb + row
            const tw_u32x2 lo = *(const tw_u32x2*)(stage + row * PITCH + pc * 16);
            const tw_u32x2 hi = *(const tw_u32x2*)(stage + row * PITCH + pc * 16 + 8);
            const unsigned dcol = (unsigned)__builtin_amdgcn_ds_bpermute(row * 4, (int)dpos[cb]);
            if (dcol != 0xFFFFFFFFu) put_piece((long)origin + (long)dcol, tw_u32x4{lo.x, lo.y, hi.x, hi.y});
        }
    }
    tw_compiler_fence();
    if (cb0 != 0) return;
    // lines of zeros for the pruned columns of the span
    const int* zp = (const int*)(p.blob + p.off_zero_ptr);
    const int* zc = (const int*)(p.blob + p.off_zero_cols);
    const int z0 = fetch_int(zp, d.tile), z1 = fetch_int(zp, d.tile + 1);
    // (`xbuf`: the rows of the span's residual-only columns that this tile has multiplied itself, [column][token])
    const signed char* zx = (const signed char*)(p.blob + p.off_zero_xc);
    for (int j = z0 + rr; j < z1; j += RPI) {
        const int col = zc[j];
        const int xs = xbuf != nullptr ? (int)zx[j] : -1;
        if (xs >= 0) {
            put_piece((long)col, *(const tw_u32x4*)(xbuf + xs * 64 + 8 * pc));
            continue;
        }
        unsigned v = 0u;
        if constexpr (FUSED) {   // a pruned column holds act(bias) for every token
            const unsigned hv = tw_cvt<DT>(tw_activate(p.bias != nullptr ? tw_to_f32<DT>(p.bias[col]) : 0.f, p.act));
            v = hv | (hv << 16);
        }
        put_piece((long)col, tw_u32x4{v, v, v, v});
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

// Element-wise residual of the TEW hybrid (Sec. IV-A): the weights kept outside the tile-wise pattern, in the
// tile's kept columns, are added to the tile's accumulators after the tile's own steps, by linearity.  The paper
// runs this part as a separate sparse product on the scalar cores; here it runs on the matrix cores out of the
// same LDS copy of A: per column block of 32 columns the packer lists the K rows in which the block has residual
// weights, 16 to a step, with the block's weights of those rows (mostly zeros).  One residual step is one such
// step of every column block: NCB gathers of A (each block has its own rows), NCB pieces of weights, MS * NCB
// MFMAs.  At 1 % of the weights a block of 32 columns touches about a quarter of the K rows, so the residual
// costs about as many MFMAs as the tile itself, where one fused multiply-add per row and weight on the vector
// units cost five times that.
// Same pipeline as run_steps: weights kDepth steps ahead, K rows kIdx steps ahead, the gather kRing - 1 column
// blocks ahead of the MFMAs that use it.
// Steps [s0, s1), not empty, of the tables `goff` (uint16 [steps][8][NCB][2]) and `bw` (16-bit [steps][NCB][64][8]).
template <int NCB>
struct BlockRegs {
    static constexpr int kDepth = 2, kIdx = NCB <= 2 ? 6 : 3;
    unsigned kk[kIdx][NCB];
    tw_u16x8 bq[kDepth][NCB];
};
template <int NCB>
__device__ __forceinline__ void block_load_k(BlockRegs<NCB>& r, int slot, const unsigned char* gk, int s, int last) {
    s = s < last ? s : last;
    const unsigned char* q = gk + (long)s * (32 * NCB);
    if constexpr (NCB == 4) {
        const tw_u32x4 t = *(const tw_u32x4*)q;
        r.kk[slot][0] = t.x; r.kk[slot][1] = t.y; r.kk[slot][2] = t.z; r.kk[slot][3] = t.w;
    } else if constexpr (NCB == 2) {
        const tw_u32x2 t = *(const tw_u32x2*)q;
        r.kk[slot][0] = t.x; r.kk[slot][1] = t.y;
    } else {
        r.kk[slot][0] = *(const unsigned*)q;
    }
}
// Requests the first steps of [s0, s1) (not empty).  The requests keep this order (first needed first): a wait for
// the first one must not wait for them all, and the loop's wait counts are the weaker of what its entry and its
// back edge allow.
template <int NCB>
__device__ __forceinline__ void request_block_steps(BlockRegs<NCB>& r, const unsigned char* goff, const unsigned char* bw,
                                                    int s0, int s1, int lane_in) {
    const int lane = fresh(lane_in);
    const unsigned char* gk = goff + ((lane >> 5) * 4 + ((lane & 15) >> 2)) * (NCB * 4);
    const unsigned char* bl = bw + lane * 16;
    const int last = s1 - 1;
#pragma unroll
    for (int i = 0; i < BlockRegs<NCB>::kIdx; ++i) {
        block_load_k<NCB>(r, i, gk, s0 + i, last);
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int i = 0; i < BlockRegs<NCB>::kDepth; ++i) {
        const int s = s0 + i < last ? s0 + i : last;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            r.bq[i][cb] = *(const tw_u16x8*)(bl + ((long)s * NCB + cb) * 1024);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}
// Expects the first steps in `r` (request_block_steps).
template <int DT, int MS, int NCB>
__device__ __forceinline__ void run_block_steps(tw_f32x16 (&acc)[MS][NCB], BlockRegs<NCB>& r, const unsigned char* at,
                                                unsigned at_pitch, const unsigned char* goff, const unsigned char* bw,
                                                int s0, int s1, int lane_in) {
    const int lane = fresh(lane_in);
    const int h = lane >> 5, j = lane & 15;
    const unsigned lanebase = (unsigned)(((lane >> 4) & 1) * 16 + (j & 3) * 4) * 2;
    const unsigned char* gk = goff + (h * 4 + (j >> 2)) * (NCB * 4);   // this lane's K rows of a step
    const unsigned char* bl = bw + lane * 16;
    const int last = s1 - 1;
    constexpr int kDepth = BlockRegs<NCB>::kDepth, kIdx = BlockRegs<NCB>::kIdx, kUnroll = 6;
    auto& kk = r.kk;
    auto& bq = r.bq;
    auto load_k = [&](int slot, int s) { block_load_k<NCB>(r, slot, gk, s, last); };
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
    constexpr int kRing = 2;   // (four buffers, the gather three column blocks ahead: no faster, 16 registers more)
    static_assert((kUnroll * NCB) % kRing == 0 && (kRing - 1 + NCB - 1) / NCB < kIdx, "ring of gather buffers");
    tw_u16x8 a[kRing][MS];
#pragma unroll
    for (int m = 0; m < kRing; ++m)
#pragma unroll
        for (int ms = 0; ms < MS; ++ms) a[m][ms] = tw_u16x8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int m = 0; m < kRing - 1; ++m) gather(a[m], kk[m / NCB][m % NCB]);
    auto step = [&](int i, int s) {
        const int sb = (s + kDepth) < last ? (s + kDepth) : last;
        const unsigned char* bnext = bl + ((long)sb * NCB) * 1024;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            const int m = i * NCB + cb, ahead = cb + kRing - 1;
            gather(a[(m + kRing - 1) % kRing], kk[(i + ahead / NCB) % kIdx][ahead % NCB]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ms = 0; ms < MS; ++ms)
                acc[ms][cb] = tw_mfma<DT>(a[m % kRing][ms], bq[i % kDepth][cb], acc[ms][cb]);
            __builtin_amdgcn_sched_barrier(0);
            bq[i % kDepth][cb] = *(const tw_u16x8*)(bnext + cb * 1024);
            __builtin_amdgcn_sched_barrier(0);
        }
        load_k(i % kIdx, s + kIdx);
        __builtin_amdgcn_sched_barrier(0);
    };
    int s = s0;
    for (; s + kUnroll <= s1; s += kUnroll) {
#pragma unroll
        for (int i = 0; i < kUnroll; ++i) step(i, s + i);
    }
    const int rest = s1 - s;
#pragma unroll
    for (int i = 0; i < kUnroll - 1; ++i)
        if (i < rest) step(i, s + i);
}

template <int DT, int MS, int NCB>
__device__ __forceinline__ void add_ew_residual(const TwGemmParams& p, int tile, int chunk, tw_f32x16 (&acc)[MS][NCB],
                                                const unsigned char* at, unsigned at_pitch, int lane) {
    const int* ep = (const int*)(p.blob + p.off_ew_ptr);
    const int pi = tile * p.n_chunks + chunk;      // residual steps of this tile inside this K chunk (`at` holds the chunk)
    const int s0 = fetch_int(ep, pi), s1 = fetch_int(ep, pi + 1);
    if (s0 != s1) {
        BlockRegs<NCB> r;
        request_block_steps<NCB>(r, p.blob + p.off_ew_goff, p.blob + p.off_ew_b, s0, s1, lane);
        run_block_steps<DT, MS, NCB>(acc, r, at, at_pitch, p.blob + p.off_ew_goff, p.blob + p.off_ew_b, s0, s1, lane);
    }
}

// Residual-only columns inside a tile's span (weights restored in a column that the tile-wise pattern pruned
// altogether), row-major boundary: the first TW_XC_INLINE of a tile are multiplied like one more column block
// (packed column j = the tile's j-th such column; per K chunk the steps hold the K rows in which any of them has a
// weight) and put into `xbuf` (16-bit, [column][row % 8][row / 8]: the eight rows that one lane of the epilogue
// puts into the staging window, one per pass, lie side by side; act(. + bias) applied if FUSED), from where the
// tile's epilogue takes them.  With K streamed their fp32 sums wait between the chunks in the wave's staging
// area, which only the epilogue uses otherwise.
struct XcSteps {
    int s0, s1;
    BlockRegs<1> r;
};
__device__ __forceinline__ int xc_count(const TileU& d) { return (int)((unsigned)d.xc >> 26); }
// original column of the tile's residual-only columns l / 8 and l / 8 + 8 for lane l (what the epilogue needs)
__device__ __forceinline__ void xc_column_numbers(const TwGemmParams& p, const TileU& d, int (&col)[TW_XC_INLINE / 8], int lane) {
    const int x0 = d.xc & 0x3FFFFFF, nx = xc_count(d);
    const int* xcol = (const int*)(p.blob + p.off_xc_col);
#pragma unroll
    for (int g = 0; g < TW_XC_INLINE / 8; ++g) {
        col[g] = 0;
        const int j = 8 * g + (fresh(lane) >> 3);
        if (nx > 0) col[g] = xcol[x0 + (j < nx ? j : nx - 1)];   // wave-uniform condition
    }
}
__device__ __forceinline__ void xc_request(const TwGemmParams& p, const TileU& d, int chunk, XcSteps& x, int lane) {
    x.s0 = x.s1 = 0;
    if (xc_count(d) == 0) return;                            // wave-uniform
    const int* xp = (const int*)(p.blob + p.off_xm_ptr) + d.tile * p.n_chunks + chunk;
    x.s0 = fetch_int(xp, 0);
    x.s1 = fetch_int(xp, 1);
    if (x.s0 != x.s1) request_block_steps<1>(x.r, p.blob + p.off_xm_goff, p.blob + p.off_xm_b, x.s0, x.s1, lane);
}
template <int DT, int MS, bool FUSED>
__device__ __forceinline__ void xc_store(const TwGemmParams& p, const TileU& d, const tw_f32x16 (&acc)[MS][1],
                                         unsigned short* xbuf, int lane) {
    const int n = lane & 31, h = lane >> 5;
    if (n < xc_count(d)) {
        float bias = 0.f;
        if constexpr (FUSED)
            if (p.bias != nullptr) bias = tw_to_f32<DT>(p.bias[((const int*)(p.blob + p.off_xc_col))[(d.xc & 0x3FFFFFF) + n]]);
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
            for (int i = 0; i < 4; ++i) {                    // rows 32*ms + 8*q + 4*h + i, q = 0..3
                float v[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    v[q] = acc[ms][0][4 * q + i];
                    if constexpr (FUSED) v[q] = tw_activate(v[q] + bias, p.act);
                }
                tw_u32x2 o;
                o.x = (unsigned)tw_cvt<DT>(v[0]) | ((unsigned)tw_cvt<DT>(v[1]) << 16);
                o.y = (unsigned)tw_cvt<DT>(v[2]) | ((unsigned)tw_cvt<DT>(v[3]) << 16);
                *(tw_u32x2*)(xbuf + n * 64 + (4 * h + i) * 8 + 4 * ms) = o;
            }
    }
}
// Transposed boundary: a column is a row of Ct, `xbuf` is [column][token] and the epilogue writes its rows in place
// of the lines of zeros.
template <int DT, int MS, bool FUSED>
__device__ __forceinline__ void xc_store_t(const TwGemmParams& p, const TileU& d, const tw_f32x16 (&acc)[MS][1],
                                           unsigned short* xbuf, int lane) {
    const int n = lane & 31, h = lane >> 5;
    if (n < xc_count(d)) {
        float bias = 0.f;
        if constexpr (FUSED)
            if (p.bias != nullptr) bias = tw_to_f32<DT>(p.bias[((const int*)(p.blob + p.off_xc_col))[(d.xc & 0x3FFFFFF) + n]]);
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
            for (int q = 0; q < 4; ++q) {                    // tokens 32*ms + 8*q + 4*h .. + 3
                float v[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    v[i] = acc[ms][0][4 * q + i];
                    if constexpr (FUSED) v[i] = tw_activate(v[i] + bias, p.act);
                }
                tw_u32x2 o;
                o.x = (unsigned)tw_cvt<DT>(v[0]) | ((unsigned)tw_cvt<DT>(v[1]) << 16);
                o.y = (unsigned)tw_cvt<DT>(v[2]) | ((unsigned)tw_cvt<DT>(v[3]) << 16);
                *(tw_u32x2*)(xbuf + n * 64 + 32 * ms + 8 * q + 4 * h) = o;
            }
    }
}
// K resident: everything at once
template <int DT, int MS, bool FUSED, bool TRANS>
__device__ __forceinline__ void xc_columns(const TwGemmParams& p, const TileU& d, XcSteps& x, const unsigned char* at,
                                           unsigned at_pitch, unsigned short* xbuf, int lane) {
    if (xc_count(d) == 0) return;                            // wave-uniform
    tw_f32x16 acc[MS][1];
    zero_acc<MS, 1>(acc);
    if (x.s0 != x.s1)
        run_block_steps<DT, MS, 1>(acc, x.r, at, at_pitch, p.blob + p.off_xm_goff, p.blob + p.off_xm_b, x.s0, x.s1, lane);
    if constexpr (TRANS) xc_store_t<DT, MS, FUSED>(p, d, acc, xbuf, lane);
    else xc_store<DT, MS, FUSED>(p, d, acc, xbuf, lane);
}
// K streamed: the sums of the 16 columns between chunks, fp32, piece (ms, q) of lane (h, n < 16) at float offset
// (((4 * ms + q) * 32 + 16 * h + n) * 4 of `area` (4 KB with 64 rows)
static_assert(TW_XC_INLINE == 16 && 2 * 4 * 32 * 16 <= (int)kStageBytes, "partial sums of the residual-only columns fit the staging area");
template <int MS>
__device__ __forceinline__ void xc_zero_partial(const TileU& d, unsigned char* area, int lane) {
    if (xc_count(d) == 0) return;                            // wave-uniform
#pragma unroll
    for (int i = 0; i < MS * 2; ++i) *(tw_u32x4*)(area + (i * 64 + lane) * 16) = tw_u32x4{0u, 0u, 0u, 0u};
}
template <int MS>
__device__ __forceinline__ void xc_load_partial(tw_f32x16 (&acc)[MS][1], const unsigned char* area, int lane) {
    zero_acc<MS, 1>(acc);
    const int n = lane & 31, h = lane >> 5;
    if (n < 16) {
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const tw_f32x4 v = *(const tw_f32x4*)(area + (((4 * ms + q) * 32 + 16 * h + n) * 16));
                acc[ms][0][4 * q + 0] = v.x; acc[ms][0][4 * q + 1] = v.y; acc[ms][0][4 * q + 2] = v.z; acc[ms][0][4 * q + 3] = v.w;
            }
    }
}
template <int DT, int MS>
__device__ __forceinline__ void xc_chunk(const TwGemmParams& p, const TileU& d, int chunk, const unsigned char* at,
                                         unsigned at_pitch, unsigned char* area, int lane) {
    XcSteps x;
    xc_request(p, d, chunk, x, lane);
    if (x.s0 == x.s1) return;                                // wave-uniform
    tw_f32x16 acc[MS][1];
    xc_load_partial<MS>(acc, area, lane);
    run_block_steps<DT, MS, 1>(acc, x.r, at, at_pitch, p.blob + p.off_xm_goff, p.blob + p.off_xm_b, x.s0, x.s1, lane);
    const int n = lane & 31, h = lane >> 5;
    if (n < 16) {
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *(tw_f32x4*)(area + (((4 * ms + q) * 32 + 16 * h + n) * 16)) =
                    tw_f32x4{acc[ms][0][4 * q + 0], acc[ms][0][4 * q + 1], acc[ms][0][4 * q + 2], acc[ms][0][4 * q + 3]};
    }
}
template <int DT, int MS, bool FUSED, bool TRANS>
__device__ __forceinline__ void xc_finish(const TwGemmParams& p, const TileU& d, const unsigned char* area,
                                          unsigned short* xbuf, int lane) {
    if (xc_count(d) == 0) return;                            // wave-uniform
    tw_f32x16 acc[MS][1];
    xc_load_partial<MS>(acc, area, lane);
    if constexpr (TRANS) xc_store_t<DT, MS, FUSED>(p, d, acc, xbuf, lane);
    else xc_store<DT, MS, FUSED>(p, d, acc, xbuf, lane);
}

// MODE 0: the K extent of a row block of 32*MS rows is resident in LDS, waves pull whole tiles.
// MODE 1: K streamed through two LDS buffers, row block of 64 rows (MS = 2), wave w owns tile 8*set + w.
// MODE 2: K streamed, row block of 64 rows (MS = 2), sets of 1, 2 or 4 tiles: of waves 0-3 wave w owns tile
//         tiles_per_set*set + w and multiplies, waves 4-7 do nothing but bring A into LDS, so the two kinds of
//         work overlap instead of taking turns (a wave's loads retire in order: a wave that waits for its packed
//         B also waits for every request for A it made before).
//         (Six multiplying and two loading waves were tried for weights of five or six tiles: the two
//         loading waves cannot keep up with the transposing LDS writes of the row-major boundary, 9 % slower
//         than MODE 1 on the FFN-down of BERT-base, and no gain on the transposed boundary.)
// Split K: a wave's fp32 results of its part of the K chunks, as they lie in the registers: piece (ms, cb, q) of
// lane l (registers 4q .. 4q+3 of acc[ms][cb]) at float offset (((ms * NCB + cb) * 4 + q) * 64 + l) * 4, so that
// every instruction writes (reads) 1 KB of consecutive memory.  32 KB per tile and part with 128-column tiles.
template <int MS, int NCB>
__device__ __forceinline__ void dump_partial(float* dst, const tw_f32x16 (&acc)[MS][NCB], int lane) {
    // dst is wave-uniform: said to the compiler, the 32 stores share one vector offset (the lane's) on a scalar
    // base instead of holding a vector address for every 4 KB of the range
    const uint64_t a = (uint64_t)dst;
    unsigned char* base = (unsigned char*)(((uint64_t)(unsigned)uni((int)(a >> 32)) << 32) | (unsigned)uni((int)(unsigned)a));
    const unsigned voff = (unsigned)lane * 16u;
#pragma unroll
    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *(tw_f32x4*)(base + ((ms * NCB + cb) * 4 + q) * 1024 + voff) =
                    tw_f32x4{acc[ms][cb][4 * q], acc[ms][cb][4 * q + 1], acc[ms][cb][4 * q + 2], acc[ms][cb][4 * q + 3]};
}

// EW: the variant for TEW blobs.  The code of the element-wise residual costs the kernels without it 1 to 2.5 %
// (registers: the widest variants sit at the limit of 256), so blobs without a residual run kernels without it.
template <int DT, int MS, int NCB, int MODE, bool FUSED, bool TRANS, bool NTA = true, bool EW = false>
__global__ __launch_bounds__(kThreads) void tw_gemm_kernel(const TwGemmParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const bool has_ew = EW && p.has_ew != 0;
    const unsigned xbuf_off = EW ? p.xbuf_off : 0u;
    constexpr int MSB = MS;                       // 32-row blocks in the workgroup's row block
    constexpr int BM = 32 * MSB;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = uni(tid >> 6);
    unsigned char* stage = smem + p.stage_off + wave * kStageBytes;
    volatile int* misc = (volatile int*)(smem + p.misc_off);
    const int* step_ptr = (const int*)(p.blob + p.off_step_ptr);

    // The loop over the workgroup's items.  ROLE 0: every wave does the same (MODE 0 and 1); with MODE 2
    // the multiplying waves (ROLE 1) and the loading waves (ROLE 2) run copies of their own, with the
    // same barriers, so that neither carries the other's registers.
    // The first item of a workgroup is its own index, later ones come from the atomic counter.
    auto run_items = [&](auto role_tag) {
    constexpr int ROLE = decltype(role_tag)::value;
    int my_next = (int)blockIdx.x;   // thread 0: the item of the coming turn
    // loading waves: the first chunks of the coming item, requested during this item's epilogue
    ARegs<12> pre0, pre1;
    bool preloaded = false;
    int lists_of = -1;               // loading waves: the set whose row lists are in LDS
    int par = 0;                     // MODE 2: chunk c of the item lives in LDS buffer (c + par) % 2 (see the ring below)
    for (int turn = 0;; ++turn) {
        if (tid == 0) {
            misc[0] = my_next;
            misc[1] = 0;
        }
        __syncthreads();
        const int item = misc[0];
        if (item >= p.n_items) break;
        // the item after this one is requested now, so that the atomic's latency passes during this item's
        // work; the counter is touched only when there are more items than workgroups
        if (tid == 0) my_next = p.n_items > (int)gridDim.x ? (int)gridDim.x + atomicAdd(&p.counters[0], 1) : p.n_items;

        if constexpr (MODE == 0) {
            // the whole K extent of the row block stays in LDS; waves pull tiles of this item's set
            // (TRANS: transposed boundary, the row block is a block of tokens)
            const int mb = item / p.n_seg, seg = item - mb * p.n_seg;
            const int row0 = mb * p.row_step;
            // first tile of this wave: its descriptor is requested before A is staged
            int i = 0;
            if (lane == 0) i = atomicAdd((int*)&misc[1], 1);
            int ti = seg + uni(i) * p.n_seg;
            TileU next = fetch_tile(p, ti < p.T ? ti : 0);
            if constexpr (TRANS) load_at_block<MS, 12>(p, smem, row0, 0, p.K, wave, lane, tid);
            else load_a_block<MS, 12, kPairResident>(p, smem, row0, 0, p.K, wave, lane, tid);
            __syncthreads();
            while (ti < p.T) {
                const TileU d = next;
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
                // residual-only columns of the tile's span (TEW): multiplied first, while the tile's own first
                // operands are on their way (their requests come first, so the wait for them is the shorter one)
                unsigned short* xbuf = nullptr;
                XcSteps xs;
                int xcols[TW_XC_INLINE / 8];
                if (xbuf_off != 0) {
                    xbuf = (unsigned short*)(smem + xbuf_off) + wave * (TW_XC_INLINE * 64);
                    if constexpr (!TRANS) xc_column_numbers(p, d, xcols, lane);
                    xc_request(p, d, 0, xs, lane);
                }
                StepRegs<NCB> rg;
                prefetch_first_steps<NCB>(rg, p.blob + p.off_goff + (long)d.first_step * 32,
                                          p.blob + p.off_bvals + (long)d.first_step * NCB * 1024, 0, d.nsteps, lane);
                if (xbuf != nullptr) xc_columns<DT, MS, FUSED, TRANS>(p, d, xs, smem, at_pitch_of<MS>(), xbuf, lane);
                tw_f32x16 acc[MS][NCB];
                zero_acc<MS, NCB>(acc);
                run_steps<DT, MS, NCB>(acc, rg, smem, at_pitch_of<MS>(), p.blob + p.off_goff + (long)d.first_step * 32,
                                           p.blob + p.off_bvals + (long)d.first_step * NCB * 1024, 0, d.nsteps, lane);
                if (has_ew) add_ew_residual<DT, MS, NCB>(p, d.tile, 0, acc, smem, at_pitch_of<MS>(), lane);
                if constexpr (TRANS) store_tile_t<DT, MS, NCB, FUSED>(p, d, acc, stage, dpos, row0, lane, 0, NCB, xbuf);
                else store_tile<DT, MS, NCB, FUSED>(p, d, acc, stage, dpos, row0, lane, xbuf, xcols);
            }
            __syncthreads();  // everyone is done with the LDS copy of A and with misc[]
        } else if constexpr (MODE == 2) {
            // K streamed, multiplying waves and loading waves.  Chunk c is multiplied out of buffer c % 2
            // while the loading waves write chunk c+1 into the other buffer and request chunk c+3;
            // one barrier per chunk.
            constexpr int NMUL = kWaves / 2, NLD = kWaves - NMUL;
            constexpr int PB = 12;   // requests per loading wave and chunk: 64 rows x 384 columns in 4 waves
            const int set = item / p.n_mblocks, mb = item - set * p.n_mblocks;
            const int row0 = mb * p.row_step;
            const bool loader = wave >= NMUL;
            const int ti = set * p.tiles_per_set + wave;
            const bool active = wave < p.tiles_per_set && ti < p.T;      // (tiles_per_set <= NMUL: never a loading wave)
            const TileU d = fetch_tile(p, active ? ti : 0);
            const int* sp = step_ptr + d.step_ptr;
            const unsigned char* gt = p.blob + p.off_goff + (long)d.first_step * 32;
            const unsigned char* bt = p.blob + p.off_bvals + (long)d.first_step * NCB * 1024;
            auto chunk_width = [&](int c) {
                const int k0 = c * p.k_chunk;
                return (p.K - k0) < p.k_chunk ? (p.K - k0) : p.k_chunk;
            };
            if (tid < BM / 2) {
                *(unsigned*)(smem + (unsigned)p.k_chunk * p.at_pitch + tid * 4) = 0u;
                *(unsigned*)(smem + p.abuf_bytes + (unsigned)p.k_chunk * p.at_pitch + tid * 4) = 0u;
            }
            if constexpr (ROLE == 2) {
                const int lw = wave - NMUL;
                static_assert(PB == 12, "size of the carried register sets");
                // Transposed boundary: this wave's entries of the set's row lists, all chunks, in its own
                // piece of LDS ([chunk][8 * PB] rows, then [chunk] counts); filled when the set changes.
                constexpr int kListEntries = 8 * PB;
                unsigned short* my_rows = (unsigned short*)(smem + p.urow_off) + (long)lw * p.n_chunks * (kListEntries + 2);
                int* my_cnt = (int*)(my_rows + (long)p.n_chunks * kListEntries);
                const bool use_rows = TRANS && p.urow_off != 0;
                auto load_lists = [&](int st) {
                    const unsigned short* g = (const unsigned short*)(p.blob + p.off_urow) + (long)st * p.n_chunks * p.k_chunk;
                    const int* gc = (const int*)(p.blob + p.off_ucnt) + (long)st * p.n_chunks;
                    for (int c = 0; c < p.n_chunks; ++c) {
                        for (int e = lane; e < kListEntries; e += 64)
                            my_rows[c * kListEntries + e] = g[(long)c * p.k_chunk + 8 * (lw + (e >> 3) * NLD) + (e & 7)];
                        if (lane == 0) my_cnt[c] = gc[c];
                    }
                };
                // Across items: the ring of chunks (chunk c in LDS buffer (c + par) % 2, waiting in register set c % 2)
                // runs on into the NEXT item of the workgroup when that item has the same set of tiles: ring positions
                // n_chunks, n_chunks + 1, .. are its chunks 0, 1, ..  They are requested during this item's last chunks
                // and its chunk 0 is written to LDS while the multiplying waves work on this item's last chunk (the
                // buffers alternate, so that buffer is free), which is the state that start_item would otherwise only
                // begin to build when this item's steps are over.  With an odd number of chunks the buffers (`par`) and
                // the register sets change roles from one item to the next.
                // (`cross`, `nrow0`: set after the item's first barrier, where thread 0 has said which item comes next.)
                const bool ring = p.n_chunks >= 3;
                bool cross = false;
                int nrow0 = 0;
                auto issue_or_zero = [&](ARegs<PB>& ar, int c, int r0) {
                    const bool into_next = c >= p.n_chunks && cross && c - p.n_chunks < p.n_chunks;
                    if (c < p.n_chunks || into_next) {
                        if (into_next) { c -= p.n_chunks; r0 = nrow0; }
                        if (use_rows)
                            at_issue_rows<PB>(p, ar, r0, c * p.k_chunk, my_rows + c * kListEntries, uni(my_cnt[c]), lw, lane, NLD);
                        else
                            stage_issue<MSB, PB, TRANS, NTA>(p, ar, r0, c * p.k_chunk, chunk_width(c), lw, lane, NLD);
                    } else {
#pragma unroll
                        for (int b = 0; b < PB; ++b) ar.v[b] = tw_u32x4{0u, 0u, 0u, 0u};   // defined on every path
                    }
                };
                auto commit = [&](const ARegs<PB>& ar, int c) {
                    const bool into_next = c >= p.n_chunks && cross && c - p.n_chunks < p.n_chunks;
                    if (c < p.n_chunks || into_next) {
                        unsigned char* buf = smem + ((c + par) & 1) * p.abuf_bytes;          // by ring position
                        if (into_next) c -= p.n_chunks;
                        if (use_rows)
                            at_commit_rows<PB>(p, ar, buf, my_rows + c * kListEntries, uni(my_cnt[c]), lw, lane, NLD);
                        else
                            stage_commit<MSB, PB, TRANS>(p, ar, buf, chunk_width(c), lw, lane, NLD);
                    }
                };
                // chunk j waits in register set j % 2; the loop is unrolled by two so that the sets are
                // addressed statically.  The start of an item (chunk 0 in LDS, chunks 1 and 2 requested) was
                // done at the end of the previous item where there was one.
                ARegs<PB>& ar0 = pre0;
                ARegs<PB>& ar1 = pre1;
                auto start_item = [&](int r0) {
                    issue_or_zero(ar0, 0, r0);
                    issue_or_zero(ar1, 1, r0);
                    commit(ar0, 0);
                    issue_or_zero(ar0, 2, r0);
                };
                if (!preloaded) {
                    if (use_rows && set != lists_of) { load_lists(set); lists_of = set; }
                    start_item(row0);
                }
                __syncthreads();
                if (ring) {
                    const int nxt = misc[2];
                    cross = nxt < p.n_items && nxt / p.n_mblocks == set;
                    nrow0 = (nxt % p.n_mblocks) * p.row_step;
                }
                for (int c = 0; c < p.n_chunks; c += 2) {
                    commit(ar1, c + 1);
                    issue_or_zero(ar1, c + 3, row0);
                    __syncthreads();
                    if (c + 1 < p.n_chunks) {
                        commit(ar0, c + 2);
                        issue_or_zero(ar0, c + 4, row0);
                    }
                    __syncthreads();
                }
                // the multiplying waves are through with both buffers; the next item's first chunks are brought in
                // while they store this item's tiles, unless the ring has done that already
                __syncthreads();
                const int nxt = misc[2];
                preloaded = nxt < p.n_items;
                par ^= p.n_chunks & 1;
                if (preloaded && cross) {
                    if (p.n_chunks & 1) {        // ring positions n+1 and n+2 are the next item's chunks 1 and 2: sets 1 and 0 there
#pragma unroll
                        for (int b = 0; b < PB; ++b) { const tw_u32x4 t = ar0.v[b]; ar0.v[b] = ar1.v[b]; ar1.v[b] = t; }
                    }
                } else if (preloaded) {
                    const int nset = nxt / p.n_mblocks;
                    if (use_rows && nset != lists_of) { load_lists(nset); lists_of = nset; }
                    start_item((nxt % p.n_mblocks) * p.row_step);
                }
            } else {
                unsigned dpos[NCB];
                {
                    const unsigned* dp = (const unsigned*)(p.blob + p.off_dpos) + ((long)d.tile * 32 + (lane & 31)) * NCB;
#pragma unroll
                    for (int cb = 0; cb < NCB; ++cb) dpos[cb] = dp[cb];
                }
                tw_f32x16 acc[MS][NCB];
                zero_acc<MS, NCB>(acc);
                // residual-only columns of the tile's span (TEW): their sums wait in the staging area between chunks
                unsigned short* xbuf = nullptr;
                int xcols[TW_XC_INLINE / 8];
                if (xbuf_off != 0 && active) {
                    xbuf = (unsigned short*)(smem + xbuf_off) + wave * (TW_XC_INLINE * 64);
                    if constexpr (!TRANS) xc_column_numbers(p, d, xcols, lane);
                    xc_zero_partial<MS>(d, stage, lane);
                }
                // the first steps of a chunk are requested at the end of the previous chunk's steps, so
                // they arrive while the workgroup meets at the barrier
                StepRegs<NCB> rg;
                // first steps of the chunks: b0 = first step of chunk c, b1 of chunk c+1, b2 of chunk c+2, read one
                // chunk ahead with scalar loads so that no chunk waits for them
                int b0 = fetch_int(sp, 0), b1 = fetch_int(sp, 1), b2 = fetch_int(sp, p.n_chunks < 2 ? p.n_chunks : 2);
                auto prefetch_steps = [&](int c0, int c1) {
                    if (active && c0 < c1) {
                        prefetch_first_steps<NCB>(rg, gt, bt, c0, c1, lane);
                    } else {                               // defined on every path
#pragma unroll
                        for (int i = 0; i < kIdxAhead; ++i) rg.kk[i] = 0u;
#pragma unroll
                        for (int i = 0; i < prefetch_depth<NCB>(); ++i)
#pragma unroll
                            for (int cb = 0; cb < NCB; ++cb) rg.bq[i][cb] = tw_u16x8{0, 0, 0, 0, 0, 0, 0, 0};
                    }
                };
                auto steps_of = [&](int c) {
                    const unsigned char* buf = smem + ((c + par) & 1) * p.abuf_bytes;
                    if (active && b0 < b1)
                        run_steps<DT, MS, NCB>(acc, rg, buf, at_pitch_of<MS>(), gt, bt, b0, b1, lane);
                    if (has_ew && active) add_ew_residual<DT, MS, NCB>(p, d.tile, c, acc, buf, at_pitch_of<MS>(), lane);
                    if (xbuf != nullptr) xc_chunk<DT, MS>(p, d, c, buf, at_pitch_of<MS>(), stage, lane);
                    // on to chunk c+1
                    b0 = b1; b1 = b2;
                    b2 = fetch_int(sp, c + 3 < p.n_chunks ? c + 3 : p.n_chunks);
                    if (c + 1 < p.n_chunks) prefetch_steps(b0, b1); else prefetch_steps(0, 0);
                };
                prefetch_steps(b0, b1);
                if (tid == 0) misc[2] = my_next;   // the loading waves look one item ahead (requested at the top of this turn)
                __syncthreads();
                for (int c = 0; c < p.n_chunks; c += 2) {
                    steps_of(c);
                    __syncthreads();
                    if (c + 1 < p.n_chunks) steps_of(c + 1);
                    __syncthreads();
                }
                __syncthreads();
                par ^= p.n_chunks & 1;
                if (active) {
                    if (xbuf != nullptr) xc_finish<DT, MS, FUSED, TRANS>(p, d, stage, xbuf, lane);
                    if constexpr (TRANS) store_tile_t<DT, MS, NCB, FUSED>(p, d, acc, stage, dpos, row0, lane, 0, NCB, xbuf);
                    else store_tile<DT, MS, NCB, FUSED>(p, d, acc, stage, dpos, row0, lane, xbuf, xcols);
                }
            }
        } else {
            // K is streamed in chunks through two LDS buffers: the requests for chunk c+1 go out before
            // the steps of chunk c and are written to the other buffer after them, one barrier per chunk.
            // Split K (MODE 3, few row blocks): the item also names a part of the chunks, [c_first, c_first + n_loc),
            // and a set may have fewer than eight tiles (the other waves then only bring in A); the tiles' fp32
            // results go to the workspace and a second kernel adds the parts up.  A kernel variant of its own, so
            // that the unsplit kernel carries none of this.
            constexpr bool SPLIT = MODE == 3;
            const int sp_item = item / p.n_mblocks, mb = item - sp_item * p.n_mblocks;
            const int part = SPLIT ? sp_item / p.n_seg : 0, set = sp_item - part * p.n_seg;
            const int c_first = SPLIT ? part * p.chunks_per_part : 0;
            const int n_loc = !SPLIT ? p.n_chunks
                              : (p.n_chunks - c_first) < p.chunks_per_part ? (p.n_chunks - c_first) : p.chunks_per_part;
            const int row0 = mb * p.row_step;
            const int ti = set * (SPLIT ? p.tiles_per_set : kWaves) + wave;
            const bool active = (!SPLIT || wave < p.tiles_per_set) && ti < p.T;
            const TileU d = fetch_tile(p, active ? ti : 0);
            constexpr int AB = 6;    // requests per wave and chunk: 64 rows x 384 columns in 8 waves
            // (chunk j of the item is chunk c_first + j of K and lives in LDS buffer j % 2)
            auto chunk_width = [&](int j) {
                const int k0 = (c_first + j) * p.k_chunk;
                return (p.K - k0) < p.k_chunk ? (p.K - k0) : p.k_chunk;
            };
            auto issue_or_zero = [&](ARegs<AB>& ar, int j) {
                if (j < n_loc) {
                    stage_issue<MSB, AB, TRANS, NTA>(p, ar, row0, (c_first + j) * p.k_chunk, chunk_width(j), wave, lane);
                } else {
#pragma unroll
                    for (int b = 0; b < AB; ++b) ar.v[b] = tw_u32x4{0u, 0u, 0u, 0u};   // defined on every path
                }
            };
            auto commit = [&](const ARegs<AB>& ar, int j) {
                if (j < n_loc) stage_commit<MSB, AB, TRANS>(p, ar, smem + (j & 1) * p.abuf_bytes, chunk_width(j), wave, lane);
            };
            // Split K: the item's first chunk is requested before anything waits for the tile's descriptor (the
            // descriptor, the table of first steps and the first packed weights are three dependent round trips to
            // memory, and an item is only a few chunks long); written to LDS below, behind the first requests for
            // packed weights.  (Not in the unsplit kernel: the registers it takes there cost more than it gains.)
            ARegs<AB> first;
            if constexpr (SPLIT) {
                issue_or_zero(first, 0);
            } else {
                const int kw = chunk_width(0);
                if constexpr (TRANS) load_at_block<MSB, AB, NTA>(p, smem, row0, c_first * p.k_chunk, kw, wave, lane, tid);
                else load_a_block<MSB, AB, kPairStream, NTA>(p, smem, row0, c_first * p.k_chunk, kw, wave, lane, tid);
                a_zero_row(p, smem + p.abuf_bytes, BM, tid);
            }
            unsigned dpos[NCB];
            if constexpr (!SPLIT) {
                const unsigned* dp = (const unsigned*)(p.blob + p.off_dpos) + ((long)d.tile * 32 + (lane & 31)) * NCB;
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb) dpos[cb] = dp[cb];
            }
            tw_f32x16 acc[MS][NCB];
            zero_acc<MS, NCB>(acc);
            // residual-only columns of the tile's span (TEW): their sums wait in the staging area between chunks
            // (a split-K plan leaves them to the pass of their own)
            unsigned short* xbuf = nullptr;
            int xcols[TW_XC_INLINE / 8];
            if constexpr (!SPLIT) {
                if (xbuf_off != 0 && active) {
                    xbuf = (unsigned short*)(smem + xbuf_off) + wave * (TW_XC_INLINE * 64);
                    if constexpr (!TRANS) xc_column_numbers(p, d, xcols, lane);
                    xc_zero_partial<MS>(d, stage, lane);
                }
            }
            const int* sp = step_ptr + d.step_ptr;
            const unsigned char* gt = p.blob + p.off_goff + (long)d.first_step * 32;
            const unsigned char* bt = p.blob + p.off_bvals + (long)d.first_step * NCB * 1024;
            // Requests run kAhead chunks ahead of the steps: two where the registers allow it (narrow
            // tiles), so that a chunk is always on its way from memory, else one.
            constexpr int kAhead = (MS * NCB <= 4) ? 2 : 1;
            // first steps of chunk c (b0), c+1 (b1) and c+2 (b2), read one chunk ahead with scalar loads
            int b0 = fetch_int(sp, c_first), b1 = fetch_int(sp, c_first + 1),
                b2 = fetch_int(sp, c_first + 2 < p.n_chunks ? c_first + 2 : p.n_chunks);
            // the first steps of a chunk are requested at the end of the previous chunk's steps, so they arrive
            // while the chunk after it is written to LDS and the workgroup meets at the barrier
            StepRegs<NCB> rg;
            auto prefetch_steps = [&](int c0, int c1) {
                if (active && c0 < c1) {
                    prefetch_first_steps<NCB>(rg, gt, bt, c0, c1, lane);
                } else {                               // defined on every path
#pragma unroll
                    for (int i = 0; i < kIdxAhead; ++i) rg.kk[i] = 0u;
#pragma unroll
                    for (int i = 0; i < prefetch_depth<NCB>(); ++i)
#pragma unroll
                        for (int cb = 0; cb < NCB; ++cb) rg.bq[i][cb] = tw_u16x8{0, 0, 0, 0, 0, 0, 0, 0};
                }
            };
            auto steps_of = [&](int j) {
                const int c = c_first + j;
                if (active && b0 < b1)
                    run_steps<DT, MS, NCB>(acc, rg, smem + (j & 1) * p.abuf_bytes, at_pitch_of<MS>(), gt, bt, b0, b1, lane);
                if (has_ew && active) add_ew_residual<DT, MS, NCB>(p, d.tile, c, acc, smem + (j & 1) * p.abuf_bytes, at_pitch_of<MS>(), lane);
                if constexpr (!SPLIT)
                    if (xbuf != nullptr) xc_chunk<DT, MS>(p, d, c, smem + (j & 1) * p.abuf_bytes, at_pitch_of<MS>(), stage, lane);
                b0 = b1; b1 = b2;
                b2 = fetch_int(sp, c + 3 < p.n_chunks ? c + 3 : p.n_chunks);
                if (j + 1 < n_loc) prefetch_steps(b0, b1); else prefetch_steps(0, 0);
            };
            prefetch_steps(b0, b1);
            if constexpr (SPLIT) {
                commit(first, 0);
                a_zero_row(p, smem, BM, tid);
                a_zero_row(p, smem + p.abuf_bytes, BM, tid);
            }
            if constexpr (kAhead == 1) {
                __syncthreads();
                for (int j = 0; j < n_loc; ++j) {
                    ARegs<AB> ar;
                    issue_or_zero(ar, j + 1);
                    steps_of(j);
                    commit(ar, j + 1);
                    __syncthreads();
                }
            } else {
                // chunk j waits in ring register set j % 2; the loop is unrolled by two so that the sets
                // are addressed statically
                ARegs<AB> ar0, ar1;
                issue_or_zero(ar1, 1);
                __syncthreads();
                for (int j = 0; j < n_loc; j += 2) {
                    issue_or_zero(ar0, j + 2);
                    steps_of(j);
                    commit(ar1, j + 1);
                    __syncthreads();
                    if (j + 1 < n_loc) {
                        issue_or_zero(ar1, j + 3);
                        steps_of(j + 1);
                        commit(ar0, j + 2);
                    }
                    __syncthreads();
                }
            }
            if (active) {
                if constexpr (SPLIT) {
                    dump_partial<MS, NCB>(p.partials + ((((long)part * p.n_mblocks + mb) * p.T + ti) * (long)(MS * NCB * 1024)), acc, lane);
                } else {
                    if (xbuf != nullptr) xc_finish<DT, MS, FUSED, TRANS>(p, d, stage, xbuf, lane);
                    if constexpr (TRANS) store_tile_t<DT, MS, NCB, FUSED>(p, d, acc, stage, dpos, row0, lane, 0, NCB, xbuf);
                    else store_tile<DT, MS, NCB, FUSED>(p, d, acc, stage, dpos, row0, lane, xbuf, xcols);
                }
            }
        }
    }
    };
    if constexpr (MODE == 2) {
        if (wave >= kWaves / 2) run_items(std::integral_constant<int, 2>{});
        else run_items(std::integral_constant<int, 1>{});
    } else {
        run_items(std::integral_constant<int, 0>{});
    }
    // the last workgroup to leave puts the counters back to zero for the next call
    if (tid == 0 && p.n_items > (int)gridDim.x) {
        __threadfence();
        const int done = atomicAdd(&p.counters[1], 1);
        if (done == (int)gridDim.x - 1) {
            atomicExch(&p.counters[0], 0);
            atomicExch(&p.counters[1], 0);
        }
    }
}

// Second kernel of a split-K product.  A workgroup is one wave and takes one piece of one (row block, tile): on the
// row-major boundary one pass of the tile's epilogue (eight rows, all column blocks), on the transposed boundary
// one column block (all 64 tokens).  It adds that piece's partial results of all parts in the order of the parts
// (a fixed order: the result does not depend on which workgroup of the first kernel finished first) and stores it
// through the epilogue of the main kernel (column scatter, zeros of pruned columns, fused bias and activation).
// The pieces are this small because a compute unit brings in only about 16 KB per microsecond from memory (its
// queue of outstanding misses times the latency): a wave that summed a whole tile (32 KB per part) would take as
// long as the chunks it saves.
template <int DT, int NCB, bool FUSED, bool TRANS>
__global__ __launch_bounds__(64) void tw_splitk_reduce_kernel(const TwGemmParams p) {
    constexpr int MS = 2;
    constexpr int SUB = TRANS ? NCB : 4 * MS;               // pieces per tile
    constexpr int NL = TRANS ? 4 * MS : NCB;                // 1 KB loads per piece and part
    __shared__ __attribute__((aligned(16))) unsigned char stage[kStageBytes];
    const int lane = threadIdx.x & 63;
    const int unit = (int)blockIdx.x;                       // ((row block * T) + tile) * SUB + piece
    const int sub = unit % SUB, mt = unit / SUB;
    const int mb = mt / p.T, ti = mt - mb * p.T;
    const int row0 = mb * p.row_step;
    const TileU d = fetch_tile(p, ti);
    const long part_stride = (long)p.n_mblocks * p.T * (MS * NCB * 1024);
    const float* src = p.partials + ((long)mb * p.T + ti) * (long)(MS * NCB * 1024) + lane * 4;
    // load i of the piece: row-major (ms, q) = sub, cb = i; transposed cb = sub, (ms, q) = i
    int off[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const int msq = TRANS ? i : sub, cb = TRANS ? sub : i;
        off[i] = (((msq >> 2) * NCB + cb) * 4 + (msq & 3)) * 256;
    }
    // (the first part is requested before anything waits for the tile's descriptor)
    tw_f32x4 s[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) s[i] = *(const tw_f32x4*)(src + off[i]);
    unsigned dpos[NCB];
    {
        const unsigned* dp = (const unsigned*)(p.blob + p.off_dpos) + ((long)d.tile * 32 + (lane & 31)) * NCB;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) dpos[cb] = dp[cb];
    }
#pragma unroll 2
    for (int part = 1; part < p.n_parts; ++part) {
        tw_f32x4 v[NL];
#pragma unroll
        for (int i = 0; i < NL; ++i) v[i] = *(const tw_f32x4*)(src + part * part_stride + off[i]);
#pragma unroll
        for (int i = 0; i < NL; ++i) s[i] += v[i];
    }
    tw_f32x16 acc[MS][NCB];
    zero_acc<MS, NCB>(acc);
#pragma unroll
    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int msq = 4 * ms + q;
                if ((TRANS ? cb : msq) == sub) {            // wave-uniform
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[ms][cb][4 * q + e] = s[TRANS ? msq : cb][e];
                }
            }
    if constexpr (TRANS) store_tile_t<DT, MS, NCB, FUSED>(p, d, acc, stage, dpos, row0, lane, sub, sub + 1);
    else store_tile<DT, MS, NCB, FUSED>(p, d, acc, stage, dpos, row0, lane, nullptr, nullptr, sub, sub + 1);
}

}  // namespace

// ---- kernel tables
// The kernels can be compiled as eight translation units (-DTW_PART=1..4: fp16 / bf16 x plain / fused epilogue, 5..8:
// the same for TEW blobs) beside the host code (-DTW_PART=0), so that a build runs them in parallel; without TW_PART one unit holds
// everything.  The tables hand out host-side kernel addresses, so no type of this file crosses a unit boundary.
namespace tw_parts {
// (nta: the streamed kernels' variant whose requests for activations carry the streaming hint)
// (EW: the variant with the code of the element-wise residual, for TEW blobs)
template <int DT, bool FUSED, bool EW> const void* pick_mode(int mode, int ms, int ncb, bool nta);     // row-major boundary
template <int DT, bool FUSED, bool EW> const void* pick_mode_t(int mode, int ms, int ncb, bool nta);   // transposed boundary
template <int DT, bool FUSED> const void* pick_reduce(int ncb, bool transposed);               // second kernel of split K
}  // namespace tw_parts

#if !defined(TW_PART) || TW_PART != 0
namespace {
template <int DT, int MS, int MODE, bool FUSED, bool TRANS, bool EW, bool NTA = true>
const void* pick_ncb(int ncb) {
    switch (ncb) {
        case 1: return (const void*)tw_gemm_kernel<DT, MS, 1, MODE, FUSED, TRANS, NTA, EW>;
        case 2: return (const void*)tw_gemm_kernel<DT, MS, 2, MODE, FUSED, TRANS, NTA, EW>;
        case 4: return (const void*)tw_gemm_kernel<DT, MS, 4, MODE, FUSED, TRANS, NTA, EW>;
        default: return nullptr;
    }
}
}  // namespace
namespace tw_parts {
template <int DT, bool FUSED, bool EW>
const void* pick_mode(int mode, int ms, int ncb, bool nta) {
    if (mode == 0) return ms == 2 ? pick_ncb<DT, 2, 0, FUSED, false, EW>(ncb) : pick_ncb<DT, 1, 0, FUSED, false, EW>(ncb);
    if (ms != 2) return nullptr;                  // the streamed kernels take 64-row blocks
    if (mode == 1) return nta ? pick_ncb<DT, 2, 1, FUSED, false, EW, true>(ncb) : pick_ncb<DT, 2, 1, FUSED, false, EW, false>(ncb);
    if (mode == 3) {                              // split K: the epilogue is the second kernel's, so only the plain variant exists
        if constexpr (!FUSED) return nta ? pick_ncb<DT, 2, 3, false, false, EW, true>(ncb) : pick_ncb<DT, 2, 3, false, false, EW, false>(ncb);
        else return nullptr;
    }
    return nta ? pick_ncb<DT, 2, 2, FUSED, false, EW, true>(ncb) : pick_ncb<DT, 2, 2, FUSED, false, EW, false>(ncb);
}
// transposed boundary: resident K with blocks of 64 or 32 tokens, streamed K always with 64
template <int DT, bool FUSED, bool EW>
const void* pick_mode_t(int mode, int ms, int ncb, bool nta) {
    if (mode == 0) return ms == 2 ? pick_ncb<DT, 2, 0, FUSED, true, EW>(ncb) : pick_ncb<DT, 1, 0, FUSED, true, EW>(ncb);
    if (ms != 2) return nullptr;
    if (mode == 1) return nta ? pick_ncb<DT, 2, 1, FUSED, true, EW, true>(ncb) : pick_ncb<DT, 2, 1, FUSED, true, EW, false>(ncb);
    if (mode == 3) {
        if constexpr (!FUSED) return nta ? pick_ncb<DT, 2, 3, false, true, EW, true>(ncb) : pick_ncb<DT, 2, 3, false, true, EW, false>(ncb);
        else return nullptr;
    }
    return nta ? pick_ncb<DT, 2, 2, FUSED, true, EW, true>(ncb) : pick_ncb<DT, 2, 2, FUSED, true, EW, false>(ncb);
}
template <int DT, bool FUSED>
const void* pick_reduce(int ncb, bool transposed) {
    switch (ncb) {
        case 1: return transposed ? (const void*)tw_splitk_reduce_kernel<DT, 1, FUSED, true> : (const void*)tw_splitk_reduce_kernel<DT, 1, FUSED, false>;
        case 2: return transposed ? (const void*)tw_splitk_reduce_kernel<DT, 2, FUSED, true> : (const void*)tw_splitk_reduce_kernel<DT, 2, FUSED, false>;
        case 4: return transposed ? (const void*)tw_splitk_reduce_kernel<DT, 4, FUSED, true> : (const void*)tw_splitk_reduce_kernel<DT, 4, FUSED, false>;
        default: return nullptr;
    }
}
}  // namespace tw_parts
#endif

#ifdef TW_PART
#define TW_TABLES_EW(KW, DT, FUSED, EW)                                          \
    KW template const void* tw_parts::pick_mode<DT, FUSED, EW>(int, int, int, bool);  \
    KW template const void* tw_parts::pick_mode_t<DT, FUSED, EW>(int, int, int, bool);
#define TW_TABLES_REDUCE(KW, DT, FUSED) KW template const void* tw_parts::pick_reduce<DT, FUSED>(int, bool);
#define TW_TABLES_ALL(KW, DT, FUSED) TW_TABLES_EW(KW, DT, FUSED, false) TW_TABLES_EW(KW, DT, FUSED, true) TW_TABLES_REDUCE(KW, DT, FUSED)
#if TW_PART == 0
TW_TABLES_ALL(extern, TW_F16, false) TW_TABLES_ALL(extern, TW_F16, true) TW_TABLES_ALL(extern, TW_BF16, false) TW_TABLES_ALL(extern, TW_BF16, true)
#elif TW_PART == 1
TW_TABLES_EW(, TW_F16, false, false) TW_TABLES_REDUCE(, TW_F16, false)
#elif TW_PART == 2
TW_TABLES_EW(, TW_F16, true, false) TW_TABLES_REDUCE(, TW_F16, true)
#elif TW_PART == 3
TW_TABLES_EW(, TW_BF16, false, false) TW_TABLES_REDUCE(, TW_BF16, false)
#elif TW_PART == 4
TW_TABLES_EW(, TW_BF16, true, false) TW_TABLES_REDUCE(, TW_BF16, true)
#elif TW_PART == 5
TW_TABLES_EW(, TW_F16, false, true)
#elif TW_PART == 6
TW_TABLES_EW(, TW_F16, true, true)
#elif TW_PART == 7
TW_TABLES_EW(, TW_BF16, false, true)
#elif TW_PART == 8
TW_TABLES_EW(, TW_BF16, true, true)
#else
#error "TW_PART is 0 (host code) or 1..8 (kernels)"
#endif
#endif

#if !defined(TW_PART) || TW_PART == 0
namespace {

// C[m, n] = act(bias[n]) (zero without a bias) for a weight with no surviving column.
template <int DT>
__global__ void tw_fill_kernel(unsigned short* C, long ldc, int M, int N, const unsigned short* bias, int act) {
    const long n = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long total = (long)M * N;
    for (long i = n; i < total; i += (long)gridDim.x * blockDim.x) {
        const long col = i % N;
        C[(i / N) * ldc + col] = bias ? tw_cvt<DT>(tw_activate(tw_to_f32<DT>(bias[col]), act)) : (unsigned short)0;
    }
}

// Ct[n, m] = act(bias[n]) (zero without a bias): the transposed output of a weight with no surviving column.
template <int DT>
__global__ void tw_fill_rows_kernel(unsigned short* Ct, long ldct, int N, int M, const unsigned short* bias, int act) {
    const long t = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long total = (long)N * M;
    for (long i = t; i < total; i += (long)gridDim.x * blockDim.x) {
        const long n = i / M;
        Ct[n * ldct + (i % M)] = bias ? tw_cvt<DT>(tw_activate(tw_to_f32<DT>(bias[n]), act)) : (unsigned short)0;
    }
}

// ---- residual weights of a TEW blob in columns that keep no tile-wise weight (Sec. IV-A "Hybrid Pattern") ----
// The paper stores the element-wise part in CSC form and runs it as a sparse product of its own, added by
// linearity.  For the columns that own a packed column of a tile that happens inside the tiles' kernel; a
// column that the tile-wise pattern pruned altogether has none, so its few entries run here, after that
// kernel (which wrote the column's zeros, or act(bias)): C[m, n] = act(bias[n] + sum_e v_e * A[m, k_e]).
struct XcolParams {
    const unsigned short* A;
    unsigned short* C;
    const unsigned short* bias;
    const int* col;
    const int* ptr;
    const int* k;
    const unsigned short* v;
    const int* rank;            // position of a column among those of its tile
    long lda, ldc;
    int M, K, n_cols, act;
    int skip_below;             // columns with rank < skip_below were added by the tiles' kernel already
};

// Row-major boundary.  A workgroup takes 64 rows of A and 64 of the columns; wave w, lane r: row r, columns
// 16*w .. 16*w+15 of the group.  A comes through LDS in chunks of 256 K positions (coalesced 16-byte loads, the
// next chunk on its way in registers while this one is worked on), so that a lane's scattered 2-byte reads hit
// LDS, not memory; the entries of a column are walked in ascending K, chunk by chunk.  The wave holds 64 entries
// of each of its 16 columns, one entry per lane (fetched again when a column has used its 64 up), counts with a
// ballot how many of them lie inside the chunk and hands those round with v_readlane, four LDS reads in flight.
// (Fetched entry by entry, a column's 40 entries were 80 dependent round trips to memory: 220 us on the FFN-down
// of BERT-base against 60 now.)
constexpr int kXcChunk = 256, kXcPitch = 2 * kXcChunk + 8, kXcColsPerWg = 64;
template <int DT>
__global__ __launch_bounds__(256) void tw_xcol_kernel(const XcolParams p) {
    __shared__ __attribute__((aligned(16))) unsigned char at[64 * kXcPitch];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row0 = blockIdx.x * 64;
    const int j0 = blockIdx.y * kXcColsPerWg + 16 * wave;      // this wave's first column of the list
    float acc[16];
    int e[16], e1[16], base[16];                                // wave-uniform: next entry, end, entry that lane 0 holds
    int kreg[16];
    float vreg[16];
    auto fetch = [&](int i) {                                   // entries base[i] + lane of column i (clamped to its last)
        const int idx = base[i] + lane < e1[i] ? base[i] + lane : e1[i] - 1;
        const bool any = base[i] < e1[i];                        // wave-uniform
        kreg[i] = any ? p.k[idx] : 0x7fffffff;
        vreg[i] = any ? tw_to_f32<DT>(p.v[idx]) : 0.f;
    };
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int j = j0 + i;
        acc[i] = 0.f;
        const bool mine = j < p.n_cols && p.rank[j] >= p.skip_below;
        e[i] = base[i] = __builtin_amdgcn_readfirstlane(mine ? p.ptr[j] : 0);
        e1[i] = __builtin_amdgcn_readfirstlane(mine ? p.ptr[j + 1] : 0);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) fetch(i);
    const int kpad = (p.K + 7) & ~7;                             // rows are readable up to the next multiple of 8
    const unsigned char* arow = at + lane * kXcPitch;
    // staging of a chunk: 64 rows x 32 pieces of 16 bytes, eight per thread
    constexpr int kPieces = 64 * (kXcChunk / 8) / 256;
    tw_u32x4 stage[kPieces];
    auto request = [&](int c0) {
#pragma unroll
        for (int q = 0; q < kPieces; ++q) {
            const int id = tid + 256 * q;
            const int r = id / (kXcChunk / 8), pc = id % (kXcChunk / 8);
            int g = row0 + r;
            g = g < p.M ? g : p.M - 1;
            stage[q] = tw_u32x4{0u, 0u, 0u, 0u};
            if (c0 + 8 * pc < kpad) stage[q] = tw_load16_stream(p.A + (long)g * p.lda + c0 + 8 * pc);
        }
    };
    request(0);
    for (int c0 = 0; c0 < p.K; c0 += kXcChunk) {
        const int cend = c0 + kXcChunk;
        __syncthreads();                                         // everyone is through with the previous chunk
#pragma unroll
        for (int q = 0; q < kPieces; ++q) {
            const int id = tid + 256 * q;
            const int r = id / (kXcChunk / 8), pc = id % (kXcChunk / 8);
            *(tw_u32x2*)(at + r * kXcPitch + pc * 16) = tw_u32x2{stage[q].x, stage[q].y};
            *(tw_u32x2*)(at + r * kXcPitch + pc * 16 + 8) = tw_u32x2{stage[q].z, stage[q].w};
        }
        __syncthreads();
        if (cend < p.K) request(cend);                           // on its way while this chunk's entries are added
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            while (e[i] < e1[i]) {                               // (wave-uniform control flow)
                const int off = e[i] - base[i];                  // 0 .. 63: first unused entry among the 64 held
                const int held = e1[i] - base[i] < 64 ? e1[i] - base[i] : 64;
                // the held entries inside the chunk are consecutive from `off`: K ascends within a column
                const unsigned long long in = __builtin_amdgcn_ballot_w64(lane >= off && lane < held && kreg[i] < cend);
                const int n = __builtin_popcountll(in);
                auto a_of = [&](int t) {
                    const int k = __builtin_amdgcn_readlane(kreg[i], off + t);
                    return tw_to_f32<DT>(*(const unsigned short*)(arow + (k - c0) * 2));
                };
                auto w_of = [&](int t) {
                    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, vreg[i]), off + t));
                };
                int t = 0;
                for (; t + 4 <= n; t += 4) {
                    const float a0 = a_of(t), a1 = a_of(t + 1), a2 = a_of(t + 2), a3 = a_of(t + 3);
                    acc[i] += w_of(t) * a0;
                    acc[i] += w_of(t + 1) * a1;
                    acc[i] += w_of(t + 2) * a2;
                    acc[i] += w_of(t + 3) * a3;
                }
                for (; t < n; ++t) acc[i] += w_of(t) * a_of(t);
                e[i] += n;
                if (off + n < 64 || e[i] >= e1[i]) break;       // entries of a later chunk remain, or the column is done
                base[i] = e[i];                                  // all 64 used up: the column's next 64
                fetch(i);
            }
        }
    }
    const int m = row0 + lane;
    if (m < p.M) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int j = j0 + i;
            if (j < p.n_cols && p.rank[j] >= p.skip_below) {
                const int n = p.col[j];
                const float b = p.bias ? tw_to_f32<DT>(p.bias[n]) : 0.f;
                p.C[(long)m * p.ldc + n] = tw_cvt<DT>(tw_activate(acc[i] + b, p.act));
            }
        }
    }
}

// Transposed boundary: a column of C is a row of Ct and a K position a row of At, so a thread takes one token
// and the reads are coalesced as they are.  blockIdx.y walks the columns of the list.
template <int DT>
__global__ __launch_bounds__(256) void tw_xcol_t_kernel(const XcolParams p) {
    const long m = (long)blockIdx.x * 256 + threadIdx.x;
    if (m >= p.M) return;
    for (int j = blockIdx.y; j < p.n_cols; j += gridDim.y) {
        if (p.rank[j] < p.skip_below) continue;
        float acc = 0.f;
        int e = p.ptr[j];
        const int e1 = p.ptr[j + 1];
        // eight requests in flight per thread (one at a time, a column's 40 entries were 40 round trips to memory);
        // the products are added in the order of the entries either way
        for (; e + 8 <= e1; e += 8) {
            unsigned short a[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) a[u] = p.A[(long)p.k[e + u] * p.lda + m];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += tw_to_f32<DT>(p.v[e + u]) * tw_to_f32<DT>(a[u]);
        }
        for (; e < e1; ++e)
            acc += tw_to_f32<DT>(p.v[e]) * tw_to_f32<DT>(p.A[(long)p.k[e] * p.lda + m]);
        const int n = p.col[j];
        const float b = p.bias ? tw_to_f32<DT>(p.bias[n]) : 0.f;
        p.C[(long)n * p.ldc + m] = tw_cvt<DT>(tw_activate(acc + b, p.act));
    }
}

// Enqueues the pass over the residual's columns without tile-wise weights, if the blob has any.
int launch_xcols(const TwHeader* h, const void* blob_dev, const void* A, long lda, void* C, long ldc, int M,
                 const void* bias, int act, bool transposed, hipStream_t stream, bool inline_done = false) {
    if (h->xc_n <= 0 || M <= 0) return TW_OK;
    if (inline_done && h->xc_overflow == 0) return TW_OK;   // the tiles' kernel added them all
    const unsigned char* b = (const unsigned char*)blob_dev;
    XcolParams p;
    p.A = (const unsigned short*)A; p.C = (unsigned short*)C; p.bias = (const unsigned short*)bias;
    p.col = (const int*)(b + h->off_xc_col); p.ptr = (const int*)(b + h->off_xc_ptr);
    p.k = (const int*)(b + h->off_xc_k); p.v = (const unsigned short*)(b + h->off_xc_v);
    p.rank = (const int*)(b + h->off_xc_rank);
    p.lda = lda; p.ldc = ldc; p.M = M; p.K = h->K; p.n_cols = h->xc_n; p.act = act;
    p.skip_below = inline_done ? TW_XC_INLINE : 0;
    void* args[] = {(void*)&p};
    hipError_t rc;
    if (transposed) {
        const unsigned gy = (unsigned)(h->xc_n < 65535 ? h->xc_n : 65535);
        const void* fn = h->dtype == TW_F16 ? (const void*)tw_xcol_t_kernel<TW_F16> : (const void*)tw_xcol_t_kernel<TW_BF16>;
        rc = hipLaunchKernel(fn, dim3((unsigned)((M + 255) / 256), gy), dim3(256), args, 0, stream);
    } else {
        const long gy = ((long)h->xc_n + kXcColsPerWg - 1) / kXcColsPerWg;
        if (gy > 65535) return TW_ERR_UNSUPPORTED;
        const void* fn = h->dtype == TW_F16 ? (const void*)tw_xcol_kernel<TW_F16> : (const void*)tw_xcol_kernel<TW_BF16>;
        rc = hipLaunchKernel(fn, dim3((unsigned)((M + 63) / 64), (unsigned)gy), dim3(256), args, 0, stream);
    }
    return rc == hipSuccess ? TW_OK : TW_ERR_HIP;
}

struct Plan {
    int mode;       // kernel MODE
    int ms;         // the kernel's MS
    int n_mblocks, n_seg, n_items;
    int tiles_per_set;   // streamed K: tiles a workgroup holds
    int row_step;        // rows per row block (see TwGemmParams)
    unsigned at_pitch, abuf_bytes, stage_off, misc_off, lds_bytes;
    unsigned urow_off;   // transposed boundary, loading waves: LDS offset of their row lists (0: whole chunks are read)
    unsigned xbuf_off;   // row-major boundary, K resident, TEW blob with residual-only columns: LDS offset of the waves' areas for them
    int n_parts, chunks_per_part;   // split K (see TwGemmParams); n_parts = 1: none
    size_t partial_bytes;           // workspace the parts' fp32 results take, behind the counters
};


constexpr unsigned kLdsLimit = 160 * 1024;
// Estimates of the planner for streamed K when a launch has fewer items than compute units, in microseconds
// (fitted to the FFN-down of BERT-base and of BERT-large and to a lowered convolution, K = 2304 .. 4096 in 6 to 11
// chunks, M = 64 .. 6000, both boundaries).  Unsplit: kItemUs for the launch and the start of an item, then per
// chunk in sequence kChunkUs (what it takes a compute unit to bring in 64 rows x 384 columns of A; kChunkUsT on
// the transposed boundary, where whole rows go to LDS; kNarrowChunk of it for tiles of at most 64 columns, whose
// requests run two chunks ahead).  Split: kSplitItemUs (nothing overlaps the first chunk), a chunk takes longer
// the more workgroups stream at once (1 + kLoadedChunk at a full round), the tiles' partial results leave a
// compute unit at kCuStoreBytesPerUs; the second kernel costs kReduceUs plus, per wave that a compute unit gets,
// kReduceWaveUs and its loads at kCuLoadBytesPerUs.  A split must promise kSplitMargin of the unsplit time or less.
constexpr double kItemUs = 4.5, kChunkUs = 3.3, kChunkUsT = 2.8, kNarrowChunk = 0.85, kSplitItemUs = 5.5,
                 kLoadedChunk = 0.4, kCuStoreBytesPerUs = 38e3, kReduceUs = 2.5, kReduceWaveUs = 0.25,
                 kCuLoadBytesPerUs = 24e3, kSplitMargin = 0.9;

unsigned at_bytes(int msb, int k_chunk) {
    const unsigned pitch = 64u * msb + 8u;
    return ((unsigned)(k_chunk + 9) * pitch + 15u) & ~15u;
}
unsigned lds_need(int msb, int k_chunk, int buffers) {
    return buffers * at_bytes(msb, k_chunk) + kWaves * kStageBytes + 16u;
}

int make_plan(const TwHeader* h, int M, int n_cu, Plan& pl, bool transposed = false, size_t ws_avail = ~(size_t)0) {
    const bool resident = h->n_chunks == 1;
    const int buffers = resident ? 1 : 2;
    if (lds_need(1, h->k_chunk, buffers) > kLdsLimit) return TW_ERR_UNSUPPORTED;
    const int T = h->T;
    // msb: 32-row blocks in a workgroup's row block; tpw: tiles a workgroup of the streamed kernel holds
    auto items_for = [&](int msb, int tpw, int& n_mblocks, int& n_seg) {
        n_mblocks = (M + 32 * msb - 1) / (32 * msb);
        if (resident) {
            // split a row block's tiles over several workgroups only when there are too few row blocks
            n_seg = 1;
            if (n_mblocks < n_cu) n_seg = (n_cu + n_mblocks - 1) / n_mblocks;
            if (n_seg > T) n_seg = T;
            if (n_seg < 1) n_seg = 1;
            return (long)n_mblocks * n_seg;
        }
        n_seg = (T + tpw - 1) / tpw;
        return (long)n_mblocks * n_seg;
    };
    int msb = 2, tpw = kWaves;
    int nmb, nseg;
    if (lds_need(2, h->k_chunk, buffers) > kLdsLimit) msb = 1;
    pl.mode = resident ? 0 : 1;
    if (resident) {
        // 64-row blocks halve the traffic of packed B, but only pay when they still fill the GPU
        if (msb == 2 && items_for(2, tpw, nmb, nseg) < n_cu) msb = 1;
    } else if (msb == 2) {
        // Streamed K, 64-row blocks.  Eight tiles per workgroup (a wave per tile) when that gives every compute
        // unit an item and there are more than four tiles.  Else four waves multiply and four only load A
        // (MODE 2), with as many tiles per workgroup (4, 2, 1) as still fill the GPU: fewer tiles per workgroup
        // mean more workgroups per row block, each reading the block's rows of A again (from the caches).
        // Measured: skewed FFN-down of BERT-large, M = 8192, T = 8: 45 us with sets of four against 57 us with
        // 32-row blocks and a wave per tile; FFN-down of BERT-base, M = 512: see the design notes.
        if (T <= kWaves / 2 || items_for(2, kWaves, nmb, nseg) < n_cu) {
            pl.mode = 2;
            tpw = kWaves / 2;
            while (tpw > 1 && items_for(2, tpw, nmb, nseg) < n_cu) tpw >>= 1;
            // (an item takes about as long with fewer tiles, its time is the time to bring A in: one round of
            // workgroups that leaves compute units idle beats two rounds)
            if (tpw < kWaves / 2 && items_for(2, tpw, nmb, nseg) > n_cu) tpw <<= 1;
        }
    }
    if (!resident && msb != 2) return TW_ERR_UNSUPPORTED;   // (the streamed kernels take 64-row blocks; 384-row chunks fit)
    pl.ms = msb;
    long items = items_for(msb, tpw, nmb, nseg);
    if (items > 0x7fffffffL) return TW_ERR_UNSUPPORTED;
    pl.row_step = 32 * msb;
    // Row-major boundary, two to four rounds of 64-row blocks, the last one partly empty (M = 20001: 313 blocks
    // on 256 compute units): lower row blocks fill the last round, and every block then brings in and stores
    // fewer rows (40 instead of 64: 86 us instead of 100 us on the FFN-up of BERT-base).  With more rounds the
    // empty part of the last one weighs little and the extra blocks cost as much as they gain (the conv
    // workload, 6.1 rounds: no change with 56-row blocks).  The transposed boundary keeps 64 tokens: a block's
    // tokens are whole 128-byte lines of the output there.
    if (!transposed && msb == 2 && items > n_cu && items <= 4L * n_cu && items % n_cu != 0) {
        const long rounds = (items + n_cu - 1) / n_cu;
        const long blocks = rounds * n_cu / nseg;                 // row blocks that fit into that many rounds
        int rows = (int)(((M + blocks - 1) / blocks + 7) / 8 * 8);
        if (rows > 32 && rows < 64) {
            pl.row_step = rows;
            nmb = (M + rows - 1) / rows;
            items = (long)nmb * nseg;
        }
    }
    if (!resident && 4 * msb * ((((h->k_chunk + 7) >> 3) + 7) >> 3) > kWaves * 6) return TW_ERR_UNSUPPORTED;   // a chunk is one batch
    pl.n_mblocks = nmb; pl.n_seg = nseg; pl.n_items = (int)items;
    pl.at_pitch = 64u * msb + 8u;
    pl.abuf_bytes = at_bytes(msb, h->k_chunk);
    pl.stage_off = buffers * pl.abuf_bytes;
    pl.misc_off = pl.stage_off + kWaves * kStageBytes;
    pl.lds_bytes = pl.misc_off + 16u;
    pl.tiles_per_set = resident ? 0 : tpw;
    // Transposed boundary, at most four tiles, streamed: the loading waves read only the K rows the tiles keep,
    // from lists they hold in LDS.  (The blob's row lists are per set of TW_SET_TILES(T) tiles: with other sets
    // the loading waves bring in whole chunks.)
    pl.urow_off = 0;
    if (transposed && pl.mode == 2 && T <= kWaves / 2 && tpw == kWaves / 2) {
        const unsigned need = (kWaves / 2) * (unsigned)h->n_chunks * (8 * 12 + 2) * 2;
        if (pl.lds_bytes + need <= kLdsLimit) { pl.urow_off = pl.lds_bytes; pl.lds_bytes += need; }
    }
    // per-wave areas for the residual-only columns that the tiles add themselves (TEW), if there is room left
    pl.xbuf_off = 0;
    if (h->xc_n > 0) {
        const unsigned need = kWaves * TW_XC_INLINE * 64 * 2;
        if (pl.lds_bytes + need <= kLdsLimit) { pl.xbuf_off = pl.lds_bytes; pl.lds_bytes += need; }
    }
    // Split K.  With streamed K and few row blocks the plan above leaves most compute units idle while each
    // workgroup walks all chunks in sequence, and a compute unit brings A in at about 16 KB per microsecond only
    // (its queue of outstanding misses times the memory latency), 3 us per chunk.  The alternative: MODE 1 with
    // the chunks cut into parts of equal length and the tiles into sets of `tpw`, an item per (part, set, row
    // block), all in one round; the tiles' fp32 results go to the workspace and a second kernel adds them in a
    // fixed order and stores C.  Both the number of parts and the tiles per set are chosen by the estimate below;
    // the split is taken when its estimate is lower and the caller's workspace holds the partial results.
    // (Not where the tiles add the residual-only columns of a TEW blob themselves: a split leaves those to the pass
    // of their own, which reads all of A once more - 92 against 46 us on the FFN-down of BERT-base at 512 rows.)
    pl.n_parts = 1; pl.chunks_per_part = h->n_chunks; pl.partial_bytes = 0;
    if (!resident && msb == 2 && h->n_chunks >= 2 && (pl.xbuf_off == 0 || transposed)) {
        const long nmb1 = (M + 63) / 64;
        const size_t tile_bytes = (size_t)2 * h->ncb * 4096;          // fp32 results of a tile: 64 rows x G columns
        const int sub = transposed ? h->ncb : 8;                      // pieces of a tile in the second kernel
        const long units2 = nmb1 * T * sub;
        const double rounds0 = (double)((items + n_cu - 1) / n_cu);
        const double chunk_us = transposed ? kChunkUsT : kChunkUs;
        double best = rounds0 * (kItemUs + h->n_chunks * chunk_us * (h->ncb <= 2 ? kNarrowChunk : 1.0));
        int best_cpp = 0, best_tpw = 0;
        for (int sets = 1; sets <= T && nmb1 * sets * 2 <= n_cu; ++sets) {   // (at least two parts in one round)
            const int tpw1 = (T + sets - 1) / sets;
            if (tpw1 > kWaves || (sets > 1 && (T + sets - 2) / (sets - 1) == tpw1)) continue;   // (as many tiles per set with fewer sets)
            for (int cpp = h->n_chunks - 1; cpp >= 1; --cpp) {
                const int parts = (h->n_chunks + cpp - 1) / cpp;
                if (nmb1 * sets * parts > n_cu) break;
                if (cpp > 1 && (h->n_chunks + cpp - 2) / (cpp - 1) == parts) continue;   // a shorter part with as many parts follows
                const size_t bytes = (size_t)parts * nmb1 * T * tile_bytes;
                if (256 + bytes > ws_avail) continue;
                const double waves2 = (double)((units2 + n_cu - 1) / n_cu);     // of the second kernel, per compute unit
                const double loaded = 1.0 + kLoadedChunk * (double)(nmb1 * sets * parts) / n_cu;
                const double cost = kSplitItemUs + cpp * chunk_us * loaded + tpw1 * (double)tile_bytes / kCuStoreBytesPerUs +
                                    kReduceUs + waves2 * (kReduceWaveUs + parts * (double)(tile_bytes / sub) / kCuLoadBytesPerUs);
                if (cost < kSplitMargin * best) { best = cost / kSplitMargin; best_cpp = cpp; best_tpw = tpw1; }
            }
        }
        if (best_cpp > 0) {
            pl.mode = 1; pl.tiles_per_set = best_tpw; pl.row_step = 64; pl.urow_off = 0; pl.xbuf_off = 0;
            pl.chunks_per_part = best_cpp;
            pl.n_parts = (h->n_chunks + best_cpp - 1) / best_cpp;
            pl.n_mblocks = (int)nmb1; pl.n_seg = (T + best_tpw - 1) / best_tpw;
            pl.n_items = (int)(nmb1 * pl.n_seg * pl.n_parts);
            pl.partial_bytes = (size_t)pl.n_parts * nmb1 * T * tile_bytes;
            pl.lds_bytes = pl.misc_off + 16u;
        }
    }
    return TW_OK;
}

// the kernel for (dtype, mode, MS, NCB, fused epilogue): a host-side address for hipLaunchKernel and hipFuncSetAttribute
template <bool EW>
const void* pick_kernel_t_of(int dt, int mode, int ms, int ncb, bool fused, bool nta) {
    using namespace tw_parts;
    if (fused) return dt == TW_F16 ? pick_mode_t<TW_F16, true, EW>(mode, ms, ncb, nta) : pick_mode_t<TW_BF16, true, EW>(mode, ms, ncb, nta);
    return dt == TW_F16 ? pick_mode_t<TW_F16, false, EW>(mode, ms, ncb, nta) : pick_mode_t<TW_BF16, false, EW>(mode, ms, ncb, nta);
}
template <bool EW>
const void* pick_kernel_of(int dt, int mode, int ms, int ncb, bool fused, bool nta) {
    using namespace tw_parts;
    if (fused) return dt == TW_F16 ? pick_mode<TW_F16, true, EW>(mode, ms, ncb, nta) : pick_mode<TW_BF16, true, EW>(mode, ms, ncb, nta);
    return dt == TW_F16 ? pick_mode<TW_F16, false, EW>(mode, ms, ncb, nta) : pick_mode<TW_BF16, false, EW>(mode, ms, ncb, nta);
}
// (ew: the blob carries an element-wise residual)
const void* pick_kernel_t(int dt, int mode, int ms, int ncb, bool fused, bool nta, bool ew) {
    return ew ? pick_kernel_t_of<true>(dt, mode, ms, ncb, fused, nta) : pick_kernel_t_of<false>(dt, mode, ms, ncb, fused, nta);
}
const void* pick_kernel(int dt, int mode, int ms, int ncb, bool fused, bool nta, bool ew) {
    return ew ? pick_kernel_of<true>(dt, mode, ms, ncb, fused, nta) : pick_kernel_of<false>(dt, mode, ms, ncb, fused, nta);
}
const void* pick_reduce_kernel(int dt, int ncb, bool fused, bool transposed) {
    using namespace tw_parts;
    if (fused) return dt == TW_F16 ? pick_reduce<TW_F16, true>(ncb, transposed) : pick_reduce<TW_BF16, true>(ncb, transposed);
    return dt == TW_F16 ? pick_reduce<TW_F16, false>(ncb, transposed) : pick_reduce<TW_BF16, false>(ncb, transposed);
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
constexpr int kMaxKernels = 512;
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
    // the counters, and behind them the partial results of a split-K plan (the larger of the two boundaries'), as
    // planned for the current GPU (256 compute units when there is none to ask)
    size_t need = 256;
    if (M > 0 && h->T > 0 && h->n_chunks > 1) {
        int n_cu = 256;
        const int dev = current_device();
        if (dev >= 0 && device_cus(dev) > 0) n_cu = device_cus(dev);
        for (int tr = 0; tr < 2; ++tr) {
            Plan pl;
            if (make_plan(h, M, n_cu, pl, tr != 0) == TW_OK && 256 + pl.partial_bytes > need) need = 256 + pl.partial_bytes;
        }
    }
    *ws_bytes = need;
    return TW_OK;
}

extern "C" int tw_gemm_plan(const void* blob_host, int M, int n_cu, int transposed, tw_plan_t* plan) {
    if (!blob_host || !plan || M < 0 || n_cu <= 0) return TW_ERR_ARG;
    const TwHeader* h = (const TwHeader*)blob_host;
    if (h->magic != TW_MAGIC || h->version != TW_FORMAT_VERSION) return TW_ERR_BUF;
    memset(plan, 0, sizeof(*plan));
    if (M == 0 || h->T == 0) return TW_OK;      // nothing to multiply: a fill kernel at most
    Plan pl;
    const int rc = make_plan(h, M, n_cu, pl, transposed != 0);
    if (rc) return rc;
    plan->mode = pl.mode;
    plan->rows_per_block = pl.row_step;
    plan->tiles_per_set = pl.tiles_per_set;
    plan->n_row_blocks = pl.n_mblocks;
    plan->n_sets = pl.n_seg;
    plan->n_items = pl.n_items;
    plan->grid = pl.n_items < n_cu ? pl.n_items : n_cu;
    plan->lds_bytes = pl.lds_bytes;
    plan->row_lists = pl.urow_off != 0;
    plan->k_parts = pl.n_parts;
    return TW_OK;
}

extern "C" int tw_gemm(const void* blob_host, const void* blob_dev, const void* A, int M, int lda, void* C,
                       int ldc, void* workspace, size_t ws_bytes, void* hip_stream) {
    return tw_gemm_bias_act(blob_host, blob_dev, A, M, lda, nullptr, TW_ACT_NONE, C, ldc, workspace, ws_bytes,
                            hip_stream);
}

namespace {
// what tw_gemm and its variants on the row-major boundary refuse before anything is enqueued
int check_gemm_args(const void* blob_host, const void* blob_dev, const void* A, int M, int lda, const void* bias,
                    tw_act act, const void* C, int ldc, const void* workspace, size_t ws_bytes) {
    if (!blob_host || !blob_dev || !A || !C || !workspace || M < 0) return TW_ERR_ARG;
    if (act != TW_ACT_NONE && act != TW_ACT_RELU && act != TW_ACT_GELU) return TW_ERR_ARG;
    if (((uintptr_t)bias & 1) != 0) return TW_ERR_ALIGN;
    const TwHeader* h = (const TwHeader*)blob_host;
    if (h->magic != TW_MAGIC || h->version != TW_FORMAT_VERSION) return TW_ERR_BUF;
    if (ws_bytes < 256) return TW_ERR_BUF;
    if (lda < h->K || ldc < h->N) return TW_ERR_ARG;
    if ((lda & 7) != 0 || ((uintptr_t)A & 15) != 0 || ((uintptr_t)C & 1) != 0) return TW_ERR_ALIGN;
    if (((uintptr_t)blob_dev & 255) != 0 || ((uintptr_t)workspace & 255) != 0) return TW_ERR_ALIGN;
    return TW_OK;
}

// ---- scratch memory of the entry point that allocates nothing and takes no workspace (tw_gemm_static) ----
// The scheduler's counters (its first 256 bytes) and the fp32 partial results of a split-K plan (the rest; the
// planner takes a split only if they fit) live in this array instead of a buffer of the caller.  Only the counters
// need a defined start value; the partial results are written before they are read.  Every GPU holds its own
// copy at its own address; host code must use the address that hipGetSymbolAddress returns with that GPU
// current (the array's name is only a host-side stand-in), so it is looked up once per device and kept.
__device__ __align__(256) unsigned char tw_static_scratch[TW_STATIC_SCRATCH_BYTES];
std::atomic<void*> g_static_scratch[kMaxDevices];

int static_scratch(int dev, void** out) {
    void* ptr = g_static_scratch[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(tw_static_scratch)) != hipSuccess || !ptr) return TW_ERR_HIP;
        g_static_scratch[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return TW_OK;
}

// the counters start every call at zero, whatever an earlier call left behind (a kernel, not a memset: the
// call may be recorded into a graph)
__global__ void tw_clear_kernel(unsigned* w, int n) {
    if ((int)threadIdx.x < n) w[threadIdx.x] = 0u;
}
}  // namespace

extern "C" int tw_gemm_static(const void* blob_host, const void* blob_dev, const void* A, int M, int lda, void* C,
                              int ldc, void* hip_stream) {
    const int dev = current_device();
    if (dev < 0) return TW_ERR_HIP;
    void* scratch = nullptr;
    int rc = static_scratch(dev, &scratch);
    if (rc) return rc;
    rc = check_gemm_args(blob_host, blob_dev, A, M, lda, nullptr, TW_ACT_NONE, C, ldc, scratch, TW_STATIC_SCRATCH_BYTES);
    if (rc) return rc;
    if (M == 0) return TW_OK;
    unsigned* w_ = (unsigned*)scratch;
    int n_ = 64;
    void* cargs[] = {(void*)&w_, (void*)&n_};
    if (hipLaunchKernel((const void*)tw_clear_kernel, dim3(1), dim3(64), cargs, 0, (hipStream_t)hip_stream) != hipSuccess)
        return TW_ERR_HIP;
    return tw_gemm_bias_act(blob_host, blob_dev, A, M, lda, nullptr, TW_ACT_NONE, C, ldc, scratch, TW_STATIC_SCRATCH_BYTES,
                            hip_stream);
}

extern "C" int tw_gemm_bias_act(const void* blob_host, const void* blob_dev, const void* A, int M, int lda,
                                const void* bias, tw_act act, void* C, int ldc, void* workspace, size_t ws_bytes,
                                void* hip_stream) {
    {
        const int rc0 = check_gemm_args(blob_host, blob_dev, A, M, lda, bias, act, C, ldc, workspace, ws_bytes);
        if (rc0) return rc0;
    }
    const TwHeader* h = (const TwHeader*)blob_host;
    if (M == 0) return TW_OK;
    hipStream_t stream = (hipStream_t)hip_stream;

    if (h->T == 0) {
        const long total = (long)M * h->N;
        int blocks = (int)((total + 255) / 256);
        if (blocks > 4096) blocks = 4096;
        unsigned short* c_ = (unsigned short*)C;
        long ldc_ = ldc;
        int m_ = M, n_ = h->N, act_ = (int)act;
        const unsigned short* bias_ = (const unsigned short*)bias;
        void* fargs[] = {(void*)&c_, (void*)&ldc_, (void*)&m_, (void*)&n_, (void*)&bias_, (void*)&act_};
        const void* ffn = h->dtype == TW_F16 ? (const void*)tw_fill_kernel<TW_F16> : (const void*)tw_fill_kernel<TW_BF16>;
        if (hipLaunchKernel(ffn, dim3(blocks), dim3(256), fargs, 0, stream) != hipSuccess) return TW_ERR_HIP;
        return launch_xcols(h, blob_dev, A, lda, C, ldc, M, bias, (int)act, false, stream);
    }

    const int dev = current_device();
    if (dev < 0) return TW_ERR_HIP;
    const int n_cu = device_cus(dev);
    if (n_cu <= 0) return TW_ERR_HIP;
    Plan pl;
    int rc = make_plan(h, M, n_cu, pl, false, ws_bytes);
    if (rc) return rc;
    const bool split = pl.n_parts > 1;
    const bool fused_epilogue = bias != nullptr || act != TW_ACT_NONE;
    const bool fused = fused_epilogue && !split;      // split K: the epilogue is the second kernel's
    // streamed K: the activations carry the streaming hint only when one workgroup reads a row block's rows
    const bool nta = pl.mode == 0 || pl.n_seg == 1;
    const int kmode = split ? 3 : pl.mode;             // the kernel's MODE
    const void* fn = pick_kernel(h->dtype, kmode, pl.ms, h->ncb, fused, nta, h->ew_nnz > 0);
    if (!fn) return TW_ERR_UNSUPPORTED;
    const void* fn_reduce = nullptr;
    if (split) {
        fn_reduce = pick_reduce_kernel(h->dtype, h->ncb, fused_epilogue, false);
        if (!fn_reduce) return TW_ERR_UNSUPPORTED;
    }
    const int variant = kmode == 0 ? (pl.ms == 2 ? 0 : 1) : 2 * kmode + (nta ? 0 : 1);   // 0..7
    const int kernel_id = (h->ew_nnz > 0 ? 240 : 0) + (fused ? 60 : 0) + (h->dtype == TW_F16 ? 0 : 30) + 3 * variant + (h->ncb == 4 ? 0 : h->ncb == 2 ? 1 : 2);
    rc = ensure_lds(dev, kernel_id, fn);
    if (rc) return rc;

    TwGemmParams p;
    p.blob = (const unsigned char*)blob_dev;
    p.A = (const unsigned short*)A;
    p.C = (unsigned short*)C;
    p.counters = (int*)workspace;
    p.bias = (const unsigned short*)bias; p.act = (int)act;
    p.lda = lda; p.ldc = ldc;
    p.M = M; p.K = h->K; p.N = h->N; p.T = h->T;
    p.k_chunk = h->k_chunk; p.n_chunks = h->n_chunks; p.G = h->G;
    p.n_mblocks = pl.n_mblocks; p.n_seg = pl.n_seg; p.n_items = pl.n_items; p.tiles_per_set = pl.tiles_per_set; p.row_step = pl.row_step;
    p.at_pitch = pl.at_pitch; p.abuf_bytes = pl.abuf_bytes;
    p.stage_off = pl.stage_off; p.misc_off = pl.misc_off;
    p.off_sched_desc = h->off_sched_desc; p.off_step_ptr = h->off_step_ptr; p.off_goff = h->off_goff;
    p.off_dpos = h->off_dpos; p.off_bvals = h->off_bvals;
    p.off_zero_ptr = h->off_zero_ptr; p.off_zero_cols = h->off_zero_cols;
    p.off_urow = h->off_urow; p.off_ucnt = h->off_ucnt; p.urow_off = 0;
    p.off_ew_ptr = h->off_ew_ptr; p.off_ew_goff = h->off_ew_goff; p.off_ew_b = h->off_ew_b; p.has_ew = h->ew_nnz > 0;
    p.off_xm_ptr = h->off_xm_ptr; p.off_xm_goff = h->off_xm_goff; p.off_xm_b = h->off_xm_b; p.off_zero_xc = h->off_zero_xc;
    p.stream_stores = ((uintptr_t)C & 127) == 0 && (ldc & 63) == 0;
    p.off_xc_tile_ptr = h->off_xc_tile_ptr; p.off_xc_col = h->off_xc_col; p.off_xc_ptr = h->off_xc_ptr;
    p.off_xc_k = h->off_xc_k; p.off_xc_v = h->off_xc_v; p.xbuf_off = pl.xbuf_off;
    p.n_parts = pl.n_parts; p.chunks_per_part = pl.chunks_per_part;
    p.partials = (float*)((unsigned char*)workspace + 256);
    const int grid = pl.n_items < n_cu ? pl.n_items : n_cu;
    void* args[] = {(void*)&p};
    if (hipLaunchKernel(fn, dim3(grid), dim3(kThreads), args, pl.lds_bytes, stream) != hipSuccess) return TW_ERR_HIP;
    if (split) {
        const long units = (long)pl.n_mblocks * h->T * 8;                 // a wave per pass of a tile
        if (hipLaunchKernel(fn_reduce, dim3((unsigned)units), dim3(64), args, 0, stream) != hipSuccess) return TW_ERR_HIP;
    }
    return launch_xcols(h, blob_dev, A, lda, C, ldc, M, bias, (int)act, false, stream, pl.xbuf_off != 0);
}

extern "C" int tw_gemm_t(const void* blob_host, const void* blob_dev, const void* At, int M, int ldat, void* Ct,
                         int ldct, void* workspace, size_t ws_bytes, void* hip_stream) {
    return tw_gemm_t_bias_act(blob_host, blob_dev, At, M, ldat, nullptr, TW_ACT_NONE, Ct, ldct, workspace, ws_bytes,
                              hip_stream);
}

extern "C" int tw_gemm_t_bias_act(const void* blob_host, const void* blob_dev, const void* At, int M, int ldat,
                                  const void* bias, tw_act act, void* Ct, int ldct, void* workspace, size_t ws_bytes,
                                  void* hip_stream) {
    if (!blob_host || !blob_dev || !At || !Ct || !workspace || M < 0) return TW_ERR_ARG;
    if (act != TW_ACT_NONE && act != TW_ACT_RELU && act != TW_ACT_GELU) return TW_ERR_ARG;
    if (((uintptr_t)bias & 1) != 0) return TW_ERR_ALIGN;
    const bool fused_epilogue = bias != nullptr || act != TW_ACT_NONE;
    const TwHeader* h = (const TwHeader*)blob_host;
    if (h->magic != TW_MAGIC || h->version != TW_FORMAT_VERSION) return TW_ERR_BUF;
    if (ws_bytes < 256) return TW_ERR_BUF;
    if (ldat < M || ldct < M) return TW_ERR_ARG;
    if ((ldat & 7) != 0 || (ldct & 7) != 0 || ((uintptr_t)At & 15) != 0 || ((uintptr_t)Ct & 15) != 0) return TW_ERR_ALIGN;
    if (((uintptr_t)blob_dev & 255) != 0 || ((uintptr_t)workspace & 255) != 0) return TW_ERR_ALIGN;
    if (M == 0) return TW_OK;
    hipStream_t stream = (hipStream_t)hip_stream;

    if (h->T == 0) {   // every row of Ct is zero
        const long total = (long)h->N * M;
        int blocks = (int)((total + 255) / 256);
        if (blocks > 4096) blocks = 4096;
        unsigned short* c_ = (unsigned short*)Ct;
        long ldc_ = ldct;
        int n_ = h->N, m_ = M, act_ = (int)act;
        const unsigned short* bias_ = (const unsigned short*)bias;
        void* fargs[] = {(void*)&c_, (void*)&ldc_, (void*)&n_, (void*)&m_, (void*)&bias_, (void*)&act_};
        const void* ffn = h->dtype == TW_F16 ? (const void*)tw_fill_rows_kernel<TW_F16> : (const void*)tw_fill_rows_kernel<TW_BF16>;
        if (hipLaunchKernel(ffn, dim3(blocks), dim3(256), fargs, 0, stream) != hipSuccess) return TW_ERR_HIP;
        return launch_xcols(h, blob_dev, At, ldat, Ct, ldct, M, bias, (int)act, true, stream);
    }

    const int dev = current_device();
    if (dev < 0) return TW_ERR_HIP;
    const int n_cu = device_cus(dev);
    if (n_cu <= 0) return TW_ERR_HIP;
    Plan pl;
    int rc = make_plan(h, M, n_cu, pl, /*transposed=*/true, ws_bytes);
    if (rc) return rc;
    const bool split = pl.n_parts > 1;
    const bool fused = fused_epilogue && !split;      // split K: the epilogue is the second kernel's
    const bool nta = pl.mode == 0 || pl.n_seg == 1;
    const int kmode = split ? 3 : pl.mode;             // the kernel's MODE
    const void* fn = pick_kernel_t(h->dtype, kmode, pl.ms, h->ncb, fused, nta, h->ew_nnz > 0);
    if (!fn) return TW_ERR_UNSUPPORTED;
    const void* fn_reduce = nullptr;
    if (split) {
        fn_reduce = pick_reduce_kernel(h->dtype, h->ncb, fused_epilogue, true);
        if (!fn_reduce) return TW_ERR_UNSUPPORTED;
    }
    const int variant = kmode == 0 ? (pl.ms == 2 ? 0 : 1) : 2 * kmode + (nta ? 0 : 1);   // 0..7
    const int kernel_id = (h->ew_nnz > 0 ? 240 : 0) + 120 + (fused ? 60 : 0) + (h->dtype == TW_F16 ? 0 : 30) + 3 * variant + (h->ncb == 4 ? 0 : h->ncb == 2 ? 1 : 2);
    rc = ensure_lds(dev, kernel_id, fn);
    if (rc) return rc;

    TwGemmParams p;
    p.blob = (const unsigned char*)blob_dev;
    p.A = (const unsigned short*)At;
    p.C = (unsigned short*)Ct;
    p.counters = (int*)workspace;
    p.bias = (const unsigned short*)bias; p.act = (int)act;
    p.lda = ldat; p.ldc = ldct;
    p.M = M; p.K = h->K; p.N = h->N; p.T = h->T;
    p.k_chunk = h->k_chunk; p.n_chunks = h->n_chunks; p.G = h->G;
    p.n_mblocks = pl.n_mblocks; p.n_seg = pl.n_seg; p.n_items = pl.n_items; p.tiles_per_set = pl.tiles_per_set; p.row_step = pl.row_step;
    p.at_pitch = pl.at_pitch; p.abuf_bytes = pl.abuf_bytes;
    p.stage_off = pl.stage_off; p.misc_off = pl.misc_off;
    p.off_sched_desc = h->off_sched_desc; p.off_step_ptr = h->off_step_ptr; p.off_goff = h->off_goff;
    p.off_dpos = h->off_dpos; p.off_bvals = h->off_bvals;
    p.off_zero_ptr = h->off_zero_ptr; p.off_zero_cols = h->off_zero_cols;
    p.off_urow = h->off_urow; p.off_ucnt = h->off_ucnt;
    p.off_ew_ptr = h->off_ew_ptr; p.off_ew_goff = h->off_ew_goff; p.off_ew_b = h->off_ew_b; p.has_ew = h->ew_nnz > 0;
    p.off_xm_ptr = h->off_xm_ptr; p.off_xm_goff = h->off_xm_goff; p.off_xm_b = h->off_xm_b; p.off_zero_xc = h->off_zero_xc;
    p.urow_off = pl.urow_off;
    p.off_xc_tile_ptr = h->off_xc_tile_ptr; p.off_xc_col = h->off_xc_col; p.off_xc_ptr = h->off_xc_ptr;
    p.off_xc_k = h->off_xc_k; p.off_xc_v = h->off_xc_v; p.xbuf_off = pl.xbuf_off;
    p.stream_stores = ((uintptr_t)Ct & 127) == 0 && (ldct & 63) == 0;
    p.n_parts = pl.n_parts; p.chunks_per_part = pl.chunks_per_part;
    p.partials = (float*)((unsigned char*)workspace + 256);
    const unsigned lds_bytes = pl.lds_bytes;
    const int grid = pl.n_items < n_cu ? pl.n_items : n_cu;
    void* args[] = {(void*)&p};
    if (hipLaunchKernel(fn, dim3(grid), dim3(kThreads), args, lds_bytes, stream) != hipSuccess) return TW_ERR_HIP;
    if (split) {
        const long units = (long)pl.n_mblocks * h->T * h->ncb;            // a wave per column block of a tile
        if (hipLaunchKernel(fn_reduce, dim3((unsigned)units), dim3(64), args, 0, stream) != hipSuccess) return TW_ERR_HIP;
    }
    return launch_xcols(h, blob_dev, At, ldat, Ct, ldct, M, bias, (int)act, true, stream, pl.xbuf_off != 0);
}

// ---- the transposes at the two ends of a network that runs on the transposed boundary (Sec. VI) ----
namespace {
__global__ __launch_bounds__(256) void tw_transpose_kernel(const unsigned short* src, long lds_, int rows, int cols,
                                                           unsigned short* dst, long ldd, int vec) {
    // 64 x 64 tile through LDS, kept TRANSPOSED there: tile[c][r], rows of 144 bytes (16-byte aligned pieces, and
    // consecutive rows 4 banks apart)
    constexpr int kPitch = 144;
    __shared__ __attribute__((aligned(16))) unsigned char tile[64 * kPitch];
    const int c0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
    const int t = threadIdx.x;
    if (vec && r0 + 64 <= rows && c0 + 64 <= cols) {
        // whole tile, 16-byte aligned rows on both sides: 16-byte loads and stores, 2-byte LDS writes in between
        const int j = t & 7;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int r = (t >> 3) + 32 * i;
            const tw_u32x4 v = tw_load16_stream(src + (long)(r0 + r) * lds_ + c0 + 8 * j);   // read once, written once
            const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 8; ++e)
                *(unsigned short*)(tile + (8 * j + e) * kPitch + r * 2) = (unsigned short)(w[e >> 1] >> (16 * (e & 1)));
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int c = (t >> 3) + 32 * i;
            // (rows of dst on 128-byte boundaries: the eight lanes of a row write a whole line)
            if (vec == 2) tw_store16_stream(dst + (long)(c0 + c) * ldd + r0 + 8 * j, *(const tw_u32x4*)(tile + c * kPitch + j * 16));
            else *(tw_u32x4*)tw_opaque(dst + (long)(c0 + c) * ldd + r0 + 8 * j) = *(const tw_u32x4*)(tile + c * kPitch + j * 16);
        }
        return;
    }
    // edge tiles and unaligned matrices: element by element
    const int tx = t & 63, ty = t >> 6;
    for (int r = ty; r < 64; r += 4)
        if (r0 + r < rows && c0 + tx < cols) *(unsigned short*)(tile + tx * kPitch + r * 2) = src[(long)(r0 + r) * lds_ + c0 + tx];
    __syncthreads();
    for (int c = ty; c < 64; c += 4)
        if (c0 + c < cols && r0 + tx < rows) dst[(long)(c0 + c) * ldd + r0 + tx] = *(const unsigned short*)(tile + c * kPitch + tx * 2);
}
}  // namespace

extern "C" int tw_transpose(const void* src, int ld_src, int rows, int cols, void* dst, int ld_dst, void* hip_stream) {
    if (!src || !dst || rows < 0 || cols < 0 || ld_src < cols || ld_dst < rows) return TW_ERR_ARG;
    if (((uintptr_t)src & 1) != 0 || ((uintptr_t)dst & 1) != 0) return TW_ERR_ALIGN;
    if (rows == 0 || cols == 0) return TW_OK;
    const long gx = ((long)cols + 63) / 64, gy = ((long)rows + 63) / 64;
    if (gy > 65535) return TW_ERR_UNSUPPORTED;
    int vec = (((uintptr_t)src | (uintptr_t)dst) & 15) == 0 && (ld_src & 7) == 0 && (ld_dst & 7) == 0;
    if (vec && ((uintptr_t)dst & 127) == 0 && (ld_dst & 63) == 0) vec = 2;
    const unsigned short* s_ = (const unsigned short*)src;
    unsigned short* d_ = (unsigned short*)dst;
    long lds2 = ld_src, ldd2 = ld_dst;
    int vec_ = vec;
    void* targs[] = {(void*)&s_, (void*)&lds2, (void*)&rows, (void*)&cols, (void*)&d_, (void*)&ldd2, (void*)&vec_};
    return hipLaunchKernel((const void*)tw_transpose_kernel, dim3((unsigned)gx, (unsigned)gy), dim3(256), targs, 0,
                           (hipStream_t)hip_stream) == hipSuccess ? TW_OK : TW_ERR_HIP;
}
#endif  // host code
