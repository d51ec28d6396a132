// Device-side building blocks shared by the TW and the dense kernels (gfx950 only).
//
// MFMA used: v_mfma_f32_32x32x16_{f16,bf16}.  Operand layout (64-lane wave, lane l):
//   first operand  (32 x 16): row  i = l % 32, contraction slots 8*(l/32) .. 8*(l/32)+7
//   second operand (16 x 32): col  j = l % 32, contraction slots 8*(l/32) .. 8*(l/32)+7
//   result 32 x 32, 16 floats per lane: register r holds row i = 8*(r/4) + 4*(l/32) + r%4, col j = l%32
// The kernels put the WEIGHT tile in the first operand (i = output column n) and the ACTIVATIONS
// in the second (j = output row m), so a lane owns one row m of C and, per group of four
// registers, four consecutive columns: stores to row-major C need no cross-lane transpose.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/tw.h"

typedef _Float16 tw_f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 tw_bf16x8 __attribute__((ext_vector_type(8)));
typedef float tw_f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned short tw_u16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short tw_u16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int tw_u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int tw_u32x2 __attribute__((ext_vector_type(2)));
typedef tw_u32x4 __attribute__((aligned(2))) tw_u32x4_a2;
typedef tw_u32x2 __attribute__((aligned(2))) tw_u32x2_a2;
typedef unsigned int __attribute__((aligned(2))) tw_u32_a2;

template <int DT>
__device__ __forceinline__ tw_f32x16 tw_mfma(tw_u16x8 w, tw_u16x8 a, tw_f32x16 c) {
    if constexpr (DT == TW_F16) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(tw_f16x8, w),
                                                      __builtin_bit_cast(tw_f16x8, a), c, 0, 0, 0);
    } else {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(tw_bf16x8, w),
                                                       __builtin_bit_cast(tw_bf16x8, a), c, 0, 0, 0);
    }
}

// fp32 -> 16-bit storage type, round to nearest even.
template <int DT>
__device__ __forceinline__ unsigned short tw_cvt(float x) {
    if constexpr (DT == TW_F16) {
        _Float16 h = (_Float16)x;
        return __builtin_bit_cast(unsigned short, h);
    } else {
        __bf16 b = (__bf16)x;
        return __builtin_bit_cast(unsigned short, b);
    }
}

// 16-bit storage type -> fp32 (exact).
template <int DT>
__device__ __forceinline__ float tw_to_f32(unsigned short bits) {
    if constexpr (DT == TW_F16) {
        return (float)__builtin_bit_cast(_Float16, bits);
    } else {
        return __builtin_bit_cast(float, (unsigned)bits << 16);
    }
}

// GELU in its exact form x * Phi(x) = x/2 * (1 + erf(x / sqrt 2)), in fp32, with erf by the rational
// approximation 7.1.26 of Abramowitz and Stegun,
//   erf(y) = 1 - (a1 t + a2 t^2 + a3 t^3 + a4 t^4 + a5 t^5) exp(-y^2),  t = 1 / (1 + p y),  y >= 0,
// absolute error below 1.5e-7: far below the rounding of the 16-bit result, and straight-line code (the library
// routine is a page of branches, which costs registers when it is inlined 128 times).  With y = |x| / sqrt 2 and
// q = (a1 t + ... + a5 t^5) exp(-x^2 / 2) / 2 both signs of x give  gelu(x) = max(x, 0) - |x| q,  which needs no
// sign transfer and no 1 + erf; the constants carry the factors 1/2, 1/sqrt 2 and log2(e), the exponential is the
// hardware's base-2 one.  The vector ALU bounds the fused GELU, so every operation here shows in the time.
__device__ __forceinline__ float tw_gelu(float x) {
    const float ax = __builtin_fabsf(x);
    const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(0.23164189f, ax, 1.f));        // p / sqrt 2
    float poly = 0.5307027145f;                                                           // a5 / 2, a4 / 2, ...
    poly = __builtin_fmaf(poly, t, -0.7265760135f);
    poly = __builtin_fmaf(poly, t, 0.7107068705f);
    poly = __builtin_fmaf(poly, t, -0.142248368f);
    poly = __builtin_fmaf(poly, t, 0.127414796f);
    const float e = __builtin_amdgcn_exp2f(-0.72134752f * (x * x));                       // exp(-x^2 / 2)
    const float q = poly * t * e;
    return __builtin_fmaf(-ax, q, __builtin_fmaxf(x, 0.f));
}

// Activation of the fused epilogue, in fp32.  act is wave-uniform.
__device__ __forceinline__ float tw_activate(float x, int act) {
    if (act == TW_ACT_RELU) return x > 0.f ? x : 0.f;
    if (act == TW_ACT_GELU) return tw_gelu(x);
    return x;
}

// Orders this wave's LDS traffic: everything issued before is complete and visible to the
// wave's other lanes afterwards.  Not a workgroup barrier.
__device__ __forceinline__ void tw_wave_lds_sync() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_wave_barrier();
}

// Staging area of one wave in the epilogue.  The dense kernel uses it as 32 rows x 64 columns of
// 16-bit values, rows 136 bytes apart (the 8 extra bytes spread rows over the LDS banks); the TW
// kernel as 8 rows x 256 columns, rows 528 bytes apart.
#define TW_STAGE_PITCH 136
#define TW_STAGE_BYTES 4864
#define TW_STAGE_COLS 64

// 16-byte store with the streaming hint (the line is not kept in the L2 after the write).  For stores that
// complete whole 128-byte lines of the output this is faster than the plain store: on the BERT-base FFN-up shape
// 9 us of 55 (the whole lines no longer push the lines that two tiles share out of the L2 before their second
// half arrives), 3 us of 46 with tiles on a fixed grid, 2 us of 42 on the transposed boundary, 9 us of 96 in the
// dense kernel.  A line that another store completes later must NOT be written this way: the pieces then reach
// memory one by one (the same workload with every store streaming: 68 us instead of 55).
// (Written with the compiler's builtin, not inline assembly: the compiler has to know that this is a store, or it
// reuses the data registers too early.)
__device__ __forceinline__ void tw_store16_stream(void* p, tw_u32x4 v) {
    __builtin_nontemporal_store(v, (tw_u32x4_a2*)p);
}
// Returns p, but hides where it came from.  Used where a plain store and a streaming store of the same value to the
// same address sit in the two arms of a branch: otherwise the optimiser folds the arms into one plain store.
template <typename T>
__device__ __forceinline__ T* tw_opaque(T* p) {
    asm volatile("" : "+v"(p));
    return p;
}

// 16-byte load with the streaming hint, for data that is read once (the activations): it does not push the
// packed weights, which every workgroup re-reads, out of the L2.
__device__ __forceinline__ tw_u32x4 tw_load16_stream(const void* p) {
    return __builtin_nontemporal_load((const tw_u32x4*)p);
}


// Writes one 32-row block of a wave's results to C[row0.., col0 .. col0+width) through the wave's
// LDS staging area, 64 columns at a time (used where result column c goes to column col0 + c).
//   acc[cb][r]   fp32 results: lane l owns row (l%32) and column c = 32*cb + 8*(r/4) + 4*(l/32) + r%4
// bias (may be null): element col0 + c is added to column c before the activation `act`.
// stream: col0 and the rows of C are multiples of 64 elements from a 128-byte boundary, so a full window of 64
// columns is a whole line per row and may be written with streaming stores.
template <int DT, int NCB>
__device__ __forceinline__ void tw_store_block(const tw_f32x16 (&acc)[NCB], unsigned char* stage, unsigned short* C,
                                               long ldc, int row0, int M, int col0, int width, int lane,
                                               const unsigned short* bias = nullptr, int act = 0, bool stream = false) {
    const int mrow = lane & 31, h = lane >> 5;
    unsigned char* myrow = stage + mrow * TW_STAGE_PITCH;
    for (int w0 = 0; w0 < width; w0 += TW_STAGE_COLS) {
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int c_lo = 32 * cb + 8 * q;          // wave-uniform: columns c_lo .. c_lo+7
                if (c_lo < w0 || c_lo >= w0 + TW_STAGE_COLS) continue;
                float x[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) x[e] = acc[cb][4 * q + e];
                if (bias != nullptr || act != 0) {           // wave-uniform
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int c = c_lo + 4 * h + e;
                        const float b = (bias != nullptr && c < width) ? tw_to_f32<DT>(bias[col0 + c]) : 0.f;
                        x[e] = tw_activate(x[e] + b, act);
                    }
                }
                tw_u32x2 v;
                v.x = (unsigned)tw_cvt<DT>(x[0]) | ((unsigned)tw_cvt<DT>(x[1]) << 16);
                v.y = (unsigned)tw_cvt<DT>(x[2]) | ((unsigned)tw_cvt<DT>(x[3]) << 16);
                *(tw_u32x2*)(myrow + (c_lo + 4 * h - w0) * 2) = v;
            }
        }
        tw_wave_lds_sync();
        // 8 lanes cover the 64 columns of a row with 16-byte pieces, 8 rows per pass
        const int j = lane & 7;
        const int left = width - w0;                 // columns of this window that exist (may exceed 64)
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int r = (lane >> 3) + 8 * p;
            const int grow = row0 + r;
            const tw_u32x2 lo = *(const tw_u32x2*)(stage + r * TW_STAGE_PITCH + j * 16);
            const tw_u32x2 hi = *(const tw_u32x2*)(stage + r * TW_STAGE_PITCH + j * 16 + 8);
            if (grow < M && 8 * j + 8 <= left) {
                // whole 128-byte lines (the caller says whether rows of C start on line boundaries)
                if (stream && left >= TW_STAGE_COLS) tw_store16_stream(C + (long)grow * ldc + col0 + w0 + 8 * j, tw_u32x4{lo.x, lo.y, hi.x, hi.y});
                else *(tw_u32x4_a2*)tw_opaque(C + (long)grow * ldc + col0 + w0 + 8 * j) = tw_u32x4{lo.x, lo.y, hi.x, hi.y};
            }
        }
        // ragged end of the row: fewer than 8 columns left in the last group, one row per lane
        if (left < TW_STAGE_COLS && (left & 7) != 0) {
            const int rem = left & 7, cbeg = left & ~7;
            const int grow = row0 + mrow;
            if (h == 0 && grow < M) {
                unsigned short* dstp = C + (long)grow * ldc + col0 + w0 + cbeg;
                for (int e = 0; e < rem; ++e) dstp[e] = *(const unsigned short*)(myrow + (cbeg + e) * 2);
            }
        }
        tw_wave_lds_sync();
    }
}
