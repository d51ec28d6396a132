// tw_dense_gemm: C = A . B, the dense yardstick of the TW kernel (the paper's baseline is a tiled
// dense GEMM on the matrix unit, Sec. IV-A Fig. 4 step 1 and Sec. VI "Tiling").  Same MFMA
// instruction, same operand roles, same epilogue as tw_gemm; B is ordinary row-major K x N.
//
// Workgroup: a (64 * MSW) x 256 block of C, 8 waves as 2 (rows) x 4 (columns), wave tile (32 * MSW) x 64;
// MSW = 4 (256 rows) where that still gives every compute unit a block, else 2 or 1 (the paper's tiling
// leaves the thread-block shape to the implementation, Sec. VI "Tiling").
// K advances 64 at a time through two LDS buffers; global loads of step i+1 are in flight
// while step i is multiplied.  The activation operand is read from LDS 16 bytes per lane, the
// weight operand with transposing reads (ds_read_b64_tr_b16) of the row-major B tile.
#include <hip/hip_runtime.h>

#include <atomic>

#include "../../include/tw.h"
#include "tw_device.hpp"

namespace {

typedef short tw_i16x4 __attribute__((ext_vector_type(4)));
constexpr int kThreads = 512;
constexpr int BN = 256, KB = 64;
constexpr int A_PITCH = KB * 2 + 16;   // 144 B: 16-byte reads of 16 consecutive rows hit distinct banks
constexpr int B_PITCH = BN * 2 + 64;   // 576 B: four consecutive K rows start 16 banks apart, as the transposing reads want
constexpr int B_BYTES = KB * B_PITCH;  // 36864
// MSW: 32-row blocks of a wave's tile; the workgroup's block has BM = 64 * MSW rows
template <int MSW> constexpr int bm_of() { return 64 * MSW; }
template <int MSW> constexpr int a_bytes_of() { return bm_of<MSW>() * A_PITCH; }            // 36864 for 256 rows
template <int MSW> constexpr int buf_bytes_of() { return a_bytes_of<MSW>() + B_BYTES; }
template <int MSW> constexpr int lds_bytes_of() {                                           // 147456 for 256 rows
    return 2 * buf_bytes_of<MSW>() > 8 * TW_STAGE_BYTES ? 2 * buf_bytes_of<MSW>() : 8 * TW_STAGE_BYTES;
}

struct DenseParams {
    const unsigned short* A;
    const unsigned short* B;
    unsigned short* C;
    long lda, ldb, ldc;
    int M, N, K;
    int nbm, nbn;
    const unsigned short* bias;   // N values added before the activation, or null
    int act;                      // tw_act
    int stream;                   // rows of C start on 128-byte boundaries: whole lines go out as streaming stores
};

template <int MSW>
struct Staged {
    tw_u32x4 a[MSW];
    tw_u32x4 b[4];
};

template <bool NT = false>
__device__ __forceinline__ tw_u32x4 load8_guard(const unsigned short* p, int valid) {
    // valid >= 8: one 16-byte load; 0 < valid < 8: element-wise, zero filled; <= 0: zeros
    if (valid >= 8) {
        if constexpr (NT) return tw_load16_stream(p);
        else return *(const tw_u32x4*)p;
    }
    unsigned short e[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) e[i] = i < valid ? p[i] : (unsigned short)0;
    return tw_u32x4{e[0] | ((unsigned)e[1] << 16), e[2] | ((unsigned)e[3] << 16), e[4] | ((unsigned)e[5] << 16),
                    e[6] | ((unsigned)e[7] << 16)};
}

// NTA: the activations are read by one column of blocks only (N <= 256), so they carry the streaming hint
template <int MSW, bool NTA>
__device__ __forceinline__ void global_fetch(const DenseParams& p, int m0, int n0, int k0, int tid, Staged<MSW>& st) {
    // A tile: 64 * MSW rows x 8 pieces of 16 B; thread handles pieces id = tid + 512*i
#pragma unroll
    for (int i = 0; i < MSW; ++i) {
        const int id = tid + kThreads * i;
        const int r = id >> 3, u = id & 7;
        int gm = m0 + r;
        gm = gm < p.M ? gm : p.M - 1;
        const int k = k0 + u * 8;
        st.a[i] = load8_guard<NTA>(p.A + (long)gm * p.lda + k, p.K - k);
    }
    // B tile: 64 rows x 32 pieces
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int id = tid + kThreads * i;
        const int r = id >> 5, u = id & 31;
        const int k = k0 + r, n = n0 + u * 8;
        if (k < p.K)
            st.b[i] = load8_guard(p.B + (long)k * p.ldb + n, p.N - n);
        else
            st.b[i] = tw_u32x4{0u, 0u, 0u, 0u};
    }
}

template <int MSW>
__device__ __forceinline__ void lds_commit(unsigned char* buf, int tid, const Staged<MSW>& st) {
#pragma unroll
    for (int i = 0; i < MSW; ++i) {
        const int id = tid + kThreads * i;
        const int r = id >> 3, u = id & 7;
        *(tw_u32x4*)(buf + r * A_PITCH + u * 16) = st.a[i];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int id = tid + kThreads * i;
        const int r = id >> 5, u = id & 31;
        *(tw_u32x4*)(buf + a_bytes_of<MSW>() + r * B_PITCH + u * 16) = st.b[i];
    }
}

template <int DT, int MSW, bool NTA>
__global__ __launch_bounds__(kThreads) void tw_dense_kernel(const DenseParams p) {
    constexpr int BM = bm_of<MSW>(), A_BYTES = a_bytes_of<MSW>(), BUF_BYTES = buf_bytes_of<MSW>();
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int h = lane >> 5, l32 = lane & 31;

    // workgroups that land on the same XCD (ids equal modulo 8) get neighbouring blocks of C,
    // so they share rows of A and columns of B in that XCD's L2
    int bid = blockIdx.x;
    const int total = p.nbm * p.nbn;
    if ((total & 7) == 0) bid = (bid & 7) * (total >> 3) + (bid >> 3);
    const int mb = bid / p.nbn, nb = bid - mb * p.nbn;
    const int m0 = mb * BM, n0 = nb * BN;

    tw_f32x16 acc[MSW][2];
#pragma unroll
    for (int ms = 0; ms < MSW; ++ms)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[ms][cb][r] = 0.f;

    const int nk = (p.K + KB - 1) / KB;
    Staged<MSW> st;
    global_fetch<MSW, NTA>(p, m0, n0, 0, tid, st);
    lds_commit(smem, tid, st);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        unsigned char* cur = smem + (kt & 1) * BUF_BYTES;
        unsigned char* nxt = smem + ((kt + 1) & 1) * BUF_BYTES;
        const bool more = kt + 1 < nk;
        if (more) global_fetch<MSW, NTA>(p, m0, n0, (kt + 1) * KB, tid, st);

        const unsigned char* la = cur + (wm * 32 * MSW + l32) * A_PITCH + h * 16;
        // weight operand by transposing reads of the row-major (K-major) B tile: in each 16-lane block,
        // lane j addresses K row 8h + 4r + j/4 at the four columns 4*(j%4) .. of the block's 16 columns
        const int j = lane & 15;
        const unsigned char* lb = cur + A_BYTES + (8 * h + (j >> 2)) * B_PITCH +
                                  (wn * 64 + ((lane >> 4) & 1) * 16 + (j & 3) * 4) * 2;
#pragma unroll
        for (int ks = 0; ks < KB / 16; ++ks) {
            tw_u16x8 w[2], a[MSW];
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                const tw_i16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) tw_i16x4*)(lb + (ks * 16) * B_PITCH + cb * 64));
                const tw_i16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) tw_i16x4*)(lb + (ks * 16 + 4) * B_PITCH + cb * 64));
                w[cb] = tw_u16x8{(unsigned short)lo4[0], (unsigned short)lo4[1], (unsigned short)lo4[2],
                                 (unsigned short)lo4[3], (unsigned short)hi4[0], (unsigned short)hi4[1],
                                 (unsigned short)hi4[2], (unsigned short)hi4[3]};
            }
#pragma unroll
            for (int ms = 0; ms < MSW; ++ms) a[ms] = *(const tw_u16x8*)(la + ms * 32 * A_PITCH + ks * 32);
#pragma unroll
            for (int ms = 0; ms < MSW; ++ms)
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) acc[ms][cb] = tw_mfma<DT>(w[cb], a[ms], acc[ms][cb]);
        }
        if (more) lds_commit(nxt, tid, st);
        __syncthreads();
    }

    // epilogue through per-wave staging areas laid over the (now idle) operand buffers
    unsigned char* stage = smem + wave * TW_STAGE_BYTES;
    const int col0 = n0 + wn * 64;
    const int width = (p.N - col0) < 64 ? (p.N - col0) : 64;
    if (width > 0) {
#pragma unroll
        for (int ms = 0; ms < MSW; ++ms)
            tw_store_block<DT, 2>(acc[ms], stage, p.C, p.ldc, m0 + wm * 32 * MSW + ms * 32, p.M, col0, width, lane,
                                  p.bias, p.act, p.stream != 0);
    }
}

template <int MSW>
const void* pick(tw_dtype dt, bool nta) {
    if (dt == TW_F16) return nta ? (const void*)tw_dense_kernel<TW_F16, MSW, true> : (const void*)tw_dense_kernel<TW_F16, MSW, false>;
    return nta ? (const void*)tw_dense_kernel<TW_BF16, MSW, true> : (const void*)tw_dense_kernel<TW_BF16, MSW, false>;
}

}  // namespace

extern "C" int tw_dense_gemm(const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K,
                             tw_dtype dt, void* hip_stream) {
    return tw_dense_gemm_bias_act(A, lda, B, ldb, nullptr, TW_ACT_NONE, C, ldc, M, N, K, dt, hip_stream);
}

extern "C" int tw_dense_gemm_bias_act(const void* A, int lda, const void* B, int ldb, const void* bias, tw_act act,
                                      void* C, int ldc, int M, int N, int K, tw_dtype dt, void* hip_stream) {
    if (!A || !B || !C || M < 0 || N <= 0 || K <= 0) return TW_ERR_ARG;
    if (act != TW_ACT_NONE && act != TW_ACT_RELU && act != TW_ACT_GELU) return TW_ERR_ARG;
    if (((uintptr_t)bias & 1) != 0) return TW_ERR_ALIGN;
    if (dt != TW_F16 && dt != TW_BF16) return TW_ERR_ARG;
    if (lda < K || ldb < N || ldc < N) return TW_ERR_ARG;
    if ((lda & 7) || (ldb & 7) || (ldc & 7)) return TW_ERR_ALIGN;
    if (((uintptr_t)A & 15) || ((uintptr_t)B & 15) || ((uintptr_t)C & 15)) return TW_ERR_ALIGN;
    if (M == 0) return TW_OK;
    DenseParams p;
    p.A = (const unsigned short*)A; p.B = (const unsigned short*)B; p.C = (unsigned short*)C;
    p.lda = lda; p.ldb = ldb; p.ldc = ldc;
    p.M = M; p.N = N; p.K = K;
    p.bias = (const unsigned short*)bias; p.act = (int)act;
    p.stream = ((uintptr_t)C & 127) == 0 && (ldc & 63) == 0;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return TW_ERR_HIP;
    static std::atomic<int> n_cus[64];
    int n_cu = n_cus[dev].load(std::memory_order_relaxed);
    if (n_cu <= 0) {
        if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0) return TW_ERR_HIP;
        n_cus[dev].store(n_cu, std::memory_order_relaxed);
    }
    // Rows per block: 256, 128 or 64, whichever needs the least time by a simple model: rounds of workgroups
    // times the block height, with 25 % (80 %) on top for the lower blocks, which read the weights more often.
    // (768 -> 768 at M = 16384 makes 192 blocks of 256 rows: one round at three quarters of the chip beats the
    // two rounds of 128-row blocks; 4096 -> 1024 at M = 8192 makes 128 blocks: 128-row blocks fill the chip.)
    p.nbn = (N + BN - 1) / BN;
    int msw = 4;
    double best = 0.0;
    for (int cand = 4; cand >= 1; cand >>= 1) {
        const long blk = (long)((M + 64 * cand - 1) / (64 * cand)) * p.nbn;
        const double cost = (double)((blk + n_cu - 1) / n_cu) * cand * (cand == 4 ? 1.0 : cand == 2 ? 1.25 : 1.8);
        if (cand == 4 || cost < best) { best = cost; msw = cand; }
    }
    p.nbm = (M + 64 * msw - 1) / (64 * msw);
    const long blocks = (long)p.nbm * p.nbn;
    if (blocks > 0x7fffffffL) return TW_ERR_UNSUPPORTED;
    const void* fn;
    int lds;
    const bool nta = p.nbn == 1;
    if (msw == 4) { fn = pick<4>(dt, nta); lds = lds_bytes_of<4>(); }
    else if (msw == 2) { fn = pick<2>(dt, nta); lds = lds_bytes_of<2>(); }
    else { fn = pick<1>(dt, nta); lds = lds_bytes_of<1>(); }
    static std::atomic<unsigned char> lds_set[64][2][10];
    const int slot = 2 * msw + (nta ? 1 : 0);
    if (!lds_set[dev][dt][slot].load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess) return TW_ERR_HIP;
        lds_set[dev][dt][slot].store(1, std::memory_order_release);
    }
    void* args[] = {(void*)&p};
    return hipLaunchKernel(fn, dim3((unsigned)blocks), dim3(kThreads), args, lds, (hipStream_t)hip_stream) == hipSuccess
               ? TW_OK : TW_ERR_HIP;
}
