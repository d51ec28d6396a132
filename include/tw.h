/*
 * libtw - tile-wise (TW) sparse GEMM for AMD MI355X (gfx950).  C ABI.
 *
 * The operation (paper Sec. IV-A and Sec. VI): a weight matrix B (K x N) is cut into column tiles
 * of granularity G; whole columns may be pruned first, the surviving columns are re-grouped G at
 * a time, and every tile then keeps its own subset of the K rows.  With M the 0/1 mask of kept
 * weights the product is
 *
 *        C (M x N)  =  A (M x K) . (B * mask)
 *
 * which runs as one reduced-K dense GEMM per tile over the activation columns that tile keeps
 * (Fig. 4 step 4).  A and C stay dense (Sec. VI "Tiling"); B is compacted offline.
 *
 * Conventions
 *   - All matrices are row-major; ld* are row strides in ELEMENTS.  Elements of A, B, C are
 *     16-bit: IEEE binary16 (TW_F16) or bfloat16 (TW_BF16).  Products are accumulated in fp32
 *     and rounded to nearest-even once, at the store.
 *   - "host" pointers are ordinary memory, "device" pointers are HIP device memory of the
 *     current device.  The library never allocates or frees device memory and never
 *     synchronises: every device call only enqueues work on the given stream.
 *   - Every function returns TW_OK (0) or a negative tw_status; on error nothing is written
 *     to output buffers and nothing is enqueued.  No exceptions cross the boundary.
 *   - The packed weight is one relocatable byte blob (offsets, no pointers).  The same bytes
 *     are used on the host (launch parameters, tw_info, tw_unpack) and, copied by the caller,
 *     on the device.  Alignment of a blob buffer: 256 bytes on the device, 16 on the host.
 *   - Functions are thread-safe; the library keeps no mutable global state apart from the
 *     per-device kernel attributes it sets once.
 *   - Non-finite activations at positions a tile does NOT keep never reach the result (they
 *     are skipped, not multiplied by zero).
 */
#ifndef TW_H_
#define TW_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { TW_F16 = 0, TW_BF16 = 1 } tw_dtype;

typedef enum {
    TW_OK = 0,
    TW_ERR_ARG = -1,           /* null pointer, non-positive size, ld too small, unknown dtype   */
    TW_ERR_NOT_TILEWISE = -2,  /* the mask needs more than 2*ceil(N/G) tiles                     */
    TW_ERR_BUF = -3,           /* blob / workspace buffer too small, or not a blob               */
    TW_ERR_ALIGN = -4,         /* pointer or ld not aligned as required                          */
    TW_ERR_HIP = -5,           /* a HIP runtime call failed                                      */
    TW_ERR_UNSUPPORTED = -6    /* granularity or shape the kernels do not cover                  */
} tw_status;

/* Description of a packed weight.  The off_* members are byte offsets from the start of the blob
 * to int32 arrays in canonical form (exactly one correct value each):
 *   col_idx[n_kept_cols]  original index of every surviving column, ascending
 *   tile_col_ptr[T+1]     tile t holds surviving columns [tile_col_ptr[t], tile_col_ptr[t+1])
 *   tile_row_ptr[T+1]     tile t keeps rows row_idx[tile_row_ptr[t] .. tile_row_ptr[t+1])
 *   row_idx[sum k_t]      kept K rows of every tile, ascending within the tile
 *   tile_span[T+1]        tile t owns original columns [tile_span[t], tile_span[t+1]); pruned
 *                         columns inside are written as zeros by tw_gemm (tile_span[0] = 0,
 *                         tile_span[T] = N; a single 0 when T = 0)
 *   sched_order[T]        tiles by kept rows, descending (stable): the load-balancing order  */
typedef struct tw_info_t {
    int32_t version;
    int32_t dtype;
    int32_t K, N, G, T;
    int32_t n_kept_cols;
    int32_t k_chunk;           /* K rows of A staged in LDS at a time by tw_gemm                  */
    int64_t nnz;               /* kept weights of the tile-wise pattern                          */
    int64_t ew_nnz;            /* weights of the element-wise residual (tw_pack_tew), else 0     */
    int64_t padded_macs_per_row; /* multiply-adds per row of A the kernel really issues (>= nnz)  */
    uint64_t blob_bytes;
    uint64_t off_col_idx, off_tile_col_ptr, off_tile_row_ptr, off_row_idx, off_tile_span,
             off_sched_order;
} tw_info_t;

/* ---- host side, offline (Sec. VI "Tiling": pruned rows/columns of B are removed before inference) ---- */

/* Size in bytes of the blob tw_pack would write for this mask.
 * mask: host, K x N bytes, row-major, N per row; nonzero = kept.  G: tile granularity (32, 64 or 128).
 * Tiling rule (Sec. IV-A "Pruning Order"): a column survives iff it keeps a weight; surviving
 * columns, ascending, are swept left to right and a tile is closed when it has G columns or when
 * the next column keeps a different set of rows.  TW_ERR_NOT_TILEWISE if that gives more than
 * 2*ceil(N/G) tiles. */
int tw_pack_size(const uint8_t* mask, int K, int N, int G, tw_dtype dt, size_t* blob_bytes);

/* Build the blob: per-tile kept-row lists, compacted 16-bit tiles (bit-exact copies of the kept
 * weights, laid out for the MFMA operand loads), gather tables and the kept-K-sorted schedule.
 * B: host, K x N elements of type dt, row-major, ldb >= N.  blob: host buffer of blob_bytes
 * (>= tw_pack_size), 16-byte aligned, owned by the caller. */
int tw_pack(const void* B, int ldb, const uint8_t* mask, int K, int N, int G, tw_dtype dt,
            void* blob, size_t blob_bytes);

/* The TEW hybrid (Sec. IV-A "Hybrid Pattern"): on top of the tile-wise pattern `mask`, the weights marked
 * in `ew_mask` (K x N bytes; entries where mask is set as well are ignored) are kept as an element-wise
 * residual and added by tw_gemm and its variants (by linearity, A.(B*(mask|ew)) = A.(B*mask) + A.(B*ew)).
 * Residual weights in a column that keeps tile-wise weights are stored per tile and block of 32 packed columns
 * (the K rows that the block touches, 16 to a step, with the block's weights of those rows) and multiplied on
 * the matrix cores inside the tiles' kernel; residual weights in a column that the tile-wise pattern prunes
 * altogether are stored by column (the CSC form the paper names) and added by a second, small kernel that
 * tw_gemm enqueues behind the first, or (up to 16 such columns per tile, no split-K plan) by the tile that owns
 * the span.  ew_mask = NULL is tw_pack. */
int tw_pack_tew_size(const uint8_t* mask, const uint8_t* ew_mask, int K, int N, int G, tw_dtype dt,
                     size_t* blob_bytes);
int tw_pack_tew(const void* B, int ldb, const uint8_t* mask, const uint8_t* ew_mask, int K, int N, int G,
                tw_dtype dt, void* blob, size_t blob_bytes);

/* Which weights the hybrid puts back: the floor(delta*K*N + 0.5) weights of largest magnitude among all the
 * weights that `mask` prunes, wherever they lie (magnitude as importance score, ties to the lower (k, n));
 * ew_mask_out: K x N bytes, receives 0/1.  Host only. */
int tw_restore_ew(const void* B, int ldb, int K, int N, tw_dtype dt, const uint8_t* mask, double delta,
                  uint8_t* ew_mask_out);

/* Inverse of tw_pack, bit-exact: B_out (host, K x N, ldb) receives the kept weights and +0 at
 * pruned positions; mask_out (host, K x N bytes) receives 1/0.  Either output may be NULL.
 * For a TEW blob both include the element-wise residual (mask | ew_mask). */
int tw_unpack(const void* blob, void* B_out, int ldb, uint8_t* mask_out);

/* Fill *out from a host blob. */
int tw_info(const void* blob, tw_info_t* out);

/* One-shot magnitude pruning of a dense weight into the TW pattern: one stage of the paper's pruning
 * algorithm (Sec. V, Alg. 1) with the weight magnitude as importance score (the "most intuitive"
 * score of Sec. V), without apriori tuning and without fine-tuning.  Host only.
 *   1. column stage: the importance of a column is the sum of its magnitudes; the floor(col_prune*N
 *      + 0.5) least important columns are pruned (the lower index first among equals);
 *   2. the surviving columns are regrouped G at a time (Sec. IV-A); the importance of a row segment
 *      (one row of one tile) is the mean magnitude over its columns;
 *   3. row stage: row segments of ALL tiles are pruned in ascending importance (tile, then row,
 *      first among equals) until zeros / (K*N) >= sparsity; every tile keeps at least one row.
 * B: K x N row-major 16-bit values (ldb elements per row); mask_out: K x N bytes, receives 0/1.
 * Scores are accumulated in double, k ascending for columns and columns ascending for segments.
 * Returns TW_ERR_ARG for null pointers, non-positive sizes, or fractions outside [0, 1). */
int tw_prune(const void* B, int ldb, int K, int N, int G, tw_dtype dt, double col_prune,
             double sparsity, uint8_t* mask_out);

/* ---- device side ---- */

/* Bytes of device workspace tw_gemm and tw_gemm_t want for M rows: 256 bytes of scheduler counters and, where
 * the plan for the current GPU splits K (see tw_plan_t.k_parts), the parts' fp32 results behind them.  Only the
 * first 256 bytes are required: with less than the full size the product runs unsplit (slower for few rows and
 * a long K, never wrong).  The first 256 bytes must be zero before the first use; tw_gemm leaves them zero when
 * the enqueued work has finished, so one buffer serves any number of calls that do not overlap in time.  The
 * rest needs no initialisation. */
int tw_gemm_workspace(const void* blob_host, int M, size_t* ws_bytes);

/* How tw_gemm (transposed = 0) or tw_gemm_t (transposed != 0) would run this weight on M rows (tokens) on a GPU
 * with n_cu compute units: the host-side decision only, no GPU call.  Sec. VI ("Load Imbalance Mitigation",
 * "Tiling") leaves the thread-block shape and the distribution of tiles to the implementation; this is this one's. */
typedef struct tw_plan_t {
    int32_t mode;            /* 0: the K extent of a row block stays in on-chip memory, waves pull whole tiles;
                                1: K streamed in chunks, a wave per tile;
                                2: K streamed, four waves multiply (a tile each), four only load A */
    int32_t rows_per_block;  /* rows of A (tokens) of a work item: 64 or 32; tw_gemm may take a multiple of 8
                                between them so that the row blocks fill the last round of workgroups */
    int32_t tiles_per_set;   /* streamed K: tiles a workgroup holds (mode 1: 8; mode 2: 4, 2 or 1; a split-K plan: 1 to 8);
                                0 with mode 0 */
    int32_t n_row_blocks;    /* ceil(M / rows_per_block) */
    int32_t n_sets;          /* mode 0: workgroups that share the tiles of a row block; else sets of tiles */
    int32_t n_items;         /* work items = n_row_blocks * n_sets * k_parts */
    int32_t grid;            /* workgroups launched: min(n_items, n_cu), each pulls items until none is left */
    uint32_t lds_bytes;      /* on-chip memory per workgroup */
    int32_t row_lists;       /* tw_gemm_t, mode 2: the loading waves read only the K rows that the tiles keep */
    int32_t k_parts;         /* streamed K, few row blocks: the K chunks are split into this many parts, each a work item
                                of its own (n_items = n_row_blocks * n_sets * k_parts) whose fp32 results go to the
                                workspace; a second kernel adds them in the order of the parts.  1: no split.  (What
                                tw_gemm does with a workspace of tw_gemm_workspace bytes; with a smaller one it
                                does not split.) */
    int32_t reserved[6];
} tw_plan_t;
/* Errors: TW_ERR_ARG (null pointer, negative M, n_cu <= 0), TW_ERR_BUF (not a blob of this format version),
 * TW_ERR_UNSUPPORTED (what tw_gemm / tw_gemm_t would refuse for this blob and M).  M = 0 or a blob without
 * tiles gives an all-zero plan. */
int tw_gemm_plan(const void* blob_host, int M, int n_cu, int transposed, tw_plan_t* plan);

/* C = A . (B * mask) (Sec. VI, Listing 1's role).  Enqueues on `hip_stream` (a hipStream_t, may be
 * NULL for the default stream) and returns.
 *   blob_host  host copy of the blob (read during the call only)
 *   blob_dev   device copy of the same bytes, 256-byte aligned
 *   A          device, M x K, lda >= K, lda % 8 == 0, 16-byte aligned base.  Rows are read in
 *              16-byte pieces, i.e. up to the next multiple of 8 columns: the buffer must hold
 *              M x lda elements (what lies between K and that multiple is read and ignored)
 *   C          device, M x N, ldc >= N; EVERY element of C[0:M, 0:N] is written (zeros in pruned
 *              columns); 2-byte aligned rows suffice
 *   workspace  device, at least 256 bytes (tw_gemm_workspace bytes for the fastest plan), 256-byte aligned, its
 *              first 256 bytes zeroed as described above
 * M >= 0 (M = 0 enqueues nothing).  Calls on one workspace must not overlap in time (use one
 * workspace per stream).  The call enqueues kernels only (one; one more for a split-K plan, one more for a TEW
 * blob with residual weights in pruned columns) (no memset, no copy, no allocation), so it can be
 * recorded into a HIP graph; the first call that uses a kernel variant on a device raises that kernel's
 * dynamic-LDS limit (a function attribute), so make one call of each kind before a stream capture.  The best speed needs a C base and ldc that are multiples of 64 elements
 * (128-byte lines); any other layout is correct and slower.
 * Errors: TW_ERR_ARG (null pointer, negative M, lda/ldc too small), TW_ERR_BUF (not a blob of this
 * format version, workspace below 256 bytes), TW_ERR_ALIGN, TW_ERR_UNSUPPORTED (more than 2^31 work items),
 * TW_ERR_HIP (the launch failed); nothing is enqueued when an error is returned. */
int tw_gemm(const void* blob_host, const void* blob_dev, const void* A, int M, int lda,
            void* C, int ldc, void* workspace, size_t ws_bytes, void* hip_stream);

/* tw_gemm for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The scratch memory that tw_gemm takes from the
 * caller's workspace (the scheduler's counters and, for few rows and a long K, the fp32 partial results of a
 * split-K plan) lives in a device array inside the library instead, TW_STATIC_SCRATCH_BYTES per GPU, held until
 * the process ends; the call allocates nothing and frees nothing.  It enqueues a one-workgroup kernel that
 * zeroes the counters, then what tw_gemm enqueues for a workspace of that size: no blob and no M need more than
 * the counters, and a split-K plan is taken only when its partial results fit the array (tw_gemm_plan's k_parts
 * is for a workspace of tw_gemm_workspace bytes; with less the product runs with fewer parts or unsplit, never
 * out of bounds).  All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 * streams, two threads) race and give wrong results; calls on one stream, one after the other, are fine.
 * Arguments, results and errors as tw_gemm; TW_ERR_HIP also if the array's address cannot be obtained. */
#define TW_STATIC_SCRATCH_BYTES (8u << 20)
int tw_gemm_static(const void* blob_host, const void* blob_dev, const void* A, int M, int lda,
                   void* C, int ldc, void* hip_stream);

/* C = act(A . (B * mask) + bias): tw_gemm with the bias addition and the activation that follow a
 * weight GEMM inside a Transformer or CNN layer fused into its epilogue (Sec. VI "Kernel Fusion": the
 * non-GEMM operators around the GEMMs are fused so that they do not eat the GEMM's gain; here the
 * part that attaches to the GEMM itself is folded into it, the rest of a layer is out of scope).
 *   bias  device, N elements of the blob's dtype, 2-byte aligned, or NULL for no bias
 *   act   TW_ACT_NONE, TW_ACT_RELU (max(x, 0)) or TW_ACT_GELU (x/2 * (1 + erf(x / sqrt 2)))
 * The sum of the fp32 accumulator and the bias, and the activation, are evaluated in fp32 and rounded
 * once to the storage type.  A pruned column n of C holds act(bias[n]) in every row.  Everything else
 * as tw_gemm; TW_ERR_ARG also for an unknown act.  tw_gemm is this call with bias = NULL, act = NONE. */
typedef enum { TW_ACT_NONE = 0, TW_ACT_RELU = 1, TW_ACT_GELU = 2 } tw_act;
int tw_gemm_bias_act(const void* blob_host, const void* blob_dev, const void* A, int M, int lda,
                     const void* bias, tw_act act, void* C, int ldc, void* workspace, size_t ws_bytes,
                     void* hip_stream);

/* The same product on the transposed boundary (Sec. VI "Memory Accesses Coalescing": the paper stores
 * the activations and the result transposed, so that skipping a pruned K position skips a whole row and
 * the pruned columns of C become whole rows): Ct = (A . (B * mask))^T from At = A^T.
 *   At  device, K x M row-major (a row per K position, M tokens), ldat >= M, ldat % 8 == 0, 16-byte
 *       aligned; rows are read in 16-byte pieces up to the pitch
 *   Ct  device, N x M row-major, ldct >= M, ldct % 8 == 0, 16-byte aligned; EVERY element of
 *       Ct[0:N, 0:M] is written, rows of pruned columns as zeros.  Fastest with 128-byte aligned rows
 *       (base and ldct multiples of 64 elements).
 * Everything else as tw_gemm. */
int tw_gemm_t(const void* blob_host, const void* blob_dev, const void* At, int M, int ldat,
              void* Ct, int ldct, void* workspace, size_t ws_bytes, void* hip_stream);

/* Ct = act(A . (B * mask) + bias)^T: tw_gemm_t with the fused epilogue of tw_gemm_bias_act (bias: N elements,
 * one per ROW of Ct; a pruned column's row holds act(bias[n]) for every token). */
int tw_gemm_t_bias_act(const void* blob_host, const void* blob_dev, const void* At, int M, int ldat,
                       const void* bias, tw_act act, void* Ct, int ldct, void* workspace, size_t ws_bytes,
                       void* hip_stream);

/* dst[c, r] = src[r, c] for a rows x cols matrix of 16-bit elements (device pointers, row-major, ld in
 * elements): the transposes at the two ends of a network whose layers run on the transposed boundary
 * (Sec. VI "Kernel Fusion" counts them, unfused, at about 10 % of the latency). */
int tw_transpose(const void* src, int ld_src, int rows, int cols, void* dst, int ld_dst, void* hip_stream);

/* Dense reference C = A . B on the same MFMA pipeline (the paper's dense baseline, Sec. VI
 * "Tiling" / Sec. VII-A).  A: device M x K (lda % 8 == 0), B: device K x N row-major
 * (ldb % 8 == 0), C: device M x N (ldc % 8 == 0); bases 16-byte aligned. */
int tw_dense_gemm(const void* A, int lda, const void* B, int ldb, void* C, int ldc,
                  int M, int N, int K, tw_dtype dt, void* hip_stream);

/* C = act(A . B + bias), the dense yardstick with the same fused epilogue (bias: N elements of dt). */
int tw_dense_gemm_bias_act(const void* A, int lda, const void* B, int ldb, const void* bias, tw_act act,
                           void* C, int ldc, int M, int N, int K, tw_dtype dt, void* hip_stream);

const char* tw_strerror(int status);
int tw_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TW_H_ */
