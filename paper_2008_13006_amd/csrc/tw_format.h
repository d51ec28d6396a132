// Internal layout of the packed-weight blob shared by the host packer and the HIP kernels.
// Everything is addressed by byte offsets from the blob start, so the bytes are relocatable.
#pragma once
#include <stdint.h>

#define TW_MAGIC 0x31425754u /* "TWB1" */
#define TW_FORMAT_VERSION 1

// MFMA step geometry the packed values are laid out for: one step contracts 16 kept rows
// (v_mfma_f32_32x32x16) against column blocks of 32 columns.
#define TW_KSTEP 16
#define TW_COLBLK 32
// Byte offset (inside an LDS row of A) that padded contraction slots gather from: the row's
// zeroed pad, directly behind the k_chunk staged elements.  Stored as k_chunk*2 in the tables.

struct TwHeader {
    uint32_t magic;
    uint32_t version;
    int32_t dtype, K, N, G, T, n_kept_cols;
    int64_t nnz;
    uint64_t blob_bytes;
    int32_t k_chunk;      // K rows of A resident in LDS at a time
    int32_t n_chunks;     // ceil(K / k_chunk)
    int32_t ncb;          // column blocks per tile = G / 32
    int32_t reserved0;
    int64_t total_steps;  // sum over tiles of 16-row steps (incl. padding)
    uint64_t off_col_idx, off_tile_col_ptr, off_tile_row_ptr, off_row_idx, off_tile_span,
        off_sched_order;
    uint64_t off_tile_desc;  // TwTileDesc[T], canonical tile order
    uint64_t off_step_ptr;   // int32 [T][n_chunks+1]: first step of every chunk, per tile
    uint64_t off_goff;       // uint16 [total_steps][16]: LDS byte offsets of the gathered rows
    uint64_t off_dcol;       // uint16 [T][2][ncb][4][4]: destination column (relative to the span
                             //   start) of packed column c = 32*cb + 8*q + 4*h + e, stored at
                             //   [h][cb][q][e]; 0xFFFF for c >= w
    uint64_t off_bvals;      // 16-bit weights: per tile, per step, per column block, per lane 8 values
    uint8_t pad[256 - 4 * 2 - 4 * 6 - 8 * 2 - 4 * 4 - 8 - 8 * 6 - 8 * 5];
};
static_assert(sizeof(TwHeader) == 256, "header is 256 bytes");

struct TwTileDesc {
    int32_t w;           // kept columns (1..G)
    int32_t k;           // kept rows
    int32_t span_start;  // first original column owned
    int32_t span_w;      // number of original columns owned
    int32_t nsteps;      // 16-row steps, all chunks
    int32_t flags;       // bit 0: kept columns are exactly span_start .. span_start+w-1
    int32_t step_ptr;    // index of this tile's row in the step_ptr table (int32 units)
    int32_t first_step;  // index of this tile's first step in the goff table
    uint64_t bvals_off;  // byte offset from blob start of this tile's packed values
    uint32_t dcol_off;   // byte offset from blob start of this tile's dcol table
    uint32_t reserved;
    uint8_t pad[64 - 4 * 8 - 8 - 4 * 2];
};
static_assert(sizeof(TwTileDesc) == 64, "tile descriptor is 64 bytes");

#define TW_TILE_NOGAP 1

// Chunking policy: the whole K extent stays resident when it fits next to the epilogue staging
// area with 32-row blocks; otherwise A is streamed in double-buffered chunks.
#define TW_K_RESIDENT_MAX 1984
#define TW_K_STREAM_CHUNK 384
