// Internal layout of the packed-weight blob shared by the host packer and the HIP kernels.
// Everything is addressed by byte offsets from the blob start, so the bytes are relocatable.
#pragma once
#include <stdint.h>

#define TW_MAGIC 0x31425754u /* "TWB1" */
#define TW_FORMAT_VERSION 14

// MFMA step geometry the packed values are laid out for: one step contracts 16 kept rows
// (v_mfma_f32_32x32x16) against column blocks of 32 columns.
#define TW_KSTEP 16
// Waves per workgroup of the TW kernel (the packer shapes the dispatch order for it).
#ifndef TW_WAVES_PER_WG
#define TW_WAVES_PER_WG 8
#endif
#define TW_COLBLK 32
// Residual-only columns (TEW) that a tile's epilogue computes itself, per tile (see off_xc_rank).
#define TW_XC_INLINE 16
// Tiles per workgroup of the streamed kernels: a wave per tile, or with at most half as many tiles
// half of the waves multiply and the others only bring A into LDS.
#define TW_SET_TILES(T) ((T) <= TW_WAVES_PER_WG / 2 ? TW_WAVES_PER_WG / 2 : TW_WAVES_PER_WG)
// Padded contraction slots gather row `k_chunk` of the LDS copy of A, which the kernel keeps zero.

struct TwHeader {
    uint32_t magic;
    uint32_t version;
    int32_t dtype, K, N, G, T, n_kept_cols;
    int64_t nnz;
    uint64_t blob_bytes;
    int32_t k_chunk;      // K rows of A resident in LDS at a time
    int32_t n_chunks;     // ceil(K / k_chunk)
    int32_t ncb;          // column blocks per tile = G / 32
    int32_t xc_n;         // columns that hold only element-wise residual weights (see off_xc_col)
    int64_t total_steps;  // sum over tiles of 16-row steps (incl. padding)
    uint64_t off_col_idx, off_tile_col_ptr, off_tile_row_ptr, off_row_idx, off_tile_span,
        off_sched_order;
    uint64_t off_tile_desc;  // TwTileDesc[T], canonical tile order
    uint64_t off_step_ptr;   // int32 [T][n_chunks+1]: first step of every chunk, per tile
    uint64_t off_goff;       // uint16 [total_steps][16]: chunk-local K index of every contraction slot,
                             //   slot s = 8*h + 4*r + q stored at [h][q][r] (the order the lanes of a
                             //   transposing LDS read consume them); k_chunk for padded slots
    uint64_t off_dpos;       // uint32 [T][32][ncb]: destination column of packed column c = 32*cb + n, stored
                             //   at [n][cb], counted from the 8-aligned column at or below the tile's
                             //   span start; 0xFFFFFFFF for c >= w
    uint64_t off_bvals;      // 16-bit weights: per tile, per step, per column block, per lane 8 values
    uint64_t off_sched_desc; // TwSchedDesc[T], dispatch order (what the kernel walks)
    uint64_t off_zero_ptr;   // int32 [T+1]: per tile (canonical order), start of its list in zero_cols
    uint64_t off_zero_cols;  // int32 []: the pruned columns inside every tile's span, ascending (the rows of
                             //   the transposed output that the tile writes as zeros)
    uint64_t off_urow;       // streamed K only: uint16 [n_sets][n_chunks][k_chunk]: per set of tiles that a
                             //   workgroup of the streamed kernel holds (TW_SET_TILES(T) tiles in dispatch order)
                             //   and per chunk, the chunk-local K rows that any tile of the set keeps (in its tile-wise
                             //   pattern, in its element-wise residual or in the residual-only columns it adds itself), ascending
    uint64_t off_ucnt;       // int32 [n_sets][n_chunks]: their number
    // element-wise residual of the TEW hybrid (Sec. IV-A): the weights kept outside the tile-wise pattern, in the
    // tile's kept columns.  They are multiplied on the matrix cores like the tile itself, column block by column
    // block: per (tile, K chunk, column block) the K rows in which any of the block's 32 columns has a residual
    // weight, 16 to a step (in fours that a transposing LDS read takes from different banks, as far as such fours
    // go), with the block's weights of those rows (zero where there is none).  A residual step of a (tile, chunk)
    // is one such step of every column block; blocks with fewer rows are padded (zero row, weight 0).
    int64_t ew_nnz;          //   number of residual weights (0: none), those of off_xc_* included
    uint64_t off_ew_ptr;     //   int32 [T*n_chunks+1]: first residual step of every (tile, chunk), tiles in canonical order
    uint64_t off_ew_goff;    //   uint16 [rsteps][8][ncb][2]: chunk-local K row of slot 8*h + 4*r + q of column block cb at
                             //   [4*h + q][cb][r] (a lane reads the indices of all its column blocks in one piece);
                             //   k_chunk (the zero row) for unused slots
    uint64_t off_ew_b;       //   16-bit [rsteps][ncb][64][8]: the weights, per column block laid out like a step of bvals
    uint64_t off_ew_mask;    //   uint32 [rsteps][ncb][16]: bit n of word s: slot s of the block holds a residual weight of
                             //   packed column 32*cb + n (host side: a stored weight may be zero)
    // residual weights in columns that the tile-wise pattern prunes altogether: stored by column (the CSC form the
    // paper names for the element-wise part, Sec. IV-A) and added by a pass of their own after the tiles' kernel
    uint64_t off_xc_col;     //   int32 [xc_n]: original column, ascending
    uint64_t off_xc_ptr;     //   int32 [xc_n+1]: first entry of every such column
    uint64_t off_xc_k;       //   int32 [entries]: K row of the entry, ascending within a column
    uint64_t off_xc_v;       //   16-bit [entries]: its weight
    uint64_t off_xc_tile_ptr;//   int32 [T+1]: the columns of the list that lie in the span of tile t (canonical order) are
                             //   [xc_tile_ptr[t], xc_tile_ptr[t+1]) (the list is ascending and spans are disjoint)
    uint64_t off_xc_rank;    //   int32 [xc_n]: position of the column among those of its tile; the tile adds the first
                             //   TW_XC_INLINE itself (see off_xm_ptr), the rest (and everything in a split-K plan) goes
                             //   to the pass of its own
    int32_t xc_overflow;     //   columns with rank >= TW_XC_INLINE
    int32_t reserved1;
    // the first TW_XC_INLINE residual-only columns of every tile once more, as one column block for the matrix
    // cores (packed column j = the tile's j-th such column), in steps like those of off_ew_goff / off_ew_b
    uint64_t off_xm_ptr;     //   int32 [T*n_chunks+1]: first step of every (tile, chunk), tiles in canonical order
    uint64_t off_xm_goff;    //   uint16 [steps][16]: chunk-local K rows, slot order of off_goff; k_chunk for unused slots
    uint64_t off_xm_b;       //   16-bit [steps][64][8]: the weights
    uint64_t off_zero_xc;    // int8 [], parallel to zero_cols: position of the column among the residual-only columns of
                             //   its tile if the tile adds it itself (0 .. TW_XC_INLINE-1), else -1
    uint8_t pad[384 - 4 * 2 - 4 * 6 - 8 * 2 - 4 * 4 - 8 - 8 * 6 - 8 * 21 - 4 * 2 - 8 * 4];
};
static_assert(sizeof(TwHeader) == 384, "header is 384 bytes");

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
    uint32_t reserved1;
    uint32_t reserved2;
    uint8_t pad[64 - 4 * 8 - 8 - 4 * 2];
};
static_assert(sizeof(TwTileDesc) == 64, "tile descriptor is 64 bytes");

#define TW_TILE_NOGAP 1

// What the kernel needs of a tile, 32 bytes, in dispatch order.
struct TwSchedDesc {
    int32_t w;           // kept columns
    int32_t span_start;  // first original column owned
    int32_t span_w;      // original columns owned
    int32_t nsteps;      // 16-row steps, all chunks
    int32_t tile;        // canonical tile number (selects the dpos table)
    int32_t step_ptr;    // row of the step_ptr table (int32 units)
    int32_t first_step;  // first step in the goff / bvals tables
    int32_t xc;          // residual-only columns in the tile's span (TEW): xc_tile_ptr[tile] in the low 26 bits, above
                         //   them min(their number, TW_XC_INLINE)
};

// Chunking policy: the whole K extent of a 32-row block stays resident in LDS when it fits next to
// the epilogue staging area; otherwise A is streamed in chunks.
#define TW_K_RESIDENT_MAX 1536
#define TW_K_STREAM_CHUNK 384
