// Internal declarations shared by the translation units of libsga.so (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "sga.h"

namespace sga {

constexpr int kHeadDim = 64;          // the only supported d
constexpr int kWave = 64;             // CDNA wavefront width

// ---- split-row parameters (gather path) -----------------------------------
constexpr int kSplitThreshold = 8192; // rows with more neighbours are split
constexpr int kSplitChunk = 2048;     // target edges per chunk
constexpr int kMaxSplit = 64;         // at most this many chunks per row

// ---- tile path parameters -----------------------------------------------------
constexpr int kTile = 32;                 // query rows per tile = keys per block
constexpr int kPairEdges = 128;           // a tile qualifies if it averages >= this many edges per block
constexpr int kTileSplitThreshold = 64;   // tiles with more key blocks are split
constexpr int kTileChunk = 16;            // target key blocks per chunk
constexpr int kTileMaxSplit = 128;        // at most this many chunks per tile
constexpr int kTileItemSlots = 2048;      // upper bound of split-tile work items per call
constexpr int kTilePartialFloats = kTile * 64 + 2 * kTile;   // o[32][64], m[32], l[32]

// ---- workspace layout -------------------------------------------------------
// [0, 256)            counters (uint32): see WsCounter
// items               cap_items x int2 {row, chunk}                    (gather split)
// long_rows           cap_items x int4 {row, base, nchunks, chunk_len}
// partials            cap_items x H x kPartialStride floats {acc[d], m, l}
// tile_nblk           n_tiles x int32: key blocks of the tile, or -1 (tile goes to the gather path)
// pair_blk            cap_pairs x int32: key block id (| full flag); tile t owns slots
//                     [row_ptr[32t]/128, row_ptr[32(t+1)]/128)
// pair_mask           cap_pairs x 32 x uint32: bit j of word r = edge (row 32t+r, key 32b+j)
// titems / tlong / tpartials: the split-tile analogue of items / long_rows / partials
enum WsCounter : int {
  kCtrChunksNeeded = 0,   // sum of chunk counts of all long rows
  kCtrItemsAlloc = 1,     // bump allocator over items
  kCtrLongRows = 2,       // number of long rows recorded
  kCtrTileChunksNeeded = 3,
  kCtrTileItems = 4,      // bump allocator over split-tile work items
  kCtrTileLong = 5,       // number of split tiles recorded
  kNumCounters = 64
};

struct WorkspacePlan {
  // gather split
  int64_t cap_items;
  size_t off_items, off_long, off_partials;
  // tile path
  int64_t n_tiles;        // ceil(L / 32)
  int64_t cap_pairs;      // capacity of the (tile, key block) pair arrays
  int64_t cap_titems;     // capacity of split-tile work items
  size_t off_tile_nblk, off_pair_blk, off_pair_mask, off_titems, off_tlong,
      off_tpartials;
  size_t total_bytes;
};

constexpr int kPartialStride = 68;    // floats per row partial: acc[64], m, l, 2 pad

// Sizes every region for (L, H, nnz); nnz < 0 means implicit mask (no tile lists).
// Evaluated identically on the host (sga_workspace_bytes) and inside the kernels
// (with nnz = row_ptr[L]), so no layout has to be passed around.
__host__ __device__ inline WorkspacePlan plan_workspace(int64_t L, int32_t H, int64_t nnz) {
  WorkspacePlan p{};
  size_t off = 256;   // counters
  const int64_t e = nnz < 0 ? 0 : nnz;
  int64_t n_long = e / (kSplitThreshold + 1);
  if (n_long > L) n_long = L;
  int64_t cap = e / kSplitChunk + n_long;
  if (cap > (int64_t)kMaxSplit * n_long) cap = (int64_t)kMaxSplit * n_long;
  p.cap_items = cap;
  p.off_items = off;
  off = (off + (size_t)cap * 8 + 255) & ~size_t(255);
  p.off_long = off;
  off = (off + (size_t)cap * 16 + 255) & ~size_t(255);
  p.off_partials = off;
  off = (off + (size_t)cap * H * kPartialStride * sizeof(float) + 255) & ~size_t(255);
  // tile path
  p.n_tiles = (L + kTile - 1) / kTile;
  p.cap_pairs = nnz < 0 ? 0 : e / kPairEdges + 1;
  p.off_tile_nblk = off;
  off = (off + (size_t)p.n_tiles * sizeof(int32_t) + 255) & ~size_t(255);
  p.off_pair_blk = off;
  off = (off + (size_t)p.cap_pairs * sizeof(int32_t) + 255) & ~size_t(255);
  p.off_pair_mask = off;
  off = (off + (size_t)p.cap_pairs * kTile * sizeof(uint32_t) + 255) & ~size_t(255);
  int64_t n_tlong = p.cap_pairs / (kTileSplitThreshold + 1);
  if (n_tlong > p.n_tiles) n_tlong = p.n_tiles;
  int64_t tcap = p.cap_pairs / kTileChunk + n_tlong;
  if (tcap > (int64_t)kTileMaxSplit * n_tlong) tcap = (int64_t)kTileMaxSplit * n_tlong;
  if (tcap > kTileItemSlots) tcap = kTileItemSlots;
  p.cap_titems = tcap;
  p.off_titems = off;
  off = (off + (size_t)tcap * 8 + 255) & ~size_t(255);
  p.off_tlong = off;
  off = (off + (size_t)tcap * 16 + 255) & ~size_t(255);
  p.off_tpartials = off;
  off = (off + (size_t)tcap * H * kTilePartialFloats * sizeof(float) + 255) & ~size_t(255);
  p.total_bytes = off;
  return p;
}

struct AttnArgs {
  const void* Q;
  const void* K;
  const void* V;
  void* O;
  float* lse;
  int64_t L;
  int32_t H;
  float scale;
  int32_t dtype;
  hipStream_t stream;
  // explicit
  const int64_t* row_ptr;
  const int32_t* col_idx;
  // implicit (window family): neighbours j = i + stride*k, |k| <= window
  int32_t window;
  int32_t stride;
  // workspace
  void* ws;
  size_t ws_bytes;
};

// gather path (attention_gather.hip)
void clear_workspace_counters(void* ws, hipStream_t stream);
// skip_tiled: rows whose 32-row tile was produced by the tile path (tile_nblk >= 0 in the
// workspace) are skipped, and a small grid strides over the rows.
sga_status launch_gather_explicit(const AttnArgs& a, bool allow_split, bool skip_tiled);
sga_status launch_gather_implicit(const AttnArgs& a);

// tile path (attention_tile.hip)
sga_status launch_tile_explicit(const AttnArgs& a);
sga_status launch_tile_implicit(const AttnArgs& a);

// mask builder (mask_builder.hip)
sga_status mask_validate(const sga_mask_desc* d);
int64_t mask_total_edges(const sga_mask_desc& d);
sga_status launch_build_mask(const sga_mask_desc& d, int64_t* row_ptr, int32_t* col_idx,
                             hipStream_t stream);

inline sga_status hip_status(hipError_t e) { return e == hipSuccess ? SGA_OK : SGA_ERR_HIP; }

}  // namespace sga
