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

// ---- workspace layout -------------------------------------------------------
// [0, 256)            counters (uint32): see WsCounter
// items               cap_items x int2 {row, chunk | nchunks << 8}     (gather split)
// long_rows           cap_items x int4 {row, base, nchunks, chunk_len}
// partials            cap_items x H x (d + 2) floats {m, l, acc[d]}
// tile region         block lists and bit masks of the tile path (see attention_tile.hip)
enum WsCounter : int {
  kCtrChunksNeeded = 0,   // sum of chunk counts of all long rows
  kCtrItemsAlloc = 1,     // bump allocator over items
  kCtrLongRows = 2,       // number of long rows recorded
  kCtrTileItems = 3,      // bump allocator over split-tile work items
  kCtrTileLong = 4,       // number of split tiles recorded
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
  size_t off_tile_nblk, off_tile_base, off_pair_blk, off_pair_mask, off_titems, off_tlong,
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
  p.n_tiles = (L + 31) / 32;
  p.cap_pairs = nnz < 0 ? 0 : e / 128 + 1;
  p.off_tile_nblk = off;
  off = (off + (size_t)p.n_tiles * sizeof(int32_t) + 255) & ~size_t(255);
  p.off_pair_blk = off;
  off = (off + (size_t)p.cap_pairs * sizeof(int32_t) + 255) & ~size_t(255);
  p.off_pair_mask = off;
  off = (off + (size_t)p.cap_pairs * 32 * sizeof(uint32_t) + 255) & ~size_t(255);
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
// tile_done: optional device byte per 32-row tile; rows of tiles marked 1 are skipped.
sga_status launch_gather_explicit(const AttnArgs& a, bool allow_split, const uint8_t* tile_done);
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
