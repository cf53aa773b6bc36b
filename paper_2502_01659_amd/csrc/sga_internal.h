// Internal declarations shared by the translation units of libsga.so (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "sga.h"

namespace sga {

constexpr int kHeadDim = 64;          // head dimension of the tile (MFMA) kernels; the per-row
                                      // kernels also take 32, 128 and 256
constexpr int kWave = 64;             // CDNA wavefront width

// ---- split-row parameters (gather path) -----------------------------------
constexpr int kSplitThreshold = 2048; // rows with more neighbours are split
constexpr int kSplitChunk = 2048;     // target edges per chunk
constexpr int kSplitChunkMin = 256;   // ... of a call with little work in total (split_chunk)
constexpr int kMaxSplit = 64;         // at most this many chunks per row by L2 share, and ranges of an implicit global row
// ... and by edge count: a row of millions of neighbours (one global token of a long sequence
// whose tile does not qualify for the tile path) must spread over the chip, not over 64
// wavefronts (L = 4,194,304, one global token, fp16: 2.65 -> 0.8 ms)
constexpr int kMaxSplitLong = 1024;
// Keys whose K and V rows do not fit one L2 (each of the 8 XCDs has its own 4 MB): rows of at
// least kL2ChunkEdges * n neighbours are then cut into n = l2_chunks() chunks, a multiple of 8, and
// chunk c of every row runs on XCD c % 8.  A chunk of a row's sorted neighbour list covers a
// range of keys, so each L2 then serves about an n-th of K and V instead of all of it (for a
// uniformly random mask exactly that; any other mask is split the same way, only with less to
// gain).  The partial states of this finer split may take up to kL2PartialBudget bytes; a call
// that could need more keeps the coarser split by edge count.
constexpr int64_t kL2FitBytes = int64_t(3) << 20;
constexpr int64_t kL2ShareBytes = int64_t(2) << 20;       // K and V bytes per chunk and XCD aimed at
constexpr int kL2ChunkEdges = 128;
constexpr int64_t kL2PartialBudget = int64_t(64) << 20;
__host__ __device__ inline int l2_chunks(int64_t L, int32_t d, int32_t dtype) {
  const int64_t kv = 2 * L * d * (dtype == SGA_F32 ? 4 : 2);
  if (kv <= kL2FitBytes) return 0;
  int64_t n = 8 * ((kv + 8 * kL2ShareBytes - 1) / (8 * kL2ShareBytes));
  return (int)(n > kMaxSplit ? kMaxSplit : n);
}
constexpr int kMaxImplicitGlobal = 64;  // global rows the implicit non-local kernels can split
// Implicit window masks on few tiles (a short sequence, one head): a tile's key blocks are cut
// into up to kMaxWindowSplit ranges that separate wavefronts reduce to partial states, so that
// the call fills the chip.  The workspace holds the partials of up to kWindowSplitTiles
// (tile, head) pairs; larger calls have tiles enough and are not cut.
constexpr int kMaxWindowSplit = 8;
constexpr int kWindowSplitTiles = 4096;

// ---- tile path parameters -----------------------------------------------------
constexpr int kTile = 32;                 // query rows per tile = keys per block
constexpr int kCutEdges = 16384;          // tiles with fewer edges are never cut into segments
constexpr int kPairEdges = 128;           // a tile qualifies if it averages >= this many edges per block
constexpr int kProbeBlocks = 16;          // ... and a list is given up early if its first kProbeBlocks blocks
constexpr int kProbeEdges = 112;          //     average fewer than kProbeEdges edges (kPairEdges less a margin)
constexpr int kMaxTilePartials = 32768;   // partial states of split tiles per call
constexpr int kTilePartialFloats = kTile * 64 + 2 * kTile;   // o[32][64], m[32], l[32]

// Edges per unit of tile work.  Tile t owns the work items [f(t), f(t+1)) with
// f(t) = t + (edges before tile t)/S, i.e. one item plus one per multiple of S its edge range
// crosses; the first max(1, edges(t)/S) of them are the tile's segments, the rest stay idle.
// The mapping follows from row_ptr alone and needs neither a scan nor atomics.  A dense
// 32x32 block is 1024 edges: S is 32 dense blocks of fp32 MFMA work or 256 of fp16 work.
// S is a power of two (the kernels divide edge counts by it with a shift): 2^15 or 2^18 edges.
// A call with less work in total (nnz * H edges) gets shorter items, down to 2^12 or 2^15
// edges, until it has about 1024 (fp32) or 4096 (fp16) of them: otherwise a call with a few
// dense rows leaves its few long items to a handful of wavefronts while the rest of the chip
// idles.  An item of S edges takes a wavefront S / (nnz * H / 4096) of the time the whole chip
// needs for the call, and the tiles that are cut at all (rows of global tokens) are half empty,
// which doubles that.  (Microbenchmark grid, fp32, one head, a few global tokens at L = 8192:
// 0.76 -> 0.14 ms with 1024 items; the longformer mask with fp16 storage, L = 65,536, H = 8:
// 0.28 -> 0.16 ms with 4096 instead of 1024, L = 262,144, H = 4: 0.65 -> 0.32 ms.  fp32 items
// pay about 5 microseconds between the claim and the first block, as much as 3 blocks of
// matrix work: 4096 items made the global masks of the microbenchmark grid up to 1.5 times
// slower, and 8192 cost workload 2 1.4 %.)
// Edges per chunk of a split row: kSplitChunk, halved down to kSplitChunkMin while the call
// (nnz * H edges) has fewer than about 1024 such chunks, for the same reason as seg_shift.
__host__ __device__ inline int split_chunk(int64_t nnz, int32_t H) {
  int c = kSplitChunk;
  const int64_t e = (nnz < 0 ? 0 : nnz) * (int64_t)H;
  while (c > kSplitChunkMin && e / c < 1024) c >>= 1;
  return c;
}
__host__ __device__ inline int seg_shift_min(int32_t dtype) { return dtype == SGA_F32 ? 12 : 15; }
__host__ __device__ inline int seg_shift(int32_t dtype, int64_t nnz, int32_t H) {
  int sh = dtype == SGA_F32 ? 15 : 18;
  const int64_t e = (nnz < 0 ? 0 : nnz) * (int64_t)H;
  while (sh > seg_shift_min(dtype) && (e >> sh) < (dtype == SGA_F32 ? 1024 : 4096)) --sh;
  return sh;
}

// ---- workspace layout -------------------------------------------------------
// [0, 256)            counters (uint32): see WsCounter
// long_rows           cap_items x int4 {row, first partial slot, nchunks, chunk_len}   (gather split)
// partials            cap_items x H x kPartialStride floats {acc[d], m, l}
//                     (implicit non-local mask: kMaxImplicitGlobal rows x kMaxSplit chunks)
// items_rec           n_work x TileItem: the work items of the tile path
// tile_bad            n_tiles x int32: != 0 -> tile is left to the gather path
// bad_list            n_tiles x int32: the tiles with tile_bad != 0, in any order (kCtrTilesBad of them)
// tile_pbase          n_tiles x int32: first partial slot of a multi-segment tile
// multi_tiles         cap_tparts x {tile, first partial slot, segments, -}: the multi-segment tiles (merge list, any order)
// pair_blk            cap_pairs x int32: key block id (| full flag); tile t owns slots
//                     [row_ptr[32t]/128, row_ptr[32(t+1)]/128), split evenly among its segments
// pair_mask           cap_pairs x 32 x uint32: bit j of word r = edge (row 32t+r, key 32b+j)
// tpartials           cap_tparts x H x max(1, d / 64) x kTilePartialFloats floats
// work_next           H x uint32: next unclaimed tile work item of each head (dynamic scheduling),
//                     then H x uint32: wavefronts (workgroups) of the head that found no item left
enum WsCounter : int {
  kCtrChunksNeeded = 0,   // sum of chunk counts of all long rows
  kCtrItemsAlloc = 1,     // bump allocator over the partial slots of split rows
  kCtrLongRows = 2,       // number of long rows recorded
  kCtrTilePartsNeeded = 3,  // sum of segment counts of all multi-segment tiles
  kCtrTilePartsAlloc = 4,   // bump allocator over tile partial slots
  kCtrTilesBad = 5,         // tiles whose block lists overflowed (left to the gather path)
  kCtrMultiTiles = 6,       // multi-segment tiles recorded in the merge list
  kCtrMaxChunks = 7,        // most chunks any split row has (bounds the chunk kernel's unit loop)
  kCtrFineNeeded = 8,       // the same three for the finer split (see row_split_shape)
  kCtrFineAlloc = 9,
  kCtrMaxChunksFine = 10,
  kNumCounters = 64
};

// One work item of the tile path, written by the CSR -> tile graph pass and read (one record,
// one load) by the attention kernel.
struct alignas(32) TileItem {
  int32_t tile;     // tile index, or -1 for an idle item
  int32_t nblk;     // key blocks in the item's list, or -1 if the list overflowed its slots
  int32_t seg;      // segment of the tile's key-block span ...
  int32_t nseg;     // ... out of this many
  int64_t slot0;    // first (tile, key block) pair slot of the list
  int64_t pad;
};

struct WorkspacePlan {
  // gather split
  int64_t cap_items;
  size_t off_long, off_partials;
  // tile path
  int64_t n_tiles;        // ceil(L / 32)
  int64_t n_work;         // tile work items (segments)
  int64_t cap_pairs;      // capacity of the (tile, key block) pair arrays
  int64_t cap_tparts;     // capacity of tile partial states
  int seg_shift;          // log2 of S, the edges per work item of the tile path
  int split_chunk;        // target edges per chunk of a split row
  int l2_chunks;          // != 0: rows of >= kL2ChunkEdges * l2_chunks neighbours are cut into this many chunks
  size_t off_items_rec, off_tile_bad, off_bad_list, off_tile_pbase, off_multi_tiles, off_pair_blk, off_pair_mask,
      off_tpartials, off_work_next, off_wparts;
  int64_t cap_wparts;     // (tile, head) pairs whose window partials fit (implicit masks)
  size_t total_bytes;
};

// A row partial of the split-row path is d + 4 floats: acc[d], m, l, 2 pad.

// Sizes every region for (L, H, nnz, dtype); nnz < 0 means implicit mask (no tile lists).
// Evaluated identically on the host (sga_workspace_bytes) and inside the kernels
// (with nnz = row_ptr[L]), so no layout has to be passed around.  (force_shift: the size of a
// layout with that log2 S and the shortest row chunks instead of those the arguments select.)
__host__ __device__ inline WorkspacePlan plan_workspace(int64_t L, int32_t H, int64_t nnz,
                                                        int32_t dtype, int32_t d = kHeadDim,
                                                        int force_shift = -1) {
  WorkspacePlan p{};
  p.seg_shift = force_shift >= 0 ? force_shift : seg_shift(dtype, nnz, H);
  p.split_chunk = force_shift >= 0 ? kSplitChunkMin : split_chunk(nnz, H);
  size_t off = 256;   // counters
  const int64_t e = nnz < 0 ? 0 : nnz;
  int64_t n_long = e / (kSplitThreshold + 1);
  if (n_long > L) n_long = L;
  int64_t cap = e / p.split_chunk + n_long;
  if (cap > (int64_t)kMaxSplitLong * n_long) cap = (int64_t)kMaxSplitLong * n_long;
  p.l2_chunks = nnz < 0 ? 0 : l2_chunks(L, d, dtype);
  if (p.l2_chunks) {
    int64_t rows = e / ((int64_t)kL2ChunkEdges * p.l2_chunks);      // rows that can qualify
    if (rows > L) rows = L;
    const int64_t cap_l2 = rows * p.l2_chunks;
    if (cap_l2 * H * (d + 4) * (int64_t)sizeof(float) > kL2PartialBudget) p.l2_chunks = 0;
    else if (cap_l2 > cap) cap = cap_l2;
  }
  // implicit masks: only the dense rows of the global (non-local) mask are split
  if (nnz < 0) cap = (int64_t)kMaxImplicitGlobal * kMaxSplit;
  p.cap_items = cap;
  p.off_long = off;
  off = (off + (size_t)cap * 32 + 255) & ~size_t(255);      // (the records of the finer split follow the cap records)
  p.off_partials = off;
  off = (off + (size_t)cap * H * (d + 4) * sizeof(float) + 255) & ~size_t(255);
  // tile path
  const bool tiles = nnz >= 0;
  p.n_tiles = tiles ? (L + kTile - 1) / kTile : 0;
  p.n_work = tiles ? p.n_tiles + (e >> p.seg_shift) : 0;
  p.cap_pairs = tiles ? e / kPairEdges + 1 : 0;
  p.cap_tparts = tiles ? (e >> p.seg_shift) + 1 : 0;
  if (p.cap_tparts > kMaxTilePartials) p.cap_tparts = kMaxTilePartials;
  p.off_items_rec = off;
  off = (off + (size_t)p.n_work * sizeof(TileItem) + 255) & ~size_t(255);
  p.off_tile_bad = off;
  off = (off + (size_t)p.n_tiles * 4 + 255) & ~size_t(255);
  p.off_bad_list = off;
  off = (off + (size_t)p.n_tiles * 4 + 255) & ~size_t(255);
  p.off_tile_pbase = off;
  off = (off + (size_t)p.n_tiles * 4 + 255) & ~size_t(255);
  p.off_multi_tiles = off;
  off = (off + (size_t)p.cap_tparts * 16 + 255) & ~size_t(255);     // {tile, first partial slot, segments, -}
  p.off_pair_blk = off;
  off = (off + (size_t)p.cap_pairs * sizeof(int32_t) + 255) & ~size_t(255);
  p.off_pair_mask = off;
  off = (off + (size_t)p.cap_pairs * kTile * sizeof(uint32_t) + 255) & ~size_t(255);
  p.off_tpartials = off;
  const int64_t slices = d > kHeadDim ? d / kHeadDim : 1;   // a wide tile leaves one record per 64 channels
  off = (off + (size_t)p.cap_tparts * H * slices * kTilePartialFloats * sizeof(float) + 255) & ~size_t(255);
  p.off_work_next = off;
  off = (off + (tiles ? (size_t)H * 8 : 0) + 255) & ~size_t(255);
  // implicit window masks: partial states of cut tiles (short sequences only)
  p.cap_wparts = 0;
  if (nnz < 0 && d >= kHeadDim) {
    const int64_t pairs = ((L + kTile - 1) / kTile + 256) * H;     // (tiles of every class: + a margin) x heads
    if (pairs <= kWindowSplitTiles) p.cap_wparts = pairs;
  }
  p.off_wparts = off;
  off = (off + (size_t)p.cap_wparts * kMaxWindowSplit * slices * kTilePartialFloats * sizeof(float) + 255) &
        ~size_t(255);
  p.total_bytes = off;
  return p;
}

// Rows the per-row kernels split into chunks (partial states + ordered merge): more than
// kSplitThreshold neighbours, or enough of them for the split by L2 share (see l2_chunks).
__host__ __device__ inline bool row_is_split(int64_t deg, const WorkspacePlan& p) {
  return deg > kSplitThreshold || (p.l2_chunks && deg >= (int64_t)kL2ChunkEdges * p.l2_chunks);
}
// ... into nchunks chunks of len edges (the last one shorter), len a multiple of 32.
// The slots are sized for chunks of split_chunk edges with every row of the mask split; where
// the split rows hold a small part of the edges (a few dense rows beside a window), the same
// slots take chunks of kSplitChunkMin edges: the call uses this finer split (fine = true)
// if the chunks of all its rows then still fit, else the coarser one for every row.  (One
// global token at L = 65,536, 8 heads, fp32: 32 chunks of 2,048 edges per head kept 256
// wavefronts busy for 0.29 ms, each waiting for its own gathers.)
__host__ __device__ inline void row_split_shape(int64_t deg, const WorkspacePlan& p, bool fine, int32_t& nchunks,
                                                int32_t& len) {
  const int chunk = fine ? kSplitChunkMin : p.split_chunk;
  int64_t n = (deg + chunk - 1) / chunk;
  if (n > kMaxSplitLong) n = kMaxSplitLong;
  // (a row of more than kMaxSplit chunks by edge count keeps them: there are few such rows in a
  // call, and each has to spread over the chip before it can share an L2 with its neighbours)
  if (n <= kMaxSplit && p.l2_chunks && deg >= (int64_t)kL2ChunkEdges * p.l2_chunks) n = p.l2_chunks;
  int64_t l = (deg + n - 1) / n;
  l = (l + 31) / 32 * 32;
  len = (int32_t)l;
  nchunks = (int32_t)((deg + l - 1) / l);
}

// First work item of tile t: f(t) = t + row_ptr[min(32t, L)] / S.
__device__ __forceinline__ int64_t work_first(const int64_t* __restrict__ row_ptr, int64_t L,
                                              int sh, int64_t t) {
  const int64_t r = t * kTile;
  return t + (row_ptr[r < L ? r : L] >> sh);
}

// Segments tile t is cut into: max(1, edges(t) / S); a tile below kCutEdges edges (every tile of
// a window mask up to +-255) stays whole also where a small call has S below that.
__device__ __forceinline__ int32_t tile_segments(const int64_t* __restrict__ row_ptr, int64_t L,
                                                 int sh, int64_t t) {
  const int64_t r0 = t * kTile, r1 = r0 + kTile < L ? r0 + kTile : L;
  const int64_t e = row_ptr[r1] - row_ptr[r0];
  const int64_t n = e >> sh;
  return n < 1 || e < kCutEdges ? 1 : (int32_t)n;
}

// True when the tile path of this call produces the rows of tile t: its block lists fitted
// their slots and, if it is a multi-segment tile, the call's partial states fitted theirs.
__device__ __forceinline__ bool tile_handled(const WorkspacePlan& pl, const void* ws,
                                             const int64_t* __restrict__ row_ptr, int64_t L,
                                             int32_t dtype, int64_t t) {
  const char* base = static_cast<const char*>(ws);
  if (reinterpret_cast<const int32_t*>(base + pl.off_tile_bad)[t] != 0) return false;
  if (tile_segments(row_ptr, L, pl.seg_shift, t) == 1) return true;
  return (int64_t) reinterpret_cast<const uint32_t*>(ws)[kCtrTilePartsNeeded] <= pl.cap_tparts;
}

// True when the tile path of this call left no row to the gather path.
__device__ __forceinline__ bool tiles_cover_everything(const WorkspacePlan& pl, const void* ws) {
  const uint32_t* ctr = reinterpret_cast<const uint32_t*>(ws);
  return ctr[kCtrTilesBad] == 0 && (int64_t)ctr[kCtrTilePartsNeeded] <= pl.cap_tparts;
}

template <typename T> struct DtypeOf;
template <> struct DtypeOf<float> { static constexpr int32_t code = SGA_F32; };
template <> struct DtypeOf<__half> { static constexpr int32_t code = SGA_F16; };

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
  int32_t d;           // head dimension
  hipStream_t stream;
  // explicit
  const int64_t* row_ptr;
  const int32_t* col_idx;
  // implicit (window family): neighbours j = i + stride*k, |k| <= window
  int32_t window;
  int32_t stride;
  int32_t mask_kind;   // implicit: sga_mask_kind
  int32_t n_global;    // implicit non-local mask
  int32_t block;       // implicit 2-D dilated mask
  // continue from the (O, lse) state already in the output buffers instead of overwriting it
  bool accumulate;
  // fp32 storage: products as three fp16 matrix-core terms instead of fp32 MFMA (tile path)
  bool split;
  // implicit non-local mask: the tile kernels may be used (the caller did not ask for the
  // per-row kernels)
  bool tiles_allowed;
  // workspace
  void* ws;
  size_t ws_bytes;
  // prepared graph (sga_graph_prepare): the workspace already holds the tile graph and the
  // chunk items of the split rows, and the host knows what they contain
  bool prepared;
  uint32_t plan_multi_tiles;   // multi-segment tiles whose partial states fit (0: no merge launch)
  bool plan_tiles_cover_all;   // no row is left to the per-row kernels
  bool plan_no_tiles;          // no tile qualified: the tile kernels have nothing to do
  uint32_t plan_long_rows;     // split rows among the leftover rows whose chunk items fit
};

// gather path (attention_gather.hip)
// Zeroes the counters (and, when row_ptr is given, the per-tile flags of the tile path).
void clear_workspace(const AttnArgs& a, bool tile_flags);
// skip_tiled: rows whose 32-row tile was produced by the tile path (tile_bad == 0 in the
// workspace) are skipped, and a small grid strides over the rows.
sga_status launch_gather_explicit(const AttnArgs& a, bool allow_split, bool skip_tiled);
sga_status launch_gather_implicit(const AttnArgs& a);

// tile path (attention_tile.hip)
sga_status launch_tile_explicit(const AttnArgs& a);
// CSR -> tile graph pass alone (sga_graph_prepare); a.ws holds a full workspace
void launch_tile_analyze(const AttnArgs& a);
// reservation of the chunk items of the split rows the tile path leaves over (sga_graph_prepare)
void launch_split_prepass(const AttnArgs& a, bool skip_tiled);
sga_status launch_tile_implicit(const AttnArgs& a);
// Implicit non-local mask on the tile kernels (d = 64, 128, 256): the rows >= g against the global keys,
// and the partial states of the g global rows over *n_chunks ranges of the key blocks, in the
// layout nonlocal_merge_kernel reads (the caller launches that merge).
void launch_tile_nonlocal(const AttnArgs& a, int64_t g, float* partials, int32_t* n_chunks);

// mask builder (mask_builder.hip)
sga_status mask_validate(const sga_mask_desc* d);
int64_t mask_total_edges(const sga_mask_desc& d);
sga_status launch_build_mask(const sga_mask_desc& d, int64_t* row_ptr, int32_t* col_idx,
                             hipStream_t stream);
// Enqueues the checks of sga_validate_csr; verdict[0] and verdict[1] (uint64) end as the smallest bad row
// found in the row offsets and in the columns, or ~0.
sga_status launch_validate_csr(const int64_t* row_ptr, const int32_t* col_idx, int64_t L, int64_t col_capacity,
                               unsigned long long* verdict, hipStream_t stream);

// Benchmark hook (api.hip): when enabled, brackets the dominant attention kernel of a forward
// call with a pair of events on the call's stream.
void profile_mark_begin(hipStream_t stream, const char* kernel);
void profile_mark_end(hipStream_t stream);

// Sequential composition on one shared state (Section V-F runs a local, a global and a CSR
// kernel one after another on the same O, l, m of Algorithm 1).  The state handed from call to
// call is the normalised O_i and lse_i = m_i + ln l_i of the edges visited so far (the two
// statistics only ever enter the recurrence through this sum).  Given the earlier state and the
// (O, lse) of the edges this call visited, the continued state is
//   lse' = ln(e^lse_prev + e^lse_now),  O' = w_prev O_prev + w_now O_now,  w_x = e^(lse_x - lse').
struct CarryWeights {
  float w_prev, w_now, lse;
};
__device__ __forceinline__ CarryWeights carry_weights(float lse_prev, float lse_now) {
  const float M = fmaxf(lse_prev, lse_now);
  if (!(M > -INFINITY)) return {0.f, 0.f, -INFINITY};     // no edge visited so far
  constexpr float kLog2eC = 1.4426950408889634f, kLn2C = 0.6931471805599453f;
  const float a = __builtin_amdgcn_exp2f((lse_prev - M) * kLog2eC);
  const float b = __builtin_amdgcn_exp2f((lse_now - M) * kLog2eC);
  const float inv = 1.0f / (a + b);
  return {a * inv, b * inv, M + __builtin_amdgcn_logf(a + b) * kLn2C};
}

inline sga_status hip_status(hipError_t e) { return e == hipSuccess ? SGA_OK : SGA_ERR_HIP; }

}  // namespace sga
