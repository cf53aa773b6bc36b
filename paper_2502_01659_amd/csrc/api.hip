// C ABI of libsga.so: argument validation and dispatch.  See include/sga.h for the contract.
#include "sga_internal.h"

#include <atomic>
#include <vector>

using namespace sga;

namespace {

// Profiling state (benchmark use only; not thread-safe).  Event pairs are created while a
// recording runs and destroyed when it is switched off.
struct ProfileState {
  bool on = false;
  bool failed = false;          // an event could not be created: reported by sga_profile_collect
  size_t used = 0;
  const char* kernel = "";      // name of the kernel inside the most recent pair
  std::vector<hipEvent_t> start, stop;
};
ProfileState g_prof;

// ---- scratch of the entry point that allocates nothing ------------------------------------------
// One array per device, in the library's own device image: it exists from the moment the image is
// loaded on a device until the process ends.  In host code `scratch` is only a handle for
// hipGetSymbolAddress; the address a kernel can use is resolved once per device and kept here.
constexpr size_t kScratchBytes = size_t(64) << 20;
__device__ __align__(256) static unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device (resolved on the first call per device).
sga_status scratch_of_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return SGA_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return SGA_ERR_UNSUPPORTED;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return SGA_ERR_HIP;
    }
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return SGA_OK;
}

constexpr uint32_t kPlanMagic = 0x53474150u;   // marks a record written by sga_graph_prepare

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

sga_status check_common(const void* Q, const void* K, const void* V, const void* O, int64_t L,
                        int32_t H, int32_t d, int32_t dtype, int32_t path, const void* ws,
                        size_t ws_bytes) {
  if (!Q || !K || !V || !O) return SGA_ERR_INVALID_ARG;
  if (L < 1 || L >= (int64_t(1) << 31) || H < 1 || H > 65535) return SGA_ERR_INVALID_ARG;
  if (dtype != SGA_F32 && dtype != SGA_F16) return SGA_ERR_INVALID_ARG;
  if (path != SGA_PATH_AUTO && path != SGA_PATH_GATHER && path != SGA_PATH_TILE &&
      path != SGA_PATH_TILE_SPLIT)
    return SGA_ERR_INVALID_ARG;
  if (path == SGA_PATH_TILE_SPLIT && (dtype != SGA_F32 || d != kHeadDim)) return SGA_ERR_UNSUPPORTED;
  if (d != 32 && d != 64 && d != 128 && d != 256) return SGA_ERR_UNSUPPORTED;
  if (path == SGA_PATH_TILE && d < kHeadDim) return SGA_ERR_UNSUPPORTED;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O)) return SGA_ERR_INVALID_ARG;
  if (ws && (reinterpret_cast<uintptr_t>(ws) & 255u)) return SGA_ERR_INVALID_ARG;
  if (!ws && ws_bytes != 0) return SGA_ERR_INVALID_ARG;
  return SGA_OK;
}

}  // namespace

namespace sga {

void profile_mark_begin(hipStream_t stream, const char* kernel) {
  if (!g_prof.on || g_prof.failed) return;
  if (g_prof.used == g_prof.start.size()) {
    hipEvent_t a, b;
    // (no system-scope fence at the records: they only take time stamps on the stream)
    if (hipEventCreateWithFlags(&a, hipEventDisableSystemFence) != hipSuccess) {
      g_prof.failed = true;
      return;
    }
    if (hipEventCreateWithFlags(&b, hipEventDisableSystemFence) != hipSuccess) {
      (void)hipEventDestroy(a);
      g_prof.failed = true;
      return;
    }
    g_prof.start.push_back(a);
    g_prof.stop.push_back(b);
  }
  g_prof.kernel = kernel;
  (void)hipEventRecord(g_prof.start[g_prof.used], stream);
}

void profile_mark_end(hipStream_t stream) {
  if (!g_prof.on || g_prof.failed || g_prof.used >= g_prof.stop.size()) return;
  (void)hipEventRecord(g_prof.stop[g_prof.used], stream);
  ++g_prof.used;
}

}  // namespace sga

extern "C" {

sga_status sga_profile_enable(int32_t on) {
  g_prof.on = on != 0;
  g_prof.used = 0;
  g_prof.failed = false;
  g_prof.kernel = "";
  if (!g_prof.on) {             // the recording's events go with it
    for (hipEvent_t e : g_prof.start) (void)hipEventDestroy(e);
    for (hipEvent_t e : g_prof.stop) (void)hipEventDestroy(e);
    g_prof.start.clear();
    g_prof.stop.clear();
  }
  return SGA_OK;
}

sga_status sga_profile_collect(float* ms_out, int32_t capacity, int32_t* n_out) {
  if (!n_out || (capacity > 0 && !ms_out) || capacity < 0) return SGA_ERR_INVALID_ARG;
  *n_out = 0;
  if (g_prof.failed) return SGA_ERR_HIP;
  for (size_t i = 0; i < g_prof.used; ++i) {
    if (hipEventSynchronize(g_prof.stop[i]) != hipSuccess) return SGA_ERR_HIP;
    if ((int64_t)i >= capacity) continue;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, g_prof.start[i], g_prof.stop[i]) != hipSuccess) return SGA_ERR_HIP;
    ms_out[i] = ms;
  }
  *n_out = (int32_t)g_prof.used;
  g_prof.used = 0;
  return SGA_OK;
}

const char* sga_profile_last_kernel(void) { return g_prof.kernel; }

const char* sga_status_string(sga_status s) {
  switch (s) {
    case SGA_OK: return "ok";
    case SGA_ERR_INVALID_ARG: return "invalid argument";
    case SGA_ERR_UNSUPPORTED: return "unsupported configuration";
    case SGA_ERR_WORKSPACE: return "workspace or output capacity too small";
    case SGA_ERR_OVERFLOW: return "size overflow";
    case SGA_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

sga_status sga_mask_nnz(const sga_mask_desc* desc, int64_t* nnz_out) {
  if (!nnz_out) return SGA_ERR_INVALID_ARG;
  const sga_status st = mask_validate(desc);
  if (st != SGA_OK) return st;
  *nnz_out = mask_total_edges(*desc);
  return SGA_OK;
}

sga_status sga_build_mask(const sga_mask_desc* desc, int64_t* row_ptr, int32_t* col_idx,
                          int64_t col_capacity, void* stream) {
  const sga_status st = mask_validate(desc);
  if (st != SGA_OK) return st;
  if (!row_ptr || !col_idx) return SGA_ERR_INVALID_ARG;
  if (col_capacity < mask_total_edges(*desc)) return SGA_ERR_WORKSPACE;
  (void)hipGetLastError();   // drop stale errors of earlier, unrelated runtime calls
  return launch_build_mask(*desc, row_ptr, col_idx, static_cast<hipStream_t>(stream));
}

sga_status sga_validate_csr(const int64_t* row_ptr, const int32_t* col_idx, int64_t L,
                            int64_t col_capacity, void* scratch, int64_t* bad_row_out, void* stream) {
  if (!row_ptr || !col_idx || !scratch || (reinterpret_cast<uintptr_t>(scratch) & 7)) return SGA_ERR_INVALID_ARG;
  if (L < 1 || L >= (int64_t(1) << 31) || col_capacity < 0) return SGA_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  (void)hipGetLastError();   // drop stale errors of earlier, unrelated runtime calls
  unsigned long long* verdict = static_cast<unsigned long long*>(scratch);
  const sga_status launched = launch_validate_csr(row_ptr, col_idx, L, col_capacity, verdict, st);
  if (launched != SGA_OK) return launched;
  unsigned long long found[2] = {0, 0};   // in the row offsets, in the columns
  if (hipMemcpyAsync(found, verdict, sizeof(found), hipMemcpyDeviceToHost, st) != hipSuccess ||
      hipStreamSynchronize(st) != hipSuccess)
    return SGA_ERR_HIP;
  const unsigned long long bad = found[0] < found[1] ? found[0] : found[1];
  if (bad_row_out) *bad_row_out = bad == ~0ull ? -1 : (int64_t)bad;
  return bad == ~0ull ? SGA_OK : SGA_ERR_INVALID_ARG;
}

sga_status sga_workspace_bytes(int64_t L, int32_t H, int32_t d, int32_t dtype, int64_t nnz,
                               size_t* bytes_out) {
  if (!bytes_out) return SGA_ERR_INVALID_ARG;
  if (L < 1 || L >= (int64_t(1) << 31) || H < 1 || H > 65535) return SGA_ERR_INVALID_ARG;
  if (dtype != SGA_F32 && dtype != SGA_F16) return SGA_ERR_INVALID_ARG;
  if (d != 32 && d != 64 && d != 128 && d != 256) return SGA_ERR_UNSUPPORTED;
  if (nnz < -1 || nnz > L * L) return SGA_ERR_INVALID_ARG;
  // (a caller that passes an upper bound of the edge count still gets enough for the shorter
  // work items the kernels may choose from the real count)
  const size_t chosen = plan_workspace(L, H, nnz, dtype, d).total_bytes;
  const size_t shortest = plan_workspace(L, H, nnz, dtype, d, seg_shift_min(dtype)).total_bytes;
  *bytes_out = chosen > shortest ? chosen : shortest;
  return SGA_OK;
}

}  // extern "C"

namespace {

sga_status run_explicit_call(const void* Q, const void* K, const void* V, const int64_t* row_ptr,
                             const int32_t* col_idx, void* O, int64_t L, int32_t H, int32_t d,
                             float scale, void* stream, int32_t dtype, float* lse, void* workspace,
                             size_t workspace_bytes, int32_t path, bool accumulate,
                             const sga_graph_plan* plan = nullptr, bool prepared = false) {
  const sga_status st = check_common(Q, K, V, O, L, H, d, dtype, path, workspace, workspace_bytes);
  if (st != SGA_OK) return st;
  if (!row_ptr || !col_idx) return SGA_ERR_INVALID_ARG;
  if (accumulate && !lse) return SGA_ERR_INVALID_ARG;
  if (prepared) {
    // the plan must have been prepared for exactly these buffers and this problem
    if (!plan || plan->struct_bytes != sizeof(sga_graph_plan) || plan->magic != kPlanMagic)
      return SGA_ERR_INVALID_ARG;
    if (plan->L != L || plan->H != H || plan->d != d || plan->dtype != dtype || plan->row_ptr != row_ptr ||
        plan->col_idx != col_idx || plan->workspace != workspace || plan->workspace_bytes != workspace_bytes)
      return SGA_ERR_INVALID_ARG;
    if (path == SGA_PATH_GATHER) return SGA_ERR_INVALID_ARG;
  }
  AttnArgs a{};
  a.Q = Q; a.K = K; a.V = V; a.O = O; a.lse = lse;
  a.L = L; a.H = H; a.scale = scale; a.dtype = dtype; a.d = d;
  a.stream = static_cast<hipStream_t>(stream);
  a.row_ptr = row_ptr; a.col_idx = col_idx;
  a.ws = workspace; a.ws_bytes = workspace_bytes;
  a.accumulate = accumulate;
  a.split = path == SGA_PATH_TILE_SPLIT;
  if ((path == SGA_PATH_TILE || path == SGA_PATH_TILE_SPLIT) && (!workspace || workspace_bytes < 256))
    return SGA_ERR_WORKSPACE;
  // the MFMA tile kernels work on 64-channel slices (d = 64, 128, 256); d = 32 runs on the per-row kernels
  const bool gather_only = path == SGA_PATH_GATHER || d < kHeadDim;
  (void)hipGetLastError();   // drop stale errors of earlier, unrelated runtime calls
  if (prepared) {
    const bool parts_fit = (plan->flags & SGA_GRAPH_TILE_PARTS_FIT) != 0;
    a.prepared = true;
    a.plan_multi_tiles = parts_fit ? plan->multi_tiles : 0;
    a.plan_tiles_cover_all = (plan->flags & SGA_GRAPH_TILES_COVER_ALL) != 0;
    a.plan_no_tiles = (int64_t)plan->tiles_left == (L + kTile - 1) / kTile;
    a.plan_long_rows = (plan->flags & SGA_GRAPH_ROW_CHUNKS_FIT) ? plan->long_rows : 0;
    return launch_tile_explicit(a);
  }
  if (workspace && workspace_bytes >= 256) clear_workspace(a, !gather_only);
  if (gather_only) return launch_gather_explicit(a, true, false);
  return launch_tile_explicit(a);
}

sga_status run_implicit_call(const void* Q, const void* K, const void* V, const sga_mask_desc* desc,
                             void* O, int64_t L, int32_t H, int32_t d, float scale, void* stream,
                             int32_t dtype, float* lse, void* workspace, size_t workspace_bytes,
                             int32_t path, bool accumulate) {
  sga_status st = check_common(Q, K, V, O, L, H, d, dtype, path, workspace, workspace_bytes);
  if (st != SGA_OK) return st;
  st = mask_validate(desc);
  if (st != SGA_OK) return st;
  if (desc->L != L) return SGA_ERR_INVALID_ARG;
  if (accumulate && !lse) return SGA_ERR_INVALID_ARG;
  const int32_t kind = desc->kind;
  if (kind != SGA_MASK_SLIDING && kind != SGA_MASK_DILATED && kind != SGA_MASK_NONLOCAL &&
      kind != SGA_MASK_DILATED_2D)
    return SGA_ERR_UNSUPPORTED;
  AttnArgs a{};
  a.Q = Q; a.K = K; a.V = V; a.O = O; a.lse = lse;
  a.L = L; a.H = H; a.scale = scale; a.dtype = dtype; a.d = d;
  a.stream = static_cast<hipStream_t>(stream);
  a.mask_kind = kind;
  a.stride = (kind == SGA_MASK_DILATED || kind == SGA_MASK_DILATED_2D) ? desc->stride : 1;
  const int64_t wmax = (L - 1) / a.stride;
  a.window = (int32_t)(desc->window < wmax ? desc->window : wmax);
  // 2-D dilated blocks: the selected rows of a block all see each other
  if (kind == SGA_MASK_DILATED_2D) a.window = (int32_t)(((desc->block < L ? desc->block : L) - 1) / a.stride);
  a.n_global = desc->n_global;
  a.block = desc->block;
  a.ws = workspace; a.ws_bytes = workspace_bytes;
  a.accumulate = accumulate;
  a.split = path == SGA_PATH_TILE_SPLIT;
  a.tiles_allowed = path != SGA_PATH_GATHER;
  (void)hipGetLastError();   // drop stale errors of earlier, unrelated runtime calls
  if (kind == SGA_MASK_NONLOCAL) {
    const int64_t g = desc->n_global < L ? desc->n_global : L;
    if (g > kMaxImplicitGlobal) return SGA_ERR_UNSUPPORTED;
    if (g > 0 && (!workspace || workspace_bytes < plan_workspace(L, H, -1, dtype, d).total_bytes))
      return SGA_ERR_WORKSPACE;
    return launch_gather_implicit(a);
  }
  if (path == SGA_PATH_GATHER || d < kHeadDim)
    return launch_gather_implicit(a);
  // 2-D dilated blocks with fewer than 16 selected rows would leave most of a 32-query tile
  // empty: the per-row kernels handle them
  if (kind == SGA_MASK_DILATED_2D && path == SGA_PATH_AUTO && a.window + 1 < 16)
    return launch_gather_implicit(a);
  return launch_tile_implicit(a);
}

}  // namespace

extern "C" {

sga_status sga_attention_forward(const void* Q, const void* K, const void* V, const int64_t* row_ptr,
                                 const int32_t* col_idx, void* O, int64_t L, int32_t H, int32_t d,
                                 float scale, void* stream, int32_t dtype, float* lse,
                                 void* workspace, size_t workspace_bytes, int32_t path) {
  return run_explicit_call(Q, K, V, row_ptr, col_idx, O, L, H, d, scale, stream, dtype, lse, workspace,
                           workspace_bytes, path, false);
}

sga_status sga_attention_forward_implicit(const void* Q, const void* K, const void* V,
                                          const sga_mask_desc* desc, void* O, int64_t L, int32_t H,
                                          int32_t d, float scale, void* stream, int32_t dtype,
                                          float* lse, void* workspace, size_t workspace_bytes,
                                          int32_t path) {
  return run_implicit_call(Q, K, V, desc, O, L, H, d, scale, stream, dtype, lse, workspace,
                           workspace_bytes, path, false);
}

sga_status sga_attention_accumulate(const void* Q, const void* K, const void* V, const int64_t* row_ptr,
                                    const int32_t* col_idx, void* O, int64_t L, int32_t H, int32_t d,
                                    float scale, void* stream, int32_t dtype, float* lse,
                                    void* workspace, size_t workspace_bytes, int32_t path) {
  return run_explicit_call(Q, K, V, row_ptr, col_idx, O, L, H, d, scale, stream, dtype, lse, workspace,
                           workspace_bytes, path, true);
}

sga_status sga_attention_accumulate_implicit(const void* Q, const void* K, const void* V,
                                             const sga_mask_desc* desc, void* O, int64_t L, int32_t H,
                                             int32_t d, float scale, void* stream, int32_t dtype,
                                             float* lse, void* workspace, size_t workspace_bytes,
                                             int32_t path) {
  return run_implicit_call(Q, K, V, desc, O, L, H, d, scale, stream, dtype, lse, workspace,
                           workspace_bytes, path, true);
}

sga_status sga_graph_prepare(const int64_t* row_ptr, const int32_t* col_idx, int64_t L, int32_t H,
                             int32_t d, int32_t dtype, void* workspace, size_t workspace_bytes,
                             void* stream, sga_graph_plan* plan_out) {
  if (!row_ptr || !col_idx || !plan_out) return SGA_ERR_INVALID_ARG;
  if (L < 1 || L >= (int64_t(1) << 31) || H < 1 || H > 65535) return SGA_ERR_INVALID_ARG;
  if (dtype != SGA_F32 && dtype != SGA_F16) return SGA_ERR_INVALID_ARG;
  if (d != 64 && d != 128 && d != 256) return SGA_ERR_UNSUPPORTED;   // the tile kernels' sizes
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return SGA_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  (void)hipGetLastError();
  // the edge count sizes the workspace layout; only the device knows it
  int64_t nnz = -1;
  if (hipMemcpyAsync(&nnz, row_ptr + L, sizeof(nnz), hipMemcpyDeviceToHost, st) != hipSuccess ||
      hipStreamSynchronize(st) != hipSuccess)
    return SGA_ERR_HIP;
  if (nnz < 0 || nnz > L * L) return SGA_ERR_INVALID_ARG;
  const WorkspacePlan pl = plan_workspace(L, H, nnz, dtype, d);
  if (pl.total_bytes > workspace_bytes) return SGA_ERR_WORKSPACE;
  AttnArgs a{};
  a.L = L; a.H = H; a.dtype = dtype; a.d = d; a.stream = st;
  a.row_ptr = row_ptr; a.col_idx = col_idx;
  a.ws = workspace; a.ws_bytes = workspace_bytes;
  clear_workspace(a, true);
  launch_tile_analyze(a);
  if (L > kSplitThreshold) launch_split_prepass(a, true);
  uint32_t ctr[kNumCounters];
  if (hipGetLastError() != hipSuccess ||
      hipMemcpyAsync(ctr, workspace, sizeof(ctr), hipMemcpyDeviceToHost, st) != hipSuccess ||
      hipStreamSynchronize(st) != hipSuccess)
    return SGA_ERR_HIP;
  sga_graph_plan p{};
  p.struct_bytes = sizeof(sga_graph_plan);
  p.magic = kPlanMagic;
  p.L = L; p.nnz = nnz; p.H = H; p.d = d; p.dtype = dtype;
  p.tiles_left = ctr[kCtrTilesBad];
  p.multi_tiles = ctr[kCtrMultiTiles];
  p.tile_parts = ctr[kCtrTilePartsNeeded];
  p.long_rows = ctr[kCtrLongRows];
  p.row_chunks = ctr[kCtrChunksNeeded];
  const bool parts_fit = (int64_t)p.tile_parts <= pl.cap_tparts;
  const bool chunks_fit = (int64_t)p.row_chunks <= pl.cap_items;
  p.flags = (parts_fit ? SGA_GRAPH_TILE_PARTS_FIT : 0) | (chunks_fit ? SGA_GRAPH_ROW_CHUNKS_FIT : 0) |
            (p.tiles_left == 0 && parts_fit ? SGA_GRAPH_TILES_COVER_ALL : 0);
  p.row_ptr = row_ptr; p.col_idx = col_idx;
  p.workspace = workspace; p.workspace_bytes = workspace_bytes;
  *plan_out = p;
  return SGA_OK;
}

sga_status sga_attention_forward_prepared(const void* Q, const void* K, const void* V,
                                          const int64_t* row_ptr, const int32_t* col_idx, void* O,
                                          int64_t L, int32_t H, int32_t d, float scale, void* stream,
                                          int32_t dtype, float* lse, void* workspace,
                                          size_t workspace_bytes, int32_t path,
                                          const sga_graph_plan* plan) {
  return run_explicit_call(Q, K, V, row_ptr, col_idx, O, L, H, d, scale, stream, dtype, lse, workspace,
                           workspace_bytes, path, false, plan, true);
}

sga_status sga_attention_accumulate_prepared(const void* Q, const void* K, const void* V,
                                             const int64_t* row_ptr, const int32_t* col_idx, void* O,
                                             int64_t L, int32_t H, int32_t d, float scale,
                                             void* stream, int32_t dtype, float* lse,
                                             void* workspace, size_t workspace_bytes, int32_t path,
                                             const sga_graph_plan* plan) {
  return run_explicit_call(Q, K, V, row_ptr, col_idx, O, L, H, d, scale, stream, dtype, lse, workspace,
                           workspace_bytes, path, true, plan, true);
}

sga_status sga_static_scratch_init(void) {
  void* p = nullptr;
  return scratch_of_current_device(&p);
}

size_t sga_static_scratch_bytes(void) { return kScratchBytes; }

sga_status sga_attention_forward_static(const void* Q, const void* K, const void* V,
                                        const int64_t* row_ptr, const int32_t* col_idx, void* O,
                                        int64_t L, int32_t H, int32_t d, float scale, void* stream,
                                        int32_t dtype, float* lse, int64_t nnz, int32_t path) {
  // the library's own scratch array takes the place of the caller's workspace
  size_t need = 0;
  const sga_status sized = sga_workspace_bytes(L, H, d, dtype, nnz, &need);
  if (sized != SGA_OK) return sized;
  if (nnz < 0) return SGA_ERR_INVALID_ARG;
  if (need > kScratchBytes) return SGA_ERR_WORKSPACE;      // beyond the stated maximum
  void* ws = nullptr;
  const sga_status found = scratch_of_current_device(&ws);
  if (found != SGA_OK) return found;
  return run_explicit_call(Q, K, V, row_ptr, col_idx, O, L, H, d, scale, stream, dtype, lse, ws,
                           kScratchBytes, path, false);
}

}  // extern "C"
