// Gather path of Algorithm 1: one wavefront per query row, per-edge K/V row gathers.
//
// Lane layout.  A K or V row is d*4 B (fp32) or d*2 B (fp16), d in {32, 64, 128, 256}; a
// group of LPK lanes reads one row with one 16-byte load per lane (LPK = d/4 for fp32, d/8
// for fp16: 16 and 8 at d = 64), so a wavefront pulls G = 64/LPK rows per load instruction
// and every row is a fully coalesced gather.  The dot product Q_i.K_j is reduced inside the lane
// group with DPP adds (no LDS); each group keeps its own running (m, l, acc) state of
// the recurrence in Algorithm 1 for the keys it has seen, and the G group states are
// merged with wavefront shuffles once per row.  The accumulator is kept un-normalised
// and divided by l once at the end, which is the same real number as the per-step
// normalisation printed in Algorithm 1.
//
// Rows with more than kSplitThreshold neighbours (global tokens) are split into chunks
// that separate wavefronts reduce to partial (m, l, acc) states; a merge kernel combines
// the partials in chunk order, so the result is deterministic.
#include "sga_internal.h"

namespace sga {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kMinusHuge = -1.0e30f;   // finite stand-in for m = -inf (keeps m - m finite)
constexpr int kUnroll = 4;               // keys per lane group per loop trip

template <int CTRL>
__device__ __forceinline__ float dpp(float x) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, false));
}

// Sum over the LPK consecutive lanes of a group; every lane of the group gets the total.
template <int LPK>
__device__ __forceinline__ float group_sum(float x) {
  static_assert(LPK == 4 || LPK == 8 || LPK == 16 || LPK == 32 || LPK == 64, "lanes per row");
  x += dpp<0xB1>(x);    // quad_perm [1,0,3,2]
  x += dpp<0x4E>(x);    // quad_perm [2,3,0,1]
  if (LPK >= 8) x += dpp<0x141>(x);    // row_half_mirror: lane k <-> 7-k of each 8
  if (LPK >= 16) x += dpp<0x140>(x);   // row_mirror: lane k <-> 15-k of each 16
  if (LPK >= 32) x += __shfl_xor(x, 16, kWave);
  if (LPK >= 64) x += __shfl_xor(x, 32, kWave);
  return x;
}

template <typename T, int D>
struct Row;

template <int D>
struct Row<float, D> {
  static constexpr int VEC = 4, LPK = D / VEC;
  __device__ static void load(const float* p, float (&v)[4]) {
    const float4 t = *reinterpret_cast<const float4*>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  }
  __device__ static void store(float* p, const float (&v)[4]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  }
};

template <int D>
struct Row<__half, D> {
  static constexpr int VEC = 8, LPK = D / VEC;
  __device__ static void load(const __half* p, float (&v)[8]) {
    const uint4 t = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const __half2 h = __builtin_bit_cast(__half2, w[k]);
      v[2 * k] = __low2float(h);
      v[2 * k + 1] = __high2float(h);
    }
  }
  __device__ static void store(__half* p, const float (&v)[8]) {
    uint32_t w[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
      w[k] = __builtin_bit_cast(uint32_t, __floats2half2_rn(v[2 * k], v[2 * k + 1]));
    *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
  }
};

__device__ __forceinline__ float load_scalar(const float* p) { return *p; }
__device__ __forceinline__ float load_scalar(const __half* p) { return __half2float(*p); }
__device__ __forceinline__ void store_scalar(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_scalar(__half* p, float v) { *p = __float2half_rn(v); }

struct WindowNeighbours {   // Get_Neighbors, implicit: j = first + e*step
  int64_t first, step;
  __device__ int64_t operator()(int64_t e) const { return first + e * step; }
};

// Running state of one lane group for the channels this lane owns.
template <int VEC>
struct State {
  float m, l, acc[VEC];
  __device__ void init() {
    m = kMinusHuge;
    l = 0.f;
#pragma unroll
    for (int c = 0; c < VEC; ++c) acc[c] = 0.f;
  }
};

// One step of the recurrence for kUnroll keys per lane group, K and V rows already in registers.
template <int LPK, int VEC>
__device__ __forceinline__ void attend_loaded(const float (&q)[VEC], const float (&kf)[kUnroll][VEC],
                                              const float (&vf)[kUnroll][VEC], const bool (&valid)[kUnroll],
                                              State<VEC>& st) {
  float s[kUnroll];
  float smax = st.m;
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    float part = 0.f;
#pragma unroll
    for (int c = 0; c < VEC; ++c) part = __builtin_fmaf(q[c], kf[u][c], part);
    part = group_sum<LPK>(part);
    s[u] = valid[u] ? part : -INFINITY;
    smax = fmaxf(smax, s[u]);
  }
  const float alpha = __builtin_amdgcn_exp2f(st.m - smax);
  st.l *= alpha;
#pragma unroll
  for (int c = 0; c < VEC; ++c) st.acc[c] *= alpha;
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const float p = __builtin_amdgcn_exp2f(s[u] - smax);
    st.l += p;
#pragma unroll
    for (int c = 0; c < VEC; ++c) st.acc[c] = __builtin_fmaf(p, vf[u][c], st.acc[c]);
  }
  st.m = smax;
}

// Visit edges [e0, e1) of one row.  q holds this lane's channels of Q_i * scale * log2(e).
template <typename T, int D, typename Nbr>
__device__ __forceinline__ void attend_range(const T* __restrict__ Kh, const T* __restrict__ Vh,
                                             const float (&q)[Row<T, D>::VEC], const Nbr& nbr,
                                             int64_t e0, int64_t e1, int lane,
                                             State<Row<T, D>::VEC>& st) {
  constexpr int LPK = Row<T, D>::LPK, VEC = Row<T, D>::VEC, G = kWave / LPK;
  const int grp = lane / LPK;
  const int cofs = (lane % LPK) * VEC;
  for (int64_t base = e0; base < e1; base += G * kUnroll) {
    float kf[kUnroll][VEC], vf[kUnroll][VEC];
    bool valid[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int64_t e = base + u * G + grp;
      valid[u] = e < e1;
      const int64_t j = nbr(valid[u] ? e : e1 - 1);   // out-of-range lanes re-read a real neighbour
      Row<T, D>::load(Kh + j * D + cofs, kf[u]);
      Row<T, D>::load(Vh + j * D + cofs, vf[u]);
    }
    attend_loaded<LPK, VEC>(q, kf, vf, valid, st);
  }
}

// attend_range over a slice of col_idx (explicit Get_Neighbors).  The column indices are read 64
// at a time with one coalesced load (lane l holds column base + l) and handed to the lane groups
// through the LDS crossbar, and the next 64 are requested before the current ones are used: the
// K/V row gathers then no longer wait for an index load of their own each, and a third of the
// vector memory instructions go away.
// kNear: one head's K (and V) is below 4 GiB, so row offsets fit 32 bits.
template <typename T, int D, bool kNear>
__device__ __forceinline__ void attend_columns(const T* __restrict__ Kh, const T* __restrict__ Vh,
                                               const float (&q)[Row<T, D>::VEC],
                                               const int32_t* __restrict__ cols, int64_t e0, int64_t e1,
                                               int lane, State<Row<T, D>::VEC>& st) {
  constexpr int LPK = Row<T, D>::LPK, VEC = Row<T, D>::VEC, G = kWave / LPK;
  constexpr int kStep = G * kUnroll;                 // edges per step of the recurrence
  static_assert(kWave % kStep == 0, "a batch of 64 columns is a whole number of steps");
  if (e0 >= e1) return;
  const int grp = lane / LPK;
  const int cofs = (lane % LPK) * VEC;
  const int64_t last = e1 - 1;
  int32_t cur = cols[e0 + lane < last ? e0 + lane : last];
  for (int64_t base = e0; base < e1; base += kWave) {
    const int64_t nb = base + kWave;
    int32_t nxt = 0;
    if (nb < e1) nxt = cols[nb + lane < last ? nb + lane : last];
    const int n_here = e1 - base < kWave ? (int)(e1 - base) : kWave;     // columns of this batch
#pragma unroll
    for (int sub = 0; sub < kWave / kStep; ++sub) {
      if (sub * kStep >= n_here) break;
      float kf[kUnroll][VEC], vf[kUnroll][VEC];
      bool valid[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const int el = sub * kStep + u * G + grp;
        valid[u] = el < n_here;
        const int32_t j = __shfl(cur, valid[u] ? el : n_here - 1, kWave);   // out-of-range lanes re-read a real neighbour
        if (kNear) {
          // one 32-bit byte offset serves the K and the V row (wave-uniform base + per-lane offset)
          const uint32_t off = (uint32_t)j * (uint32_t)(D * sizeof(T)) + (uint32_t)(cofs * sizeof(T));
          Row<T, D>::load(reinterpret_cast<const T*>(reinterpret_cast<const char*>(Kh) + off), kf[u]);
          Row<T, D>::load(reinterpret_cast<const T*>(reinterpret_cast<const char*>(Vh) + off), vf[u]);
        } else {
          Row<T, D>::load(Kh + (int64_t)j * D + cofs, kf[u]);
          Row<T, D>::load(Vh + (int64_t)j * D + cofs, vf[u]);
        }
      }
      attend_loaded<LPK, VEC>(q, kf, vf, valid, st);
    }
    cur = nxt;
  }
}

// Merge the G lane-group states of a wavefront; afterwards every group holds the row's state.
template <int LPK, int VEC>
__device__ __forceinline__ void merge_groups(State<VEC>& st) {
#pragma unroll
  for (int off = LPK; off < kWave; off <<= 1) {
    const float m2 = __shfl_xor(st.m, off, kWave);
    const float l2 = __shfl_xor(st.l, off, kWave);
    const float mn = fmaxf(st.m, m2);
    const float a1 = __builtin_amdgcn_exp2f(st.m - mn);
    const float a2 = __builtin_amdgcn_exp2f(m2 - mn);
    st.l = st.l * a1 + l2 * a2;
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
      const float o = __shfl_xor(st.acc[c], off, kWave);
      st.acc[c] = st.acc[c] * a1 + o * a2;
    }
    st.m = mn;
  }
}

template <typename T, int D>
__device__ __forceinline__ void load_query(const T* Qrow, float scale, int lane,
                                           float (&q)[Row<T, D>::VEC]) {
  Row<T, D>::load(Qrow + (lane % Row<T, D>::LPK) * Row<T, D>::VEC, q);
  const float c = scale * kLog2e;
#pragma unroll
  for (int k = 0; k < Row<T, D>::VEC; ++k) q[k] *= c;
}

// Normalise and store a row; with `accumulate` the row continues the (O, lse) state already
// in the output buffers (sequential composition on one state, Section V-F).
template <typename T, int D>
__device__ __forceinline__ void finish_row(T* Orow, float* lse_i, int lane,
                                           State<Row<T, D>::VEC>& st, bool accumulate) {
  constexpr int LPK = Row<T, D>::LPK, VEC = Row<T, D>::VEC;
  merge_groups<LPK, VEC>(st);
  const bool empty = !(st.l > 0.f);
  float inv = empty ? 0.f : 1.0f / st.l;
  float lse_row = empty ? -INFINITY : (st.m + __builtin_amdgcn_logf(st.l)) * kLn2;
  float w_prev = 0.f;
  if (accumulate) {     // every lane reads the earlier lse before lane 0 replaces it
    const CarryWeights cw = carry_weights(*lse_i, lse_row);
    inv *= cw.w_now;
    w_prev = cw.w_prev;
    lse_row = cw.lse;
  }
  float o[VEC];
#pragma unroll
  for (int c = 0; c < VEC; ++c) o[c] = st.acc[c] * inv;
  if (lane < LPK) {
    if (accumulate) {
      float old[VEC];
      Row<T, D>::load(Orow + lane * VEC, old);
#pragma unroll
      for (int c = 0; c < VEC; ++c) o[c] = __builtin_fmaf(w_prev, old[c], o[c]);
    }
    Row<T, D>::store(Orow + lane * VEC, o);
  }
  if (lse_i && lane == 0) *lse_i = lse_row;
}

__host__ __device__ inline void split_shape(int64_t deg, int chunk, int32_t& nchunks, int32_t& len) {
  int64_t n = (deg + chunk - 1) / chunk;
  if (n > kMaxSplit) n = kMaxSplit;
  int64_t l = (deg + n - 1) / n;
  l = (l + 31) / 32 * 32;
  len = (int32_t)l;
  nchunks = (int32_t)((deg + l - 1) / l);
}

// ---- kernels ----------------------------------------------------------------

// Zeroes the counters and (tile_flags != 0) the per-tile flags of the tile path.
__global__ __launch_bounds__(256) void clear_workspace_kernel(void* ws, size_t ws_bytes,
                                                              const int64_t* row_ptr, int64_t L,
                                                              int32_t H, int32_t dtype, int32_t d,
                                                              int tile_flags) {
  uint32_t* ctr = reinterpret_cast<uint32_t*>(ws);
  if (blockIdx.x == 0 && threadIdx.x < kNumCounters) ctr[threadIdx.x] = 0;
  if (!tile_flags) return;
  const WorkspacePlan pl = plan_workspace(L, H, row_ptr[L], dtype, d);
  if (pl.total_bytes > ws_bytes) return;
  int32_t* bad = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + pl.off_tile_bad);
  for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < pl.n_tiles;
       t += (int64_t)gridDim.x * blockDim.x)
    bad[t] = 0;
  uint32_t* next = reinterpret_cast<uint32_t*>(static_cast<char*>(ws) + pl.off_work_next);
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < 2 * (int64_t)H;
       i += (int64_t)gridDim.x * blockDim.x)
    next[i] = 0;          // claim counters and exit counters of the heads
}

// One thread per row: rows that are split reserve their partial slots and enter the list of
// long rows.
__global__ __launch_bounds__(256) void split_prepass_kernel(const int64_t* __restrict__ row_ptr,
                                                            int64_t L, int32_t H, int32_t dtype,
                                                            int32_t d, void* ws, size_t ws_bytes,
                                                            int skip_tiled) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= L) return;
  const int64_t deg = row_ptr[i + 1] - row_ptr[i];
  if (deg <= kSplitThreshold / 2) return;           // (no rule splits a row this short)
  const WorkspacePlan pl = plan_workspace(L, H, row_ptr[L], dtype, d);
  if (pl.total_bytes > ws_bytes || !row_is_split(deg, pl)) return;
  if (skip_tiled && (tiles_cover_everything(pl, ws) || tile_handled(pl, ws, row_ptr, L, dtype, i / kTile)))
    return;
  uint32_t* ctr = reinterpret_cast<uint32_t*>(ws);
  int32_t n, len, nf, lenf;
  row_split_shape(deg, pl, false, n, len);
  row_split_shape(deg, pl, true, nf, lenf);
  if (nf <= n) {
    nf = n;
    lenf = len;
  }
  atomicAdd(&ctr[kCtrChunksNeeded], (uint32_t)n);
  atomicMax(&ctr[kCtrMaxChunks], (uint32_t)n);
  atomicAdd(&ctr[kCtrFineNeeded], (uint32_t)nf);
  atomicMax(&ctr[kCtrMaxChunksFine], (uint32_t)nf);
  const uint32_t base = atomicAdd(&ctr[kCtrItemsAlloc], (uint32_t)n);
  const uint32_t basef = atomicAdd(&ctr[kCtrFineAlloc], (uint32_t)nf);
  if ((int64_t)base + n > pl.cap_items) return;
  const uint32_t slot = atomicAdd(&ctr[kCtrLongRows], 1u);
  int4* lr = reinterpret_cast<int4*>(static_cast<char*>(ws) + pl.off_long);
  lr[slot] = make_int4((int)i, (int)base, n, len);
  // (read only if the finer chunks of every row fit, and then basef + nf <= cap_items)
  lr[pl.cap_items + slot] = make_int4((int)i, (int)basef, nf, lenf);
}

// The list of long rows that this call uses: the finer split if all its chunks fit.
__device__ __forceinline__ const int4* long_rows(const WorkspacePlan& pl, const void* ws, uint32_t& max_chunks) {
  const uint32_t* ctr = reinterpret_cast<const uint32_t*>(ws);
  const bool fine = (int64_t)ctr[kCtrFineNeeded] <= pl.cap_items;
  max_chunks = ctr[fine ? kCtrMaxChunksFine : kCtrMaxChunks];
  return reinterpret_cast<const int4*>(static_cast<const char*>(ws) + pl.off_long) + (fine ? pl.cap_items : 0);
}

// True when the long rows of this call are handled by the chunk kernels.
__device__ __forceinline__ bool split_active(const int64_t* row_ptr, int64_t L, int32_t H,
                                             int32_t dtype, int32_t d, const void* ws,
                                             size_t ws_bytes) {
  if (!ws) return false;
  const WorkspacePlan pl = plan_workspace(L, H, row_ptr[L], dtype, d);
  if (pl.total_bytes > ws_bytes) return false;
  const uint32_t need = reinterpret_cast<const uint32_t*>(ws)[kCtrChunksNeeded];
  return (int64_t)need <= pl.cap_items;
}

// True when this call's tile path produced row i (its 32-row tile has a block list).
__device__ __forceinline__ bool row_done_by_tiles(const int64_t* row_ptr, int64_t L, int32_t H,
                                                  int32_t dtype, int32_t d, const void* ws,
                                                  size_t ws_bytes, int64_t i) {
  const WorkspacePlan pl = plan_workspace(L, H, row_ptr[L], dtype, d);
  if (pl.total_bytes > ws_bytes) return false;
  return tile_handled(pl, ws, row_ptr, L, dtype, i / kTile);
}

// (wg of n_wg: this workgroup's place among those that share the rows of a head)
template <typename T, int D>
__device__ __forceinline__ void gather_csr_body(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, T* __restrict__ O,
    float* __restrict__ lse, const int64_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
    int64_t L, float scale, const void* ws, size_t ws_bytes, int use_split, int skip_tiled,
    int accumulate, uint32_t wg, uint32_t n_wg) {
  const int lane = threadIdx.x & (kWave - 1);
  const int waves = blockDim.x / kWave;
  const int64_t h = blockIdx.y;
  const int32_t H = (int32_t)gridDim.y;
  const int64_t hoff = h * L * D;
  // After the tile path the rows left are those of the tiles it gave up (the list the CSR -> tile
  // pass wrote) and, if the partial states of the multi-segment tiles did not fit, of those
  // tiles (the merge list): the wavefronts stride over these tiles' rows instead of testing
  // every row of the sequence (L = 262,144 with one tile left: 430 -> 10 microseconds).
  int64_t n_units = L;                  // rows, or 32 x listed tiles
  const int32_t* bad_list = nullptr;
  const int4* multi_list = nullptr;
  int64_t n_bad = 0, n_multi = 0;
  bool listed = false, parts_fit = true;
  WorkspacePlan pl{};
  if (skip_tiled) {
    pl = plan_workspace(L, H, row_ptr[L], DtypeOf<T>::code, D);
    if (pl.total_bytes <= ws_bytes) {
      if (tiles_cover_everything(pl, ws)) return;
      const uint32_t* ctr = reinterpret_cast<const uint32_t*>(ws);
      parts_fit = (int64_t)ctr[kCtrTilePartsNeeded] <= pl.cap_tparts;
      n_bad = ctr[kCtrTilesBad];
      n_multi = parts_fit ? 0 : ctr[kCtrMultiTiles];
      if (n_multi <= pl.cap_tparts) {     // (a merge list that overflowed is incomplete: test every row then)
        listed = true;
        bad_list = reinterpret_cast<const int32_t*>(static_cast<const char*>(ws) + pl.off_bad_list);
        multi_list = reinterpret_cast<const int4*>(static_cast<const char*>(ws) + pl.off_multi_tiles);
        n_units = (n_bad + n_multi) * kTile;
      }
    }
  }
  for (int64_t u = (int64_t)wg * waves + (threadIdx.x / kWave); u < n_units;
       u += (int64_t)n_wg * waves) {
    int64_t i = u;
    if (listed) {
      const int64_t ti = u / kTile;
      const int64_t t = ti < n_bad ? bad_list[ti] : multi_list[ti - n_bad].x;
      // (a multi-segment tile that was also given up is in both lists when the parts do not fit)
      if (ti < n_bad && !parts_fit && tile_segments(row_ptr, L, pl.seg_shift, t) > 1) continue;
      i = t * kTile + (u - ti * kTile);
      if (i >= L) continue;
    } else if (skip_tiled && row_done_by_tiles(row_ptr, L, H, DtypeOf<T>::code, D, ws, ws_bytes, i)) {
      continue;
    }
    const int64_t r0 = row_ptr[i], r1 = row_ptr[i + 1];
    if (use_split && r1 - r0 > kSplitThreshold / 2 && split_active(row_ptr, L, H, DtypeOf<T>::code, D, ws, ws_bytes) &&
        row_is_split(r1 - r0, plan_workspace(L, H, row_ptr[L], DtypeOf<T>::code, D)))
      continue;
    float q[Row<T, D>::VEC];
    load_query<T, D>(Q + hoff + i * D, scale, lane, q);
    State<Row<T, D>::VEC> st;
    st.init();
    if (L * D * (int64_t)sizeof(T) < (int64_t(1) << 32))
      attend_columns<T, D, true>(K + hoff, V + hoff, q, col_idx + r0, 0, r1 - r0, lane, st);
    else
      attend_columns<T, D, false>(K + hoff, V + hoff, q, col_idx + r0, 0, r1 - r0, lane, st);
    finish_row<T, D>(O + hoff + i * D, lse ? lse + h * L + i : nullptr, lane, st, accumulate != 0);
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void gather_csr_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, T* __restrict__ O,
    float* __restrict__ lse, const int64_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
    int64_t L, float scale, const void* ws, size_t ws_bytes, int use_split, int skip_tiled,
    int accumulate) {
  gather_csr_body<T, D>(Q, K, V, O, lse, row_ptr, col_idx, L, scale, ws, ws_bytes, use_split, skip_tiled,
                        accumulate, blockIdx.x, gridDim.x);
}

template <typename T, int D>
__global__ __launch_bounds__(256) void gather_window_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, T* __restrict__ O,
    float* __restrict__ lse, int64_t L, int64_t W, int64_t s, float scale, int accumulate) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t i = (int64_t)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
  if (i >= L) return;
  const int64_t h = blockIdx.y;
  const int64_t hoff = h * L * D;
  const int64_t kl = min(W, i / s), kr = min(W, (L - 1 - i) / s);
  float q[Row<T, D>::VEC];
  load_query<T, D>(Q + hoff + i * D, scale, lane, q);
  State<Row<T, D>::VEC> st;
  st.init();
  WindowNeighbours nbr{i - kl * s, s};
  attend_range<T, D>(K + hoff, V + hoff, q, nbr, 0, kl + kr + 1, lane, st);
  finish_row<T, D>(O + hoff + i * D, lse ? lse + h * L + i : nullptr, lane, st, accumulate != 0);
}

// Implicit Get_Neighbors for the masks whose rows are one arithmetic run of keys that is not a
// centred window: the 2-D dilated blocks of Section II-C, and the rows below the global rows
// of the "global (non-local)" mask of Section IV-B.  One wavefront per row; a row without
// neighbours is written as the initial state (or left as it is when accumulating).
struct RowRun {
  int64_t first, step, count;
};

__device__ __forceinline__ RowRun row_run(int32_t kind, int64_t i, int64_t L, int64_t W, int64_t s,
                                          int64_t g, int64_t B) {
  if (kind == SGA_MASK_DILATED_2D) {
    const int64_t blk = i / B, r = i - blk * B;
    if (r % s != 0) return {0, 1, 0};
    const int64_t len = min(B, L - blk * B);
    return {blk * B, s, (len + s - 1) / s};
  }
  // non-local, row i >= g: global columns 0..g-1 that lie left of the window
  const int64_t n = min(g, i - W);
  return {0, 1, n > 0 ? n : 0};
}

template <typename T, int D>
__global__ __launch_bounds__(256) void gather_runs_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, T* __restrict__ O,
    float* __restrict__ lse, int64_t L, int32_t kind, int64_t W, int64_t s, int64_t g, int64_t B,
    int64_t row0, float scale, int accumulate) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t i = row0 + (int64_t)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
  if (i >= L) return;
  const int64_t h = blockIdx.y;
  const int64_t hoff = h * L * D;
  const RowRun run = row_run(kind, i, L, W, s, g, B);
  float q[Row<T, D>::VEC];
  load_query<T, D>(Q + hoff + i * D, scale, lane, q);
  State<Row<T, D>::VEC> st;
  st.init();
  if (run.count > 0) {
    WindowNeighbours nbr{run.first, run.step};
    attend_range<T, D>(K + hoff, V + hoff, q, nbr, 0, run.count, lane, st);
  }
  finish_row<T, D>(O + hoff + i * D, lse ? lse + h * L + i : nullptr, lane, st, accumulate != 0);
}

// Combine the n partial (m, l, acc) states of one row in their stored order (deterministic) and
// write the row: one wavefront, lane c owns channels c, c + 64, ...
template <typename T, int D>
__device__ __forceinline__ void merge_row_partials(const float* p0, int64_t step, int n, T* Orow,
                                                   float* lse_i, int lane, bool accumulate) {
  constexpr int kCh = (D + kWave - 1) / kWave;
  float M = kMinusHuge;
  for (int c = 0; c < n; ++c) M = fmaxf(M, p0[c * step + D]);
  float l = 0.f, acc[kCh];
#pragma unroll
  for (int k = 0; k < kCh; ++k) acc[k] = 0.f;
  for (int c = 0; c < n; ++c) {
    const float w = __builtin_amdgcn_exp2f(p0[c * step + D] - M);
    l = __builtin_fmaf(p0[c * step + D + 1], w, l);
#pragma unroll
    for (int k = 0; k < kCh; ++k)
      if (lane + k * kWave < D) acc[k] = __builtin_fmaf(p0[c * step + lane + k * kWave], w, acc[k]);
  }
  const bool empty = !(l > 0.f);
  const float inv = empty ? 0.f : 1.0f / l;
  float lse_row = empty ? -INFINITY : (M + __builtin_amdgcn_logf(l)) * kLn2;
  CarryWeights cw{0.f, 1.f, lse_row};
  if (accumulate) {      // every lane reads the earlier lse before lane 0 replaces it
    cw = carry_weights(*lse_i, lse_row);
    lse_row = cw.lse;
  }
#pragma unroll
  for (int k = 0; k < kCh; ++k) {
    const int ch = lane + k * kWave;
    if (ch < D) {
      float o = acc[k] * inv * cw.w_now;
      if (accumulate) o = __builtin_fmaf(cw.w_prev, load_scalar(Orow + ch), o);
      store_scalar(Orow + ch, o);
    }
  }
  if (lse_i && lane == 0) *lse_i = lse_row;
}

// Global rows i < g of the non-local mask attend every key outside their window: about L
// neighbours each.  grid = (chunks, g, H): a wavefront reduces the keys of one chunk of the
// key range (the window cut out) to a partial (m, l, acc) state ...
template <typename T, int D>
__global__ __launch_bounds__(64) void nonlocal_chunk_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, int64_t L, int64_t W,
    int64_t chunk_len, float scale, float* __restrict__ partials) {
  const int lane = threadIdx.x;
  const int64_t c = blockIdx.x, i = blockIdx.y, h = blockIdx.z;
  const int64_t H = gridDim.z, n_chunks = gridDim.x;
  const int64_t hoff = h * L * D;
  const int64_t lo = c * chunk_len, hi = min(L, lo + chunk_len);      // keys [lo, hi)
  float q[Row<T, D>::VEC];
  load_query<T, D>(Q + hoff + i * D, scale, lane, q);
  State<Row<T, D>::VEC> st;
  st.init();
  const int64_t a1 = min(hi, i - W);             // keys [lo, a1) lie left of the window
  if (a1 > lo) {
    WindowNeighbours nbr{lo, 1};
    attend_range<T, D>(K + hoff, V + hoff, q, nbr, 0, a1 - lo, lane, st);
  }
  const int64_t b0 = max(lo, i + W + 1);         // keys [b0, hi) lie right of it
  if (hi > b0) {
    WindowNeighbours nbr{b0, 1};
    attend_range<T, D>(K + hoff, V + hoff, q, nbr, 0, hi - b0, lane, st);
  }
  merge_groups<Row<T, D>::LPK, Row<T, D>::VEC>(st);
  float* p = partials + ((i * n_chunks + c) * H + h) * (D + 4);
  if (lane < Row<T, D>::LPK) {
#pragma unroll
    for (int k = 0; k < Row<T, D>::VEC; ++k) p[lane * Row<T, D>::VEC + k] = st.acc[k];
  }
  if (lane == 0) {
    p[D] = st.m;
    p[D + 1] = st.l;
  }
}

// ... and one workgroup per (global row, head) combines the row's partials: each of its four
// wavefronts reduces a quarter of the chunks, in chunk order, to one partial state in LDS, and
// the first wavefront combines the four in wavefront order and writes the row (a fixed order:
// deterministic).
template <typename T, int D>
__global__ __launch_bounds__(256) void nonlocal_merge_kernel(T* __restrict__ O, float* __restrict__ lse,
                                                             int64_t L, int32_t n_chunks,
                                                             const float* __restrict__ partials,
                                                             int accumulate) {
  constexpr int kCh = (D + kWave - 1) / kWave;
  __shared__ float quarter[4][D + 4];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int64_t i = blockIdx.x, h = blockIdx.y, H = gridDim.y;
  const int64_t step = H * (D + 4);
  const int per = (n_chunks + 3) / 4;
  const int c0 = wave * per < n_chunks ? wave * per : n_chunks;
  const int c1 = c0 + per < n_chunks ? c0 + per : n_chunks;
  const float* p0 = partials + ((i * n_chunks + c0) * H + h) * (D + 4);
  float M = kMinusHuge;
  for (int c = 0; c < c1 - c0; ++c) M = fmaxf(M, p0[c * step + D]);
  float l = 0.f, acc[kCh];
#pragma unroll
  for (int k = 0; k < kCh; ++k) acc[k] = 0.f;
  for (int c = 0; c < c1 - c0; ++c) {
    const float w = __builtin_amdgcn_exp2f(p0[c * step + D] - M);
    l = __builtin_fmaf(p0[c * step + D + 1], w, l);
#pragma unroll
    for (int k = 0; k < kCh; ++k)
      if (lane + k * kWave < D) acc[k] = __builtin_fmaf(p0[c * step + lane + k * kWave], w, acc[k]);
  }
#pragma unroll
  for (int k = 0; k < kCh; ++k)
    if (lane + k * kWave < D) quarter[wave][lane + k * kWave] = acc[k];
  if (lane == 0) {
    quarter[wave][D] = M;
    quarter[wave][D + 1] = l;
  }
  __syncthreads();
  if (wave == 0)
    merge_row_partials<T, D>(&quarter[0][0], D + 4, 4, O + h * L * D + i * D, lse ? lse + h * L + i : nullptr, lane,
                             accumulate != 0);
}

// One wavefront per (chunk of a long row, head): partial state of a slice of the row.  Chunk c
// of every row is computed on XCD c % 8 (workgroups go to the XCDs round-robin in launch order
// and gridDim.x is a multiple of 8): chunks are ranges of the rows' sorted neighbour lists, so
// an XCD's L2 sees the same part of the key range from every row.  The work units of XCD x are
// the pairs (long row s, j) with chunk c = x + 8j, numbered j * n_long + s (rows of few chunks
// have no unit for the larger j) and dealt to the XCD's wavefronts in turn.
template <typename T, int D>
__device__ __forceinline__ void gather_chunk_body(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const int64_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx, int64_t L, float scale,
    void* ws, size_t ws_bytes, uint32_t wg, uint32_t n_wg) {
  const int32_t H = (int32_t)gridDim.y;
  constexpr int32_t dtype = DtypeOf<T>::code;
  if (!split_active(row_ptr, L, H, dtype, D, ws, ws_bytes)) return;
  const WorkspacePlan pl = plan_workspace(L, H, row_ptr[L], dtype, D);
  const uint32_t n_long = reinterpret_cast<const uint32_t*>(ws)[kCtrLongRows];
  uint32_t max_chunks;
  const int4* lr = long_rows(pl, ws, max_chunks);
  float* partials = reinterpret_cast<float*>(static_cast<char*>(ws) + pl.off_partials);
  const int lane = threadIdx.x & (kWave - 1);
  const int waves = blockDim.x / kWave;
  const int64_t h = blockIdx.y;
  const int64_t hoff = h * L * D;
  const uint32_t xcd = wg & 7;
  const uint64_t n_units = (uint64_t)n_long * ((max_chunks + 7) / 8);
  for (uint64_t u = (uint64_t)(wg >> 3) * waves + threadIdx.x / kWave; u < n_units;
       u += (uint64_t)(n_wg >> 3) * waves) {
    const int4 rec = lr[u % n_long];                         // {row, first partial slot, chunks, chunk length}
    const int32_t c = (int32_t)(xcd + 8 * (u / n_long));
    if (c >= rec.z) continue;
    const int64_t i = rec.x;
    const int64_t r0 = row_ptr[i], deg = row_ptr[i + 1] - r0;
    const int64_t e0 = (int64_t)c * rec.w;
    const int64_t e1 = min(deg, e0 + rec.w);
    float q[Row<T, D>::VEC];
    load_query<T, D>(Q + hoff + i * D, scale, lane, q);
    State<Row<T, D>::VEC> st;
    st.init();
    if (L * D * (int64_t)sizeof(T) < (int64_t(1) << 32))
      attend_columns<T, D, true>(K + hoff, V + hoff, q, col_idx + r0, e0, e1, lane, st);
    else
      attend_columns<T, D, false>(K + hoff, V + hoff, q, col_idx + r0, e0, e1, lane, st);
    merge_groups<Row<T, D>::LPK, Row<T, D>::VEC>(st);
    float* p = partials + ((int64_t)(rec.y + c) * H + h) * (D + 4);
    if (lane < Row<T, D>::LPK) {
#pragma unroll
      for (int k = 0; k < Row<T, D>::VEC; ++k) p[lane * Row<T, D>::VEC + k] = st.acc[k];
    }
    if (lane == 0) {
      p[D] = st.m;
      p[D + 1] = st.l;
    }
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void gather_chunk_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const int64_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx, int64_t L, float scale,
    void* ws, size_t ws_bytes) {
  gather_chunk_body<T, D>(Q, K, V, row_ptr, col_idx, L, scale, ws, ws_bytes, blockIdx.x, gridDim.x);
}

// The two kernels above in one launch (neither reads what the other writes): the first n_rows
// workgroups of a head (a multiple of 8, so that the chunk workgroups keep their XCDs) take the
// leftover rows, the others the chunks of the split rows.  For the call that does not know yet
// whether anything is left for either: one launch that finds nothing to do instead of two.
template <typename T, int D>
__global__ __launch_bounds__(256) void gather_rows_and_chunks_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, T* __restrict__ O,
    float* __restrict__ lse, const int64_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
    int64_t L, float scale, void* ws, size_t ws_bytes, int skip_tiled, int accumulate, uint32_t n_rows) {
  if (blockIdx.x < n_rows)
    gather_csr_body<T, D>(Q, K, V, O, lse, row_ptr, col_idx, L, scale, ws, ws_bytes, 1, skip_tiled, accumulate,
                          blockIdx.x, n_rows);
  else
    gather_chunk_body<T, D>(Q, K, V, row_ptr, col_idx, L, scale, ws, ws_bytes, blockIdx.x - n_rows,
                            gridDim.x - n_rows);
}

// Partial states p0[c * step + ...], c < n, combined in order into one partial state
// (D accumulators, m, l) at `out`; one wavefront, lane c owns channels c, c + 64, ...  The
// maxima are read 64 partials at a time and the states eight at a time, so that a row of a
// thousand chunks does not wait for a thousand loads one after the other; the sums run in
// chunk order all the same.
template <int D>
__device__ __forceinline__ void combine_partials(const float* p0, int64_t step, int n, float* out, int lane) {
  constexpr int kCh = (D + kWave - 1) / kWave;
  constexpr int kAhead = 8;
  float M = kMinusHuge;
  for (int c = lane; c < n; c += kWave) M = fmaxf(M, p0[c * step + D]);
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) M = fmaxf(M, __shfl_xor(M, off, kWave));
  float l = 0.f, acc[kCh];
#pragma unroll
  for (int k = 0; k < kCh; ++k) acc[k] = 0.f;
  for (int c0 = 0; c0 < n; c0 += kAhead) {
    float mm[kAhead], ll[kAhead], aa[kAhead][kCh];
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {
      const float* p = p0 + (c0 + u < n ? c0 + u : n - 1) * step;
      mm[u] = p[D];
      ll[u] = p[D + 1];
#pragma unroll
      for (int k = 0; k < kCh; ++k) aa[u][k] = lane + k * kWave < D ? p[lane + k * kWave] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {
      if (c0 + u < n) {
        const float w = __builtin_amdgcn_exp2f(mm[u] - M);
        l = __builtin_fmaf(ll[u], w, l);
#pragma unroll
        for (int k = 0; k < kCh; ++k) acc[k] = __builtin_fmaf(aa[u][k], w, acc[k]);
      }
    }
  }
#pragma unroll
  for (int k = 0; k < kCh; ++k)
    if (lane + k * kWave < D) out[lane + k * kWave] = acc[k];
  if (lane == 0) {
    out[D] = M;
    out[D + 1] = l;
  }
}

// Rows of up to kMaxSplit chunks: one wavefront per (long row, head) combines the row's partials
// in chunk order.  Rows of more chunks (cut by edge count into up to kMaxSplitLong): one
// workgroup per row, each of its four wavefronts combines a quarter of the partials in chunk
// order, the first one the four results in wavefront order (a fixed order whatever the
// schedule).
template <typename T, int D>
__global__ __launch_bounds__(256) void gather_merge_kernel(T* __restrict__ O, float* __restrict__ lse,
                                                           const int64_t* __restrict__ row_ptr,
                                                           int64_t L, void* ws, size_t ws_bytes,
                                                           int accumulate) {
  __shared__ float quarter[4][D + 4];
  const int32_t H = (int32_t)gridDim.y;
  constexpr int32_t dtype = DtypeOf<T>::code;
  if (!split_active(row_ptr, L, H, dtype, D, ws, ws_bytes)) return;
  const WorkspacePlan pl = plan_workspace(L, H, row_ptr[L], dtype, D);
  const uint32_t n_long = reinterpret_cast<const uint32_t*>(ws)[kCtrLongRows];
  uint32_t max_chunks;
  const int4* lr = long_rows(pl, ws, max_chunks);
  const float* partials = reinterpret_cast<const float*>(static_cast<char*>(ws) + pl.off_partials);
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int64_t h = blockIdx.y;
  const int64_t step = (int64_t)H * (D + 4);
  for (uint32_t r = blockIdx.x * 4 + wave; r < n_long; r += gridDim.x * 4) {
    const int4 rec = lr[r];
    if (rec.z > kMaxSplit) continue;
    const int64_t i = rec.x;
    merge_row_partials<T, D>(partials + ((int64_t)rec.y * H + h) * (D + 4), step, rec.z, O + h * L * D + i * D,
                             lse ? lse + h * L + i : nullptr, lane, accumulate != 0);
  }
  if (max_chunks <= (uint32_t)kMaxSplit) return;
  for (uint32_t r = blockIdx.x; r < n_long; r += gridDim.x) {      // (the same trips for the whole workgroup)
    const int4 rec = lr[r];
    if (rec.z <= kMaxSplit) continue;
    const int64_t i = rec.x;
    const float* p0 = partials + ((int64_t)rec.y * H + h) * (D + 4);
    T* Orow = O + h * L * D + i * D;
    float* lse_i = lse ? lse + h * L + i : nullptr;
    const int per = (rec.z + 3) / 4;
    const int c0 = wave * per < rec.z ? wave * per : rec.z;
    const int c1 = c0 + per < rec.z ? c0 + per : rec.z;
    __syncthreads();                 // the previous row's combine has read the shared records
    combine_partials<D>(p0 + c0 * step, step, c1 - c0, &quarter[wave][0], lane);
    __syncthreads();
    if (wave == 0) merge_row_partials<T, D>(&quarter[0][0], D + 4, 4, Orow, lse_i, lane, accumulate != 0);
  }
}

template <typename T, int D>
sga_status run_explicit(const AttnArgs& a, bool allow_split, bool skip_tiled) {
  const T* Q = static_cast<const T*>(a.Q);
  const T* K = static_cast<const T*>(a.K);
  const T* V = static_cast<const T*>(a.V);
  T* O = static_cast<T*>(a.O);
  const bool split = allow_split && a.ws && a.ws_bytes >= 256 && a.L > kSplitThreshold;
  // (a prepared graph holds the chunk items of its split rows already)
  if (split && !a.prepared) launch_split_prepass(a, skip_tiled);
  // after the tile path only leftover rows remain: a grid of about one chip-full of wavefronts
  // over all heads strides over the rows (it returns at once when the tiles covered everything)
  int64_t nwg = (a.L + 3) / 4;
  const int64_t leftover_wgs = 2048 / a.H > 256 ? 2048 / a.H : 256;
  if (skip_tiled && nwg > leftover_wgs) nwg = leftover_wgs;
  const dim3 grid((unsigned)nwg, (unsigned)a.H);
  // the benchmark hook brackets the kernel that does the work: the row kernel, or the chunk
  // kernel where a prepared graph has found every row left to it split
  const bool mark = !skip_tiled || (a.prepared && a.plan_no_tiles);
  const bool mark_chunks = mark && a.prepared && a.plan_long_rows > 0;
  const unsigned chunk_wgs = skip_tiled && a.H >= 8 ? 128 : 1024;
  const bool fused = split && skip_tiled && !a.prepared;     // (after the tile path, nothing known about what is left)
  if (fused) {
    const unsigned n_rows = ((unsigned)nwg + 7u) & ~7u;
    hipLaunchKernelGGL((gather_rows_and_chunks_kernel<T, D>), dim3(n_rows + chunk_wgs, (unsigned)a.H), dim3(256), 0,
                       a.stream, Q, K, V, O, a.lse, a.row_ptr, a.col_idx, a.L, a.scale, a.ws, a.ws_bytes, 1,
                       a.accumulate ? 1 : 0, n_rows);
  } else {
    if (mark && !mark_chunks) profile_mark_begin(a.stream, "gather_csr_kernel");
    hipLaunchKernelGGL((gather_csr_kernel<T, D>), grid, dim3(256), 0, a.stream, Q, K, V, O, a.lse,
                       a.row_ptr, a.col_idx, a.L, a.scale, a.ws, a.ws_bytes, split ? 1 : 0,
                       skip_tiled ? 1 : 0, a.accumulate ? 1 : 0);
    if (mark && !mark_chunks) profile_mark_end(a.stream);
  }
  if (split && (!a.prepared || a.plan_long_rows > 0)) {
    if (!fused) {
      if (mark_chunks) profile_mark_begin(a.stream, "gather_chunk_kernel");
      hipLaunchKernelGGL((gather_chunk_kernel<T, D>), dim3(chunk_wgs, (unsigned)a.H), dim3(256), 0, a.stream, Q,
                         K, V, a.row_ptr, a.col_idx, a.L, a.scale, a.ws, a.ws_bytes);
      if (mark_chunks) profile_mark_end(a.stream);
    }
    // one wavefront per long row and head, one workgroup for a row of more than kMaxSplit
    // chunks; a prepared graph knows how many rows there are
    int64_t merge_wgs = a.prepared ? (int64_t)a.plan_long_rows : (a.L + 3) / 4;
    const int64_t merge_cap = 4096 / a.H > 64 ? 4096 / a.H : 64;
    if (merge_wgs > merge_cap) merge_wgs = merge_cap;
    hipLaunchKernelGGL((gather_merge_kernel<T, D>), dim3((unsigned)merge_wgs, (unsigned)a.H), dim3(256), 0, a.stream, O,
                       a.lse, a.row_ptr, a.L, a.ws, a.ws_bytes, a.accumulate ? 1 : 0);
  }
  return hip_status(hipGetLastError());
}

}  // namespace

void clear_workspace(const AttnArgs& a, bool tile_flags) {
  const int64_t n_tiles = (a.L + kTile - 1) / kTile;
  int64_t nwg = tile_flags ? (n_tiles + 255) / 256 : 1;
  if (nwg > 1024) nwg = 1024;
  hipLaunchKernelGGL(clear_workspace_kernel, dim3((unsigned)nwg), dim3(256), 0, a.stream, a.ws,
                     a.ws_bytes, a.row_ptr, a.L, a.H, a.dtype, a.d, tile_flags ? 1 : 0);
}

void launch_split_prepass(const AttnArgs& a, bool skip_tiled) {
  hipLaunchKernelGGL(split_prepass_kernel, dim3((unsigned)((a.L + 255) / 256)), dim3(256), 0, a.stream,
                     a.row_ptr, a.L, a.H, a.dtype, a.d, a.ws, a.ws_bytes, skip_tiled ? 1 : 0);
}

sga_status launch_gather_explicit(const AttnArgs& a, bool allow_split, bool skip_tiled) {
  switch (a.d) {
    case 32:
      return a.dtype == SGA_F32 ? run_explicit<float, 32>(a, allow_split, skip_tiled)
                                : run_explicit<__half, 32>(a, allow_split, skip_tiled);
    case 64:
      return a.dtype == SGA_F32 ? run_explicit<float, 64>(a, allow_split, skip_tiled)
                                : run_explicit<__half, 64>(a, allow_split, skip_tiled);
    case 128:
      return a.dtype == SGA_F32 ? run_explicit<float, 128>(a, allow_split, skip_tiled)
                                : run_explicit<__half, 128>(a, allow_split, skip_tiled);
    case 256:
      return a.dtype == SGA_F32 ? run_explicit<float, 256>(a, allow_split, skip_tiled)
                                : run_explicit<__half, 256>(a, allow_split, skip_tiled);
    default:
      return SGA_ERR_UNSUPPORTED;
  }
}

template <typename T, int D>
static sga_status run_implicit(const AttnArgs& a) {
  const T* Q = static_cast<const T*>(a.Q);
  const T* K = static_cast<const T*>(a.K);
  const T* V = static_cast<const T*>(a.V);
  T* O = static_cast<T*>(a.O);
  const int acc = a.accumulate ? 1 : 0;
  if (a.mask_kind == SGA_MASK_SLIDING || a.mask_kind == SGA_MASK_DILATED) {
    const dim3 grid((unsigned)((a.L + 3) / 4), (unsigned)a.H);
    profile_mark_begin(a.stream, "gather_window_kernel");
    hipLaunchKernelGGL((gather_window_kernel<T, D>), grid, dim3(256), 0, a.stream, Q, K, V, O, a.lse, a.L,
                       (int64_t)a.window, (int64_t)a.stride, a.scale, acc);
    profile_mark_end(a.stream);
    return hip_status(hipGetLastError());
  }
  // rows that are one arithmetic run: all rows of the 2-D dilated mask, rows >= g of the
  // non-local mask
  const int64_t g = a.mask_kind == SGA_MASK_NONLOCAL ? (a.n_global < a.L ? a.n_global : a.L) : 0;
  if constexpr (D >= kHeadDim) {
    if (a.mask_kind == SGA_MASK_NONLOCAL && a.tiles_allowed) {
      // matrix-core tiles: 32 rows >= g at a time against the one or two key blocks that hold the
      // global tokens; the g global rows as one or two tiles over ranges of all key blocks, with
      // partial states that the merge below combines in range order
      float* partials = g > 0 ? reinterpret_cast<float*>(static_cast<char*>(a.ws) +
                                                         plan_workspace(a.L, a.H, -1, a.dtype, D).off_partials)
                              : nullptr;
      int32_t n_chunks = 0;
      launch_tile_nonlocal(a, g, partials, &n_chunks);
      if (g > 0)
        hipLaunchKernelGGL((nonlocal_merge_kernel<T, D>), dim3((unsigned)g, (unsigned)a.H), dim3(256), 0, a.stream,
                           O, a.lse, a.L, n_chunks, partials, acc);
      return hip_status(hipGetLastError());
    }
  }
  if (a.L > g) {
    const dim3 grid((unsigned)((a.L - g + 3) / 4), (unsigned)a.H);
    profile_mark_begin(a.stream, "gather_runs_kernel");
    hipLaunchKernelGGL((gather_runs_kernel<T, D>), grid, dim3(256), 0, a.stream, Q, K, V, O, a.lse, a.L,
                       a.mask_kind, (int64_t)a.window, (int64_t)a.stride, g, (int64_t)a.block, g, a.scale,
                       acc);
    profile_mark_end(a.stream);
  }
  if (g > 0) {
    // the g global rows: split over the key range, partial states in the workspace
    int32_t n_chunks, len;
    split_shape(a.L, kSplitChunk, n_chunks, len);
    float* partials = reinterpret_cast<float*>(static_cast<char*>(a.ws) +
                                               plan_workspace(a.L, a.H, -1, a.dtype, D).off_partials);
    hipLaunchKernelGGL((nonlocal_chunk_kernel<T, D>), dim3((unsigned)n_chunks, (unsigned)g, (unsigned)a.H),
                       dim3(64), 0, a.stream, Q, K, V, a.L, (int64_t)a.window, (int64_t)len, a.scale,
                       partials);
    hipLaunchKernelGGL((nonlocal_merge_kernel<T, D>), dim3((unsigned)g, (unsigned)a.H), dim3(256), 0, a.stream,
                       O, a.lse, a.L, n_chunks, partials, acc);
  }
  return hip_status(hipGetLastError());
}

sga_status launch_gather_implicit(const AttnArgs& a) {
  switch (a.d) {
    case 32: return a.dtype == SGA_F32 ? run_implicit<float, 32>(a) : run_implicit<__half, 32>(a);
    case 64: return a.dtype == SGA_F32 ? run_implicit<float, 64>(a) : run_implicit<__half, 64>(a);
    case 128: return a.dtype == SGA_F32 ? run_implicit<float, 128>(a) : run_implicit<__half, 128>(a);
    case 256: return a.dtype == SGA_F32 ? run_implicit<float, 256>(a) : run_implicit<__half, 256>(a);
    default: return SGA_ERR_UNSUPPORTED;
  }
}

}  // namespace sga
