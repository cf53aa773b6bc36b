// Mask -> graph: CSR row offsets and sorted column indices of the mask families of
// Section II-C and of the "global (non-local)" mask of Section IV-B (explicit form of
// Get_Neighbors, Section IV-B "CSR").
//
// Every row of every family is a short ordered list of arithmetic column runs
// ("segments": start, length, step), so
//   - the row offset is a closed-form prefix sum evaluated independently per row
//     (no scan over the rows is needed), and
//   - a group of consecutive rows is filled by one wavefront that derives the
//     group's segments once and then streams the rows out with coalesced int32
//     stores; rows that attend every key are written by a kernel of their own,
//     many workgroups per row.
#include "sga_internal.h"

namespace sga {
namespace {

constexpr int kMaxRandom = 16;
constexpr int kMaxSegments = kMaxRandom + 2;
constexpr uint64_t kGold = 0x9E3779B97F4A7C15ull;

__host__ __device__ inline uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

__host__ __device__ inline int64_t imin(int64_t a, int64_t b) { return a < b ? a : b; }
__host__ __device__ inline int64_t imax(int64_t a, int64_t b) { return a > b ? a : b; }

// sum_{t=0}^{n-1} min(W, t div s)
__host__ __device__ inline int64_t clipped_steps_prefix(int64_t n, int64_t W, int64_t s) {
  if (n >= W * s) return s * (W * (W - 1) / 2) + (n - W * s) * W;
  const int64_t q = n / s, r = n - q * s;
  return s * (q * (q - 1) / 2) + r * q;
}

// Edges in rows [0, i) of the window family: row t has 1 + min(W, t div s) + min(W, (L-1-t) div s).
__host__ __device__ inline int64_t window_prefix(int64_t i, int64_t L, int64_t W, int64_t s) {
  return i + clipped_steps_prefix(i, W, s) + clipped_steps_prefix(L, W, s) -
         clipped_steps_prefix(L - i, W, s);
}

// sum_{t=0}^{n-1} min(L, t + w + 1)
__host__ __device__ inline int64_t upper_prefix(int64_t n, int64_t L, int64_t w) {
  const int64_t n1 = imin(n, imax(0, L - w));
  return n1 * (n1 - 1) / 2 + n1 * (w + 1) + (n - n1) * L;
}

// sum_{t=0}^{n-1} max(t - w, g)
__host__ __device__ inline int64_t lower_prefix(int64_t n, int64_t w, int64_t g) {
  const int64_t n2 = imin(n, g + w);
  return n2 * g + (n * (n - 1) / 2 - n2 * (n2 - 1) / 2) - (n - n2) * w;
}

// Edges in rows [0, i) of "window w plus g leading global tokens" over L tokens, with
// `extra` further neighbours on every non-global row (0 here; the random picks at block level).
// Row t < g has L neighbours; row t >= g has g + min(L, t+w+1) - max(t-w, g) + extra.
__host__ __device__ inline int64_t global_local_prefix(int64_t i, int64_t L, int64_t w, int64_t g,
                                                       int64_t extra) {
  if (i <= g) return i * L;
  return g * L + (g + extra) * (i - g) + (upper_prefix(i, L, w) - upper_prefix(g, L, w)) -
         (lower_prefix(i, w, g) - lower_prefix(g, w, g));
}

struct MaskParams {
  int32_t kind;
  int64_t L;
  int64_t W;       // clamped half-width in steps
  int64_t s;       // stride
  int64_t g;       // clamped global token count
  int64_t B, nb, wb, G, R;
  uint64_t seed;
};

__host__ __device__ inline int64_t row_offset(const MaskParams& p, int64_t i) {
  switch (p.kind) {
    case SGA_MASK_SLIDING:
    case SGA_MASK_DILATED:
      return window_prefix(i, p.L, p.W, p.s);
    case SGA_MASK_GLOBAL_LOCAL:
      return global_local_prefix(i, p.L, p.W, p.g, 0);
    case SGA_MASK_NONLOCAL:   // the global+local mask without its window
      return global_local_prefix(i, p.L, p.W, p.g, 0) - window_prefix(i, p.L, p.W, 1);
    case SGA_MASK_DILATED_2D: {
      // blocks before row i's block are whole: ceil(B/s)^2 edges each; inside the block the
      // selected rows (every s-th) before row i have one edge per selected column
      const int64_t blk = i / p.B, r = i - blk * p.B;
      const int64_t per_full = (p.B + p.s - 1) / p.s;
      const int64_t len = imin(p.B, p.L - blk * p.B);
      const int64_t n_sel = (len + p.s - 1) / p.s;
      return blk * per_full * per_full + ((r + p.s - 1) / p.s) * n_sel;
    }
    default: {  // block mask: all rows of a query block have the same degree
      const int64_t b = i / p.B;
      const int64_t before = global_local_prefix(b, p.nb, p.wb, p.G, p.R);
      const int64_t cnt = global_local_prefix(b + 1, p.nb, p.wb, p.G, p.R) - before;
      return p.B * (p.B * before + (i - b * p.B) * cnt);
    }
  }
}

MaskParams make_params(const sga_mask_desc& d) {
  MaskParams p{};
  p.kind = d.kind;
  p.L = d.L;
  p.s = (d.kind == SGA_MASK_DILATED || d.kind == SGA_MASK_DILATED_2D) ? d.stride : 1;
  p.W = imin(d.window, (d.L - 1) / p.s);
  p.g = imin(d.n_global, d.L);
  p.B = d.block > 0 ? d.block : 1;
  p.nb = d.L / p.B;
  p.wb = imin(d.window_blocks, p.nb > 0 ? p.nb - 1 : 0);
  p.G = imin(d.n_global_blocks, p.nb);
  p.R = d.n_random_blocks;
  p.seed = d.seed;
  return p;
}

__device__ __forceinline__ void row_ptr_part(const MaskParams& p, int64_t* __restrict__ row_ptr,
                                             int64_t bid) {
  const int64_t i = bid * blockDim.x + threadIdx.x;
  if (i <= p.L) row_ptr[i] = row_offset(p, i);
}

struct Segment {
  int32_t start, len, step;
};

// Rows that attend every key (global tokens / global query blocks) come first: rows [0, n_full).
__host__ __device__ inline int64_t full_rows(const MaskParams& p) {
  if (p.kind == SGA_MASK_GLOBAL_LOCAL) return p.g;
  if (p.kind == SGA_MASK_BIGBIRD) return p.G * p.B;
  return 0;
}

// Rows of a group share one segment list: the B rows of a query block (block mask), else one row.
__host__ __device__ inline int64_t group_rows(const MaskParams& p) {
  return p.kind == SGA_MASK_BIGBIRD ? p.B : 1;
}

// One wavefront per row group: lane 0 derives the group's segments once, then the wavefront
// streams every row of the group with coalesced 256-byte stores.  Full rows are left to
// fill_full_rows_kernel.
// (row offsets are evaluated in closed form, not read from row_ptr, so that this part does not
// depend on the part of the launch that writes row_ptr)
__device__ __forceinline__ void fill_part(const MaskParams& p, int32_t* __restrict__ col_idx, int64_t bid,
                                          Segment (*seg_all)[kMaxSegments], int* n_seg_all,
                                          int64_t (*picks_all)[kMaxRandom]) {
  const int wave = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
  Segment* seg = seg_all[wave];
  int64_t* picks = picks_all[wave];
  const int64_t R = group_rows(p);
  const int64_t group = bid * 4 + wave;
  const int64_t i = group * R;                      // first row of the group
  if (i >= p.L || i < full_rows(p)) return;
  if (lane == 0) {
    int n = 0;
    if (p.kind == SGA_MASK_SLIDING || p.kind == SGA_MASK_DILATED) {
      const int64_t kl = imin(p.W, i / p.s), kr = imin(p.W, (p.L - 1 - i) / p.s);
      seg[n++] = {(int32_t)(i - kl * p.s), (int32_t)(kl + kr + 1), (int32_t)p.s};
    } else if (p.kind == SGA_MASK_GLOBAL_LOCAL) {
      const int64_t lo = imax(0, i - p.W), hi = imin(p.L - 1, i + p.W);
      if (lo <= p.g) {
        seg[n++] = {0, (int32_t)(hi + 1), 1};
      } else {
        if (p.g > 0) seg[n++] = {0, (int32_t)p.g, 1};
        seg[n++] = {(int32_t)lo, (int32_t)(hi - lo + 1), 1};
      }
    } else if (p.kind == SGA_MASK_NONLOCAL) {
      if (i < p.g) {
        if (i - p.W - 1 >= 0) seg[n++] = {0, (int32_t)(i - p.W), 1};
        if (i + p.W + 1 <= p.L - 1) seg[n++] = {(int32_t)(i + p.W + 1), (int32_t)(p.L - 1 - i - p.W), 1};
      } else {
        const int64_t hi = imin(p.g - 1, i - p.W - 1);
        if (hi >= 0) seg[n++] = {0, (int32_t)(hi + 1), 1};
      }
    } else if (p.kind == SGA_MASK_DILATED_2D) {
      const int64_t blk = i / p.B, r = i - blk * p.B;
      if (r % p.s == 0) {
        const int64_t len = imin(p.B, p.L - blk * p.B);
        seg[n++] = {(int32_t)(blk * p.B), (int32_t)((len + p.s - 1) / p.s), (int32_t)p.s};
      }
    } else {
      const int64_t b = group;
      const int64_t lo = imax(0, b - p.wb), hi = imin(p.nb - 1, b + p.wb);
      // random key blocks: rejection sampling over the counter-based stream of block b
      const uint64_t key = mix64(p.seed + kGold * (uint64_t)(b + 1));
      int got = 0;
      uint64_t a = 0;
      while (got < (int)p.R) {
        const int64_t cand = (int64_t)(mix64(key + kGold * (a + 1)) % (uint64_t)p.nb);
        ++a;
        bool taken = cand < p.G || (cand >= lo && cand <= hi);
        for (int t = 0; t < got; ++t) taken = taken || picks[t] == cand;
        if (!taken) {
          // keep picks sorted (insertion)
          int pos = got;
          while (pos > 0 && picks[pos - 1] > cand) {
            picks[pos] = picks[pos - 1];
            --pos;
          }
          picks[pos] = cand;
          ++got;
        }
      }
      int t = 0;
      if (lo <= p.G) {
        // global blocks and the window form one run [0, hi]
        seg[n++] = {0, (int32_t)((hi + 1) * p.B), 1};
      } else {
        if (p.G > 0) seg[n++] = {0, (int32_t)(p.G * p.B), 1};
        for (; t < got && picks[t] < lo; ++t)
          seg[n++] = {(int32_t)(picks[t] * p.B), (int32_t)p.B, 1};
        seg[n++] = {(int32_t)(lo * p.B), (int32_t)((hi - lo + 1) * p.B), 1};
      }
      for (; t < got; ++t) seg[n++] = {(int32_t)(picks[t] * p.B), (int32_t)p.B, 1};
    }
    n_seg_all[wave] = n;
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  const int n = n_seg_all[wave];
  const int64_t rows = imin(R, p.L - i);
  // the rows of a group hold the same columns, so they follow each other at equal distances
  int64_t row_len = 0;
  for (int k = 0; k < n; ++k) row_len += seg[k].len;
  const int64_t base = row_offset(p, i);
  for (int64_t r = 0; r < rows; ++r) {
    int32_t* out = col_idx + base + r * row_len;
    for (int k = 0; k < n; ++k) {
      const Segment sg = seg[k];
      for (int32_t t = lane; t < sg.len; t += kWave) out[t] = sg.start + t * sg.step;
      out += sg.len;
    }
  }
}

// Rows [0, n_full) attend every key: col_idx of such a row is 0, 1, ..., L-1.  One workgroup per
// chunk of 4096 columns of one full row; 16 consecutive entries per thread.
__device__ __forceinline__ void full_rows_part(const MaskParams& p, int32_t* __restrict__ col_idx,
                                               int64_t row, int64_t chunk) {
  int32_t* out = col_idx + row_offset(p, row);
  const int64_t base = chunk * 4096;
#pragma unroll
  for (int u = 0; u < 16; ++u) {
    const int64_t j = base + u * 256 + threadIdx.x;
    if (j < p.L) out[j] = (int32_t)j;
  }
}

// The whole mask -> CSR pass in one launch: workgroups [0, n_rp) write row_ptr, the next n_fill
// write the column runs of the ordinary rows, the rest the full rows (chunks_per_row workgroups
// each).  The three parts do not depend on each other.
__global__ __launch_bounds__(256) void build_mask_kernel(MaskParams p, int64_t* __restrict__ row_ptr,
                                                         int32_t* __restrict__ col_idx, uint32_t n_rp,
                                                         uint32_t n_fill, uint32_t chunks_per_row) {
  __shared__ Segment seg_all[4][kMaxSegments];
  __shared__ int n_seg_all[4];
  __shared__ int64_t picks_all[4][kMaxRandom];
  const uint32_t bid = blockIdx.x;
  if (bid < n_rp) {
    row_ptr_part(p, row_ptr, bid);
  } else if (bid < n_rp + n_fill) {
    fill_part(p, col_idx, bid - n_rp, seg_all, n_seg_all, picks_all);
  } else {
    const uint32_t idx = bid - n_rp - n_fill;
    full_rows_part(p, col_idx, idx / chunks_per_row, idx % chunks_per_row);
  }
}

}  // namespace

sga_status mask_validate(const sga_mask_desc* d) {
  if (!d) return SGA_ERR_INVALID_ARG;
  if (d->struct_bytes != sizeof(sga_mask_desc)) return SGA_ERR_INVALID_ARG;
  if (d->L < 1 || d->L >= (int64_t(1) << 31)) return SGA_ERR_INVALID_ARG;
  if (d->window < 0) return SGA_ERR_INVALID_ARG;
  switch (d->kind) {
    case SGA_MASK_SLIDING:
      return SGA_OK;
    case SGA_MASK_DILATED:
      return d->stride >= 1 ? SGA_OK : SGA_ERR_INVALID_ARG;
    case SGA_MASK_GLOBAL_LOCAL:
    case SGA_MASK_NONLOCAL:
      return d->n_global >= 0 ? SGA_OK : SGA_ERR_INVALID_ARG;
    case SGA_MASK_DILATED_2D:
      return d->block >= 1 && d->stride >= 1 ? SGA_OK : SGA_ERR_INVALID_ARG;
    case SGA_MASK_BIGBIRD: {
      if (d->block < 1 || d->block > 1024 || d->L % d->block != 0) return SGA_ERR_INVALID_ARG;
      if (d->window_blocks < 0 || d->n_global_blocks < 0) return SGA_ERR_INVALID_ARG;
      if (d->n_random_blocks < 0 || d->n_random_blocks > kMaxRandom) return SGA_ERR_INVALID_ARG;
      const int64_t nb = d->L / d->block;
      const int64_t need = 2 * (int64_t)d->window_blocks + 1 + d->n_global_blocks + d->n_random_blocks;
      return nb >= need ? SGA_OK : SGA_ERR_INVALID_ARG;
    }
    default:
      return SGA_ERR_INVALID_ARG;
  }
}

namespace {

constexpr unsigned long long kNoBadRow = ~0ull;

// verdict[0]: smallest bad row found in the row offsets, verdict[1]: in the columns.
__global__ void validate_init_kernel(unsigned long long* verdict) {
  verdict[0] = kNoBadRow;
  verdict[1] = kNoBadRow;
}

// One thread per row offset: row_ptr[0] = 0, no offset below its predecessor, the last one
// within the column array.  A violation of the first or the last kind is reported as row L.
__global__ __launch_bounds__(256) void validate_rows_kernel(const int64_t* __restrict__ row_ptr, int64_t L,
                                                            int64_t col_capacity, unsigned long long* verdict) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i > L) return;
  if (i == L) {
    if (row_ptr[0] != 0 || row_ptr[L] < 0 || row_ptr[L] > col_capacity) atomicMin(verdict, (unsigned long long)L);
    return;
  }
  if (row_ptr[i] < 0 || row_ptr[i] > row_ptr[i + 1]) atomicMin(verdict, (unsigned long long)i);
}

// The row of edge e: the last row whose offset is <= e (rows without edges share an offset
// with the row after them, and the last of them owns the edge).
__device__ __forceinline__ int64_t row_of_edge(const int64_t* __restrict__ row_ptr, int64_t L, int64_t e) {
  int64_t lo = 0, hi = L;                 // row_ptr[lo] <= e < row_ptr[hi]
  while (hi - lo > 1) {
    const int64_t mid = lo + ((hi - lo) >> 1);
    if (row_ptr[mid] <= e) lo = mid; else hi = mid;
  }
  return lo;
}

// One thread per edge (grid-stride): the column lies in [0, L) and, unless the edge is the
// first of its row, above the column before it.  Only an edge that fails the second test looks
// its row up (about once per row: where the next row starts further left).  Runs only if the
// row offsets passed, so every index it forms lies inside the arrays.
__global__ __launch_bounds__(256) void validate_cols_kernel(const int64_t* __restrict__ row_ptr,
                                                            const int32_t* __restrict__ col_idx, int64_t L,
                                                            unsigned long long* verdict) {
  if (verdict[0] != kNoBadRow) return;    // (written by the launch before this one only)
  const int64_t nnz = row_ptr[L];
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < nnz; e += (int64_t)gridDim.x * blockDim.x) {
    const int32_t c = col_idx[e];
    const bool outside = c < 0 || c >= L;
    const bool descends = e > 0 && c <= col_idx[e - 1];
    if (outside || descends) {
      const int64_t r = row_of_edge(row_ptr, L, e);
      if (outside || row_ptr[r] != e) atomicMin(verdict + 1, (unsigned long long)r);
    }
  }
}

}  // namespace

sga_status launch_validate_csr(const int64_t* row_ptr, const int32_t* col_idx, int64_t L, int64_t col_capacity,
                               unsigned long long* verdict, hipStream_t stream) {
  hipLaunchKernelGGL(validate_init_kernel, dim3(1), dim3(1), 0, stream, verdict);
  hipLaunchKernelGGL(validate_rows_kernel, dim3((unsigned)((L + 1 + 255) / 256)), dim3(256), 0, stream, row_ptr, L,
                     col_capacity, verdict);
  int64_t wgs = (col_capacity + 255) / 256;
  if (wgs > 16384) wgs = 16384;
  if (wgs < 1) wgs = 1;
  hipLaunchKernelGGL(validate_cols_kernel, dim3((unsigned)wgs), dim3(256), 0, stream, row_ptr, col_idx, L, verdict);
  return hip_status(hipGetLastError());
}

int64_t mask_total_edges(const sga_mask_desc& d) {
  const MaskParams p = make_params(d);
  return row_offset(p, p.L);
}

sga_status launch_build_mask(const sga_mask_desc& d, int64_t* row_ptr, int32_t* col_idx,
                             hipStream_t stream) {
  const MaskParams p = make_params(d);
  const int64_t n_rp = (p.L + 1 + 255) / 256;
  const int64_t groups = (p.L + group_rows(p) - 1) / group_rows(p);
  const int64_t n_fill = (groups + 3) / 4;
  const int64_t n_full = full_rows(p) < p.L ? full_rows(p) : p.L;
  const int64_t chunks = (p.L + 4095) / 4096;
  const int64_t total = n_rp + n_fill + n_full * chunks;
  if (total >= (int64_t(1) << 31)) return SGA_ERR_OVERFLOW;   // (more than 2^31 workgroups: L^2 / 4096 full-row chunks)
  hipLaunchKernelGGL(build_mask_kernel, dim3((unsigned)total), dim3(256), 0, stream, p, row_ptr, col_idx,
                     (uint32_t)n_rp, (uint32_t)n_fill, (uint32_t)(chunks > 0 ? chunks : 1));
  return hip_status(hipGetLastError());
}

}  // namespace sga
