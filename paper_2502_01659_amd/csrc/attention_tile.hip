// Tile path of Algorithm 1: 32 query rows x 32 keys per MFMA tile.
//
// The graph is regrouped into a "tile graph": for every tile of 32 consecutive query rows,
// the sorted list of 32-key blocks that hold at least one of its edges, each with a 32x32
// bit mask (word r, bit j = edge between row 32t+r and key 32b+j).  Explicit CSR masks are
// converted on the device by tile_analyze_kernel into workspace slots derived from row_ptr
// alone (no scan, no host round trip); window masks generate the same lists by index
// arithmetic inside the attention kernel (implicit Get_Neighbors).
//
// One wavefront owns one tile and walks its block list.  Per block it computes, on the
// matrix cores,
//     S^T[key][query] = K_blk Q_tile^T                       (SDDMM restricted to the block)
//     O^T[chan][query] += V_blk^T P^T                        (SpMM)
// with the online-softmax recurrence of Algorithm 1 applied per block instead of per key.
// Both products are laid out transposed so that a lane always owns one query (lane % 32):
// the running max m, the running sum l, the rescale factor and the mask word of a query
// live in that query's lanes and no cross-lane traffic is needed except one exchange
// between the two half-waves per block.  Entries outside the mask are set to -inf before
// the softmax, so they contribute exactly 0; blocks whose 1024 bits are all set skip the
// masking.
//
// fp32 storage uses v_mfma_f32_32x32x2_f32 (true fp32 products), fp16 storage uses
// v_mfma_f32_32x32x16_f16 with fp32 accumulation; P is rounded to fp16 only as the MFMA
// operand, l is summed in fp32.
//
// Tiles with many edges (global-token rows) are cut into segments of their key-block span;
// each segment is one more work item of the same launches, leaves a partial (m, l, acc)
// state, and tile_merge_kernel combines the partials in segment order (deterministic).
// Window masks on short sequences (few tiles, many key blocks each) are cut the same way by a
// host rule, into ranges of key blocks whose partial states window_merge_kernel combines.
#include "sga_internal.h"

#include <type_traits>

namespace sga {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kMinusHuge = -1.0e30f;
constexpr int kFullBit = 1 << 30;
constexpr int kBitmapBlocks = 32;   // key blocks per window of the CSR -> tile pass's bitmap walk
constexpr int kBitmapAfter = 4;     // ... which takes over after this many blocks if all but one had scattered columns
constexpr int kBitmapUnits = 2;     // ... each lane taking this many units of 16 columns at a time

// Key (within a 32-key block) held in accumulator register r of half-wave h after an
// MFMA 32x32 whose M index is the key: rows 8*(r/4) + 4*h + r%4.
__device__ __forceinline__ constexpr int acc_row(int r, int h) { return 8 * (r / 4) + 4 * h + (r % 4); }

// Global -> LDS copy of 16 bytes per lane without passing through registers: lane l's 16 bytes
// land at dst + 16*l (dst is wave-uniform).  Completion is tracked by vmcnt.
__device__ __forceinline__ void copy16_to_lds(const void* src, char* dst) {
  __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)src,
                                   (void __attribute__((address_space(3)))*)dst, 16, 0, 0);
}
// The same copy issued behind the compiler's back.  While it knows of copies in flight, the
// compiler waits for all of them before any LDS read it cannot prove to be elsewhere; the
// caller of this one orders the reads itself, by counted waits.
__device__ __forceinline__ void copy16_to_lds_untracked(const void* src, char* dst) {
  const uint32_t at = __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(char __attribute__((address_space(3)))*)dst);
  uint32_t m0_kept;    // (M0 holds the LDS address of the copy; the compiler's own value is put back)
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\t"
               "s_mov_b32 m0, %0"
               : "=&s"(m0_kept) : "s"(at), "v"(src) : "memory");
}
// Same with 4 bytes per lane: lane l's word lands at dst + 4*l.
__device__ __forceinline__ void copy4_to_lds(const void* src, char* dst) {
  __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)src,
                                   (void __attribute__((address_space(3)))*)dst, 4, 0, 0);
}

// s_waitcnt vmcnt(N): all but the N most recently issued vector memory operations (global
// loads, LDS copies included) have completed.  The 6-bit count sits in bits 3:0 and 15:14.
template <int N>
__device__ __forceinline__ void wait_loads_except() {
  static_assert(N >= 0 && N <= 63, "vmcnt immediate");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// Wait ahead of the reads of a staged V block: with further copies behind it (more), all but
// the kKeepMore most recently issued vector memory operations must have completed; without, all
// of them.  kKeepMore = -1: the block is known to be complete, no wait.
template <int kKeepMore>
__device__ __forceinline__ void wait_staged_v(bool more) {
  static_assert(kKeepMore >= -1 && kKeepMore <= 63, "a count the vmcnt field can hold, or -1");
  if constexpr (kKeepMore >= 0) {
    if (more) wait_loads_except<kKeepMore>(); else wait_loads_except<0>();
  }
}

// K-ready wait of the LDS pipelines: the K copies of block k are older than the kCopies V copies
// and, if a block record was requested after them, its kGetLoads loads.
template <int kCopies, int kGetLoads>
__device__ __forceinline__ void wait_k_block(bool record_requested) {
  if (kGetLoads > 0 && record_requested) wait_loads_except<kCopies + kGetLoads>();
  else wait_loads_except<kCopies>();
}

// The value held by the lane 32 positions away (the same query in the other half-wave), by the
// gfx950 half-wave swap: one vector instruction instead of a round trip through the LDS
// permute network.  h = lane / 32.
__device__ __forceinline__ float other_half(float x, int h) {
  const unsigned xi = __builtin_bit_cast(unsigned, x);
  const auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  return __builtin_bit_cast(float, h ? r[0] : r[1]);
}

// s_waitcnt lgkmcnt(0): every LDS read issued so far has returned its data.
__device__ __forceinline__ void wait_lds_reads() { __builtin_amdgcn_s_waitcnt(0xC07F); }

// K/V pipelines of the tile kernels (template parameter kPipe).
constexpr int kPipeRegK = 0;   // K fragment prefetched into registers, V block staged in LDS
constexpr int kPipeLdsK = 1;   // K and V blocks staged in LDS, one block ahead
constexpr int kPipeSplit = 2;  // fp32 storage, products as three fp16 matrix-core terms (CoreSplit)

struct BlockInfo {   // (no padding bytes: copies of the struct stay in registers)
  int64_t row0;     // tensor row of the block's first key (wave-uniform)
  int raw;          // explicit masks: block record as loaded (row0, nvalid, full follow from it)
  int nvalid;       // keys of the block that exist (1..32); others are masked off (wave-uniform)
  uint32_t word;    // mask bits of this lane's query against the block's 32 keys
  int full;         // non-zero: all 32x32 bits set (wave-uniform)
};

__device__ __forceinline__ int64_t uniform64(int64_t v) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
  return (int64_t)(((uint64_t)hi << 32) | lo);
}

// Block list of an explicit tile, as written by tile_analyze_kernel.
struct ExplicitBlocks {
  const int32_t* blk;
  const uint32_t* mask;
  int64_t L;
  static constexpr int kGetLoads = 2;   // vector memory loads issued by one get()
  __device__ int64_t key_stride() const { return 1; }
  // get() only issues the loads (two blocks ahead of their use); resolve() turns the loaded
  // record into wave-uniform values once the block is about to be staged, so that the loads are
  // not waited for early.
  __device__ BlockInfo get(int k, int n) const {
    BlockInfo b;
    b.raw = blk[k];
    b.word = mask[(int64_t)k * kTile + n];
    return b;
  }
  __device__ void resolve(BlockInfo& b) const {
    const int id = __builtin_amdgcn_readfirstlane(b.raw);
    b.full = (id & kFullBit) != 0;
    b.row0 = (int64_t)(id & ~kFullBit) * kTile;
    const int64_t left = L - b.row0;
    b.nvalid = left < kTile ? (int)left : kTile;
  }
  // resolve() for a block that is not the last of its list: lists ascend, so only the last
  // block of a list can be the one the end of the sequence cuts short.
  __device__ void resolve_whole(BlockInfo& b) const {
    const int id = __builtin_amdgcn_readfirstlane(b.raw);
    b.full = (id & kFullBit) != 0;
    b.row0 = (int64_t)(id & ~kFullBit) * kTile;
    b.nvalid = kTile;
  }
  // Block k without its mask word, read through the scalar (constant) path: the list is only
  // written by an earlier kernel, and a scalar load neither occupies a vector register nor counts
  // among the vector memory operations, so the pipelines' counted waits stay exact.
  // (like get(), this only issues the load; resolve() completes the record)
  __device__ BlockInfo block(int k) const {
    BlockInfo b;
    b.raw = ((const int32_t __attribute__((address_space(4)))*)blk)[k];
    b.word = ~0u;
    return b;
  }
};

// Block list of a window tile in one residue class p of stride s: queries u0..u0+31 and keys
// v of the class (token = s*index + p), edge iff |u - v| <= W.  Everything but the lane's mask
// word is wave-uniform and is computed from differences that fit 32 bits.
struct WindowBlocks {
  int64_t vfirst, Lc, s, p, u0, W;   // blocks start at the tile's first key, not at multiples of 32
  static constexpr int kGetLoads = 0;
  __device__ int64_t key_stride() const { return s; }
  __device__ static int clamp64(int64_t v) { return v < -64 ? -64 : (v > 64 ? 64 : (int)v); }
  __device__ void resolve(BlockInfo&) const {}
  // Where block k lies (wave-uniform; no mask word): what the staging needs.
  __device__ BlockInfo place(int k) const {
    BlockInfo b;
    b.raw = 0;
    const int64_t v0 = vfirst + (int64_t)k * kTile;
    b.row0 = s * v0 + p;
    const int64_t left = Lc - v0;
    b.nvalid = left < kTile ? (int)left : kTile;
    b.word = 0;
    b.full = 0;
    return b;
  }
  // Block k against the tile's queries, from wave-uniform quantities alone: 0 = no query of the
  // tile sees a key of the block, 2 = every query sees every key, 1 = anything else (get() then
  // gives the lanes' mask words).  Interior blocks of a wide window are all 2 and cost no
  // per-lane arithmetic.
  __device__ int classify(int k) const {
    const int64_t v0 = vfirst + (int64_t)k * kTile;
    const int64_t left = Lc - v0, nq = Lc - u0;
    const int64_t dlo = u0 - W - v0, dhi = u0 + W - v0;
    if (left <= 0 || nq <= 0 || dhi + (kTile - 1) < 0 || dlo > kTile - 1) return 0;
    return left >= kTile && nq >= kTile && dlo + (kTile - 1) <= 0 && dhi >= kTile - 1 ? 2 : 1;
  }
  __device__ BlockInfo get(int k, int n) const {
    BlockInfo b;
    b.raw = 0;
    const int64_t v0 = vfirst + (int64_t)k * kTile;
    b.row0 = s * v0 + p;
    const int64_t left = Lc - v0;
    b.nvalid = left < kTile ? (int)left : kTile;
    // query n sees the keys [n + dlo, n + dhi] of the block, clipped to the keys that exist
    const int dlo = clamp64(u0 - W - v0), dhi = clamp64(u0 + W - v0);
    const int nq = clamp64(Lc - u0);               // queries of the tile that exist
    int lo = n + dlo, hi = n + dhi;
    lo = lo < 0 ? 0 : lo;
    hi = hi > b.nvalid - 1 ? b.nvalid - 1 : hi;
    b.word = (lo > hi || n >= nq) ? 0u : ((~0u >> (31 - hi)) & (~0u << lo));
    // every query of the tile sees every key of the block
    b.full = b.nvalid == kTile && nq >= kTile && dlo + (kTile - 1) <= 0 && dhi >= kTile - 1;
    return b;
  }
};

// The mask words of WindowBlocks for a tile whose keys all lie within a few hundred positions of
// its first key (the workgroup-staged kernel): the same quantities as 32-bit differences, so the
// per-block arithmetic runs on the scalar unit.  d0 = u0 - vfirst, rem = min(Lc - vfirst, 2^20),
// nq = queries of the tile that exist (clamped to 64), W <= 64.
struct WindowWordsNear {
  int d0, W, nq, rem;
  __device__ static int clamp(int v) { return v < -64 ? -64 : (v > 64 ? 64 : v); }
  __device__ BlockInfo get(int k, int n) const {
    BlockInfo b;
    b.raw = 0;
    b.row0 = 0;                                    // (not used: the blocks are staged by the workgroup)
    const int v0 = k * kTile;                      // first key of the block, relative to vfirst
    const int left = rem - v0;
    b.nvalid = left < kTile ? left : kTile;
    const int dlo = clamp(d0 - W - v0), dhi = clamp(d0 + W - v0);
    int lo = n + dlo, hi = n + dhi;
    lo = lo < 0 ? 0 : lo;
    hi = hi > b.nvalid - 1 ? b.nvalid - 1 : hi;
    b.word = (lo > hi || n >= nq) ? 0u : ((~0u >> (31 - hi)) & (~0u << lo));
    b.full = b.nvalid == kTile && nq >= kTile && dlo + (kTile - 1) <= 0 && dhi >= kTile - 1;
    return b;
  }
};

// Per-lane running state: lane owns query n = lane % 32; channels of O^T are spread over the
// 16 accumulator registers of both 32-channel halves.
struct TileState {
  float m;          // running max (log2 domain), identical in both half-waves
  float l;          // running sum of this half-wave's keys
  floatx16 o[2];    // o[cb][r]: channel cb*32 + acc_row(r, h), un-normalised
  __device__ void init() {
    m = kMinusHuge;
    l = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) { o[0][r] = 0.f; o[1][r] = 0.f; }
  }
};

// The running max m of Algorithm 1 only has to bound the scores for the exponentials to stay
// finite, so it is raised lazily: a block moves m (and rescales l and O) only when its largest
// score exceeds m by more than kRescaleSlack (log2 units).  Softmax numerators are then at most
// 2^kRescaleSlack, well inside fp16/fp32 range, and the quotient acc/l is unchanged.
constexpr float kRescaleSlack = 8.0f;

// c = |scale| * log2(e) of p = 2^(c*s - m).  A zero scale (uniform weights over the neighbours)
// is replaced by 2^-100: every finite product then scales to 0 within rounding, while the -inf of
// a masked entry stays -inf instead of turning into 0 * inf.
__device__ __forceinline__ float softmax_factor(float scale) {
  const float c = __builtin_fabsf(scale) * kLog2e;
  return c > 0.f ? c : 7.888609052210118e-31f;
}

// Mask, running max/sum update and (rare) rescale for one block.  sv: raw dot products of this
// lane's query with keys acc_row(r, h); c > 0 is scale * log2(e) (a negative scale is folded
// into the sign of Q by the caller), so the block maximum can be taken over the raw products
// and the scaling fused into the exponent: p = 2^(c*s - m).
__device__ __forceinline__ void softmax_block(floatx16 sv, float c, const BlockInfo& b, int h,
                                              TileState& st, float (&p)[16],
                                              floatx16* o_low = nullptr) {
  float bm = -INFINITY;
  if (!b.full) {
    const uint32_t wh = b.word >> (4 * h);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      // all-ones where the edge exists, else zero; then select the product or -inf bitwise
      const int keep = ((int)(wh << (31 - acc_row(r, 0)))) >> 31;
      const float x = sv[r];   // (a bit cast applied to the vector element itself reads element 0)
      const int bits = (__builtin_bit_cast(int, x) & keep) | ((int)0xff800000 & ~keep);
      sv[r] = __builtin_bit_cast(float, bits);
    }
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) bm = fmaxf(bm, sv[r]);
  bm = fmaxf(bm, other_half(bm, h)) * c;
  if (__any(bm > st.m + kRescaleSlack)) {
    const float m_new = bm > st.m + kRescaleSlack ? bm : st.m;
    const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);
    st.m = m_new;
    st.l *= alpha;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      st.o[0][r] *= alpha;
      st.o[1][r] *= alpha;
    }
    if (o_low) {       // low-order accumulators of the split-precision core
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        o_low[0][r] *= alpha;
        o_low[1][r] *= alpha;
      }
    }
  }
  float lsum = 0.f;
  const float neg_m = -st.m;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    p[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[r], c, neg_m));
    lsum += p[r];
  }
  st.l += lsum;
}

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float2v __attribute__((ext_vector_type(2)));

// softmax_block for fp16 storage, in three steps that callers with two independent sub-tiles
// interleave.  The numerators leave as the B operand of the PV products: rounded to fp16 two at a
// time (one packed conversion per pair, to nearest even), ph[u][e] = p of accumulator register
// 8u + e.  The running sum adds the *rounded* numerators (a dot product of each pair with (1, 1),
// accumulated in fp32), i.e. exactly the weights the products apply, so that acc / l is a true
// weighted mean of V rows.
//
// Entries outside the mask become -inf (word: mask bits of this lane's query).
__device__ __forceinline__ void mask_scores(floatx16& sv, uint32_t word, int h) {
  const uint32_t wh = word >> (4 * h);
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    // all-ones where the edge exists, else zero; then select the product or -inf bitwise
    const int keep = ((int)(wh << (31 - acc_row(r, 0)))) >> 31;
    const float x = sv[r];   // (a bit cast applied to the vector element itself reads element 0)
    const int bits = (__builtin_bit_cast(int, x) & keep) | ((int)0xff800000 & ~keep);
    sv[r] = __builtin_bit_cast(float, bits);
  }
}
// Largest scaled score of this lane's query in the block (both half-waves agree).
__device__ __forceinline__ float block_max(const floatx16& sv, float c, int h) {
  float bm = fmaxf(sv[0], sv[1]);
#pragma unroll
  for (int r = 2; r < 16; r += 2) bm = __builtin_fmaxf(__builtin_fmaxf(bm, sv[r]), sv[r + 1]);
  return fmaxf(bm, other_half(bm, h)) * c;
}
__device__ __forceinline__ bool needs_rescale(const TileState& st, float bm) {
  return bm > st.m + kRescaleSlack;
}
// Raises m to bm where bm exceeds it by more than the slack, and rescales l and O (a factor of
// exactly 1 elsewhere).
__device__ __forceinline__ void rescale_state(TileState& st, float bm) {
  const float m_new = needs_rescale(st, bm) ? bm : st.m;
  const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);
  st.m = m_new;
  st.l *= alpha;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    st.o[0][r] *= alpha;
    st.o[1][r] *= alpha;
  }
}
__device__ __forceinline__ void numerators_h(const floatx16& sv, float c, TileState& st, half8 (&ph)[2]) {
  const float neg_m = -st.m;
  const half2v ones = {(_Float16)1.0f, (_Float16)1.0f};
  float l = st.l;
#pragma unroll
  for (int r = 0; r < 16; r += 2) {
    const float2v p2 = {__builtin_amdgcn_exp2f(__builtin_fmaf(sv[r], c, neg_m)),
                        __builtin_amdgcn_exp2f(__builtin_fmaf(sv[r + 1], c, neg_m))};
    const half2v hp = __builtin_convertvector(p2, half2v);
    l = __builtin_amdgcn_fdot2(hp, ones, l, false);
    ph[r / 8][r % 8] = hp[0];
    ph[r / 8][r % 8 + 1] = hp[1];
  }
  st.l = l;
}
// The running max of fp16 tiles is raised on demand: the numerators are first taken against the
// m the state already has, and only if one of them leaves the fp16 range (it rounds to +inf, and
// so does the sum it enters; the first block of a tile, whose m is still the initial one, always
// does) is the block's maximum computed, m raised and the numerators taken again.  A numerator is
// then at most 2^16 instead of 2^kRescaleSlack, which fp16 holds at the same relative precision,
// and the common block pays neither for the maximum nor for waiting on it.
constexpr float kSumOverflow = 3.0e38f;
__device__ __forceinline__ bool sum_overflowed(const TileState& st) { return !(st.l < kSumOverflow); }
__device__ __forceinline__ void softmax_block_h(floatx16 sv, float c, bool full, uint32_t word, int h,
                                                TileState& st, half8 (&ph)[2]) {
  if (!full) mask_scores(sv, word, h);
  const float l_before = st.l;
  numerators_h(sv, c, st, ph);
  if (__any(sum_overflowed(st))) {
    st.l = l_before;
    rescale_state(st, block_max(sv, c, h));
    numerators_h(sv, c, st, ph);
  }
}
// The same for two sub-tiles whose blocks are both unmasked, as one stretch of code with one
// (rare) branch.
__device__ __forceinline__ void softmax_pair_h(const floatx16& s_a, const floatx16& s_b, float c, int h,
                                               TileState& sta, TileState& stb, half8 (&pha)[2],
                                               half8 (&phb)[2]) {
  const float la = sta.l, lb = stb.l;
  numerators_h(s_a, c, sta, pha);
  numerators_h(s_b, c, stb, phb);
  if (__any(sum_overflowed(sta) || sum_overflowed(stb))) {
    sta.l = la;
    stb.l = lb;
    rescale_state(sta, block_max(s_a, c, h));
    rescale_state(stb, block_max(s_b, c, h));
    numerators_h(s_a, c, sta, pha);
    numerators_h(s_b, c, stb, phb);
  }
}

// Source addresses of the global -> LDS block copies.  A block's rows are row0 + j*stride
// (j = 0..31); copy i of a block moves kRows consecutive keys, kLanes lanes of 16 bytes per
// row.  The per-lane part of the address is fixed for a whole work item (32-bit byte offsets
// from the block's first row); the per-block part is wave-uniform, so a copy costs no vector
// arithmetic.  Blocks cut short by the end of the sequence (nvalid < 32) re-read their last
// row instead of running past it; those keys are masked off.
//
// kD is the row length of the tensors in global memory; a block always holds 64 channels of a
// key (for kD > 64 the caller passes tensor pointers already advanced to its 64-channel slice).
template <typename T, int kD = kHeadDim>
struct StageMap {
  static constexpr int kRowBytes = kHeadDim * (int)sizeof(T);   // staged row (one 64-channel slice)
  static constexpr int kGlobalRowBytes = kD * (int)sizeof(T);   // tensor row
  static constexpr int kLanes = kRowBytes / 16;          // lanes per row
  static constexpr int kRows = kWave / kLanes;           // rows per copy
  static constexpr int kCopies = kTile / kRows;          // copies per block
  int64_t stride_bytes;                                  // bytes between consecutive keys
  uint32_t voff;                                         // V: lane's row and 16-byte chunk
  uint32_t koff[kLanes / 4 > 1 ? 4 : 1];                 // K: same with the chunk swizzled, per copy % 4

  __device__ void init(int64_t stride, int lane) {
    stride_bytes = stride * kGlobalRowBytes;
    const int lr = lane / kLanes, lc = lane % kLanes;
    const uint32_t rowoff = (uint32_t)(lr * stride_bytes);
    voff = rowoff + lc * 16;
    // chunk c of key r is stored at chunk slot c ^ (r % kLanes): the copy reads the chunk that
    // belongs into the slot this lane writes
    if (kLanes == 8) {
      koff[0] = rowoff + ((lc ^ lr) * 16);               // (8i + lr) % 8 = lr for every copy i
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) koff[i] = rowoff + ((lc ^ ((4 * i + lr) & 15)) * 16);
    }
  }
  // (a block all of whose 32 keys exist)
  __device__ void stage_v_whole(const T* __restrict__ Vh, int64_t row0, char* dst) const {
    const char* base = reinterpret_cast<const char*>(Vh) + row0 * kGlobalRowBytes;
#pragma unroll
    for (int i = 0; i < kCopies; ++i) copy16_to_lds(base + i * kRows * stride_bytes + voff, dst + i * 1024);
  }
  __device__ void stage_k_whole(const T* __restrict__ Kh, int64_t row0, char* dst) const {
    const char* base = reinterpret_cast<const char*>(Kh) + row0 * kGlobalRowBytes;
#pragma unroll
    for (int i = 0; i < kCopies; ++i)
      copy16_to_lds(base + i * kRows * stride_bytes + koff[kLanes == 8 ? 0 : i % 4], dst + i * 1024);
  }
  __device__ void stage_v(const T* __restrict__ Vh, const BlockInfo& b, int lane, char* dst) const {
    if (b.nvalid == kTile) {
      stage_v_whole(Vh, b.row0, dst);
    } else {
#pragma unroll
      for (int i = 0; i < kCopies; ++i) {
        int key = kRows * i + lane / kLanes;
        key = key < b.nvalid ? key : b.nvalid - 1;
        copy16_to_lds(reinterpret_cast<const char*>(Vh) + b.row0 * kGlobalRowBytes + key * stride_bytes +
                          (lane % kLanes) * 16,
                      dst + i * 1024);
      }
    }
  }
  __device__ void stage_k(const T* __restrict__ Kh, const BlockInfo& b, int lane, char* dst) const {
    if (b.nvalid == kTile) {
      stage_k_whole(Kh, b.row0, dst);
    } else {
#pragma unroll
      for (int i = 0; i < kCopies; ++i) {
        const int row = kRows * i + lane / kLanes;
        const int key = row < b.nvalid ? row : b.nvalid - 1;
        const int chunk = (lane % kLanes) ^ (row % kLanes);
        copy16_to_lds(reinterpret_cast<const char*>(Kh) + b.row0 * kGlobalRowBytes + key * stride_bytes +
                          chunk * 16,
                      dst + i * 1024);
      }
    }
  }
};

// Head dimensions above 64: the kD / 64 wavefronts of a workgroup own one tile together, each
// with one 64-channel slice of Q, K, V and O.  The products S^T = K Q^T of the slices are partial
// sums over the channels; every wavefront leaves its 32x32 partial in LDS and, after one
// workgroup barrier, all of them add the partials in slice order, so that every wavefront
// continues with bit-identical scores (and therefore identical m, l and P).  Two buffers
// alternate, which makes one barrier per block enough: a wavefront overwrites a buffer only
// after the barrier that every reader of its previous contents has passed.
template <int kD>
struct SliceExchange {
  static constexpr int kSlices = kD / kHeadDim;
  static constexpr int kBytes = 2 * kSlices * 4096;   // [2][slice][4][64 lanes] float4
  float4* xs;      // the workgroup's exchange buffers
  int slice;       // this wavefront's slice
  int parity;
  __device__ void init(char* lds, int slice_) {
    xs = reinterpret_cast<float4*>(lds);
    slice = slice_;
    parity = 0;
  }
  __device__ void sum_slices(floatx16& s, int lane) {
    float4* buf = xs + parity * (kSlices * 256);
    parity ^= 1;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      buf[(slice * 4 + j) * 64 + lane] = make_float4(s[4 * j], s[4 * j + 1], s[4 * j + 2], s[4 * j + 3]);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float4 t = buf[j * 64 + lane];
#pragma unroll
      for (int w = 1; w < kSlices; ++w) {
        const float4 v = buf[(w * 4 + j) * 64 + lane];
        t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w;
      }
      s[4 * j] = t.x; s[4 * j + 1] = t.y; s[4 * j + 2] = t.z; s[4 * j + 3] = t.w;
    }
  }
};

// ---- fp32 storage ---------------------------------------------------------------------------
template <int kD>
struct CoreF32T {
  using Stage = StageMap<float, kD>;
  float qf[32];   // Q[query n][h*32 + t] (of this wavefront's 64-channel slice)
  SliceExchange<kD> xchg;   // used for kD > 64 only

  __device__ void load_q(const float* Qrow, int h, bool negate) {
    const float4* src = reinterpret_cast<const float4*>(Qrow + h * 32);
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const float4 v = src[t];
      qf[4 * t] = v.x; qf[4 * t + 1] = v.y; qf[4 * t + 2] = v.z; qf[4 * t + 3] = v.w;
    }
    if (negate) {
#pragma unroll
      for (int t = 0; t < 32; ++t) qf[t] = -qf[t];
    }
  }

  // kf[t] = K[key n of the block][h*32 + t], straight from global memory: 128 contiguous bytes
  // per lane, i.e. kFragLoads loads of 16 bytes (the widest load there is; the counted waits of
  // run_regk rely on this number).  lane_off = byte offset of the lane's key row and half inside
  // a whole block.
  static constexpr int kFragLoads = 32 * (int)sizeof(float) / 16;
  __device__ static void load_k(const float* __restrict__ Kh, const BlockInfo& b, int64_t stride_bytes,
                                uint32_t lane_off, int n, int h, float (&kf)[32]) {
    const char* base = reinterpret_cast<const char*>(Kh) + b.row0 * Stage::kGlobalRowBytes;
    const float4* kp;
    if (b.nvalid == kTile) {
      kp = reinterpret_cast<const float4*>(base + lane_off);
    } else {
      const int krow = n < b.nvalid ? n : b.nvalid - 1;
      kp = reinterpret_cast<const float4*>(base + krow * stride_bytes + h * 128);
    }
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const float4 v = kp[t];
      kf[4 * t] = v.x; kf[4 * t + 1] = v.y; kf[4 * t + 2] = v.z; kf[4 * t + 3] = v.w;
    }
  }

  static constexpr int kBlockBytes = kTile * kHeadDim * 4;   // one staged K or V block

  // kf[t] = K[key n][h*32 + t] out of the staged block.  The global -> LDS copy moved keys
  // 4i..4i+3 per instruction, 16 lanes per 256-byte row (whole cache lines), and stored the
  // sixteen 16-byte chunks of a row XOR-swizzled: chunk c of key r lives at chunk slot
  // c ^ (r & 15).  This read (each lane 128 contiguous bytes of its own key row, 16 at a time)
  // then spreads 8 consecutive lanes over the 8 groups of 4 banks instead of hitting one.
  __device__ static void read_k(const char* ldsk, int n, int h, float (&kf)[32]) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int slot = (8 * h + j) ^ (n & 15);
      const float4 v = *reinterpret_cast<const float4*>(ldsk + (n * 16 + slot) * 16);
      kf[4 * j] = v.x; kf[4 * j + 1] = v.y; kf[4 * j + 2] = v.z; kf[4 * j + 3] = v.w;
    }
  }

  // S^T = K_blk Q^T, softmax, O^T += V_blk^T P^T for one block whose V rows are staged at ldsv.
  // (kKeepMore, more: see wait_staged_v)
  template <int kKeepMore>
  __device__ void block_math(const float (&kf)[32], const BlockInfo& b, float c, int n, int h,
                             TileState& st, const char* ldsv, bool more) {
    floatx16 s = {0};
#pragma unroll
    for (int t = 0; t < 32; ++t)
      s = __builtin_amdgcn_mfma_f32_32x32x2f32(kf[t], qf[t], s, 0, 0, 0);
    if (kD > kHeadDim) xchg.sum_slices(s, 32 * h + n);
    float p[16];
    softmax_block(s, c, b, h, st, p);
    wait_staged_v<kKeepMore>(more);
    __builtin_amdgcn_wave_barrier();
    const float* vread = reinterpret_cast<const float*>(ldsv) + h * 4 * kHeadDim + n;
    if (b.full) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        // A operand: V^T[channel cb*32+n][key acc_row(r,h)] = staged V[key][channel]
        const float v0 = vread[acc_row(r, 0) * kHeadDim];
        const float v1 = vread[acc_row(r, 0) * kHeadDim + 32];
        st.o[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(v0, p[r], st.o[0], 0, 0, 0);
        st.o[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(v1, p[r], st.o[1], 0, 0, 0);
      }
    } else {
      // A masked block: registers 4g..4g+3 hold the keys 8g..8g+7 of the block; a group of keys
      // that no query of the tile attends (p = 0 in every lane) is skipped, which is exact
      // (e.g. the upper half of a block that holds 16 global tokens).
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        if (__builtin_amdgcn_ballot_w64(((b.word >> (8 * g)) & 0xffu) != 0) == 0) continue;
#pragma unroll
        for (int r = 4 * g; r < 4 * g + 4; ++r) {
          const float v0 = vread[acc_row(r, 0) * kHeadDim];
          const float v1 = vread[acc_row(r, 0) * kHeadDim + 32];
          st.o[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(v0, p[r], st.o[0], 0, 0, 0);
          st.o[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(v1, p[r], st.o[1], 0, 0, 0);
        }
      }
    }
  }

  // Variant with the K block staged in LDS (many blocks per tile).  Both K and V blocks travel
  // global -> LDS without registers, as whole rows (coalesced).  Per block k: the V copy is
  // issued first; the K fragment (copied during block k-1) is read into registers and the K
  // copy of block k+1 is issued at once, so it lands behind the matrix work of block k; block
  // ids / mask words are fetched two blocks ahead.
  template <typename Src>
  __device__ void run_ldsk(const float* __restrict__ Kh, const float* __restrict__ Vh, const Src& src,
                      int k0, int k1, float c, int lane, TileState& st, char* lds) {
    if (k0 >= k1) return;
    const int n = lane & 31, h = lane >> 5;
    Stage sm;
    sm.init(src.key_stride(), lane);
    char* ldsk = lds;
    char* ldsv = lds + kBlockBytes;
    BlockInfo b = src.get(k0, n);
    BlockInfo b1 = src.get(k0 + 1 < k1 ? k0 + 1 : k0, n);
    src.resolve(b);
    __builtin_amdgcn_wave_barrier();     // reads of both buffers by an earlier work item are done
    sm.stage_k(Kh, b, lane, ldsk);
    for (int k = k0; k < k1; ++k) {
      const bool more = k + 1 < k1;      // wave-uniform
      src.resolve(b1);
      __builtin_amdgcn_wave_barrier();   // the previous block's reads of the staged V are done
      sm.stage_v(Vh, b, lane, ldsv);
      BlockInfo b2 = b1;
      if (k + 2 < k1) b2 = src.get(k + 2, n);
      wait_k_block<8, Src::kGetLoads>(k + 2 < k1);   // K block k: older than the V copies (and the record loads)
      __builtin_amdgcn_wave_barrier();
      float kf[32];
      read_k(ldsk, n, h, kf);
      wait_lds_reads();                  // the K buffer may be overwritten now
      __builtin_amdgcn_wave_barrier();
      if (more) sm.stage_k(Kh, b1, lane, ldsk);
      // V block k is older than the 8 K copies issued above (if any)
      block_math<8>(kf, b, c, n, h, st, ldsv, more);
      b = b1;
      b1 = b2;
    }
  }

  // Variant with the K fragment in registers (few blocks per tile): the K fragment of block k+1 is
  // prefetched global -> registers (each lane reads 128 contiguous bytes of its key row), the V
  // block k is copied global -> LDS behind the S^T matrix work, and block ids / mask words are
  // fetched two blocks ahead, so no load sits on the critical path of the matrix cores.  The
  // loop is unrolled over two fragment buffers, so the prefetched fragment is never copied.
  template <typename Src>
  __device__ void run_regk(const float* __restrict__ Kh, const float* __restrict__ Vh, const Src& src,
                      int k0, int k1, float c, int lane, TileState& st, char* lds) {
    if (k0 >= k1) return;
    const int n = lane & 31, h = lane >> 5;
    Stage sm;
    sm.init(src.key_stride(), lane);
    const uint32_t klane = (uint32_t)(n * sm.stride_bytes) + h * 128;
    BlockInfo b = src.get(k0, n);
    BlockInfo b1 = src.get(k0 + 1 < k1 ? k0 + 1 : k0, n);
    src.resolve(b);
    float kfa[32], kfb[32];
    load_k(Kh, b, sm.stride_bytes, klane, n, h, kfa);
    auto step = [&](int k, float (&kf)[32], float (&kf_next)[32]) {
      src.resolve(b1);
      if (k + 1 < k1) load_k(Kh, b1, sm.stride_bytes, klane, n, h, kf_next);
      __builtin_amdgcn_wave_barrier();   // the previous block's reads of the staged V are done
      sm.stage_v(Vh, b, lane, lds);
      BlockInfo b2 = b1;
      if (k + 2 < k1) b2 = src.get(k + 2, n);
      block_math<0>(kf, b, c, n, h, st, lds, false);
      b = b1;
      b1 = b2;
    };
    for (int k = k0; k < k1; k += 2) {
      step(k, kfa, kfb);
      if (k + 1 >= k1) break;
      step(k + 1, kfb, kfa);
    }
  }

  // Explicit block lists: as run_regk, with the block ids read through the scalar path and the
  // mask words of block k+1 copied global -> LDS while block k is computed (two 256-byte slots
  // behind the V block), as in CoreF16T::run_ldsk.  The only loads into vector registers are the
  // K fragments, and the step's own waits are counted: V block k, then the words of block k+1,
  // then the K fragment of block k+1 are issued in this order, so the fragment may still be in
  // flight during the PV products.  (Workload 2, measured side by side: 4 % faster than with the records loaded
  // into vector registers two blocks ahead.)
  __device__ void run_regk(const float* __restrict__ Kh, const float* __restrict__ Vh,
                           const ExplicitBlocks& src, int k0, int k1, float c, int lane, TileState& st,
                           char* lds) {
    if (k0 >= k1) return;
    const int n = lane & 31, h = lane >> 5;
    Stage sm;
    sm.init(1, lane);
    const uint32_t klane = (uint32_t)(n * sm.stride_bytes) + h * 128;
    char* ldsw = lds + kBlockBytes;              // two slots of 64 mask words (both half-waves)
    const uint32_t* wsrc = src.mask + n;         // this lane's word of block k: wsrc[32 k]
    BlockInfo b = src.block(k0);
    BlockInfo b1 = src.block(k0 + 1 < k1 ? k0 + 1 : k0);
    src.resolve(b);
    __builtin_amdgcn_wave_barrier();     // reads of the buffers by an earlier work item are done
    copy4_to_lds(wsrc + (int64_t)k0 * kTile, ldsw + (k0 & 1) * 256);
    float kfa[32], kfb[32];
    load_k(Kh, b, sm.stride_bytes, klane, n, h, kfa);
    auto step = [&](int k, float (&kf)[32], float (&kf_next)[32]) {
      const bool more = k + 1 < k1;      // wave-uniform
      src.resolve(b1);
      __builtin_amdgcn_wave_barrier();   // the previous block's reads of V and of the other word slot are done
      sm.stage_v(Vh, b, lane, lds);
      if (more) {
        copy4_to_lds(wsrc + (int64_t)(k + 1) * kTile, ldsw + ((k + 1) & 1) * 256);
        load_k(Kh, b1, sm.stride_bytes, klane, n, h, kf_next);
      }
      BlockInfo b2 = b1;
      if (k + 2 < k1) b2 = src.block(k + 2);
      // the words and the K fragment of block k are older than the operations above: the V copies
      // and, if a block follows, its word copy and fragment loads
      if (more) wait_loads_except<Stage::kCopies + 1 + kFragLoads>(); else wait_loads_except<Stage::kCopies>();
      __builtin_amdgcn_wave_barrier();
      b.word = *reinterpret_cast<const uint32_t*>(ldsw + (k & 1) * 256 + lane * 4);
      // V block k is older than the word copy and the fragment loads (if any)
      block_math<1 + kFragLoads>(kf, b, c, n, h, st, lds, more);
      b = b1;
      b1 = b2;
    };
    for (int k = k0; k < k1; k += 2) {
      step(k, kfa, kfb);
      if (k + 1 >= k1) break;
      step(k + 1, kfb, kfa);
    }
  }

  // kLdsK selects the pipeline: K block staged in LDS (coalesced whole-row copies; best with many
  // blocks per tile) or K fragment loaded straight into registers (no LDS round trip before the
  // first product; best with two or three blocks per tile).
  template <int kPipe>
  static constexpr int lds_bytes() { return kPipe == kPipeRegK ? kBlockBytes + 512 : 2 * kBlockBytes; }

  template <int kPipe, typename Src>
  __device__ void run(const float* __restrict__ Kh, const float* __restrict__ Vh, const Src& src,
                      int k0, int k1, float c, int lane, TileState& st, char* lds) {
    static_assert(kPipe == kPipeRegK || kPipe == kPipeLdsK, "fp32 pipelines");
    if (kPipe == kPipeLdsK) run_ldsk(Kh, Vh, src, k0, k1, c, lane, st, lds);
    else run_regk(Kh, Vh, src, k0, k1, c, lane, st, lds);
  }

  // Orow = acc * inv, or w_prev * Orow + acc * inv when the call continues an earlier state.
  __device__ static void store_row(float* Orow, const TileState& st, float inv, float w_prev,
                                   bool accumulate, int h) {
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float4* dst = reinterpret_cast<float4*>(Orow + cb * 32 + 8 * g + 4 * h);
        float4 v = make_float4(st.o[cb][4 * g] * inv, st.o[cb][4 * g + 1] * inv,
                               st.o[cb][4 * g + 2] * inv, st.o[cb][4 * g + 3] * inv);
        if (accumulate) {
          const float4 old = *dst;
          v.x = __builtin_fmaf(w_prev, old.x, v.x);
          v.y = __builtin_fmaf(w_prev, old.y, v.y);
          v.z = __builtin_fmaf(w_prev, old.z, v.z);
          v.w = __builtin_fmaf(w_prev, old.w, v.w);
        }
        *dst = v;
      }
  }

  // (Direct row stores: 32 bytes per row and instruction from the two half-waves.  Sending the
  // tile through LDS to store whole rows, as CoreF16T::store_tile does, changes nothing here.)
  static constexpr bool kTileStore = false;
};
using CoreF32 = CoreF32T<kHeadDim>;

// ---- fp16 storage ---------------------------------------------------------------------------
template <int kD>
struct CoreF16T {
  using Stage = StageMap<__half, kD>;
  half8 qf[4];    // Q[query n][h*32 + 8s .. +7], s = 0..3 (of this wavefront's 64-channel slice)
  SliceExchange<kD> xchg;   // used for kD > 64 only

  __device__ void load_q(const __half* Qrow, int h, bool negate) {
    const half8* src = reinterpret_cast<const half8*>(Qrow + h * 32);
#pragma unroll
    for (int s = 0; s < 4; ++s) qf[s] = src[s];
    if (negate) {
#pragma unroll
      for (int s = 0; s < 4; ++s) qf[s] = -qf[s];
    }
  }

  // The loads of load_q have completed (the caller has waited for them): taking qf as read and
  // written here keeps the compiler from waiting for them again at their first use, where
  // copies issued in between would be waited for as well.
  __device__ void q_arrived() {
#pragma unroll
    for (int s = 0; s < 4; ++s) asm volatile("" : "+v"(qf[s]));
  }

  static constexpr int kBlockBytes = kTile * kHeadDim * 2;   // one staged K or V block

  // kf[s] = K[key n][h*32 + 8s .. +7] out of the staged block: keys 8i..8i+7 per copy, 8 lanes
  // per 128-byte row, the eight 16-byte chunks of a row XOR-swizzled with the row index (see
  // CoreF32::read_k) so that these reads are free of bank conflicts.
  __device__ static void read_k(const char* ldsk, int n, int h, half8 (&kf)[4]) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int slot = (4 * h + s) ^ (n & 7);
      kf[s] = *reinterpret_cast<const half8*>(ldsk + (n * 8 + slot) * 16);
    }
  }

  // 4 keys x 1 channel per lane out of the row-major staged V block, using the LDS transpose
  // read of gfx950: inside a 16-lane group, lane i receives element (i % 4) of the 8 bytes
  // addressed by lanes i/4, 4 + i/4, 8 + i/4 and 12 + i/4.  Lane i therefore addresses key
  // (key0 + i/4) at channels 4*(i%4).. of its group's 16 channels, and ends up with channel i of
  // the group for keys key0..key0+3: the K-contiguous A operand of V^T.
  __device__ static half4 read_vt(const char* p) {
    const short4v raw =
        __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)p);
    return __builtin_bit_cast(half4, raw);
  }

  // (kKeepMore, more: see wait_staged_v)
  template <int kKeepMore>
  __device__ void block_math(const half8 (&kf)[4], const BlockInfo& b, float c, int lane, int h,
                             TileState& st, const char* ldsv, bool more) {
    half8 ph[2];
    scores(kf, b, c, lane, h, st, ph);
    wait_staged_v<kKeepMore>(more);
    __builtin_amdgcn_wave_barrier();
    accumulate(ph, lane, h, st, ldsv);
  }

  // First half of the block step: S^T = K_blk Q^T and the softmax update; ph = numerators as the
  // B operand of the PV products.
  __device__ void scores(const half8 (&kf)[4], const BlockInfo& b, float c, int lane, int h,
                         TileState& st, half8 (&ph)[2]) {
    floatx16 sacc = {0};
#pragma unroll
    for (int s = 0; s < 4; ++s)
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[s], qf[s], sacc, 0, 0, 0);
    if (kD > kHeadDim) xchg.sum_slices(sacc, lane);
    softmax_block_h(sacc, c, b.full != 0, b.word, h, st, ph);
  }

  // This lane's address of the V^T operand reads for key0 = 4h, channel group 0; the other reads
  // are constant offsets from it.
  __device__ static const char* vt_base(const char* ldsv, int lane, int h) {
    const int i = lane & 15, grp16 = (lane >> 4) & 1;
    return ldsv + (4 * h + (i >> 2)) * (kHeadDim * 2) + (grp16 * 16 + 4 * (i & 3)) * 2;
  }

  // A operand of one PV product: V^T[channel cb*32+n][slot (u,h,e)], slot key = 16u + 8(e/4) + 4h + e%4
  __device__ static half8 read_va(const char* vt, int u, int cb) {
    const half4 lo = read_vt(vt + (16 * u) * (kHeadDim * 2) + cb * 64);
    const half4 hi = read_vt(vt + (16 * u + 8) * (kHeadDim * 2) + cb * 64);
    return half8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  }

  // Second half: O^T += V_blk^T P^T with the V block staged (complete) at ldsv.
  __device__ static void accumulate(const half8 (&ph)[2], int lane, int h, TileState& st,
                                    const char* ldsv) {
    const char* vt = vt_base(ldsv, lane, h);
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
        st.o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(read_va(vt, u, cb), ph[u], st.o[cb], 0, 0, 0);
  }

  // Same pipeline as CoreF32::run_ldsk.
  template <typename Src>
  __device__ void run_ldsk(const __half* __restrict__ Kh, const __half* __restrict__ Vh, const Src& src,
                      int k0, int k1, float c, int lane, TileState& st, char* lds) {
    if (k0 >= k1) return;
    const int n = lane & 31, h = lane >> 5;
    Stage sm;
    sm.init(src.key_stride(), lane);
    char* ldsk = lds;
    char* ldsv = lds + kBlockBytes;
    BlockInfo b = src.get(k0, n);
    BlockInfo b1 = src.get(k0 + 1 < k1 ? k0 + 1 : k0, n);
    src.resolve(b);
    __builtin_amdgcn_wave_barrier();     // reads of both buffers by an earlier work item are done
    sm.stage_k(Kh, b, lane, ldsk);
    for (int k = k0; k < k1; ++k) {
      const bool more = k + 1 < k1;      // wave-uniform
      src.resolve(b1);
      __builtin_amdgcn_wave_barrier();   // the previous block's reads of the staged V are done
      sm.stage_v(Vh, b, lane, ldsv);
      BlockInfo b2 = b1;
      if (k + 2 < k1) b2 = src.get(k + 2, n);
      wait_k_block<4, Src::kGetLoads>(k + 2 < k1);   // K block k: older than the V copies (and the record loads)
      __builtin_amdgcn_wave_barrier();
      half8 kf[4];
      read_k(ldsk, n, h, kf);
      wait_lds_reads();                  // the K buffer may be overwritten now
      __builtin_amdgcn_wave_barrier();
      if (more) sm.stage_k(Kh, b1, lane, ldsk);
      // V block k (and any record load after it) is older than the 4 K copies issued above (if any)
      block_math<4>(kf, b, c, lane, h, st, ldsv, more);
      b = b1;
      b1 = b2;
    }
  }

  // Explicit block lists: as run_ldsk, with no vector load into registers inside the loop.  Block
  // ids come through the scalar path (ExplicitBlocks::block), and the 32 mask words of block k+1
  // are copied global -> LDS (one 4-byte copy per lane into one of two 256-byte slots) while block
  // k is computed.  Every vector memory operation of the loop is then an LDS copy whose
  // completion only the counted waits below ask for; a register load carried around the loop
  // would make the compiler drain all of them, the prefetched K block included, once per block.
  __device__ void run_ldsk(const __half* __restrict__ Kh, const __half* __restrict__ Vh,
                           const ExplicitBlocks& src, int k0, int k1, float c, int lane, TileState& st,
                           char* lds) {
    if (k0 >= k1) return;
    const int n = lane & 31, h = lane >> 5;
    Stage sm;
    sm.init(1, lane);
    char* ldsk = lds;
    char* ldsv = lds + kBlockBytes;
    char* ldsw = lds + 2 * kBlockBytes;          // two slots of 64 mask words (both half-waves)
    const uint32_t* wsrc = src.mask + n;         // this lane's word of block k: wsrc[32 k]
    BlockInfo b = src.block(k0);
    BlockInfo b1 = src.block(k0 + 1 < k1 ? k0 + 1 : k0);
    src.resolve(b);
    __builtin_amdgcn_wave_barrier();     // reads of the buffers by an earlier work item are done
    copy4_to_lds(wsrc + (int64_t)k0 * kTile, ldsw + (k0 & 1) * 256);
    sm.stage_k(Kh, b, lane, ldsk);
    // One block step.  kInner: blocks k+1 and k+2 exist and blocks k and k+1 are whole (true up
    // to the list's last two blocks), which leaves no branch on the position in the list and
    // none on a block cut short by the end of the sequence.
    auto step = [&](int k, auto inner) {
      constexpr bool kInner = decltype(inner)::value;
      const bool more = kInner || k + 1 < k1;      // wave-uniform
      if (kInner) src.resolve_whole(b1); else src.resolve(b1);
      __builtin_amdgcn_wave_barrier();   // the previous block's reads of V and of the other word slot are done
      if (more) copy4_to_lds(wsrc + (int64_t)(k + 1) * kTile, ldsw + ((k + 1) & 1) * 256);
      if (kInner) sm.stage_v_whole(Vh, b.row0, ldsv); else sm.stage_v(Vh, b, lane, ldsv);
      BlockInfo b2 = b1;
      if (kInner || k + 2 < k1) b2 = src.block(k + 2);
      // K block k and the words of block k are older than the copies issued in this step
      if (more) wait_loads_except<5>(); else wait_loads_except<4>();
      __builtin_amdgcn_wave_barrier();
      half8 kf[4];
      read_k(ldsk, n, h, kf);
      b.word = *reinterpret_cast<const uint32_t*>(ldsw + (k & 1) * 256 + lane * 4);
      wait_lds_reads();                  // the K buffer may be overwritten now
      __builtin_amdgcn_wave_barrier();
      if (kInner) sm.stage_k_whole(Kh, b1.row0, ldsk); else if (more) sm.stage_k(Kh, b1, lane, ldsk);
      half8 ph[2];
      scores(kf, b, c, lane, h, st, ph);
      // V block k (and the words of block k+1) are older than the 4 K copies issued above (if any)
      if (more) wait_loads_except<4>(); else wait_loads_except<0>();
      __builtin_amdgcn_wave_barrier();
      accumulate(ph, lane, h, st, ldsv);
      b = b1;
      b1 = b2;
    };
    int k = k0;
    for (; k + 2 < k1; ++k) step(k, std::true_type{});
    for (; k < k1; ++k) step(k, std::false_type{});
  }

  template <int kPipe>
  static constexpr int lds_bytes() { return 2 * kBlockBytes + 512; }

  template <int kPipe, typename Src>
  __device__ void run(const __half* __restrict__ Kh, const __half* __restrict__ Vh, const Src& src,
                      int k0, int k1, float c, int lane, TileState& st, char* lds) {
    static_assert(kPipe == kPipeLdsK, "fp16 pipeline");
    run_ldsk(Kh, Vh, src, k0, k1, c, lane, st, lds);
  }

  __device__ static void store_row(__half* Orow, const TileState& st, float inv, float w_prev,
                                   bool accumulate, int h) {
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2* dst = reinterpret_cast<uint2*>(Orow + cb * 32 + 8 * g + 4 * h);
        float v[4] = {st.o[cb][4 * g] * inv, st.o[cb][4 * g + 1] * inv, st.o[cb][4 * g + 2] * inv,
                      st.o[cb][4 * g + 3] * inv};
        if (accumulate) {
          const uint2 old = *dst;
          const __half2 o01 = __builtin_bit_cast(__half2, old.x), o23 = __builtin_bit_cast(__half2, old.y);
          v[0] = __builtin_fmaf(w_prev, __low2float(o01), v[0]);
          v[1] = __builtin_fmaf(w_prev, __high2float(o01), v[1]);
          v[2] = __builtin_fmaf(w_prev, __low2float(o23), v[2]);
          v[3] = __builtin_fmaf(w_prev, __high2float(o23), v[3]);
        }
        uint2 w;
        w.x = __builtin_bit_cast(uint32_t, __floats2half2_rn(v[0], v[1]));
        w.y = __builtin_bit_cast(uint32_t, __floats2half2_rn(v[2], v[3]));
        *dst = w;
      }
  }

  // The whole tile, normalised, in row order: tensor rows row0 + r * row_step, r < n_rows.
  // A lane holds fragments of its own query's row, so store_row touches 32 rows with 16 bytes
  // each per instruction, eight times; here the tile goes through the wavefront's LDS instead
  // (rows kTilePitch bytes apart, which spreads the writes over the banks) and leaves as whole
  // 128-byte rows, eight per instruction.  lds = kTileBytes bytes no copy is in flight to.
  // (Workloads 3, 4 and 5: 8 to 10 % off the kernel time.)
  static constexpr bool kTileStore = true;
  static constexpr int kTilePitch = 64 * 2 + 16;
  static constexpr int kTileBytes = kTile * kTilePitch;
  __device__ static void store_tile(__half* Oh, int64_t row0, int64_t row_step, int n_rows,
                                    const TileState& st, float inv, int lane, char* lds) {
    const int n = lane & 31, h = lane >> 5;
    __builtin_amdgcn_wave_barrier();     // the last block's reads of the staged blocks are done
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w;
        w.x = __builtin_bit_cast(uint32_t, __floats2half2_rn(st.o[cb][4 * g] * inv, st.o[cb][4 * g + 1] * inv));
        w.y = __builtin_bit_cast(uint32_t,
                                 __floats2half2_rn(st.o[cb][4 * g + 2] * inv, st.o[cb][4 * g + 3] * inv));
        *reinterpret_cast<uint2*>(lds + n * kTilePitch + (cb * 32 + 8 * g + 4 * h) * 2) = w;
      }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = (lane >> 3) + 8 * i;
      const uint4 v = *reinterpret_cast<const uint4*>(lds + r * kTilePitch + (lane & 7) * 16);
      if (r < n_rows)
        // (written once and not read again by this call: a streaming store keeps the L2 for K and V)
        __builtin_nontemporal_store(__builtin_bit_cast(half8, v),
                                    reinterpret_cast<half8*>(Oh + (row0 + r * row_step) * kHeadDim + (lane & 7) * 8));
    }
  }
};
using CoreF16 = CoreF16T<kHeadDim>;

// ---- fp32 storage, split-precision products -----------------------------------------------------
// Every fp32 operand x is written as hi + lo with hi = fp16(x) and lo = fp16(x - hi) (x - hi is
// exact in fp32), and a product a.b is evaluated as hi_a.hi_b + hi_a.lo_b + lo_a.hi_b on the
// fp16 matrix cores, all three terms into the same fp32 accumulator.  The dropped term
// lo_a.lo_b and the rounding of lo are below 2^-22 |a.b|, the size of an fp32 rounding error,
// so results match the true-fp32 kernels to their tolerance while the matrix work drops from
// 64 fp32 MFMAs (4096 cycles) to 24 fp16 MFMAs (768 cycles) per block.  lo is a subnormal fp16
// number for |x| < 0.25 (the matrix cores do not flush them); below |x| ~ 2^-13 it loses bits,
// an absolute error of at most 2^-25 per operand.  Inputs must lie inside the fp16 range
// (|x| < 65504); the caller opts in (SGA_PATH_TILE_SPLIT).
// K and V blocks travel global -> LDS as raw fp32 (as in CoreF32::run_ldsk); K is split when
// its fragment is read, V is split in registers and written back over its own staged block as
// two row-major fp16 blocks, which the PV products read with the LDS transpose read.
struct CoreSplit {
  using Stage = StageMap<float>;
  static constexpr int kBlockBytes = kTile * kHeadDim * 4;
  half8 qh[4], ql[4];   // Q[query n][h*32 + 8s .. +7], high and low parts

  typedef _Float16 half2v __attribute__((ext_vector_type(2)));

  // Two values at a time: hi = fp16(x) packed into one register, x - hi by the mixed-precision
  // fma (the fp16 operand is read straight out of the packed pair, no conversion back), and the
  // remainders packed again: four instructions per pair.
  __device__ static void split2(float x0, float x1, half2v& hi, half2v& lo) {
    hi = half2v{(_Float16)x0, (_Float16)x1};
    const uint32_t hp = __builtin_bit_cast(uint32_t, hi);
    float r0, r1;
    asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel_hi:[1,0,0]" : "=v"(r0) : "v"(hp), "v"(x0));
    asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r1) : "v"(hp), "v"(x1));
    lo = half2v{(_Float16)r0, (_Float16)r1};
  }

  __device__ static void split8(const float* x, half8& hi, half8& lo) {
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      half2v h2, l2;
      split2(x[e], x[e + 1], h2, l2);
      hi[e] = h2[0]; hi[e + 1] = h2[1];
      lo[e] = l2[0]; lo[e + 1] = l2[1];
    }
  }

  __device__ void load_q(const float* Qrow, int h, bool negate) {
    float q[32];
    const float4* src = reinterpret_cast<const float4*>(Qrow + h * 32);
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const float4 v = src[t];
      q[4 * t] = v.x; q[4 * t + 1] = v.y; q[4 * t + 2] = v.z; q[4 * t + 3] = v.w;
    }
    if (negate) {
#pragma unroll
      for (int t = 0; t < 32; ++t) q[t] = -q[t];
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) split8(q + 8 * s, qh[s], ql[s]);
  }

  template <int kPipe>
  static constexpr int lds_bytes() { return 2 * kBlockBytes; }

  template <int kPipe, typename Src>
  __device__ void run(const float* __restrict__ Kh, const float* __restrict__ Vh, const Src& src,
                      int k0, int k1, float c, int lane, TileState& st, char* lds) {
    if (k0 >= k1) return;
    const int n = lane & 31, h = lane >> 5;
    Stage sm;
    sm.init(src.key_stride(), lane);
    char* ldsk = lds;
    char* ldsv = lds + kBlockBytes;
    BlockInfo b = src.get(k0, n);
    BlockInfo b1 = src.get(k0 + 1 < k1 ? k0 + 1 : k0, n);
    src.resolve(b);
    __builtin_amdgcn_wave_barrier();     // reads of both buffers by an earlier work item are done
    sm.stage_k(Kh, b, lane, ldsk);
    // this lane's part of the row-major staged V block: copy i moved 16 bytes to dst + i*1024 + lane*16
    const int lr = lane >> 4, lc = lane & 15;
    const int i16 = lane & 15, grp16 = (lane >> 4) & 1;
    const char* vt = ldsv + (4 * h + (i16 >> 2)) * (kHeadDim * 2) + (grp16 * 16 + 4 * (i16 & 3)) * 2;
    for (int k = k0; k < k1; ++k) {
      const bool more = k + 1 < k1;      // wave-uniform
      src.resolve(b1);
      __builtin_amdgcn_wave_barrier();   // the previous block's reads of the V buffer are done
      sm.stage_v(Vh, b, lane, ldsv);
      BlockInfo b2 = b1;
      if (k + 2 < k1) b2 = src.get(k + 2, n);
      wait_k_block<8, Src::kGetLoads>(k + 2 < k1);   // K block k: older than the V copies (and the record loads)
      __builtin_amdgcn_wave_barrier();
      half8 kh[4], kl[4];
      {
        float kf[32];
        CoreF32::read_k(ldsk, n, h, kf);
        wait_lds_reads();                // the K buffer may be overwritten now
        __builtin_amdgcn_wave_barrier();
        if (more) sm.stage_k(Kh, b1, lane, ldsk);
#pragma unroll
        for (int s = 0; s < 4; ++s) split8(kf + 8 * s, kh[s], kl[s]);
      }
      floatx16 sacc = {0};
#pragma unroll
      for (int s = 0; s < 4; ++s) {     // smallest terms first
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_f16(kl[s], qh[s], sacc, 0, 0, 0);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_f16(kh[s], ql[s], sacc, 0, 0, 0);
      }
#pragma unroll
      for (int s = 0; s < 4; ++s)
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_f16(kh[s], qh[s], sacc, 0, 0, 0);
      float p[16];
      softmax_block(sacc, c, b, h, st, p);
      // V block k (and any record load after it) is older than the 8 K copies issued above (if any)
      if (more) wait_loads_except<8>(); else wait_loads_except<0>();
      b = b1;
      b1 = b2;
      __builtin_amdgcn_wave_barrier();
      {
        // split the staged fp32 V block in place: rows 4i + lr, channels 4*lc .. +3 per copy i
        float vraw[32];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float4 v = *reinterpret_cast<const float4*>(ldsv + i * 1024 + lane * 16);
          vraw[4 * i] = v.x; vraw[4 * i + 1] = v.y; vraw[4 * i + 2] = v.z; vraw[4 * i + 3] = v.w;
        }
        wait_lds_reads();
        __builtin_amdgcn_wave_barrier();   // every lane holds its part: the block may be overwritten
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          half4 vh, vl;
#pragma unroll
          for (int e = 0; e < 4; e += 2) {
            half2v h2, l2;
            split2(vraw[4 * i + e], vraw[4 * i + e + 1], h2, l2);
            vh[e] = h2[0]; vh[e + 1] = h2[1];
            vl[e] = l2[0]; vl[e + 1] = l2[1];
          }
          char* row = ldsv + (4 * i + lr) * (kHeadDim * 2) + lc * 8;
          *reinterpret_cast<half4*>(row) = vh;
          *reinterpret_cast<half4*>(row + kTile * kHeadDim * 2) = vl;
        }
        __builtin_amdgcn_s_waitcnt(0xC07F);   // LDS writes have landed
        __builtin_amdgcn_wave_barrier();
      }
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        half8 ph, pl;
        split8(p + 8 * u, ph, pl);
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
          const char* a0 = vt + (16 * u) * (kHeadDim * 2) + cb * 64;
          const half4 hlo = CoreF16::read_vt(a0), hhi = CoreF16::read_vt(a0 + 8 * (kHeadDim * 2));
          const half4 llo = CoreF16::read_vt(a0 + kTile * kHeadDim * 2);
          const half4 lhi = CoreF16::read_vt(a0 + kTile * kHeadDim * 2 + 8 * (kHeadDim * 2));
          const half8 vh = {hlo[0], hlo[1], hlo[2], hlo[3], hhi[0], hhi[1], hhi[2], hhi[3]};
          const half8 vl = {llo[0], llo[1], llo[2], llo[3], lhi[0], lhi[1], lhi[2], lhi[3]};
          st.o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vl, ph, st.o[cb], 0, 0, 0);
          st.o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vh, pl, st.o[cb], 0, 0, 0);
          st.o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vh, ph, st.o[cb], 0, 0, 0);
        }
      }
    }
  }

  __device__ static void store_row(float* Orow, const TileState& st, float inv, float w_prev,
                                   bool accumulate, int h) {
    CoreF32::store_row(Orow, st, inv, w_prev, accumulate, h);
  }
};

template <typename T> struct CoreOf;
template <> struct CoreOf<float> { using type = CoreF32; };
template <> struct CoreOf<__half> { using type = CoreF16; };
// the core that runs pipeline kPipe on storage type T
template <typename T, int kPipe> struct CoreFor { using type = typename CoreOf<T>::type; };
template <> struct CoreFor<float, kPipeSplit> { using type = CoreSplit; };
// the core of a 64-channel slice of kD-wide rows
template <typename T, int kD> struct WideCoreOf;
template <int kD> struct WideCoreOf<float, kD> { using type = CoreF32T<kD>; };
template <int kD> struct WideCoreOf<__half, kD> { using type = CoreF16T<kD>; };

// Normalise and store the tile's rows (row(n) = tensor row of query n, < 0 if it does not exist).
template <typename T>
__device__ __forceinline__ void finish_tile(T* Oh, float* lse_h, int64_t row, int64_t lse_idx,
                                            bool exists, TileState& st, int h, bool accumulate) {
  const float l = st.l + other_half(st.l, h);
  if (!exists) return;
  const bool empty = !(l > 0.f);
  float inv = empty ? 0.f : 1.0f / l;
  float lse_row = empty ? -INFINITY : (st.m + __builtin_amdgcn_logf(l)) * kLn2;
  float w_prev = 0.f;
  if (accumulate) {    // both half-waves read the earlier lse before half-wave 0 replaces it
    const CarryWeights cw = carry_weights(lse_h[lse_idx], lse_row);
    inv *= cw.w_now;
    w_prev = cw.w_prev;
    lse_row = cw.lse;
  }
  CoreOf<T>::type::store_row(Oh + row * kHeadDim, st, inv, w_prev, accumulate, h);
  if (lse_h && h == 0) lse_h[lse_idx] = lse_row;
}

// finish_tile for a call that starts from the initial state, rows row0 + r * row_step with
// r < n_rows existing: the tile leaves in row order through lds (Core::store_tile).
template <typename T>
__device__ __forceinline__ void finish_tile_rows(T* Oh, float* lse_h, int64_t row0, int64_t row_step,
                                                 int n_rows, TileState& st, int lane, char* lds) {
  const int n = lane & 31, h = lane >> 5;
  const float l = st.l + other_half(st.l, h);
  const bool empty = !(l > 0.f);
  const float inv = empty ? 0.f : 1.0f / l;
  CoreOf<T>::type::store_tile(Oh, row0, row_step, n_rows, st, inv, lane, lds);
  if (lse_h && h == 0 && n < n_rows)
    lse_h[row0 + n * row_step] = empty ? -INFINITY : (st.m + __builtin_amdgcn_logf(l)) * kLn2;
}

// Un-normalised partial of a chunk: o[32][64], m[32], l[32].
__device__ __forceinline__ void store_partial(float* part, TileState& st, int n, int h) {
  const float l = st.l + other_half(st.l, h);
#pragma unroll
  for (int cb = 0; cb < 2; ++cb)
#pragma unroll
    for (int g = 0; g < 4; ++g)
      *reinterpret_cast<float4*>(part + n * 64 + cb * 32 + 8 * g + 4 * h) =
          make_float4(st.o[cb][4 * g], st.o[cb][4 * g + 1], st.o[cb][4 * g + 2], st.o[cb][4 * g + 3]);
  if (h == 0) {
    part[kTile * 64 + n] = st.m;
    part[kTile * 64 + kTile + n] = l;
  }
}

// finish_tile for one 64-channel slice of a kD-wide tile (Oslice = first channel of the slice in
// the head's O).  Every slice wavefront holds the same (m, l); when the call continues an earlier
// state, all of them read the earlier lse before the workgroup barrier and slice 0 replaces it
// after it.
template <typename T, int kD>
__device__ __forceinline__ void finish_tile_wide(T* Oslice, float* lse_h, int64_t row, bool exists,
                                                 TileState& st, int h, int slice, bool accumulate) {
  const float l = st.l + other_half(st.l, h);
  const bool empty = !(l > 0.f);
  float inv = empty ? 0.f : 1.0f / l;
  float lse_row = empty ? -INFINITY : (st.m + __builtin_amdgcn_logf(l)) * kLn2;
  float w_prev = 0.f;
  if (accumulate) {
    if (exists) {
      const CarryWeights cw = carry_weights(lse_h[row], lse_row);
      inv *= cw.w_now;
      w_prev = cw.w_prev;
      lse_row = cw.lse;
    }
    __syncthreads();
  }
  if (!exists) return;
  CoreOf<T>::type::store_row(Oslice + row * kD, st, inv, w_prev, accumulate, h);
  if (lse_h && h == 0 && slice == 0) lse_h[row] = lse_row;
}

// Minimum (maximum) of v over lanes 0..31, as a wave-uniform value.  Data-parallel-primitive
// moves inside the 16-lane rows (a running minimum towards lane 15), then lane 15 of row 0 into
// row 1, and lane 31 holds the result: a chain of short vector instructions, where shuffles
// through the LDS crossbar cost a round trip each (this reduction sits in the block loop of the
// CSR -> tile pass, once per key block).
template <int CTRL, int ROWS>
__device__ __forceinline__ int dpp_from(int v) {     // lanes without a source keep v
  return __builtin_amdgcn_update_dpp(v, v, CTRL, ROWS, 0xf, false);
}
__device__ __forceinline__ int first_half_min(int v) {
  int o;
  o = dpp_from<0x111, 0xf>(v); v = o < v ? o : v;    // row_shr:1
  o = dpp_from<0x112, 0xf>(v); v = o < v ? o : v;    // row_shr:2
  o = dpp_from<0x114, 0xf>(v); v = o < v ? o : v;    // row_shr:4
  o = dpp_from<0x118, 0xf>(v); v = o < v ? o : v;    // row_shr:8
  o = dpp_from<0x142, 0xa>(v); v = o < v ? o : v;    // row_bcast:15 into rows 1 and 3
  return __builtin_amdgcn_readlane(v, 31);
}
__device__ __forceinline__ int first_half_max(int v) {
  int o;
  o = dpp_from<0x111, 0xf>(v); v = o > v ? o : v;
  o = dpp_from<0x112, 0xf>(v); v = o > v ? o : v;
  o = dpp_from<0x114, 0xf>(v); v = o > v ? o : v;
  o = dpp_from<0x118, 0xf>(v); v = o > v ? o : v;
  o = dpp_from<0x142, 0xa>(v); v = o > v ? o : v;
  return __builtin_amdgcn_readlane(v, 31);
}

// First position in [lo, hi) of the sorted column list whose column is >= key.
__device__ __forceinline__ int64_t lower_bound_col(const int32_t* __restrict__ col, int64_t lo,
                                                   int64_t hi, int64_t key) {
  while (lo < hi) {
    const int64_t mid = lo + ((hi - lo) >> 1);
    if (col[mid] < key) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// Work item w -> (tile, item index within the tile, segments of the tile).  With S = seg_edges
// and f(t) = t + row_ptr[min(32t, L)] / S, tile t owns the items [f(t), f(t+1)); items with
// index >= segments are idle.
struct WorkId {
  int64_t tile;
  int32_t seg, nseg;
};

// (Called by a whole wavefront with the same w.)  f is increasing, and for masks of even density
// the item index is close to proportional to the tile index: the 64 lanes evaluate f at the 64
// tiles around that guess in one round of loads, and only a guess that misses this window falls
// back to galloping and bisection, one dependent load per step.
__device__ __forceinline__ WorkId locate_work(const int64_t* __restrict__ row_ptr, int64_t L, int sh,
                                              int64_t n_tiles, int64_t n_work, int64_t w, int lane) {
  int64_t g = (int64_t)((double)w * (double)n_tiles / (double)n_work);
  if (g >= n_tiles) g = n_tiles - 1;
  // (the guess errs upwards where rows with many edges come first: most of the window lies below it)
  int64_t base = g - 47;
  if (base + kWave > n_tiles) base = n_tiles - kWave;
  if (base < 0) base = 0;
  const int64_t tc = base + lane;
  const int64_t fc = tc < n_tiles ? work_first(row_ptr, L, sh, tc) : INT64_MAX;
  const uint64_t below = __builtin_amdgcn_ballot_w64(fc <= w);       // a prefix of the lanes
  const int n_below = __builtin_popcountll(below);
  int64_t lo, f0;
  if (n_below > 0 && (n_below < kWave || base + kWave >= n_tiles)) {
    lo = base + n_below - 1;
    f0 = __shfl(fc, n_below - 1, kWave);
  } else {
    int64_t hi;
    if (n_below > 0) {                 // beyond the window
      lo = base + kWave - 1;
      int64_t step = 1;
      hi = n_tiles;
      while (lo + step < n_tiles) {
        if (work_first(row_ptr, L, sh, lo + step) <= w) { lo += step; step <<= 1; }
        else { hi = lo + step; break; }
      }
    } else {                           // before it
      hi = base;
      int64_t step = 1;
      lo = 0;
      while (hi - step > 0) {
        if (work_first(row_ptr, L, sh, hi - step) > w) { hi -= step; step <<= 1; }
        else { lo = hi - step; break; }
      }
    }
    while (hi - lo > 1) {
      const int64_t mid = lo + ((hi - lo) >> 1);
      if (work_first(row_ptr, L, sh, mid) <= w) lo = mid; else hi = mid;
    }
    f0 = work_first(row_ptr, L, sh, lo);
  }
  WorkId id;
  id.tile = lo;
  id.seg = (int32_t)(w - f0);
  id.nseg = tile_segments(row_ptr, L, sh, lo);
  return id;
}

// ---- CSR -> tile graph ------------------------------------------------------------------------
// One wavefront per work item (a tile, or one key-block range of a tile with many edges);
// lane r < 32 walks row 32t + r.  A 32-way merge by key block id: every round takes the
// smallest block id at the head of any row and lets each row consume its columns inside that
// block into a 32-bit word.  A row whose remaining columns are consecutive integers (windows,
// global rows) is walked arithmetically without reading col_idx again; otherwise a run of
// consecutive columns up to the end of the block costs two loads, and only scattered columns
// are read one by one.
__global__ __launch_bounds__(256) void tile_analyze_kernel(const int64_t* __restrict__ row_ptr,
                                                           const int32_t* __restrict__ col_idx,
                                                           int64_t L, int32_t H, int32_t dtype,
                                                           int32_t d, void* ws, size_t ws_bytes) {
  const WorkspacePlan pl = plan_workspace(L, H, row_ptr[L], dtype, d);
  if (pl.total_bytes > ws_bytes) return;
  // per wavefront: the bit words of kBitmapBlocks key blocks, then of the 32 rows the first
  // unit of the window in one numbering, their positions in col_idx (low, high word) and their
  // numbers of columns inside the window
  __shared__ __attribute__((aligned(16))) uint32_t bitmap_all[4][kBitmapBlocks * kTile + 4 * kTile];
  const int lane = threadIdx.x & (kWave - 1);
  const int waves = blockDim.x / kWave;
  uint32_t* bm = bitmap_all[__builtin_amdgcn_readfirstlane(threadIdx.x / kWave)];
  char* base_ws = static_cast<char*>(ws);
  TileItem* items = reinterpret_cast<TileItem*>(base_ws + pl.off_items_rec);
  int32_t* tile_bad = reinterpret_cast<int32_t*>(base_ws + pl.off_tile_bad);
  int32_t* tile_pbase = reinterpret_cast<int32_t*>(base_ws + pl.off_tile_pbase);
  int32_t* pair_blk = reinterpret_cast<int32_t*>(base_ws + pl.off_pair_blk);
  uint32_t* pair_mask = reinterpret_cast<uint32_t*>(base_ws + pl.off_pair_mask);
  uint32_t* ctr = reinterpret_cast<uint32_t*>(ws);
  for (int64_t w = (int64_t)blockIdx.x * waves + threadIdx.x / kWave; w < pl.n_work;
       w += (int64_t)gridDim.x * waves) {
    WorkId id = locate_work(row_ptr, L, pl.seg_shift, pl.n_tiles, pl.n_work, w, lane);
    if (id.seg >= id.nseg) {          // spare item of a tile whose edge range crosses a multiple of S
      if (lane == 0) items[w].tile = -1;
      continue;
    }
    if (id.nseg > 1) {
      // Four neighbouring tiles that are all cut into the same number of segments (rows of global
      // tokens: every tile spans the whole key range) trade segments among their items so that
      // consecutive items hold the same segment of the four tiles.  The items of a workgroup
      // of the static schedule then stream the same K and V blocks at the same time, instead of
      // each tile passing over all keys on its own (workload 4: the four global tiles of a head
      // otherwise fetch K and V four times).  The j-th (tile, segment) pair of the quad in
      // tile-major order computes pair number j in segment-major order: a permutation of the
      // same 4 * nseg pairs, a function of the mask alone.
      const int64_t g = id.tile & ~int64_t(3);
      bool same = g + 3 < pl.n_tiles;
      for (int64_t q = g; same && q < g + 4; ++q) same = tile_segments(row_ptr, L, pl.seg_shift, q) == id.nseg;
      if (same) {
        const int64_t j = (id.tile - g) * id.nseg + id.seg;
        id.tile = g + (j & 3);
        id.seg = (int32_t)(j >> 2);
      }
    }
    const int64_t t = id.tile;
    const int64_t row_first = t * kTile;
    const int64_t row_last = row_first + kTile < L ? row_first + kTile : L;
    const int64_t slot_t = row_ptr[row_first] / kPairEdges;
    const int64_t cap_t = row_ptr[row_last] / kPairEdges - slot_t;
    const int64_t cap = cap_t / id.nseg;
    const int64_t slot0 = slot_t + (int64_t)id.seg * cap;
    const int64_t row = row_first + lane;
    const bool active = lane < kTile && row < L;
    int64_t pos = active ? row_ptr[row] : 0;
    int64_t end = active ? row_ptr[row + 1] : 0;
    if (id.nseg > 1) {
      // this segment's share of the tile's key-block span
      const int first_c = pos < end ? col_idx[pos] : INT32_MAX;
      const int last_c = pos < end ? col_idx[end - 1] : -1;
      const int64_t bmin = first_half_min(first_c) >> 5;
      const int64_t bmax = first_half_max(last_c) >> 5;
      const int64_t span = bmax - bmin + 1;
      const int64_t B0 = bmin + span * id.seg / id.nseg;
      const int64_t B1 = bmin + span * (id.seg + 1) / id.nseg;
      if (pos < end && (int64_t)last_c - first_c == end - 1 - pos) {
        // the row is one run of consecutive columns (global-token rows): its share follows by
        // arithmetic instead of two binary searches over the column list
        const int64_t p0 = pos;
        const int64_t lo = B0 * kTile - first_c, hi = B1 * kTile - first_c;
        pos = p0 + (lo < 0 ? 0 : (lo > end - p0 ? end - p0 : lo));
        end = p0 + (hi < 0 ? 0 : (hi > end - p0 ? end - p0 : hi));
      } else {
        pos = lower_bound_col(col_idx, pos, end, B0 * kTile);
        end = lower_bound_col(col_idx, pos, end, B1 * kTile);
      }
    }
    // a row whose remaining columns are one run of consecutive integers needs no more loads;
    // the test is repeated with every column that starts a round (it costs nothing: the last
    // column is kept), so a row of a few runs turns arithmetic once its last run is reached
    int run_lo = 0, run_hi = -1;
    bool arith = false;
    const int c_last = pos < end ? col_idx[end - 1] : -1;
    int nblk = 0;
    bool overflow = false;
    int consumed = 0;                   // edges of this lane's row in the blocks written so far
    int scattered = 0;                  // blocks so far in which some row's columns were read one by one
    bool by_bitmap = false;
    while (true) {
      int cur = INT32_MAX;
      if (!arith && pos < end) {
        const int c0 = col_idx[pos];
        if ((int64_t)c_last - c0 == end - 1 - pos) {
          arith = true;
          run_lo = c0;
          run_hi = c_last;
          pos = end;
        } else {
          cur = c0 >> 5;
        }
      }
      if (arith) cur = run_lo <= run_hi ? (run_lo >> 5) : INT32_MAX;
      if (__all(arith || pos >= end)) {
        // Every row is down to one run of consecutive columns (or to nothing).  If the runs'
        // block ranges overlap or touch, the remaining blocks are the whole range from the first
        // to the last, and each row's word follows from its run alone: no minimum per block.
        const bool some = arith && run_lo <= run_hi;
        const int blo = first_half_min(some ? run_lo >> 5 : INT32_MAX);
        if (blo == INT32_MAX) break;
        const int bhi = first_half_max(some ? run_hi >> 5 : -1);
        const int lo_max = first_half_max(some ? run_lo >> 5 : -1);
        const int hi_min = first_half_min(some ? run_hi >> 5 : INT32_MAX);
        if (lo_max <= hi_min + 1) {
          for (int b = blo; b <= bhi; ++b) {
            if (nblk >= cap) {
              overflow = true;
              break;
            }
            const int lo = run_lo - (b << 5) > 0 ? run_lo - (b << 5) : 0;
            const int hi = run_hi - (b << 5) < 31 ? run_hi - (b << 5) : 31;
            const uint32_t word = some && lo <= hi ? (~0u >> (31 - hi)) & (~0u << lo) : 0u;
            const bool full = __all(lane >= kTile || word == ~0u);
            if (lane < kTile) pair_mask[(slot0 + nblk) * kTile + lane] = word;
            if (lane == 0) pair_blk[slot0 + nblk] = b | (full ? kFullBit : 0);
            ++nblk;
          }
          break;
        }
      }
      const int b = first_half_min(cur);
      if (b == INT32_MAX) break;
      if (nblk >= cap) {
        overflow = true;
        break;
      }
      uint32_t word = 0;
      bool one_by_one = false;
      if (cur == b) {
        if (arith) {
          const int lo = run_lo & 31;
          const int hi = run_hi < (b << 5) + 31 ? (run_hi & 31) : 31;
          word = (~0u >> (31 - hi)) & (~0u << lo);
          run_lo = (b + 1) << 5;
        } else {
          // if the row's columns run consecutively up to the end of the block (or of the row),
          // one more load settles the whole word: the list is sorted and free of duplicates, so
          // equal ends mean every column in between is present
          const int c0 = col_idx[pos];
          const int lo = c0 & 31;
          const int64_t left = end - pos;
          const int cnt = left < 32 - lo ? (int)left : 32 - lo;
          if (col_idx[pos + cnt - 1] == c0 + cnt - 1) {
            word = (~0u >> (32 - cnt)) << lo;
            pos += cnt;
          } else {
            // the row's columns inside block b are the next entries of its sorted list: take
            // them four per load while four remain, then one by one
            one_by_one = true;
            bool more = true;
            while (more && pos + 4 <= end) {
              int cc[4];
              __builtin_memcpy(cc, col_idx + pos, 16);
#pragma unroll
              for (int t = 0; t < 4; ++t) {
                if (more && (cc[t] >> 5) == b) {
                  word |= 1u << (cc[t] & 31);
                  ++pos;
                } else {
                  more = false;
                }
              }
            }
            while (more && pos < end) {
              const int cc = col_idx[pos];
              if ((cc >> 5) != b) break;
              word |= 1u << (cc & 31);
              ++pos;
            }
          }
        }
      }
      const bool full = __all(lane >= kTile || word == ~0u);
      if (lane < kTile) pair_mask[(slot0 + nblk) * kTile + lane] = word;
      if (lane == 0) pair_blk[slot0 + nblk] = b | (full ? kFullBit : 0);
      ++nblk;
      consumed += __builtin_popcount(word);
      if (__any(one_by_one)) ++scattered;
      // Scattered columns in nearly all of the first blocks: the rest of the list is made by
      // the bitmap walk below (the same blocks and words, from coalesced loads, many in flight,
      // instead of a chain of dependent ones per row).
      if (nblk == kBitmapAfter && scattered >= kBitmapAfter - 1) {
        by_bitmap = true;
        break;
      }
      if (nblk == kProbeBlocks) {
        // A list that averages under kProbeEdges edges per block over its first kProbeBlocks blocks
        // is given up at once (scattered columns: the rows go to the per-row kernels) instead
        // of being walked until its slots run out.  Like the slot rule this depends on the mask
        // alone.
        int total = lane < kTile ? consumed : 0;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) total += __shfl_xor(total, off, kWave);
        if (total < kProbeBlocks * kProbeEdges) {
          overflow = true;
          break;
        }
      }
    }
    if (by_bitmap) {
      // (a row walked arithmetically goes back to its position in the column list)
      if (arith) pos = end - (run_lo <= run_hi ? run_hi - run_lo + 1 : 0);
      uint32_t* first = bm + kBitmapBlocks * kTile;
      uint32_t* at_lo = first + kTile;
      uint32_t* at_hi = at_lo + kTile;
      uint32_t* count = at_hi + kTile;
      const int64_t nnz = row_ptr[L];
      while (true) {
        const int cur = pos < end ? col_idx[pos] >> 5 : INT32_MAX;
        const int b0 = first_half_min(cur);              // the window: key blocks b0 .. b0 + kBitmapBlocks - 1
        if (b0 == INT32_MAX) break;
#pragma unroll
        for (int k = 0; k < kBitmapBlocks * kTile / (4 * kWave); ++k)
          reinterpret_cast<uint4*>(bm)[k * kWave + lane] = uint4{0u, 0u, 0u, 0u};
        // where each row's columns inside the window end (at most one column per key)
        const int64_t reach = end - pos > kBitmapBlocks * kTile ? pos + kBitmapBlocks * kTile : end;
        const int64_t q = lower_bound_col(col_idx, pos, reach, ((int64_t)b0 + kBitmapBlocks) * kTile);
        const int cnt = (int)(q - pos);
        // The window's columns in units of 16 consecutive entries of one row, all units of the 32
        // rows in one numbering: a lane takes a unit with four 16-byte loads, combines the bits
        // that fall into the same word in registers, and adds each word to the bitmap with one
        // LDS atomic (neighbouring lanes hold different words, or at worst the same one).
        const int units = (cnt + 15) >> 4;
        int incl = units;
#pragma unroll
        for (int off = 1; off < kTile; off <<= 1) {
          const int up = __shfl_up(incl, off, kWave);
          if (lane >= off) incl += up;
        }
        const int total = __shfl(incl, kTile - 1, kWave);
        if (total == 0) break;                           // (cannot happen: the row that gave b0 has a column in the window)
        if (lane < kTile) {
          first[lane] = (uint32_t)(incl - units);
          at_lo[lane] = (uint32_t)pos;
          at_hi[lane] = (uint32_t)((uint64_t)pos >> 32);
          count[lane] = (uint32_t)cnt;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // (one wavefront: its LDS operations complete in order)
        for (int u0 = 0; u0 < total; u0 += kBitmapUnits * kWave) {
          int rr[kBitmapUnits], nn[kBitmapUnits];
          int cc[kBitmapUnits][16];
#pragma unroll
          for (int v = 0; v < kBitmapUnits; ++v) {
            const int unit = u0 + v * kWave + lane;
            const int uu = unit < total ? unit : total - 1;
            int r = 0;
#pragma unroll
            for (int st = kTile / 2; st > 0; st >>= 1)
              if ((int)first[r + st] <= uu) r += st;
            const int j = uu - (int)first[r];
            const int64_t at = (int64_t)(((uint64_t)at_hi[r] << 32) | at_lo[r]) + 16 * j;
            const int left = (int)count[r] - 16 * j;
            rr[v] = r;
            nn[v] = unit < total ? (left < 16 ? left : 16) : 0;
            if (at + 16 <= nnz) {
              __builtin_memcpy(cc[v], col_idx + at, 64);
            } else {
#pragma unroll
              for (int t = 0; t < 16; ++t) cc[v][t] = at + t < nnz ? col_idx[at + t] : 0;
            }
          }
#pragma unroll
          for (int v = 0; v < kBitmapUnits; ++v) {
            int held = -1;
            uint32_t word = 0;
#pragma unroll
            for (int t = 0; t < 16; ++t) {
              if (t < nn[v]) {
                const int k = (cc[v][t] >> 5) - b0;
                if (k != held) {
                  if (held >= 0) atomicOr(&bm[held * kTile + rr[v]], word);
                  held = k;
                  word = 0;
                }
                word |= 1u << (cc[v][t] & 31);
              }
            }
            if (held >= 0) atomicOr(&bm[held * kTile + rr[v]], word);
          }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        for (int k = 0; k < kBitmapBlocks; ++k) {
          const uint32_t word = lane < kTile ? bm[k * kTile + lane] : 0u;
          if (!__any(word != 0u)) continue;
          if (nblk >= cap) {
            overflow = true;
            break;
          }
          const bool full = __all(lane >= kTile || word == ~0u);
          if (lane < kTile) pair_mask[(slot0 + nblk) * kTile + lane] = word;
          if (lane == 0) pair_blk[slot0 + nblk] = (b0 + k) | (full ? kFullBit : 0);
          ++nblk;
          consumed += __builtin_popcount(word);
          if (nblk == kProbeBlocks) {                    // (the same test as in the walk above)
            int sum = consumed;
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, kWave);
            if (sum < kProbeBlocks * kProbeEdges) {
              overflow = true;
              break;
            }
          }
        }
        if (overflow) break;
        pos = q;
      }
    }
    if (lane == 0) {
      TileItem it;
      it.tile = (int32_t)t;
      it.nblk = overflow ? -1 : nblk;
      it.seg = id.seg;
      it.nseg = id.nseg;
      it.slot0 = slot0;
      it.pad = 0;
      items[w] = it;
      if (overflow && atomicOr(&tile_bad[t], 1) == 0) {
        // (the per-row kernels walk this list instead of testing every row of the sequence)
        const uint32_t bi = atomicAdd(&ctr[kCtrTilesBad], 1u);
        reinterpret_cast<int32_t*>(base_ws + pl.off_bad_list)[bi] = (int32_t)t;
      }
      if (id.seg == 0 && id.nseg > 1) {
        // reserve the tile's partial slots; if the call needs more than exist, every
        // multi-segment tile goes to the gather path (all-or-nothing keeps runs reproducible)
        atomicAdd(&ctr[kCtrTilePartsNeeded], (uint32_t)id.nseg);
        const uint32_t first = atomicAdd(&ctr[kCtrTilePartsAlloc], (uint32_t)id.nseg);
        const int32_t pbase = (int64_t)first + id.nseg <= pl.cap_tparts ? (int32_t)first : -1;
        tile_pbase[t] = pbase;
        // the merge reads one record per tile instead of a chain of dependent loads
        const uint32_t mi = atomicAdd(&ctr[kCtrMultiTiles], 1u);
        if ((int64_t)mi < pl.cap_tparts)
          reinterpret_cast<int4*>(base_ws + pl.off_multi_tiles)[mi] = make_int4((int32_t)t, pbase, id.nseg, 0);
      }
    }
  }
}

__device__ __forceinline__ bool tile_parts_fit(const WorkspacePlan& pl, const void* ws) {
  return (int64_t) reinterpret_cast<const uint32_t*>(ws)[kCtrTilePartsNeeded] <= pl.cap_tparts;
}

// A claimant (wavefront or workgroup) of the dynamic schedule found no item left.  The last of
// the head's `claimants` to arrive puts the head's claim counter and this exit counter back to
// zero (every other claimant has made its last claim by then), so the next call on the same
// workspace starts from a clean schedule without a clearing launch of its own.  One lane calls.
__device__ __forceinline__ void claim_exit(uint32_t* work_next, int32_t H, uint32_t claimants) {
  uint32_t* done = work_next + H;
  if (atomicAdd(done, 1u) == claimants - 1) {
    atomicExch(work_next, 0u);
    atomicExch(done, 0u);
  }
}

constexpr uint32_t kXcdRun = 4;   // consecutive workgroups of the static schedule that share an XCD

// Persistent wavefronts: every wavefront claims the next unprocessed work item of its head from
// a device counter until none is left (items are ordered long segments first, so the greedy
// order balances the load and no workgroup has to be re-launched between items).  A segment
// of a multi-segment tile leaves a partial state.
template <typename T, int kPipe>
__device__ __forceinline__ void tile_attend_body(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, T* __restrict__ O,
    float* __restrict__ lse, const int64_t* __restrict__ row_ptr, int64_t L, float scale, void* ws,
    size_t ws_bytes, int accumulate) {
  constexpr int kLds = CoreFor<T, kPipe>::type::template lds_bytes<kPipe>();
  __shared__ __attribute__((aligned(16))) char lds_all[4 * kLds];
  const int32_t H = (int32_t)gridDim.x;   // head-major grid: the long work items of every head are dispatched first
  const WorkspacePlan pl = plan_workspace(L, H, row_ptr[L], DtypeOf<T>::code);
  if (pl.total_bytes > ws_bytes) return;
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int n = lane & 31, h = lane >> 5;
  char* lds = lds_all + wave * kLds;
  char* base_ws = static_cast<char*>(ws);
  // a negative scale is applied as a sign flip of Q (exact), so the kernels see c >= 0
  const bool negate = scale < 0.f;
  const float c = softmax_factor(scale);
  const TileItem* items = reinterpret_cast<const TileItem*>(base_ws + pl.off_items_rec);
  const int32_t* tile_bad = reinterpret_cast<const int32_t*>(base_ws + pl.off_tile_bad);
  const int32_t* tile_pbase = reinterpret_cast<const int32_t*>(base_ws + pl.off_tile_pbase);
  const bool parts_fit = tile_parts_fit(pl, ws);
  constexpr bool kDynamic = DtypeOf<T>::code == SGA_F32;
  // Workgroups go to the 8 XCDs (each with its own L2) round-robin in launch order.  The static
  // schedule hands every XCD runs of kXcdRun consecutive workgroups of one head, so that the key
  // blocks neighbouring tiles share (window blocks, global blocks) are fetched into one L2 instead
  // of several.  (gridDim.y is a multiple of 8 * kXcdRun for this schedule.)
  uint32_t head = blockIdx.x, ywg = blockIdx.y;
  if (!kDynamic && gridDim.y % (8 * kXcdRun) == 0) {
    const uint32_t lin = blockIdx.x + gridDim.x * blockIdx.y;
    const uint32_t xcd = lin & 7, slot = lin >> 3;
    const uint32_t v = ((slot / kXcdRun) * 8 + xcd) * kXcdRun + slot % kXcdRun;
    head = v / gridDim.y;
    ywg = v % gridDim.y;
  }
  const int64_t hoff = (int64_t)head * L * kHeadDim;
  uint32_t* work_next = reinterpret_cast<uint32_t*>(base_ws + pl.off_work_next) + head;
  // fp32 items are long (4096 matrix-core cycles per block): wavefronts stay resident and claim
  // the next item of their head from a device counter (greedy balance, no re-launch gaps).
  // fp16 items are short and bound by the memory path: the 4 wavefronts of a workgroup take 4
  // neighbouring tiles at the same time (static stride), so that the key blocks they share are
  // fetched together and hit the CU's L1.
  int64_t w_static = (int64_t)ywg * 4 + wave;
  while (true) {
    int64_t w_cur;
    if (kDynamic) {
      uint32_t claimed = 0;
      if (lane == 0) claimed = atomicAdd(work_next, 1u);
      w_cur = __builtin_amdgcn_readfirstlane(claimed);
      if (w_cur >= pl.n_work) {
        if (lane == 0) claim_exit(work_next, H, gridDim.y * 4);
        break;
      }
    } else {
      w_cur = w_static;
      w_static += (int64_t)gridDim.y * 4;
      if (w_cur >= pl.n_work) break;
    }
    // the whole record in one uniform 32-byte read
    const int4 r0 = reinterpret_cast<const int4*>(items + w_cur)[0];
    const int64_t slot_raw = reinterpret_cast<const int64_t*>(items + w_cur)[2];
    const int32_t t = __builtin_amdgcn_readfirstlane(r0.x);
    const int32_t nblk = __builtin_amdgcn_readfirstlane(r0.y);
    const int32_t seg = __builtin_amdgcn_readfirstlane(r0.z);
    const int32_t nseg = __builtin_amdgcn_readfirstlane(r0.w);
    const int64_t slot0 = uniform64(slot_raw);
    if (t < 0 || nblk < 0) continue;         // idle item / list overflow: tile left to the gather path
    if (nseg > 1 && (!parts_fit || tile_bad[t])) continue;
    const int64_t row_first = (int64_t)t * kTile;
    ExplicitBlocks src{reinterpret_cast<const int32_t*>(base_ws + pl.off_pair_blk) + slot0,
                       reinterpret_cast<const uint32_t*>(base_ws + pl.off_pair_mask) + slot0 * kTile, L};
    const int64_t qrow = row_first + n;
    const bool exists = qrow < L;
    typename CoreFor<T, kPipe>::type core;
    core.load_q(Q + hoff + (exists ? qrow : L - 1) * kHeadDim, h, negate);
    TileState st;
    st.init();
    core.template run<kPipe>(K + hoff, V + hoff, src, 0, nblk, c, lane, st, lds);
    if (nseg > 1) {
      float* part = reinterpret_cast<float*>(base_ws + pl.off_tpartials) +
                    (((int64_t)tile_pbase[t] + seg) * H + head) * (int64_t)kTilePartialFloats;
      store_partial(part, st, n, h);
    } else if (accumulate || !CoreOf<T>::type::kTileStore) {
      finish_tile<T>(O + hoff, lse ? lse + (int64_t)head * L : nullptr, qrow, qrow, exists, st, h,
                     accumulate != 0);
    } else if constexpr (CoreOf<T>::type::kTileStore) {
      static_assert(CoreOf<T>::type::kTileBytes <= kLds, "output tile fits the wavefront's LDS");
      const int64_t left = L - row_first;
      finish_tile_rows<T>(O + hoff, lse ? lse + (int64_t)head * L : nullptr, row_first, 1,
                          left < kTile ? (int)left : kTile, st, lane, lds);
    }
  }
}

template <typename T, int kPipe>
__global__ __launch_bounds__(256) void tile_attend_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, T* __restrict__ O,
    float* __restrict__ lse, const int64_t* __restrict__ row_ptr, int64_t L, float scale, void* ws,
    size_t ws_bytes, int accumulate) {
  tile_attend_body<T, kPipe>(Q, K, V, O, lse, row_ptr, L, scale, ws, ws_bytes, accumulate);
}

// fp16 storage: the same body held to the registers of four wavefronts per SIMD (the fp16 items
// are short and bound by the memory path: the fourth wavefront is worth more than the two
// registers the allocator would otherwise take beyond 128).
__global__ __attribute__((amdgpu_waves_per_eu(4, 4))) __launch_bounds__(256) void tile_attend_f16_kernel(
    const __half* __restrict__ Q, const __half* __restrict__ K, const __half* __restrict__ V,
    __half* __restrict__ O, float* __restrict__ lse, const int64_t* __restrict__ row_ptr, int64_t L,
    float scale, void* ws, size_t ws_bytes, int accumulate) {
  tile_attend_body<__half, kPipeLdsK>(Q, K, V, O, lse, row_ptr, L, scale, ws, ws_bytes, accumulate);
}

// Head dimensions 128 and 256: one workgroup of kD / 64 wavefronts per work item, wavefront w
// owning channels 64w .. 64w+63 (CoreF32T / CoreF16T with SliceExchange).  Workgroups stay
// resident and claim items from the head's counter like the fp32 kernel above; wavefront 0
// claims and the item index travels through LDS.
template <typename T, int kD, int kPipe>
__global__ __launch_bounds__(kD) void tile_attend_wide_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, T* __restrict__ O,
    float* __restrict__ lse, const int64_t* __restrict__ row_ptr, int64_t L, float scale, void* ws,
    size_t ws_bytes, int accumulate) {
  using Core = typename WideCoreOf<T, kD>::type;
  constexpr int kSlices = kD / kHeadDim;
  constexpr int kLds = Core::template lds_bytes<kPipe>();
  __shared__ __attribute__((aligned(16))) char lds_all[kSlices * kLds + SliceExchange<kD>::kBytes];
  __shared__ uint32_t claim;
  const int32_t H = (int32_t)gridDim.x;
  const WorkspacePlan pl = plan_workspace(L, H, row_ptr[L], DtypeOf<T>::code, kD);
  if (pl.total_bytes > ws_bytes) return;
  const int lane = threadIdx.x & (kWave - 1);
  const int slice = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int n = lane & 31, h = lane >> 5;
  char* lds = lds_all + slice * kLds;
  char* base_ws = static_cast<char*>(ws);
  const bool negate = scale < 0.f;
  const float c = softmax_factor(scale);
  const TileItem* items = reinterpret_cast<const TileItem*>(base_ws + pl.off_items_rec);
  const int32_t* tile_bad = reinterpret_cast<const int32_t*>(base_ws + pl.off_tile_bad);
  const int32_t* tile_pbase = reinterpret_cast<const int32_t*>(base_ws + pl.off_tile_pbase);
  const bool parts_fit = tile_parts_fit(pl, ws);
  const int64_t head = blockIdx.x;
  const int64_t hoff = head * L * kD + slice * kHeadDim;   // this wavefront's slice of the head
  uint32_t* work_next = reinterpret_cast<uint32_t*>(base_ws + pl.off_work_next) + head;
  Core core;
  core.xchg.init(lds_all + kSlices * kLds, slice);
  while (true) {
    __syncthreads();           // every wavefront has read the previous claim and left its item
    if (threadIdx.x == 0) claim = atomicAdd(work_next, 1u);
    __syncthreads();
    const int64_t w_cur = __builtin_amdgcn_readfirstlane(claim);
    if (w_cur >= pl.n_work) {
      if (threadIdx.x == 0) claim_exit(work_next, H, gridDim.y);
      break;
    }
    const int4 r0 = reinterpret_cast<const int4*>(items + w_cur)[0];
    const int64_t slot_raw = reinterpret_cast<const int64_t*>(items + w_cur)[2];
    const int32_t t = __builtin_amdgcn_readfirstlane(r0.x);
    const int32_t nblk = __builtin_amdgcn_readfirstlane(r0.y);
    const int32_t seg = __builtin_amdgcn_readfirstlane(r0.z);
    const int32_t nseg = __builtin_amdgcn_readfirstlane(r0.w);
    const int64_t slot0 = uniform64(slot_raw);
    if (t < 0 || nblk < 0) continue;
    if (nseg > 1 && (!parts_fit || tile_bad[t])) continue;
    const int64_t row_first = (int64_t)t * kTile;
    ExplicitBlocks src{reinterpret_cast<const int32_t*>(base_ws + pl.off_pair_blk) + slot0,
                       reinterpret_cast<const uint32_t*>(base_ws + pl.off_pair_mask) + slot0 * kTile, L};
    const int64_t qrow = row_first + n;
    const bool exists = qrow < L;
    core.load_q(Q + hoff + (exists ? qrow : L - 1) * kD, h, negate);
    TileState st;
    st.init();
    core.template run<kPipe>(K + hoff, V + hoff, src, 0, nblk, c, lane, st, lds);
    if (nseg > 1) {
      float* part = reinterpret_cast<float*>(base_ws + pl.off_tpartials) +
                    ((((int64_t)tile_pbase[t] + seg) * H + head) * kSlices + slice) *
                        (int64_t)kTilePartialFloats;
      store_partial(part, st, n, h);
    } else {
      finish_tile_wide<T, kD>(O + hoff, lse ? lse + head * L : nullptr, qrow, exists, st, h, slice,
                              accumulate != 0);
    }
  }
}

__device__ __forceinline__ float load_out(const float* p) { return *p; }
__device__ __forceinline__ float load_out(const __half* p) { return __half2float(*p); }
__device__ __forceinline__ void store_out(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_out(__half* p, float v) { *p = __float2half_rn(v); }

// Merge of a multi-segment tile's partial states.  grid = (tiles of the merge list, head,
// rows of the tile in groups of 32 / gridDim.z).  Per row: the running maximum M over all
// segments (every thread takes every 256th segment, so all loads are in flight together), the
// weights 2^(m_c - M), and the weighted sums of l and of the accumulators.  The 4 wavefronts of
// a workgroup take every 4th segment (lane = channel within each 64-channel slice; a partial
// of a kD-wide tile is kD / 64 records, one per slice, with the same m and l), four segments per
// trip so that their loads overlap, each in ascending segment order; the four results are added
// in wavefront order, so the summation order is fixed.
template <typename T, int kD>
__global__ __launch_bounds__(256) void tile_merge_kernel(T* __restrict__ O, float* __restrict__ lse,
                                                         const int64_t* __restrict__ row_ptr, int64_t L,
                                                         void* ws, size_t ws_bytes, int accumulate) {
  constexpr int kSlices = kD / kHeadDim;
  __shared__ float sm_acc[4][kD];
  __shared__ float sm_m[4], sm_l[4];
  const int32_t H = (int32_t)gridDim.y;
  constexpr int32_t dtype = DtypeOf<T>::code;
  const WorkspacePlan pl = plan_workspace(L, H, row_ptr[L], dtype, kD);
  if (pl.total_bytes > ws_bytes || !tile_parts_fit(pl, ws)) return;
  char* base_ws = static_cast<char*>(ws);
  const uint32_t n_multi = reinterpret_cast<const uint32_t*>(ws)[kCtrMultiTiles];
  const int4* multi = reinterpret_cast<const int4*>(base_ws + pl.off_multi_tiles);     // {tile, first partial slot, segments, -}
  const int32_t* tile_bad = reinterpret_cast<const int32_t*>(base_ws + pl.off_tile_bad);
  const float* parts = reinterpret_cast<const float*>(base_ws + pl.off_tpartials);
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int64_t hd = blockIdx.y;
  for (uint32_t i = blockIdx.x; i < n_multi; i += gridDim.x) {
    const int4 rec = multi[i];
    const int64_t t = rec.x;
    if (tile_bad[t]) continue;
    const int nseg = rec.z;
    const float* p0 = parts + ((int64_t)rec.y * H + hd) * (kSlices * kTilePartialFloats);
    const int64_t step = (int64_t)H * (kSlices * kTilePartialFloats);
    const int rows_per_wg = kTile / (int)gridDim.z;
    for (int r = blockIdx.z * rows_per_wg; r < (int)(blockIdx.z + 1) * rows_per_wg; ++r) {
      const int64_t row = t * kTile + r;
      const float* pm = p0 + kTile * 64 + r;       // segment c: m = pm[c * step], l = pm[c * step + kTile]
      float M = kMinusHuge;
      for (int c = threadIdx.x; c < nseg; c += 256) M = fmaxf(M, pm[c * step]);
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off, kWave));
      __syncthreads();            // the previous row's combine has read the shared arrays
      if (lane == 0) sm_m[wave] = M;
      __syncthreads();
      M = fmaxf(fmaxf(sm_m[0], sm_m[1]), fmaxf(sm_m[2], sm_m[3]));
      float l = 0.f, acc[kSlices];
#pragma unroll
      for (int sl = 0; sl < kSlices; ++sl) acc[sl] = 0.f;
      for (int c = wave; c < nseg; c += 16) {
        float mc[4], lc[4], oc[4][kSlices];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int cc = c + 4 * u < nseg ? c + 4 * u : c;
          mc[u] = pm[cc * step];
          lc[u] = pm[cc * step + kTile];
#pragma unroll
          for (int sl = 0; sl < kSlices; ++sl) oc[u][sl] = p0[cc * step + sl * kTilePartialFloats + r * 64 + lane];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const float wgt = c + 4 * u < nseg ? __builtin_amdgcn_exp2f(mc[u] - M) : 0.f;
          l = __builtin_fmaf(lc[u], wgt, l);
#pragma unroll
          for (int sl = 0; sl < kSlices; ++sl) acc[sl] = __builtin_fmaf(oc[u][sl], wgt, acc[sl]);
        }
      }
#pragma unroll
      for (int sl = 0; sl < kSlices; ++sl) sm_acc[wave][sl * 64 + lane] = acc[sl];
      if (lane == 0) sm_l[wave] = l;
      __syncthreads();
      if (wave == 0 && row < L) {
        const float lt = ((sm_l[0] + sm_l[1]) + sm_l[2]) + sm_l[3];
        const bool empty = !(lt > 0.f);
        float lse_row = empty ? -INFINITY : (M + __builtin_amdgcn_logf(lt)) * kLn2;
        CarryWeights cw{0.f, 1.f, lse_row};
        if (accumulate) {
          cw = carry_weights(lse[hd * L + row], lse_row);
          lse_row = cw.lse;
        }
#pragma unroll
        for (int sl = 0; sl < kSlices; ++sl) {
          const float at = ((sm_acc[0][sl * 64 + lane] + sm_acc[1][sl * 64 + lane]) +
                            sm_acc[2][sl * 64 + lane]) + sm_acc[3][sl * 64 + lane];
          T* dst = O + hd * L * kD + row * kD + sl * 64 + lane;
          float o = empty ? 0.f : at / lt;
          if (accumulate) o = cw.w_prev * load_out(dst) + cw.w_now * o;
          store_out(dst, o);
        }
        if (lse && lane == 0) lse[hd * L + row] = lse_row;
      }
    }
  }
}

// A workgroup's place among the window tiles.  Whole-sequence masks (seg_len = 0): residue class
// bid % s of the sequence, group bid / s of that class.  Block-diagonal masks (seg_len > 0: the
// 2-D dilated blocks of Section II-C, where the rows at in-block multiples of s attend each
// other inside every block of seg_len tokens): block bid / n_groups, the one class that starts
// at the block's first token, group bid % n_groups.  p = token of class index 0, Lc = tokens of
// the class; token = s * index + p in both cases.
struct WindowSlot {
  int64_t p, Lc, grp;
};
__device__ __forceinline__ bool locate_window_slot(int64_t bid, int64_t L, int64_t s, int64_t n_groups,
                                                   int64_t seg_len, WindowSlot& w) {
  if (seg_len > 0) {
    const int64_t base = (bid / n_groups) * seg_len;
    if (base >= L) return false;
    const int64_t len = L - base < seg_len ? L - base : seg_len;
    w.p = base;
    w.Lc = (len + s - 1) / s;
    w.grp = bid % n_groups;
  } else {
    if (bid >= n_groups * s) return false;
    w.p = bid % s;
    if (w.p >= L) return false;
    w.Lc = (L - w.p + s - 1) / s;
    w.grp = bid / s;
  }
  return true;
}

// Rows of a 2-D dilated mask that are no in-block multiple of the stride have no neighbour:
// O = 0, lse = -inf (Algorithm 1's initial state).  One thread per 16 bytes of O.
template <typename T>
__global__ __launch_bounds__(256) void clear_unselected_rows_kernel(T* __restrict__ O,
                                                                    float* __restrict__ lse, int64_t L,
                                                                    int64_t H, int32_t d, int64_t b,
                                                                    int64_t s) {
  const int64_t per_row = d * (int64_t)sizeof(T) / 16;
  const int64_t total = H * L * per_row;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t row = (i / per_row) % L;
    if (((row % b) % s) == 0) continue;
    reinterpret_cast<uint4*>(O)[i] = make_uint4(0, 0, 0, 0);
    if (lse && i % per_row == 0) lse[i / per_row] = -INFINITY;
  }
}

// Implicit window masks.  grid.x = workgroups (4 tiles each) over all residue classes, grid.y = head.
// Workgroups are dealt round-robin to the 8 XCDs, each with its own L2, and neighbouring tiles
// share most of their K/V rows, so the linear workgroup id is remapped to give every XCD one
// contiguous range of the sequence; inside it consecutive workgroups alternate between the
// residue classes, so that the interleaved rows of all classes are touched together.
template <typename T, int kPipe>
__global__ __attribute__((amdgpu_waves_per_eu(2, 2))) __launch_bounds__(256) void tile_window_kernel(const T* __restrict__ Q,
                                                          const T* __restrict__ K,
                                                          const T* __restrict__ V, T* __restrict__ O,
                                                          float* __restrict__ lse, int64_t L, int64_t W,
                                                          int64_t s, int64_t n_groups, float scale,
                                                          int accumulate, int64_t seg_len, int nsplit,
                                                          float* __restrict__ parts) {
  constexpr int kLds = CoreFor<T, kPipe>::type::template lds_bytes<kPipe>();
  __shared__ __attribute__((aligned(16))) char lds_all[4 * kLds];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int n = lane & 31, h = lane >> 5;
  char* lds = lds_all + wave * kLds;
  // gridDim.x is a multiple of 8: XCD x handles the workgroups [x*chunk, (x+1)*chunk)
  const int64_t chunk = gridDim.x / 8;
  const int64_t bid_all = (int64_t)(blockIdx.x % 8) * chunk + blockIdx.x / 8;
  // (nsplit > 1: nsplit consecutive workgroups share four tiles, each takes one range of their
  // key blocks and leaves partial states for window_merge_kernel)
  const int64_t bid = bid_all / nsplit;
  const int part = (int)(bid_all - bid * nsplit);
  WindowSlot slot;
  if (!locate_window_slot(bid, L, s, n_groups, seg_len, slot)) return;
  const int64_t p = slot.p, Lc = slot.Lc;
  const int64_t u0 = (slot.grp * 4 + wave) * kTile;
  if (u0 >= Lc) return;
  const int64_t hd = blockIdx.y;
  const int64_t hoff = hd * L * kHeadDim;
  const int64_t vlo = u0 - W > 0 ? u0 - W : 0;
  const int64_t vhi = u0 + kTile - 1 + W < Lc - 1 ? u0 + kTile - 1 + W : Lc - 1;
  WindowBlocks src{vlo, Lc, s, p, u0, W};
  const int nblk = (int)((vhi - vlo) / kTile + 1);
  const int64_t u = u0 + n;
  const bool exists = u < Lc;
  const int64_t qrow = s * (exists ? u : Lc - 1) + p;
  typename CoreFor<T, kPipe>::type core;
  core.load_q(Q + hoff + qrow * kHeadDim, h, scale < 0.f);
  TileState st;
  st.init();
  if (nsplit > 1) {
    const int k0 = (int)((int64_t)nblk * part / nsplit), k1 = (int)((int64_t)nblk * (part + 1) / nsplit);
    core.template run<kPipe>(K + hoff, V + hoff, src, k0, k1, softmax_factor(scale), lane, st, lds);
    store_partial(parts + (((bid * 4 + wave) * gridDim.y + hd) * nsplit + part) * (int64_t)kTilePartialFloats,
                  st, n, h);
    return;
  }
  core.template run<kPipe>(K + hoff, V + hoff, src, 0, nblk, softmax_factor(scale), lane, st, lds);
  if (accumulate || !CoreOf<T>::type::kTileStore) {
    finish_tile<T>(O + hoff, lse ? lse + hd * L : nullptr, qrow, qrow, exists, st, h, accumulate != 0);
  } else if constexpr (CoreOf<T>::type::kTileStore) {
    static_assert(CoreOf<T>::type::kTileBytes <= kLds, "output tile fits the wavefront's LDS");
    finish_tile_rows<T>(O + hoff, lse ? lse + hd * L : nullptr, s * u0 + p, s,
                        Lc - u0 < kTile ? (int)(Lc - u0) : kTile, st, lane, lds);
  }
}

// Key blocks of the non-local mask (global tokens 0..g-1 without the window, Section IV-B
// "Global (non-local)") against the 32 queries that start at row0, by index arithmetic.
// kGlobalRows: the queries i < g, which see every key outside their window, blocks kb0, kb0+1, ...;
// otherwise the queries i >= g, which see the global keys j < min(g, i - W).  Queries of the
// other kind (and past the end) get empty words.
template <bool kGlobalRows>
struct NonlocalBlocks {
  int64_t L, g, W, row0;
  int64_t kb0;
  static constexpr int kGetLoads = 0;
  __device__ int64_t key_stride() const { return 1; }
  __device__ void resolve(BlockInfo&) const {}
  __device__ BlockInfo get(int k, int n) const {
    BlockInfo b;
    b.raw = 0;
    const int64_t v0 = (kb0 + k) * kTile;
    b.row0 = v0;
    const int64_t left = L - v0;
    b.nvalid = left < kTile ? (int)left : kTile;
    const uint32_t valid = b.nvalid == kTile ? ~0u : ((1u << b.nvalid) - 1u);
    const int64_t i = row0 + n;
    if (kGlobalRows) {
      // keys of the block inside the window [i - W, i + W] are no neighbours
      int64_t lo = i - W - v0, hi = i + W - v0;
      uint32_t inside = 0;
      if (hi >= 0 && lo <= kTile - 1) {
        lo = lo < 0 ? 0 : lo;
        hi = hi > kTile - 1 ? kTile - 1 : hi;
        inside = (~0u >> (31 - (int)hi)) & (~0u << (int)lo);
      }
      b.word = i < g ? (valid & ~inside) : 0u;
      // (wave-uniform) every query of the tile is a global row and no window reaches the block
      b.full = b.nvalid == kTile && row0 + kTile <= g && (row0 + kTile - 1 + W < v0 || row0 - W > v0 + kTile - 1);
    } else {
      const int64_t end = (g < i - W ? g : i - W) - v0;       // keys [0, end) of the block are neighbours
      const uint32_t below = end <= 0 ? 0u : (end >= kTile ? ~0u : ((1u << (int)end) - 1u));
      b.word = (i >= g && i < L) ? (valid & below) : 0u;
      const int64_t end0 = (g < row0 - W ? g : row0 - W) - v0;      // of the tile's first query
      b.full = b.nvalid == kTile && row0 >= g && row0 + kTile <= L && end0 >= kTile;
    }
    return b;
  }
};

// Implicit non-local mask, queries i >= g: one wavefront per 32 rows against the (g + 31) / 32
// key blocks that hold the global tokens.
template <typename T, int kPipe>
__global__ __launch_bounds__(256) void tile_nonlocal_cols_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, T* __restrict__ O,
    float* __restrict__ lse, int64_t L, int64_t W, int64_t g, float scale, int accumulate) {
  constexpr int kLds = CoreFor<T, kPipe>::type::template lds_bytes<kPipe>();
  __shared__ __attribute__((aligned(16))) char lds_all[4 * kLds];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int n = lane & 31, h = lane >> 5;
  char* lds = lds_all + wave * kLds;
  const int64_t row0 = (g / kTile + (int64_t)blockIdx.x * 4 + wave) * kTile;      // the first tile may start below g
  if (row0 >= L) return;
  const int64_t hd = blockIdx.y;
  const int64_t hoff = hd * L * kHeadDim;
  const NonlocalBlocks<false> src{L, g, W, row0, 0};
  const int nblk = (int)((g + kTile - 1) / kTile);
  const int64_t i = row0 + n;
  const bool mine = i >= g && i < L;
  typename CoreFor<T, kPipe>::type core;
  core.load_q(Q + hoff + (i < L ? i : L - 1) * kHeadDim, h, scale < 0.f);
  TileState st;
  st.init();
  core.template run<kPipe>(K + hoff, V + hoff, src, 0, nblk, softmax_factor(scale), lane, st, lds);
  finish_tile<T>(O + hoff, lse ? lse + hd * L : nullptr, i, i, mine, st, h, accumulate != 0);
}

// Implicit non-local mask, the g global rows: grid = (ranges of key blocks, tiles of global rows,
// heads), one wavefront each, which leaves the partial state of its rows over its range in the
// layout nonlocal_merge_kernel reads (row-major: D accumulators, m, l per (row, range, head)).
template <typename T, int kPipe>
__global__ __launch_bounds__(64) void tile_nonlocal_rows_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, int64_t L, int64_t W,
    int64_t g, int64_t blocks_per_range, float scale, float* __restrict__ partials) {
  constexpr int kLds = CoreFor<T, kPipe>::type::template lds_bytes<kPipe>();
  __shared__ __attribute__((aligned(16))) char lds[kLds];
  const int lane = threadIdx.x;
  const int n = lane & 31, h = lane >> 5;
  const int64_t c = blockIdx.x, n_ranges = gridDim.x, hd = blockIdx.z, H = gridDim.z;
  const int64_t row0 = (int64_t)blockIdx.y * kTile;
  const int64_t hoff = hd * L * kHeadDim;
  const int64_t nb_total = (L + kTile - 1) / kTile;
  const int64_t kb0 = c * blocks_per_range;
  const int64_t kb1 = kb0 + blocks_per_range < nb_total ? kb0 + blocks_per_range : nb_total;
  const NonlocalBlocks<true> src{L, g, W, row0, kb0};
  const int64_t i = row0 + n;
  typename CoreFor<T, kPipe>::type core;
  core.load_q(Q + hoff + (i < L ? i : L - 1) * kHeadDim, h, scale < 0.f);
  TileState st;
  st.init();
  core.template run<kPipe>(K + hoff, V + hoff, src, 0, (int)(kb1 > kb0 ? kb1 - kb0 : 0), softmax_factor(scale),
                           lane, st, lds);
  if (i >= g) return;
  const float l = st.l + other_half(st.l, h);
  float* p = partials + ((i * n_ranges + c) * H + hd) * (kHeadDim + 4);
#pragma unroll
  for (int cb = 0; cb < 2; ++cb)
#pragma unroll
    for (int q = 0; q < 4; ++q)
      *reinterpret_cast<float4*>(p + cb * 32 + 8 * q + 4 * h) =
          make_float4(st.o[cb][4 * q], st.o[cb][4 * q + 1], st.o[cb][4 * q + 2], st.o[cb][4 * q + 3]);
  if (h == 0) {
    p[kHeadDim] = st.m;
    p[kHeadDim + 1] = l;
  }
}

__device__ __forceinline__ float lane_value(float v, int src_lane) {     // v of lane src_lane (uniform index)
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), src_lane));
}

// Merge of the partial states that the window kernels leave when they cut the key blocks of
// their tiles into nsplit <= kMaxWindowSplit ranges.  grid = (tiles: 4 per workgroup of the uncut
// d = 64 launch, 1 per workgroup of the wider ones; head; quarter of the tile's rows), one
// wavefront per 64-channel slice.  Lanes 0..7 first reduce the (m, l) of the quarter's eight rows
// over the ranges, in ascending order, to the rows' weights; then lane = channel and the
// weighted accumulators are summed row by row, every load independent of the others.
template <typename T, int kD>
__global__ __launch_bounds__(kD) void window_merge_kernel(
    T* __restrict__ O, float* __restrict__ lse, const float* __restrict__ parts, int64_t L, int64_t s,
    int64_t n_groups, int accumulate, int64_t seg_len, int nsplit) {
  constexpr int kSlices = kD / kHeadDim;
  constexpr int kTilesPerWg = kSlices == 1 ? 4 : 1;    // of the launch that wrote the partial states
  constexpr int kRows = kTile / 4;
  const int lane = threadIdx.x & (kWave - 1);
  const int slice = threadIdx.x / kWave;
  const int64_t bid = blockIdx.x / kTilesPerWg, hd = blockIdx.y;
  const int tile_in_wg = blockIdx.x % kTilesPerWg;
  WindowSlot slot;
  if (!locate_window_slot(bid, L, s, n_groups, seg_len, slot)) return;
  const int64_t u0 = (slot.grp * kTilesPerWg + tile_in_wg) * kTile + blockIdx.z * kRows;
  if (u0 >= slot.Lc) return;
  const int r0 = blockIdx.z * kRows;
  const int64_t range_step = (int64_t)kSlices * kTilePartialFloats;
  const float* p0 = parts + ((((bid * kTilesPerWg + tile_in_wg) * gridDim.y + hd) * nsplit) * kSlices + slice) *
                                (int64_t)kTilePartialFloats;
  // row statistics: lane j < kRows owns row r0 + j
  const int jr = lane < kRows ? lane : 0;
  const int64_t row_j = s * (u0 + jr < slot.Lc ? u0 + jr : slot.Lc - 1) + slot.p;
  float mc[kMaxWindowSplit], lc[kMaxWindowSplit];
  float M = kMinusHuge;
#pragma unroll
  for (int c = 0; c < kMaxWindowSplit; ++c) {
    const int cc = c < nsplit ? c : 0;
    mc[c] = p0[cc * range_step + kTile * 64 + r0 + jr];
    lc[c] = c < nsplit ? p0[cc * range_step + kTile * 64 + kTile + r0 + jr] : 0.f;
    if (c < nsplit) M = fmaxf(M, mc[c]);
  }
  float l = 0.f, w[kMaxWindowSplit];
#pragma unroll
  for (int c = 0; c < kMaxWindowSplit; ++c) {
    w[c] = c < nsplit ? __builtin_amdgcn_exp2f(mc[c] - M) : 0.f;
    l = __builtin_fmaf(lc[c], w[c], l);
  }
  const bool empty = !(l > 0.f);
  float lse_row = empty ? -INFINITY : (M + __builtin_amdgcn_logf(l)) * kLn2;
  float w_now = empty ? 0.f : 1.0f / l, w_prev = 0.f;
  if (accumulate) {
    const CarryWeights cw = carry_weights(lse[hd * L + row_j], lse_row);
    w_now *= cw.w_now;
    w_prev = cw.w_prev;
    lse_row = cw.lse;
    if (kSlices > 1) __syncthreads();     // every slice has read the earlier lse before slice 0 replaces it
  }
  if (lse && slice == 0 && lane < kRows && u0 + lane < slot.Lc) lse[hd * L + row_j] = lse_row;
#pragma unroll
  for (int c = 0; c < kMaxWindowSplit; ++c) w[c] *= w_now;        // weights of the normalised sum
#pragma unroll
  for (int j = 0; j < kRows; ++j) {
    if (u0 + j >= slot.Lc) break;
    const int64_t row = s * (u0 + j) + slot.p;
    float acc = 0.f;
#pragma unroll
    for (int c = 0; c < kMaxWindowSplit; ++c) {
      if (c < nsplit)
        acc = __builtin_fmaf(p0[c * range_step + (r0 + j) * 64 + lane], lane_value(w[c], j), acc);
    }
    T* dst = O + hd * L * kD + row * kD + slice * kHeadDim + lane;
    if (accumulate) acc = __builtin_fmaf(lane_value(w_prev, j), load_out(dst), acc);
    store_out(dst, acc);
  }
}

// Window masks at head dimensions 128 and 256: one workgroup of kD / 64 wavefronts per
// 32-query tile (see tile_attend_wide_kernel); grid mapping as in tile_window_kernel with one
// tile per workgroup.
template <typename T, int kD, int kPipe>
__global__ __launch_bounds__(kD) void tile_window_wide_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, T* __restrict__ O,
    float* __restrict__ lse, int64_t L, int64_t W, int64_t s, int64_t n_tiles, float scale,
    int accumulate, int64_t seg_len, int nsplit, float* __restrict__ parts) {
  using Core = typename WideCoreOf<T, kD>::type;
  constexpr int kSlices = kD / kHeadDim;
  constexpr int kLds = Core::template lds_bytes<kPipe>();
  __shared__ __attribute__((aligned(16))) char lds_all[kSlices * kLds + SliceExchange<kD>::kBytes];
  const int lane = threadIdx.x & (kWave - 1);
  const int slice = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int n = lane & 31, h = lane >> 5;
  const int64_t chunk = gridDim.x / 8;
  const int64_t bid_all = (int64_t)(blockIdx.x % 8) * chunk + blockIdx.x / 8;
  // (nsplit > 1: nsplit consecutive workgroups share a tile, see tile_window_kernel)
  const int64_t bid = bid_all / nsplit;
  const int part = (int)(bid_all - bid * nsplit);
  // (every condition below is the same for all wavefronts of the workgroup)
  WindowSlot slot;
  if (!locate_window_slot(bid, L, s, n_tiles, seg_len, slot)) return;
  const int64_t p = slot.p, Lc = slot.Lc;
  const int64_t u0 = slot.grp * kTile;
  if (u0 >= Lc) return;
  const int64_t hd = blockIdx.y;
  const int64_t hoff = hd * L * kD + slice * kHeadDim;
  const int64_t vlo = u0 - W > 0 ? u0 - W : 0;
  const int64_t vhi = u0 + kTile - 1 + W < Lc - 1 ? u0 + kTile - 1 + W : Lc - 1;
  WindowBlocks src{vlo, Lc, s, p, u0, W};
  const int nblk = (int)((vhi - vlo) / kTile + 1);
  const int64_t u = u0 + n;
  const bool exists = u < Lc;
  const int64_t qrow = s * (exists ? u : Lc - 1) + p;
  Core core;
  core.xchg.init(lds_all + kSlices * kLds, slice);
  core.load_q(Q + hoff + qrow * kD, h, scale < 0.f);
  TileState st;
  st.init();
  if (nsplit > 1) {
    const int k0 = (int)((int64_t)nblk * part / nsplit), k1 = (int)((int64_t)nblk * (part + 1) / nsplit);
    core.template run<kPipe>(K + hoff, V + hoff, src, k0, k1, softmax_factor(scale), lane, st,
                             lds_all + slice * kLds);
    store_partial(parts + (((bid * gridDim.y + hd) * nsplit + part) * kSlices + slice) *
                              (int64_t)kTilePartialFloats,
                  st, n, h);
    return;
  }
  core.template run<kPipe>(K + hoff, V + hoff, src, 0, nblk, softmax_factor(scale), lane, st,
                           lds_all + slice * kLds);
  finish_tile_wide<T, kD>(O + hoff, lse ? lse + hd * L : nullptr, qrow, exists, st, h, slice,
                          accumulate != 0);
}

// fp16, d = 128, explicit masks: one wavefront per work item with all 128 channels of its 32
// queries (tile_attend_wide_kernel gives each 64-channel slice a wavefront, which repeats the
// softmax in every slice and exchanges the partial scores through LDS).  A key block is staged as
// four 64-channel blocks in the layout CoreF16 reads (K channels 0..63, K 64..127, V 0..63,
// V 64..127: 16 KB per wavefront), K one block ahead as in CoreF16T::run_ldsk; the scores of a
// block are one chain of eight products over the two K halves, the softmax is done once, the
// numerators meet the two V halves in eight more products.  Wavefronts claim items of their head
// from the device counter.  Partial states of multi-segment tiles are written as the two slice
// records tile_merge_kernel<__half, 128> reads.
__global__ __attribute__((amdgpu_waves_per_eu(2, 2))) __launch_bounds__(256) void tile_attend128_f16_kernel(
    const __half* __restrict__ Q, const __half* __restrict__ K, const __half* __restrict__ V,
    __half* __restrict__ O, float* __restrict__ lse, const int64_t* __restrict__ row_ptr, int64_t L,
    float scale, void* ws, size_t ws_bytes, int accumulate) {
  using Core = CoreF16T<2 * kHeadDim>;
  constexpr int kD = 2 * kHeadDim;
  constexpr int kBlk = Core::kBlockBytes;
  __shared__ __attribute__((aligned(16))) char lds_all[4][4 * kBlk];
  const int32_t H = (int32_t)gridDim.x;
  const WorkspacePlan pl = plan_workspace(L, H, row_ptr[L], SGA_F16, kD);
  if (pl.total_bytes > ws_bytes) return;
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int n = lane & 31, h = lane >> 5;
  char* ldsk = lds_all[wave];                    // K channels 0..63, then 64..127
  char* ldsv = ldsk + 2 * kBlk;                  // V likewise
  char* base_ws = static_cast<char*>(ws);
  const bool negate = scale < 0.f;
  const float c = softmax_factor(scale);
  const TileItem* items = reinterpret_cast<const TileItem*>(base_ws + pl.off_items_rec);
  const int32_t* tile_bad = reinterpret_cast<const int32_t*>(base_ws + pl.off_tile_bad);
  const int32_t* tile_pbase = reinterpret_cast<const int32_t*>(base_ws + pl.off_tile_pbase);
  const bool parts_fit = tile_parts_fit(pl, ws);
  const int64_t head = blockIdx.x;
  const int64_t hoff = head * L * kD;
  uint32_t* work_next = reinterpret_cast<uint32_t*>(base_ws + pl.off_work_next) + head;
  const __half* Kh = K + hoff;
  const __half* Vh = V + hoff;
  typename Core::Stage sm;
  sm.init(1, lane);
  const char* vt0 = Core::vt_base(ldsv, lane, h);
  float* lse_h = lse ? lse + head * L : nullptr;
  while (true) {
    uint32_t claimed = 0;
    if (lane == 0) claimed = atomicAdd(work_next, 1u);
    const int64_t w_cur = __builtin_amdgcn_readfirstlane(claimed);
    if (w_cur >= pl.n_work) {
      if (lane == 0) claim_exit(work_next, H, gridDim.y * 4);
      break;
    }
    const int4 r0 = reinterpret_cast<const int4*>(items + w_cur)[0];
    const int64_t slot_raw = reinterpret_cast<const int64_t*>(items + w_cur)[2];
    const int32_t t = __builtin_amdgcn_readfirstlane(r0.x);
    const int32_t nblk = __builtin_amdgcn_readfirstlane(r0.y);
    const int32_t seg = __builtin_amdgcn_readfirstlane(r0.z);
    const int32_t nseg = __builtin_amdgcn_readfirstlane(r0.w);
    const int64_t slot0 = uniform64(slot_raw);
    if (t < 0 || nblk < 0) continue;         // idle item / list overflow: tile left to the gather path
    if (nseg > 1 && (!parts_fit || tile_bad[t])) continue;
    const int64_t row_first = (int64_t)t * kTile;
    const ExplicitBlocks src{reinterpret_cast<const int32_t*>(base_ws + pl.off_pair_blk) + slot0,
                             reinterpret_cast<const uint32_t*>(base_ws + pl.off_pair_mask) + slot0 * kTile, L};
    const int64_t qrow = row_first + n;
    const bool exists = qrow < L;
    Core lo, hi;                             // channels 0..63 and 64..127 of the same queries
    lo.load_q(Q + hoff + (exists ? qrow : L - 1) * kD, h, negate);
    hi.load_q(Q + hoff + (exists ? qrow : L - 1) * kD + kHeadDim, h, negate);
    TileState st, st_hi;                     // m and l live in st; st_hi holds the accumulators of channels 64..127
    st.init();
    st_hi.init();
    if (nblk > 0) {
      BlockInfo b = src.get(0, n);
      BlockInfo b1 = src.get(nblk > 1 ? 1 : 0, n);
      src.resolve(b);
      __builtin_amdgcn_wave_barrier();       // reads of the buffers by the work item before are done
      sm.stage_k(Kh, b, lane, ldsk);
      sm.stage_k(Kh + kHeadDim, b, lane, ldsk + kBlk);
      for (int k = 0; k < nblk; ++k) {
        const bool more = k + 1 < nblk;      // wave-uniform
        src.resolve(b1);
        __builtin_amdgcn_wave_barrier();     // the previous block's reads of the staged V are done
        sm.stage_v(Vh, b, lane, ldsv);
        sm.stage_v(Vh + kHeadDim, b, lane, ldsv + kBlk);
        BlockInfo b2 = b1;
        if (k + 2 < nblk) b2 = src.get(k + 2, n);
        wait_k_block<8, ExplicitBlocks::kGetLoads>(k + 2 < nblk);   // K block k: older than the V copies (and the record loads)
        __builtin_amdgcn_wave_barrier();
        half8 kf[4], kg[4];
        Core::read_k(ldsk, n, h, kf);
        Core::read_k(ldsk + kBlk, n, h, kg);
        wait_lds_reads();                    // the K buffers may be overwritten now
        __builtin_amdgcn_wave_barrier();
        if (more) {
          sm.stage_k(Kh, b1, lane, ldsk);
          sm.stage_k(Kh + kHeadDim, b1, lane, ldsk + kBlk);
        }
        floatx16 sv = {0};
#pragma unroll
        for (int u = 0; u < 4; ++u) sv = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[u], lo.qf[u], sv, 0, 0, 0);
#pragma unroll
        for (int u = 0; u < 4; ++u) sv = __builtin_amdgcn_mfma_f32_32x32x16_f16(kg[u], hi.qf[u], sv, 0, 0, 0);
        if (!b.full) mask_scores(sv, b.word, h);
        half8 ph[2];
        const float l_before = st.l;
        numerators_h(sv, c, st, ph);
        if (__any(sum_overflowed(st))) {
          // (see softmax_block_h; the accumulators of the upper channels take the same factor)
          st.l = l_before;
          const float m_before = st.m;
          rescale_state(st, block_max(sv, c, h));
          const float alpha = __builtin_amdgcn_exp2f(m_before - st.m);
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            st_hi.o[0][r] *= alpha;
            st_hi.o[1][r] *= alpha;
          }
          numerators_h(sv, c, st, ph);
        }
        // V block k (and any record load after it) is older than the 8 K copies issued above (if any)
        wait_staged_v<8>(more);
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const half8 a0 = Core::read_va(vt0, u, 0), a1 = Core::read_va(vt0, u, 1);
          const half8 c0 = Core::read_va(vt0 + kBlk, u, 0), c1 = Core::read_va(vt0 + kBlk, u, 1);
          st.o[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, ph[u], st.o[0], 0, 0, 0);
          st.o[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, ph[u], st.o[1], 0, 0, 0);
          st_hi.o[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(c0, ph[u], st_hi.o[0], 0, 0, 0);
          st_hi.o[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(c1, ph[u], st_hi.o[1], 0, 0, 0);
        }
        b = b1;
        b1 = b2;
      }
    }
    if (nseg > 1) {
      float* part = reinterpret_cast<float*>(base_ws + pl.off_tpartials) +
                    ((((int64_t)tile_pbase[t] + seg) * H + head) * 2) * (int64_t)kTilePartialFloats;
      st_hi.m = st.m;
      st_hi.l = st.l;
      store_partial(part, st, n, h);
      store_partial(part + kTilePartialFloats, st_hi, n, h);
      continue;
    }
    const float l = st.l + other_half(st.l, h);
    const bool empty = !(l > 0.f);
    const float inv = empty ? 0.f : 1.0f / l;
    float lse_row = empty ? -INFINITY : (st.m + __builtin_amdgcn_logf(l)) * kLn2;
    if (accumulate) {
      if (exists) {
        // (both half-waves read the earlier lse before the first replaces it)
        const CarryWeights cw = carry_weights(lse_h[qrow], lse_row);
        Core::store_row(O + hoff + qrow * kD, st, inv * cw.w_now, cw.w_prev, true, h);
        Core::store_row(O + hoff + qrow * kD + kHeadDim, st_hi, inv * cw.w_now, cw.w_prev, true, h);
        if (h == 0) lse_h[qrow] = cw.lse;
      }
      continue;
    }
    // The tile leaves through the wavefront's LDS (every copy has landed, every read is done) as
    // whole 256-byte rows, four per instruction, with streaming stores (see CoreF16T::store_tile).
    constexpr int kPitch = kD * 2 + 16;
    static_assert(kTile * kPitch <= 4 * kBlk, "output tile fits the wavefront's LDS");
    char* tile = ldsk;
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const TileState& part = half ? st_hi : st;
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          uint2 w;
          w.x = __builtin_bit_cast(uint32_t, __floats2half2_rn(part.o[cb][4 * g] * inv, part.o[cb][4 * g + 1] * inv));
          w.y = __builtin_bit_cast(uint32_t,
                                   __floats2half2_rn(part.o[cb][4 * g + 2] * inv, part.o[cb][4 * g + 3] * inv));
          *reinterpret_cast<uint2*>(tile + n * kPitch + (half * kHeadDim + cb * 32 + 8 * g + 4 * h) * 2) = w;
        }
    }
    __builtin_amdgcn_wave_barrier();
    const int64_t left = L - row_first;
    const int n_rows = left < kTile ? (int)left : kTile;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = (lane >> 4) + 4 * i;
      const uint4 v = *reinterpret_cast<const uint4*>(tile + r * kPitch + (lane & 15) * 16);
      if (r < n_rows)
        __builtin_nontemporal_store(__builtin_bit_cast(half8, v),
                                    reinterpret_cast<half8*>(O + hoff + (row_first + r) * kD + (lane & 15) * 8));
    }
    if (lse_h && h == 0 && n < n_rows) lse_h[row_first + n] = lse_row;
    wait_lds_reads();                        // (the tile has left before the next item stages into this space)
  }
}

// The implicit non-local mask at head dimensions 128 and 256: the two kernels of the 64-channel
// form (tile_nonlocal_cols_kernel, tile_nonlocal_rows_kernel) with one workgroup of kD / 64
// wavefronts per tile, each on its 64-channel slice (see tile_attend_wide_kernel).
template <typename T, int kD, int kPipe>
__global__ __launch_bounds__(kD) void tile_nonlocal_cols_wide_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, T* __restrict__ O,
    float* __restrict__ lse, int64_t L, int64_t W, int64_t g, float scale, int accumulate) {
  using Core = typename WideCoreOf<T, kD>::type;
  constexpr int kSlices = kD / kHeadDim;
  constexpr int kLds = Core::template lds_bytes<kPipe>();
  __shared__ __attribute__((aligned(16))) char lds_all[kSlices * kLds + SliceExchange<kD>::kBytes];
  const int lane = threadIdx.x & (kWave - 1);
  const int slice = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int n = lane & 31, h = lane >> 5;
  const int64_t row0 = (g / kTile + (int64_t)blockIdx.x) * kTile;
  if (row0 >= L) return;                           // (the same for every wavefront of the workgroup)
  const int64_t hd = blockIdx.y;
  const int64_t hoff = hd * L * kD + slice * kHeadDim;
  const NonlocalBlocks<false> src{L, g, W, row0, 0};
  const int nblk = (int)((g + kTile - 1) / kTile);
  const int64_t i = row0 + n;
  Core core;
  core.xchg.init(lds_all + kSlices * kLds, slice);
  core.load_q(Q + hoff + (i < L ? i : L - 1) * kD, h, scale < 0.f);
  TileState st;
  st.init();
  core.template run<kPipe>(K + hoff, V + hoff, src, 0, nblk, softmax_factor(scale), lane, st,
                           lds_all + slice * kLds);
  finish_tile_wide<T, kD>(O + hoff, lse ? lse + hd * L : nullptr, i < L ? i : L - 1, i >= g && i < L, st, h, slice,
                          accumulate != 0);
}

template <typename T, int kD, int kPipe>
__global__ __launch_bounds__(kD) void tile_nonlocal_rows_wide_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, int64_t L, int64_t W,
    int64_t g, int64_t blocks_per_range, float scale, float* __restrict__ partials) {
  using Core = typename WideCoreOf<T, kD>::type;
  constexpr int kSlices = kD / kHeadDim;
  constexpr int kLds = Core::template lds_bytes<kPipe>();
  __shared__ __attribute__((aligned(16))) char lds_all[kSlices * kLds + SliceExchange<kD>::kBytes];
  const int lane = threadIdx.x & (kWave - 1);
  const int slice = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int n = lane & 31, h = lane >> 5;
  const int64_t c = blockIdx.x, n_ranges = gridDim.x, hd = blockIdx.z, H = gridDim.z;
  const int64_t row0 = (int64_t)blockIdx.y * kTile;
  const int64_t hoff = hd * L * kD + slice * kHeadDim;
  const int64_t nb_total = (L + kTile - 1) / kTile;
  const int64_t kb0 = c * blocks_per_range;
  const int64_t kb1 = kb0 + blocks_per_range < nb_total ? kb0 + blocks_per_range : nb_total;
  const NonlocalBlocks<true> src{L, g, W, row0, kb0};
  const int64_t i = row0 + n;
  Core core;
  core.xchg.init(lds_all + kSlices * kLds, slice);
  core.load_q(Q + hoff + (i < L ? i : L - 1) * kD, h, scale < 0.f);
  TileState st;
  st.init();
  core.template run<kPipe>(K + hoff, V + hoff, src, 0, (int)(kb1 > kb0 ? kb1 - kb0 : 0), softmax_factor(scale),
                           lane, st, lds_all + slice * kLds);
  if (i >= g) return;
  const float l = st.l + other_half(st.l, h);
  float* p = partials + ((i * n_ranges + c) * H + hd) * (kD + 4);
#pragma unroll
  for (int cb = 0; cb < 2; ++cb)
#pragma unroll
    for (int q = 0; q < 4; ++q)
      *reinterpret_cast<float4*>(p + slice * kHeadDim + cb * 32 + 8 * q + 4 * h) =
          make_float4(st.o[cb][4 * q], st.o[cb][4 * q + 1], st.o[cb][4 * q + 2], st.o[cb][4 * q + 3]);
  if (h == 0 && slice == 0) {
    p[kD] = st.m;
    p[kD + 1] = l;
  }
}

// fp16 window masks, wide bands: a workgroup owns 256 consecutive queries of a class (64 per
// wavefront: two 32-query sub-tiles that share every K fragment and V^T operand read, with two
// independent chains of products) and walks the key blocks of its
// whole window once, in step: every K and V block is copied global -> LDS once per workgroup
// (each wavefront moves one 1 KB copy of K and one of V per block instead of all eight), into a
// ring of kBandSlots blocks that runs kBandAhead blocks ahead of the block being computed.  One
// workgroup barrier per block both publishes the block (every wavefront has waited for its own
// two copies) and retires the block before it (its slot is the next one to be overwritten).
// A wavefront computes a block only where it lies inside its own window (its queries start 64w
// keys into the workgroup's range, so it idles for two blocks per wavefront index at one end or
// the other).  The copies are issued untracked: every wavefront issues exactly two per block, so
// a counted wait names the block that must have landed; past the last block the copies repeat
// the last block into a slot nobody reads any more, which keeps the count constant to the end.
constexpr int kBandSlots = 8;
constexpr int kBandAhead = 6;      // <= kBandSlots - 2: the slot written holds a block retired a barrier ago

__global__ __attribute__((amdgpu_waves_per_eu(2, 2))) __launch_bounds__(256) void tile_window_band_kernel(
    const __half* __restrict__ Q, const __half* __restrict__ K, const __half* __restrict__ V,
    __half* __restrict__ O, float* __restrict__ lse, int64_t L, int64_t W, int64_t s, int64_t n_groups,
    float scale, int accumulate, int64_t seg_len) {
  constexpr int kSlotBytes = 2 * CoreF16::kBlockBytes;       // K block, then V block
  __shared__ __attribute__((aligned(16))) char ring[kBandSlots * kSlotBytes];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int n = lane & 31, h = lane >> 5;
  const int64_t chunk = gridDim.x / 8;
  const int64_t bid = (int64_t)(blockIdx.x % 8) * chunk + blockIdx.x / 8;
  WindowSlot slot;
  if (!locate_window_slot(bid, L, s, n_groups, seg_len, slot)) return;      // (the whole workgroup leaves)
  const int64_t p = slot.p, Lc = slot.Lc;
  const int64_t q0 = slot.grp * (8 * kTile);
  if (q0 >= Lc) return;
  const int64_t hd = blockIdx.y;
  const int64_t hoff = hd * L * kHeadDim;
  const int64_t u0 = q0 + (int64_t)wave * (2 * kTile);
  const int64_t vfirst = q0 - W > 0 ? q0 - W : 0;
  const int64_t vlast = q0 + 8 * kTile - 1 + W < Lc - 1 ? q0 + 8 * kTile - 1 + W : Lc - 1;
  const int nblk = (int)((vlast - vfirst) / kTile + 1);
  // a wavefront whose queries lie past the end of the class (u0 >= Lc) still copies and meets the
  // barriers; classify() then reports no block as its own
  const WindowBlocks sa{vfirst, Lc, s, p, u0, W}, sb{vfirst, Lc, s, p, u0 + kTile, W};
  const int64_t ua = u0 + n, ub = u0 + kTile + n;
  const bool exists_a = ua < Lc, exists_b = ub < Lc;
  const int64_t qrow_a = s * (exists_a ? ua : Lc - 1) + p, qrow_b = s * (exists_b ? ub : Lc - 1) + p;
  CoreF16 core, core_b;
  core.load_q(Q + hoff + qrow_a * kHeadDim, h, scale < 0.f);
  core_b.load_q(Q + hoff + qrow_b * kHeadDim, h, scale < 0.f);
  wait_loads_except<0>();            // Q has arrived: from here on only the ring's copies are counted
  core.q_arrived();
  core_b.q_arrived();
  // this wavefront's share of a block: keys 8w .. 8w+7, eight lanes of 16 bytes per 128-byte row
  // (the K chunks swizzled as CoreF16::read_k expects)
  const int r_own = 8 * wave + (lane >> 3), c_own = lane & 7;
  const char* Kb = reinterpret_cast<const char*>(K + hoff);
  const char* Vb = reinterpret_cast<const char*>(V + hoff);
  auto issue = [&](int kb) {
    const int kc = kb < nblk ? kb : nblk - 1;
    int64_t v = vfirst + (int64_t)kc * kTile + r_own;
    v = v < Lc ? v : Lc - 1;                               // keys past the end re-read the last one (masked off)
    const int64_t row_bytes = (s * v + p) * (kHeadDim * 2);
    char* dst = ring + (kb % kBandSlots) * kSlotBytes + wave * 1024;
    copy16_to_lds_untracked(Kb + row_bytes + ((c_own ^ (r_own & 7)) * 16), dst);
    copy16_to_lds_untracked(Vb + row_bytes + c_own * 16, dst + CoreF16::kBlockBytes);
  };
  TileState sta, stb;
  sta.init();
  stb.init();
  const float c = softmax_factor(scale);
  const char* vt0 = CoreF16::vt_base(ring + CoreF16::kBlockBytes, lane, h);
  // The barrier that opens block kb: every wavefront has waited for its own copies of blocks kb
  // and kb+1 (so after it both are whole: the interior steps read K of block kb+1 for the score
  // products they issue one block ahead), and everyone is done with block kb-1; then the copy
  // kBandAhead blocks on is started, into the slot of block kb-2.
  auto publish = [&](int kb) {
    wait_loads_except<2 * (kBandAhead - 2)>();
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    issue(kb + kBandAhead);
  };
  // One block on the edge of (or outside) this wavefront's windows: publish it, compute what
  // falls inside.
  auto step = [&](int kb) {
    publish(kb);
    const char* ldsk = ring + (kb % kBandSlots) * kSlotBytes;
    const char* vt = vt0 + (kb % kBandSlots) * kSlotBytes;
    half8 pha[2], phb[2];
    {
      const int class_a = sa.classify(kb), class_b = sb.classify(kb);     // wave-uniform
      if (class_a | class_b) {
        half8 kf[4];
        CoreF16::read_k(ldsk, n, h, kf);
        if (class_a) {
          floatx16 sacc = {0};
#pragma unroll
          for (int t = 0; t < 4; ++t) sacc = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[t], core.qf[t], sacc, 0, 0, 0);
          const uint32_t word = class_a == 2 ? ~0u : sa.get(kb, n).word;
          softmax_block_h(sacc, c, class_a == 2, word, h, sta, pha);
        }
        if (class_b) {
          floatx16 sacc = {0};
#pragma unroll
          for (int t = 0; t < 4; ++t) sacc = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[t], core_b.qf[t], sacc, 0, 0, 0);
          const uint32_t word = class_b == 2 ? ~0u : sb.get(kb, n).word;
          softmax_block_h(sacc, c, class_b == 2, word, h, stb, phb);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int cb = 0; cb < 2; ++cb) {
            const half8 va = CoreF16::read_va(vt, u, cb);
            if (class_a) sta.o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(va, pha[u], sta.o[cb], 0, 0, 0);
            if (class_b) stb.o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(va, phb[u], stb.o[cb], 0, 0, 0);
          }
      }
    }
  };
  // the blocks interior to both of this wavefront's sub-tiles form one range [k_lo, k_hi)
  int k_lo = 0, k_hi = nblk;
  while (k_lo < nblk && !(sa.classify(k_lo) == 2 && sb.classify(k_lo) == 2)) ++k_lo;
  while (k_hi > k_lo && !(sa.classify(k_hi - 1) == 2 && sb.classify(k_hi - 1) == 2)) --k_hi;
  // Interior blocks, software-pipelined: the score products of block kb+1 are issued ahead of the
  // exponentials and the PV products of block kb, so that the matrix cores and the vector unit
  // have independent work side by side.  cur_* hold the scores of block kb on entry (kFirst: the
  // step computes them itself), nxt_* receive those of block kb+1 (kNext: it is interior too);
  // successive steps swap the two pairs, so no accumulator is ever copied.
  auto products = [&](int kb, floatx16& da, floatx16& db) {
    half8 kf[4];
    CoreF16::read_k(ring + (kb % kBandSlots) * kSlotBytes, n, h, kf);
    da = floatx16{0};
    db = floatx16{0};
#pragma unroll
    for (int t = 0; t < 4; ++t) da = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[t], core.qf[t], da, 0, 0, 0);
#pragma unroll
    for (int t = 0; t < 4; ++t) db = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[t], core_b.qf[t], db, 0, 0, 0);
  };
  auto piped = [&](int kb, floatx16& cur_a, floatx16& cur_b, floatx16& nxt_a, floatx16& nxt_b, auto first,
                   auto next) {
    publish(kb);
    if constexpr (decltype(first)::value) products(kb, cur_a, cur_b);
    if constexpr (decltype(next)::value) products(kb + 1, nxt_a, nxt_b);
    half8 pha[2], phb[2];
    softmax_pair_h(cur_a, cur_b, c, h, sta, stb, pha, phb);
    const char* vt = vt0 + (kb % kBandSlots) * kSlotBytes;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const half8 va0 = CoreF16::read_va(vt, u, 0), va1 = CoreF16::read_va(vt, u, 1);
      sta.o[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(va0, pha[u], sta.o[0], 0, 0, 0);
      stb.o[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(va0, phb[u], stb.o[0], 0, 0, 0);
      sta.o[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(va1, pha[u], sta.o[1], 0, 0, 0);
      stb.o[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(va1, phb[u], stb.o[1], 0, 0, 0);
    }
  };
  for (int kb = 0; kb < kBandAhead; ++kb) issue(kb);
  int kb = 0;
  for (; kb < k_lo; ++kb) step(kb);
  if (kb < k_hi) {
    constexpr std::true_type yes{};
    constexpr std::false_type no{};
    floatx16 s_a, s_b, t_a, t_b;
    if (kb + 1 < k_hi) {
      piped(kb, s_a, s_b, t_a, t_b, yes, yes);
      ++kb;                                              // the scores of block kb are in t_*
      for (; kb + 2 < k_hi; kb += 2) {
        piped(kb, t_a, t_b, s_a, s_b, no, yes);
        piped(kb + 1, s_a, s_b, t_a, t_b, no, yes);
      }
      if (kb + 1 < k_hi) {
        piped(kb, t_a, t_b, s_a, s_b, no, yes);
        piped(kb + 1, s_a, s_b, t_a, t_b, no, no);
      } else {
        piped(kb, t_a, t_b, s_a, s_b, no, no);
      }
    } else {
      piped(kb, s_a, s_b, t_a, t_b, yes, no);
    }
    kb = k_hi;
  }
  for (; kb < nblk; ++kb) step(kb);
  // every copy has landed and every wavefront is done with the ring: its space takes the output tiles
  wait_loads_except<0>();
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  if (u0 >= Lc) return;
  float* lse_h = lse ? lse + hd * L : nullptr;
  if (accumulate) {
    finish_tile<__half>(O + hoff, lse_h, qrow_a, qrow_a, exists_a, sta, h, true);
    finish_tile<__half>(O + hoff, lse_h, qrow_b, qrow_b, exists_b, stb, h, true);
  } else {
    char* lds = ring + wave * (2 * CoreF16::kTileBytes);
    const int64_t left = Lc - u0;
    finish_tile_rows<__half>(O + hoff, lse_h, s * u0 + p, s, left < kTile ? (int)left : kTile, sta, lane, lds);
    if (left > kTile)
      finish_tile_rows<__half>(O + hoff, lse_h, s * (u0 + kTile) + p, s,
                               left < 2 * kTile ? (int)(left - kTile) : kTile, stb, lane,
                               lds + CoreF16::kTileBytes);
  }
}

// fp16 window masks, wide bands, d = 128: the ring of tile_window_band_kernel with key blocks of
// 128 channels.  A block is staged as four 64-channel blocks in the layout CoreF16 reads (K
// channels 0..63, K 64..127, V 0..63, V 64..127: 16 KB), once per workgroup of 128 queries; a
// wavefront owns one 32-query sub-tile and all 128 channels of it: the scores of a block are one
// chain of eight products over the two K halves, the softmax is done once, and the numerators
// meet the two V halves in eight more products (16 matrix instructions per block against the
// same vector work as at d = 64; the kernel that gives each 64-channel slice a wavefront of its
// own repeats the softmax in every slice and exchanges the partial scores through LDS).  Four
// slots, copies three blocks ahead: the barrier that opens block kb (every wavefront has waited
// for its own four copies of block kb, and is done with block kb-1) is followed by the copy of
// block kb+3 into the slot of block kb-1.
constexpr int kBand128Slots = 4;
constexpr int kBand128Ahead = 3;      // = kBand128Slots - 1

__global__ __attribute__((amdgpu_waves_per_eu(2, 2))) __launch_bounds__(256) void tile_window_band128_kernel(
    const __half* __restrict__ Q, const __half* __restrict__ K, const __half* __restrict__ V,
    __half* __restrict__ O, float* __restrict__ lse, int64_t L, int64_t W, int64_t s, int64_t n_groups,
    float scale, int accumulate, int64_t seg_len) {
  constexpr int kD = 2 * kHeadDim;
  constexpr int kWaves = 4;          // (eight wavefronts, 256 queries and two copies each per block, were slower: 2.60 against 2.55 ms at +-2048)
  constexpr int kBlk = CoreF16::kBlockBytes;
  constexpr int kSlotBytes = 4 * kBlk;
  __shared__ __attribute__((aligned(16))) char ring[kBand128Slots * kSlotBytes];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int n = lane & 31, h = lane >> 5;
  const int64_t chunk = gridDim.x / 8;
  const int64_t bid = (int64_t)(blockIdx.x % 8) * chunk + blockIdx.x / 8;
  WindowSlot slot;
  if (!locate_window_slot(bid, L, s, n_groups, seg_len, slot)) return;      // (the whole workgroup leaves)
  const int64_t p = slot.p, Lc = slot.Lc;
  const int64_t q0 = slot.grp * (kWaves * kTile);
  if (q0 >= Lc) return;
  const int64_t hd = blockIdx.y;
  const int64_t hoff = hd * L * kD;
  const int64_t u0 = q0 + (int64_t)wave * kTile;
  const int64_t vfirst = q0 - W > 0 ? q0 - W : 0;
  const int64_t vlast = q0 + kWaves * kTile - 1 + W < Lc - 1 ? q0 + kWaves * kTile - 1 + W : Lc - 1;
  const int nblk = (int)((vlast - vfirst) / kTile + 1);
  // a wavefront whose queries lie past the end of the class (u0 >= Lc) still copies and meets the
  // barriers; classify() then reports no block as its own
  const WindowBlocks src{vfirst, Lc, s, p, u0, W};
  const int64_t u = u0 + n;
  const bool exists = u < Lc;
  const int64_t qrow = s * (exists ? u : Lc - 1) + p;
  CoreF16 lo, hi;                                  // channels 0..63 and 64..127 of the same queries
  lo.load_q(Q + hoff + qrow * kD, h, scale < 0.f);
  hi.load_q(Q + hoff + qrow * kD + kHeadDim, h, scale < 0.f);
  wait_loads_except<0>();            // Q has arrived: from here on only the ring's copies are counted
  lo.q_arrived();
  hi.q_arrived();
  // this wavefront's share of a block: keys 8w .. 8w+7 of all four 64-channel blocks, eight lanes
  // of 16 bytes per 128-byte half row (the K chunks swizzled as CoreF16::read_k expects)
  constexpr int kCopies = 4;                       // copies per wavefront and block
  const int r_own = 8 * wave + (lane >> 3), c_own = lane & 7;
  const char* Kb = reinterpret_cast<const char*>(K + hoff);
  const char* Vb = reinterpret_cast<const char*>(V + hoff);
  auto issue = [&](int kb) {
    const int kc = kb < nblk ? kb : nblk - 1;
    int64_t v = vfirst + (int64_t)kc * kTile + r_own;
    v = v < Lc ? v : Lc - 1;                               // keys past the end re-read the last one (masked off)
    const int64_t row_bytes = (s * v + p) * (kD * 2);
    char* dst = ring + (kb % kBand128Slots) * kSlotBytes + wave * 1024;
    const int k_at = (c_own ^ (r_own & 7)) * 16, v_at = c_own * 16;
    copy16_to_lds_untracked(Kb + row_bytes + k_at, dst);
    copy16_to_lds_untracked(Kb + row_bytes + kHeadDim * 2 + k_at, dst + kBlk);
    copy16_to_lds_untracked(Vb + row_bytes + v_at, dst + 2 * kBlk);
    copy16_to_lds_untracked(Vb + row_bytes + kHeadDim * 2 + v_at, dst + 3 * kBlk);
  };
  TileState st, st_hi;               // m and l live in st; st_hi holds the accumulators of channels 64..127
  st.init();
  st_hi.init();
  const float c = softmax_factor(scale);
  const char* vt0 = CoreF16::vt_base(ring + 2 * kBlk, lane, h);
  // The barrier that opens block kb: every wavefront has waited for its own copies of blocks kb
  // and kb+1 (the interior steps read K of block kb+1 for the score products they issue one block
  // ahead), and everyone is done with block kb-1, whose slot takes the copy of block kb+3.
  auto publish = [&](int kb) {
    wait_loads_except<kCopies * (kBand128Ahead - 2)>();
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    issue(kb + kBand128Ahead);
  };
  // scores of block kb: one chain of eight products over the two K halves
  auto products = [&](int kb, floatx16& sv) {
    const char* ldsk = ring + (kb % kBand128Slots) * kSlotBytes;
    half8 kf[4], kg[4];
    CoreF16::read_k(ldsk, n, h, kf);
    CoreF16::read_k(ldsk + kBlk, n, h, kg);
    sv = floatx16{0};
#pragma unroll
    for (int t = 0; t < 4; ++t) sv = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[t], lo.qf[t], sv, 0, 0, 0);
#pragma unroll
    for (int t = 0; t < 4; ++t) sv = __builtin_amdgcn_mfma_f32_32x32x16_f16(kg[t], hi.qf[t], sv, 0, 0, 0);
  };
  // numerators of a block (see softmax_block_h; the accumulators of the upper channels take the
  // same factor when the running maximum is raised), then the products with the two V halves
  auto weigh = [&](int kb, floatx16& sv) {
    half8 ph[2];
    const float l_before = st.l;
    numerators_h(sv, c, st, ph);
    if (__any(sum_overflowed(st))) {
      st.l = l_before;
      const float m_before = st.m;
      rescale_state(st, block_max(sv, c, h));
      const float alpha = __builtin_amdgcn_exp2f(m_before - st.m);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        st_hi.o[0][r] *= alpha;
        st_hi.o[1][r] *= alpha;
      }
      numerators_h(sv, c, st, ph);
    }
    const char* vt = vt0 + (kb % kBand128Slots) * kSlotBytes;
#pragma unroll
    for (int uu = 0; uu < 2; ++uu) {
      const half8 a0 = CoreF16::read_va(vt, uu, 0), a1 = CoreF16::read_va(vt, uu, 1);
      const half8 b0 = CoreF16::read_va(vt + kBlk, uu, 0), b1 = CoreF16::read_va(vt + kBlk, uu, 1);
      st.o[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, ph[uu], st.o[0], 0, 0, 0);
      st.o[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, ph[uu], st.o[1], 0, 0, 0);
      st_hi.o[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(b0, ph[uu], st_hi.o[0], 0, 0, 0);
      st_hi.o[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(b1, ph[uu], st_hi.o[1], 0, 0, 0);
    }
  };
  // a block on the edge of (or outside) this wavefront's window
  auto step = [&](int kb) {
    publish(kb);
    const int cls = src.classify(kb);                      // wave-uniform
    if (cls) {
      floatx16 sv;
      products(kb, sv);
      if (cls != 2) mask_scores(sv, src.get(kb, n).word, h);
      weigh(kb, sv);
    }
  };
  // Interior blocks, software-pipelined as in tile_window_band_kernel: the score products of
  // block kb+1 are issued ahead of the exponentials and the PV products of block kb; cur holds
  // the scores of block kb on entry (first: the step computes them itself), nxt receives those of
  // block kb+1 (next: it is interior too); successive steps swap the two.
  auto piped = [&](int kb, floatx16& cur, floatx16& nxt, auto first, auto next) {
    publish(kb);
    if constexpr (decltype(first)::value) products(kb, cur);
    if constexpr (decltype(next)::value) products(kb + 1, nxt);
    weigh(kb, cur);
  };
  int k_lo = 0, k_hi = nblk;
  while (k_lo < nblk && src.classify(k_lo) != 2) ++k_lo;
  while (k_hi > k_lo && src.classify(k_hi - 1) != 2) --k_hi;
  for (int kb = 0; kb < kBand128Ahead; ++kb) issue(kb);
  int kb = 0;
  for (; kb < k_lo; ++kb) step(kb);
  if (kb < k_hi) {
    constexpr std::true_type yes{};
    constexpr std::false_type no{};
    floatx16 s_a, s_b;
    if (kb + 1 < k_hi) {
      piped(kb, s_a, s_b, yes, yes);
      ++kb;                                              // the scores of block kb are in s_b
      for (; kb + 2 < k_hi; kb += 2) {
        piped(kb, s_b, s_a, no, yes);
        piped(kb + 1, s_a, s_b, no, yes);
      }
      if (kb + 1 < k_hi) {
        piped(kb, s_b, s_a, no, yes);
        piped(kb + 1, s_a, s_b, no, no);
      } else {
        piped(kb, s_b, s_a, no, no);
      }
    } else {
      piped(kb, s_a, s_b, yes, no);
    }
    kb = k_hi;
  }
  for (; kb < nblk; ++kb) step(kb);
  // every copy has landed and every wavefront is done with the ring: its space takes the output tiles
  wait_loads_except<0>();
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  if (u0 >= Lc) return;
  const float l = st.l + other_half(st.l, h);
  const bool empty = !(l > 0.f);
  float inv = empty ? 0.f : 1.0f / l;
  float lse_row = empty ? -INFINITY : (st.m + __builtin_amdgcn_logf(l)) * kLn2;
  float* lse_h = lse ? lse + hd * L : nullptr;
  if (accumulate) {
    if (!exists) return;
    // (both half-waves read the earlier lse before the first replaces it)
    const CarryWeights cw = carry_weights(lse_h[qrow], lse_row);
    CoreF16::store_row(O + hoff + qrow * kD, st, inv * cw.w_now, cw.w_prev, true, h);
    CoreF16::store_row(O + hoff + qrow * kD + kHeadDim, st_hi, inv * cw.w_now, cw.w_prev, true, h);
    if (h == 0) lse_h[qrow] = cw.lse;
    return;
  }
  // A lane holds fragments of its own query's row; the tile goes through LDS and leaves as whole
  // 256-byte rows, four per instruction (see CoreF16T::store_tile), with streaming stores.
  constexpr int kPitch = kD * 2 + 16;
  char* tile = ring + wave * (kTile * kPitch);
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const TileState& part = half ? st_hi : st;
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w;
        w.x = __builtin_bit_cast(uint32_t, __floats2half2_rn(part.o[cb][4 * g] * inv, part.o[cb][4 * g + 1] * inv));
        w.y = __builtin_bit_cast(uint32_t,
                                 __floats2half2_rn(part.o[cb][4 * g + 2] * inv, part.o[cb][4 * g + 3] * inv));
        *reinterpret_cast<uint2*>(tile + n * kPitch + (half * kHeadDim + cb * 32 + 8 * g + 4 * h) * 2) = w;
      }
  }
  __builtin_amdgcn_wave_barrier();
  const int64_t left = Lc - u0;
  const int n_rows = left < kTile ? (int)left : kTile;
  const int64_t row0 = s * u0 + p;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = (lane >> 4) + 4 * i;
    const uint4 v = *reinterpret_cast<const uint4*>(tile + r * kPitch + (lane & 15) * 16);
    if (r < n_rows)
      __builtin_nontemporal_store(__builtin_bit_cast(half8, v),
                                  reinterpret_cast<half8*>(O + hoff + (row0 + r * s) * kD + (lane & 15) * 8));
  }
  if (lse_h && h == 0 && n < n_rows) lse_h[row0 + n * s] = lse_row;
}

// fp16 window masks narrow enough that the keys of 128 consecutive queries fit the LDS
// (128 + 2W <= 256 keys: 8 key blocks; this kernel takes the windows of up to 6 blocks, K and V
// side by side in 48 KB at most, tile_window_kv_kernel those of 7 and 8).  A workgroup owns 128 queries
// of one residue class: its four wavefronts first copy every K and V block the workgroup
// needs global -> LDS, once (wavefront w copies blocks w, w+4), and after one barrier each
// wavefront runs its own 32-query sub-tile entirely out of LDS.  Compared with one wavefront
// staging its own blocks, neighbouring sub-tiles no longer fetch the blocks they share four
// times, and the block loop holds no memory instruction and no wait.  The LDS is sized to the
// window at launch, so narrow windows run up to four workgroups per CU.  Grid mapping as in
// tile_window_kernel.
constexpr int kWgBlocks = 8;

__global__ __launch_bounds__(256) void tile_window_wg_kernel(
    const __half* __restrict__ Q, const __half* __restrict__ K, const __half* __restrict__ V,
    __half* __restrict__ O, float* __restrict__ lse, int64_t L, int64_t W, int64_t s, int64_t n_groups,
    float scale, int accumulate, int nb_max, int64_t seg_len, int64_t Lq, int64_t Lr) {
  // nb_max K blocks, then nb_max V blocks (dynamic: narrow windows leave room for more workgroups)
  extern __shared__ __attribute__((aligned(16))) char lds_wg[];
  char* lds_k = lds_wg;
  char* lds_v = lds_wg + nb_max * CoreF16::kBlockBytes;
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int n = lane & 31, h = lane >> 5;
  // The place among the window tiles as in locate_window_slot, without its 64-bit divisions
  // (each is a chain of about a hundred dependent scalar instructions ahead of the first load):
  // workgroup indices and the stride fit 32 bits (the host checks the grid size), and the host
  // passes the class lengths.  Whole-sequence masks: Lq = L / s, Lr = L % s, class p holds
  // Lq + (p < Lr) tokens.  Block-diagonal masks: Lq = tokens of the class of a whole block,
  // Lr = of the sequence's last block.
  const uint32_t chunk = gridDim.x / 8;
  const uint32_t bid = (blockIdx.x % 8) * chunk + blockIdx.x / 8;
  int64_t p, Lc, q0;                               // class start, tokens of the class, first query
  if (seg_len > 0) {
    const uint32_t ng32 = (uint32_t)n_groups;
    const uint32_t seg = bid / ng32;
    p = (int64_t)seg * seg_len;
    if (p >= L) return;
    Lc = p + seg_len <= L ? Lq : Lr;
    q0 = (int64_t)(bid - seg * ng32) * (4 * kTile);
  } else {
    if ((int64_t)bid >= n_groups * s) return;
    const uint32_t s32 = (uint32_t)s;
    const uint32_t grp = bid / s32;
    p = bid - grp * s32;                           // residue class
    Lc = Lq + (p < Lr ? 1 : 0);
    q0 = (int64_t)grp * (4 * kTile);
  }
  // (the divisions above run on the vector unit; back in scalar registers, the per-block index
  // arithmetic that follows from these values stays on the scalar unit)
  p = uniform64(p);
  Lc = uniform64(Lc);
  q0 = uniform64(q0);
  if (q0 >= Lc) return;                            // (the whole workgroup leaves: no barrier is missed)
  const int64_t hd = blockIdx.y;
  const int64_t hoff = hd * L * kHeadDim;
  const int64_t vfirst = q0 - W > 0 ? q0 - W : 0;
  const int64_t vlast = q0 + 4 * kTile - 1 + W < Lc - 1 ? q0 + 4 * kTile - 1 + W : Lc - 1;
  const int nb = (int)((vlast - vfirst) / kTile + 1);          // <= kWgBlocks
  const int64_t u0 = q0 + (int64_t)wave * kTile;
  const int64_t u = u0 + n;
  const bool exists = u < Lc;
  const int64_t qrow = s * (exists ? u : Lc - 1) + p;
  CoreF16 core;
  core.load_q(Q + hoff + qrow * kHeadDim, h, scale < 0.f);
  CoreF16::Stage sm;
  sm.init(s, lane);
  auto stage = [&](int j) {
    BlockInfo b;
    const int64_t v0 = vfirst + (int64_t)j * kTile;
    b.raw = 0;
    b.row0 = s * v0 + p;
    b.nvalid = Lc - v0 < kTile ? (int)(Lc - v0) : kTile;
    b.word = 0;
    b.full = false;
    sm.stage_k(K + hoff, b, lane, lds_k + j * CoreF16::kBlockBytes);
    sm.stage_v(V + hoff, b, lane, lds_v + j * CoreF16::kBlockBytes);
  };
  const bool active = u0 < Lc;                     // (a wavefront without queries still meets the barriers below)
  TileState st;
  st.init();
  const int64_t rem64 = Lc - vfirst, nq64 = Lc - u0;
  const WindowWordsNear src{(int)(u0 - vfirst), (int)W, (int)(nq64 > 64 ? 64 : (nq64 > 0 ? nq64 : 0)),
                            (int)(rem64 > (1 << 20) ? (1 << 20) : rem64)};
  const int64_t lo_key = u0 - W > vfirst ? u0 - W : vfirst;
  const int64_t hi_key = u0 + kTile - 1 + W < vlast ? u0 + kTile - 1 + W : vlast;
  const int k_lo = (int)((lo_key - vfirst) / kTile);
  const int k_hi = active ? (int)((hi_key - vfirst) / kTile) : k_lo - 1;
  const float c = softmax_factor(scale);
  auto blocks = [&](int ka, int kb) {
    for (int k = ka; k <= kb; ++k) {
      const BlockInfo b = src.get(k, n);
      half8 kf[4];
      CoreF16::read_k(lds_k + k * CoreF16::kBlockBytes, n, h, kf);
      core.template block_math<-1>(kf, b, c, lane, h, st, lds_v + k * CoreF16::kBlockBytes, false);
    }
  };
  for (int j = wave; j < nb; j += 4) stage(j);
  wait_loads_except<0>();
  __syncthreads();
  blocks(k_lo, k_hi);
  float* lse_h = lse ? lse + hd * L : nullptr;
  if (accumulate) {
    if (active) finish_tile<__half>(O + hoff, lse_h, qrow, qrow, exists, st, h, true);
    return;
  }
  // every wavefront is done with the staged blocks: their space takes the four output tiles
  // (at least 4 K and 4 V blocks are allocated, 32 KB)
  __syncthreads();
  if (active)
    finish_tile_rows<__half>(O + hoff, lse_h, s * u0 + p, s, Lc - u0 < kTile ? (int)(Lc - u0) : kTile, st,
                             lane, lds_wg + wave * CoreF16::kTileBytes);
}

// softmax_block_h for a caller that accumulates the PV products later: only m and l are kept
// here (st.o is not touched); the numerators of the block are taken against the m the block leaves
// behind, which the caller records.
__device__ __forceinline__ void softmax_block_deferred(floatx16 sv, float c, bool full, uint32_t word,
                                                       int h, TileState& st, half8 (&ph)[2]) {
  if (!full) mask_scores(sv, word, h);
  const float l_before = st.l;
  numerators_h(sv, c, st, ph);
  if (__any(sum_overflowed(st))) {
    const float bm = block_max(sv, c, h);
    const float m_new = needs_rescale(st, bm) ? bm : st.m;
    st.l = l_before * __builtin_amdgcn_exp2f(st.m - m_new);
    st.m = m_new;
    numerators_h(sv, c, st, ph);
  }
}

// The same windows as tile_window_wg_kernel at their widest (7 or 8 key blocks per workgroup),
// with K and V taking turns in ONE set of LDS blocks: the workgroup copies its K blocks, every
// wavefront takes the scores and softmax numerators of its sub-tile against them (numerators and
// the running max each block left behind stay in registers: at most kKvWaveBlocks blocks meet a
// 32-query sub-tile), and after a barrier the V blocks are copied over the K blocks and the PV
// products follow, O rescaled where the recorded max changes, exactly as the online form does.
// Half the LDS (32 KB for 8 blocks) and under 128 registers: four workgroups per CU instead of
// two, so that the copies of one workgroup overlap the arithmetic of three others.
// (blocks start at the workgroup's first key, W below it: sub-tile w covers blocks w .. w + (31 + 2W) / 32
// of them, and in the first workgroup of a class, where the window is cut at key 0, at most
// 2 * ceil(W / 32) + 1: five blocks at most for W <= 64)
constexpr int kKvWaveBlocks = 5;
constexpr int kKvMinBlocks = 7;     // windows of this many blocks per workgroup take this kernel

__global__ __launch_bounds__(256) void tile_window_kv_kernel(
    const __half* __restrict__ Q, const __half* __restrict__ K, const __half* __restrict__ V,
    __half* __restrict__ O, float* __restrict__ lse, int64_t L, int64_t W, int64_t s, int64_t n_groups,
    float scale, int accumulate, int nb_max, int64_t seg_len, int64_t Lq, int64_t Lr) {
  extern __shared__ __attribute__((aligned(16))) char lds_wg[];      // max(nb_max, 5) blocks
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int n = lane & 31, h = lane >> 5;
  // (placement of the workgroup among the window tiles: see tile_window_wg_kernel)
  const uint32_t chunk = gridDim.x / 8;
  const uint32_t bid = (blockIdx.x % 8) * chunk + blockIdx.x / 8;
  int64_t p, Lc, q0;
  if (seg_len > 0) {
    const uint32_t ng32 = (uint32_t)n_groups;
    const uint32_t seg = bid / ng32;
    p = (int64_t)seg * seg_len;
    if (p >= L) return;
    Lc = p + seg_len <= L ? Lq : Lr;
    q0 = (int64_t)(bid - seg * ng32) * (4 * kTile);
  } else {
    if ((int64_t)bid >= n_groups * s) return;
    const uint32_t s32 = (uint32_t)s;
    const uint32_t grp = bid / s32;
    p = bid - grp * s32;
    Lc = Lq + (p < Lr ? 1 : 0);
    q0 = (int64_t)grp * (4 * kTile);
  }
  p = uniform64(p);
  Lc = uniform64(Lc);
  q0 = uniform64(q0);
  if (q0 >= Lc) return;                            // (the whole workgroup leaves: no barrier is missed)
  const int64_t hd = blockIdx.y;
  const int64_t hoff = hd * L * kHeadDim;
  const int64_t vfirst = q0 - W > 0 ? q0 - W : 0;
  const int64_t vlast = q0 + 4 * kTile - 1 + W < Lc - 1 ? q0 + 4 * kTile - 1 + W : Lc - 1;
  const int nb = (int)((vlast - vfirst) / kTile + 1);          // <= kWgBlocks
  const int64_t u0 = q0 + (int64_t)wave * kTile;
  const int64_t u = u0 + n;
  const bool exists = u < Lc;
  const int64_t qrow = s * (exists ? u : Lc - 1) + p;
  CoreF16 core;
  core.load_q(Q + hoff + qrow * kHeadDim, h, scale < 0.f);
  CoreF16::Stage sm;
  sm.init(s, lane);
  auto block_at = [&](int j) {
    BlockInfo b;
    const int64_t v0 = vfirst + (int64_t)j * kTile;
    b.raw = 0;
    b.row0 = s * v0 + p;
    b.nvalid = Lc - v0 < kTile ? (int)(Lc - v0) : kTile;
    b.word = 0;
    b.full = false;
    return b;
  };
  const bool active = u0 < Lc;                     // (a wavefront without queries still meets the barriers below)
  const int64_t rem64 = Lc - vfirst, nq64 = Lc - u0;
  const WindowWordsNear src{(int)(u0 - vfirst), (int)W, (int)(nq64 > 64 ? 64 : (nq64 > 0 ? nq64 : 0)),
                            (int)(rem64 > (1 << 20) ? (1 << 20) : rem64)};
  const int64_t lo_key = u0 - W > vfirst ? u0 - W : vfirst;
  const int64_t hi_key = u0 + kTile - 1 + W < vlast ? u0 + kTile - 1 + W : vlast;
  const int k_lo = (int)((lo_key - vfirst) / kTile);
  const int k_hi = active ? (int)((hi_key - vfirst) / kTile) : k_lo - 1;     // k_hi - k_lo < kKvWaveBlocks
  const float c = softmax_factor(scale);
  // K blocks of the workgroup, then this sub-tile's scores and numerators
  for (int j = wave; j < nb; j += 4) sm.stage_k(K + hoff, block_at(j), lane, lds_wg + j * CoreF16::kBlockBytes);
  wait_loads_except<0>();
  __syncthreads();
  TileState st;
  st.init();
  half8 ph[kKvWaveBlocks][2];
  float m_after[kKvWaveBlocks];
#pragma unroll
  for (int j = 0; j < kKvWaveBlocks; ++j) {
    const int k = k_lo + j;
    m_after[j] = st.m;
    if (k <= k_hi) {
      const BlockInfo b = src.get(k, n);
      half8 kf[4];
      CoreF16::read_k(lds_wg + k * CoreF16::kBlockBytes, n, h, kf);
      floatx16 sacc = {0};
#pragma unroll
      for (int t = 0; t < 4; ++t) sacc = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[t], core.qf[t], sacc, 0, 0, 0);
      softmax_block_deferred(sacc, c, b.full != 0, b.word, h, st, ph[j]);
      m_after[j] = st.m;
    }
  }
  __syncthreads();                                 // every wavefront has read its K blocks
  for (int j = wave; j < nb; j += 4) sm.stage_v(V + hoff, block_at(j), lane, lds_wg + j * CoreF16::kBlockBytes);
  wait_loads_except<0>();
  __syncthreads();
  float m_run = m_after[0];
#pragma unroll
  for (int j = 0; j < kKvWaveBlocks; ++j) {
    const int k = k_lo + j;
    if (k <= k_hi) {
      if (__any(m_after[j] != m_run)) {
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_after[j]);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          st.o[0][r] *= alpha;
          st.o[1][r] *= alpha;
        }
        m_run = m_after[j];
      }
      CoreF16::accumulate(ph[j], lane, h, st, lds_wg + k * CoreF16::kBlockBytes);
    }
  }
  float* lse_h = lse ? lse + hd * L : nullptr;
  if (accumulate) {
    if (active) finish_tile<__half>(O + hoff, lse_h, qrow, qrow, exists, st, h, true);
    return;
  }
  // every wavefront is done with the staged blocks: their space takes the four output tiles
  __syncthreads();
  if (active)
    finish_tile_rows<__half>(O + hoff, lse_h, s * u0 + p, s, Lc - u0 < kTile ? (int)(Lc - u0) : kTile, st,
                             lane, lds_wg + wave * CoreF16::kTileBytes);
}

template <typename T>
sga_status run_tile_explicit_wide(const AttnArgs& a);

template <typename T>
sga_status run_tile_explicit(const AttnArgs& a) {
  if (a.d != kHeadDim) return run_tile_explicit_wide<T>(a);
  const T* Q = static_cast<const T*>(a.Q);
  const T* K = static_cast<const T*>(a.K);
  const T* V = static_cast<const T*>(a.V);
  T* O = static_cast<T*>(a.O);
  // The number of work items depends on row_ptr[L], which only the device knows: the kernels
  // stride over the items with grids sized from L alone.
  const int64_t n_tiles = (a.L + kTile - 1) / kTile;
  int64_t nwg = (n_tiles + 3) / 4 + 64;
  if (nwg > 16384) nwg = 16384;
  if (!a.prepared) launch_tile_analyze(a);
  // fp32: resident workgroups only (256 CUs x 2 wavefronts per SIMD, shared by the heads), which
  // claim items dynamically; fp16: one pass of workgroups over the items of each head
  int64_t per_head = (nwg + 8 * kXcdRun - 1) / (8 * kXcdRun) * (8 * kXcdRun);
  if (a.dtype == SGA_F32) {
    per_head = 512 / a.H;
    if (per_head < 1) per_head = 1;
    if (per_head > nwg) per_head = nwg;
  }
  // fp32 tiles keep the K fragment in registers; fp16 tiles stage K in LDS (measured best)
  const dim3 grid((unsigned)a.H, (unsigned)per_head);
  if constexpr (DtypeOf<T>::code == SGA_F16) {
    profile_mark_begin(a.stream, "tile_attend_f16_kernel");
    hipLaunchKernelGGL(tile_attend_f16_kernel, grid, dim3(256), 0, a.stream, Q, K, V, O, a.lse, a.row_ptr,
                       a.L, a.scale, a.ws, a.ws_bytes, a.accumulate ? 1 : 0);
  } else {
    profile_mark_begin(a.stream, "tile_attend_kernel");
    auto kernel = a.split ? tile_attend_kernel<T, kPipeSplit> : tile_attend_kernel<T, kPipeRegK>;
    hipLaunchKernelGGL(kernel, grid, dim3(256), 0, a.stream, Q, K, V, O, a.lse, a.row_ptr, a.L, a.scale, a.ws,
                       a.ws_bytes, a.accumulate ? 1 : 0);
  }
  profile_mark_end(a.stream);
  // (a prepared graph knows whether any tile was cut into segments)
  if (!a.prepared || a.plan_multi_tiles > 0)
    hipLaunchKernelGGL((tile_merge_kernel<T, kHeadDim>), dim3(16, (unsigned)a.H, kTile), dim3(256), 0,
                       a.stream, O, a.lse, a.row_ptr, a.L, a.ws, a.ws_bytes, a.accumulate ? 1 : 0);
  return hip_status(hipGetLastError());
}

template <typename T, int kD>
sga_status run_tile_explicit_wide_d(const AttnArgs& a) {
  const T* Q = static_cast<const T*>(a.Q);
  const T* K = static_cast<const T*>(a.K);
  const T* V = static_cast<const T*>(a.V);
  T* O = static_cast<T*>(a.O);
  constexpr int kSlices = kD / kHeadDim;
  const int64_t n_tiles = (a.L + kTile - 1) / kTile;
  if (!a.prepared) launch_tile_analyze(a);
  // resident workgroups (2 wavefronts per SIMD over the chip), shared by the heads
  int64_t per_head = (2048 / kSlices) / a.H;
  if (per_head < 1) per_head = 1;
  if (per_head > n_tiles + 64) per_head = n_tiles + 64;
  constexpr int kPipe = DtypeOf<T>::code == SGA_F16 ? kPipeLdsK : kPipeRegK;
  if constexpr (DtypeOf<T>::code == SGA_F16 && kD == 128) {
    // one wavefront per item with all 128 channels; two workgroups of four wavefronts per CU
    int64_t wgs = 512 / a.H;
    if (wgs < 1) wgs = 1;
    if (wgs > (n_tiles + 3) / 4 + 16) wgs = (n_tiles + 3) / 4 + 16;
    profile_mark_begin(a.stream, "tile_attend128_f16_kernel");
    hipLaunchKernelGGL(tile_attend128_f16_kernel, dim3((unsigned)a.H, (unsigned)wgs), dim3(256), 0, a.stream, Q, K,
                       V, O, a.lse, a.row_ptr, a.L, a.scale, a.ws, a.ws_bytes, a.accumulate ? 1 : 0);
  } else {
    profile_mark_begin(a.stream, "tile_attend_wide_kernel");
    hipLaunchKernelGGL((tile_attend_wide_kernel<T, kD, kPipe>), dim3((unsigned)a.H, (unsigned)per_head),
                       dim3(kD), 0, a.stream, Q, K, V, O, a.lse, a.row_ptr, a.L, a.scale, a.ws, a.ws_bytes,
                       a.accumulate ? 1 : 0);
  }
  profile_mark_end(a.stream);
  if (!a.prepared || a.plan_multi_tiles > 0)
    hipLaunchKernelGGL((tile_merge_kernel<T, kD>), dim3(16, (unsigned)a.H, kTile), dim3(256), 0, a.stream,
                       O, a.lse, a.row_ptr, a.L, a.ws, a.ws_bytes, a.accumulate ? 1 : 0);
  return hip_status(hipGetLastError());
}

template <typename T>
sga_status run_tile_explicit_wide(const AttnArgs& a) {
  if (a.d == 128) return run_tile_explicit_wide_d<T, 128>(a);
  if (a.d == 256) return run_tile_explicit_wide_d<T, 256>(a);
  return SGA_ERR_UNSUPPORTED;
}

// Shape of a window launch: the classes the tiles are dealt over (residue classes of the whole
// sequence, or one class per block of a 2-D dilated mask) and the longest class.
struct WindowShape {
  int64_t seg_len;   // 0, or the block length of a 2-D dilated mask
  int64_t n_slots;   // residue classes, or blocks
  int64_t Lc;        // tokens of the longest class
};
WindowShape window_shape(const AttnArgs& a) {
  WindowShape w;
  if (a.mask_kind == SGA_MASK_DILATED_2D) {
    const int64_t span = a.block < a.L ? a.block : a.L;
    w.seg_len = a.block;
    w.n_slots = (a.L + a.block - 1) / a.block;
    w.Lc = (span + a.stride - 1) / a.stride;
  } else {
    w.seg_len = 0;
    w.n_slots = a.stride;
    w.Lc = (a.L + a.stride - 1) / a.stride;
  }
  return w;
}

// 2-D dilated masks: rows off the stride have no neighbour; a forward call writes their initial
// state, a continuing call leaves them as they are.
template <typename T>
void clear_unselected_rows(const AttnArgs& a) {
  if (a.mask_kind != SGA_MASK_DILATED_2D || a.stride == 1 || a.accumulate) return;
  const int64_t chunks = (int64_t)a.H * a.L * (a.d * (int64_t)sizeof(T) / 16);
  int64_t nwg = (chunks + 255) / 256;
  if (nwg > 8192) nwg = 8192;
  hipLaunchKernelGGL(clear_unselected_rows_kernel<T>, dim3((unsigned)nwg), dim3(256), 0, a.stream,
                     static_cast<T*>(a.O), a.lse, a.L, (int64_t)a.H, a.d, (int64_t)a.block,
                     (int64_t)a.stride);
}

// A window call with few tiles and many key blocks per tile (a short sequence with a wide
// window, one head) is cut into ranges of at least 16 key blocks per tile.  The chip runs
// `resident` tiles at a time, so k ranges cost about ceil(tiles * k / resident) rounds of
// ceil(blocks / k) blocks each, plus the partial states and their merge (taken as 4 blocks per
// range): the cheapest k <= kMaxWindowSplit wins.  The partial states go to the workspace; without
// room for them (or without a workspace) the call is not cut.  Returns k and sets *parts.
int choose_window_split(const AttnArgs& a, int64_t tile_heads, int64_t resident, float** parts) {
  *parts = nullptr;
  const int64_t blocks_per_tile = (2 * (int64_t)a.window + kTile - 1) / kTile + 1;
  if (!a.ws || tile_heads >= 4 * resident || blocks_per_tile < 32) return 1;
  const WorkspacePlan pl = plan_workspace(a.L, a.H, -1, a.dtype, a.d);
  if (pl.total_bytes > a.ws_bytes || tile_heads > pl.cap_wparts) return 1;
  int64_t want = 1, best = blocks_per_tile * ((tile_heads + resident - 1) / resident);
  for (int64_t k = 2; k <= kMaxWindowSplit && blocks_per_tile / k >= 16; ++k) {
    const int64_t cost = (tile_heads * k + resident - 1) / resident * ((blocks_per_tile + k - 1) / k) + 4 * k;
    if (cost < best) {
      best = cost;
      want = k;
    }
  }
  if (want > 1) *parts = reinterpret_cast<float*>(static_cast<char*>(a.ws) + pl.off_wparts);
  return (int)want;
}

template <typename T, int kD>
sga_status run_tile_implicit_wide_d(const AttnArgs& a) {
  const int64_t s = a.stride;
  const WindowShape shape = window_shape(a);
  const int64_t n_tiles = (shape.Lc + kTile - 1) / kTile;     // workgroups per class
  const int64_t n_wg = (n_tiles * shape.n_slots + 7) / 8 * 8;
  if (n_wg >= (int64_t(1) << 31)) return SGA_ERR_OVERFLOW;
  constexpr int kPipe = DtypeOf<T>::code == SGA_F16 ? kPipeLdsK : kPipeRegK;
  constexpr int kSlices = kD / kHeadDim;
  clear_unselected_rows<T>(a);
  const int acc = a.accumulate ? 1 : 0;
  if constexpr (DtypeOf<T>::code == SGA_F16 && kD == 128) {
    // wide bands on a call with workgroups enough to fill the chip: one wavefront per 32 queries
    // with all 128 channels, key blocks staged once per 128 queries
    const int64_t n_groups = (n_tiles + 3) / 4;
    const int64_t n_wg128 = (n_groups * shape.n_slots + 7) / 8 * 8;
    if (n_groups * shape.n_slots * a.H >= 512) {
      profile_mark_begin(a.stream, "tile_window_band128_kernel");
      hipLaunchKernelGGL(tile_window_band128_kernel, dim3((unsigned)n_wg128, (unsigned)a.H), dim3(256), 0, a.stream,
                         static_cast<const __half*>(a.Q), static_cast<const __half*>(a.K),
                         static_cast<const __half*>(a.V), static_cast<__half*>(a.O), a.lse, a.L,
                         (int64_t)a.window, s, n_groups, a.scale, acc, shape.seg_len);
      profile_mark_end(a.stream);
      return hip_status(hipGetLastError());
    }
  }
  float* parts = nullptr;
  const int nsplit = choose_window_split(a, n_wg * a.H, 2048 / kSlices, &parts);
  profile_mark_begin(a.stream, "tile_window_wide_kernel");
  hipLaunchKernelGGL((tile_window_wide_kernel<T, kD, kPipe>), dim3((unsigned)(n_wg * nsplit), (unsigned)a.H),
                     dim3(kD), 0, a.stream, static_cast<const T*>(a.Q), static_cast<const T*>(a.K),
                     static_cast<const T*>(a.V), static_cast<T*>(a.O), a.lse, a.L, (int64_t)a.window, s,
                     n_tiles, a.scale, acc, shape.seg_len, nsplit, parts);
  profile_mark_end(a.stream);
  if (nsplit > 1)
    hipLaunchKernelGGL((window_merge_kernel<T, kD>), dim3((unsigned)n_wg, (unsigned)a.H, 4), dim3(kD), 0, a.stream,
                       static_cast<T*>(a.O), a.lse, parts, a.L, s, n_tiles, acc, shape.seg_len, nsplit);
  return hip_status(hipGetLastError());
}

template <typename T>
sga_status run_tile_implicit_wide(const AttnArgs& a) {
  if (a.d == 128) return run_tile_implicit_wide_d<T, 128>(a);
  if (a.d == 256) return run_tile_implicit_wide_d<T, 256>(a);
  return SGA_ERR_UNSUPPORTED;
}

sga_status run_tile_implicit(const AttnArgs& a) {
  if (a.d != kHeadDim)
    return a.dtype == SGA_F32 ? run_tile_implicit_wide<float>(a) : run_tile_implicit_wide<__half>(a);
  const int64_t s = a.stride;
  const WindowShape shape = window_shape(a);
  const int64_t Lc = shape.Lc;
  // fp16, 128 queries' key range fits the LDS: one workgroup stages it once (128 queries per
  // workgroup, as in the fp32 kernel); wider fp16 windows: 64 queries per wavefront
  const bool wg = a.dtype == SGA_F16 && 4 * kTile + 2 * (int64_t)a.window <= kWgBlocks * kTile;
  const bool pair = a.dtype == SGA_F16 && !wg;
  const int64_t per_wave = pair ? 2 * kTile : kTile;
  const int64_t n_tiles = (Lc + per_wave - 1) / per_wave;
  const int64_t n_groups = (n_tiles + 3) / 4;           // workgroups per class
  const int64_t n_wg = (n_groups * shape.n_slots + 7) / 8 * 8;
  if (n_wg >= (int64_t(1) << 31)) return SGA_ERR_OVERFLOW;
  const dim3 grid((unsigned)n_wg, (unsigned)a.H);
  const int acc = a.accumulate ? 1 : 0;
  if (a.dtype == SGA_F32) clear_unselected_rows<float>(a); else clear_unselected_rows<__half>(a);
  const int nb_max = (int)((4 * kTile - 1 + 2 * (int64_t)a.window) / kTile + 1);   // key blocks of 128 queries
  const bool kv = wg && nb_max >= kKvMinBlocks;
  profile_mark_begin(a.stream, kv ? "tile_window_kv_kernel" : wg ? "tile_window_wg_kernel"
                               : pair ? "tile_window_band_kernel" : "tile_window_kernel");
  if (wg) {
    int64_t Lq = a.L / s, Lr = a.L % s;             // class lengths, see the kernel
    if (shape.seg_len > 0) {
      const int64_t last_len = a.L - (a.L - 1) / shape.seg_len * shape.seg_len;
      Lq = (shape.seg_len + s - 1) / s;
      Lr = (last_len + s - 1) / s;
    }
    if (kv)
      hipLaunchKernelGGL(tile_window_kv_kernel, grid, dim3(256), (size_t)(nb_max > 5 ? nb_max : 5) * CoreF16::kBlockBytes,
                         a.stream, static_cast<const __half*>(a.Q), static_cast<const __half*>(a.K),
                         static_cast<const __half*>(a.V), static_cast<__half*>(a.O), a.lse, a.L,
                         (int64_t)a.window, s, n_groups, a.scale, acc, nb_max, shape.seg_len, Lq, Lr);
    else
      hipLaunchKernelGGL(tile_window_wg_kernel, grid, dim3(256), (size_t)nb_max * 2 * CoreF16::kBlockBytes,
                         a.stream, static_cast<const __half*>(a.Q), static_cast<const __half*>(a.K),
                         static_cast<const __half*>(a.V), static_cast<__half*>(a.O), a.lse, a.L,
                         (int64_t)a.window, s, n_groups, a.scale, acc, nb_max, shape.seg_len, Lq, Lr);
  } else if (pair) {
    hipLaunchKernelGGL(tile_window_band_kernel, grid, dim3(256), 0, a.stream,
                       static_cast<const __half*>(a.Q), static_cast<const __half*>(a.K),
                       static_cast<const __half*>(a.V), static_cast<__half*>(a.O), a.lse, a.L,
                       (int64_t)a.window, s, n_groups, a.scale, acc, shape.seg_len);
  } else {
    float* parts = nullptr;
    const int nsplit = choose_window_split(a, n_wg * 4 * a.H, 2048, &parts);
    auto kernel = a.split ? tile_window_kernel<float, kPipeSplit> : tile_window_kernel<float, kPipeRegK>;
    hipLaunchKernelGGL(kernel, dim3((unsigned)(n_wg * nsplit), (unsigned)a.H), dim3(256), 0, a.stream,
                       static_cast<const float*>(a.Q), static_cast<const float*>(a.K),
                       static_cast<const float*>(a.V), static_cast<float*>(a.O), a.lse, a.L,
                       (int64_t)a.window, s, n_groups, a.scale, acc, shape.seg_len, nsplit, parts);
    if (nsplit > 1) {
      profile_mark_end(a.stream);
      hipLaunchKernelGGL((window_merge_kernel<float, kHeadDim>), dim3((unsigned)(n_wg * 4), (unsigned)a.H, 4),
                         dim3(kHeadDim), 0, a.stream, static_cast<float*>(a.O), a.lse, parts, a.L, s, n_groups,
                         acc, shape.seg_len, nsplit);
      return hip_status(hipGetLastError());
    }
  }
  profile_mark_end(a.stream);
  return hip_status(hipGetLastError());
}

}  // namespace

// The CSR -> tile pass is a chain of dependent loads per item: one wavefront per tile and a
// margin for the extra segments keeps every item's chain in flight at once.
void launch_tile_analyze(const AttnArgs& a) {
  const int64_t n_tiles = (a.L + kTile - 1) / kTile;
  int64_t nwg_analyze = n_tiles + 64;
  if (nwg_analyze < 2048) nwg_analyze = 2048;
  if (nwg_analyze > 16384) nwg_analyze = 16384;
  hipLaunchKernelGGL(tile_analyze_kernel, dim3((unsigned)nwg_analyze), dim3(256), 0, a.stream, a.row_ptr,
                     a.col_idx, a.L, a.H, a.dtype, a.d, a.ws, a.ws_bytes);
}

sga_status launch_tile_explicit(const AttnArgs& a) {
  if (!a.ws || a.ws_bytes < 256) return launch_gather_explicit(a, false, false);
  // (a prepared graph in which no tile qualified goes straight to the per-row kernels)
  if (!(a.prepared && a.plan_no_tiles)) {
    const sga_status st = a.dtype == SGA_F32 ? run_tile_explicit<float>(a) : run_tile_explicit<__half>(a);
    if (st != SGA_OK) return st;
  }
  if (a.prepared && a.plan_tiles_cover_all) return SGA_OK;
  // rows of tiles that did not qualify (or everything, if the workspace is too small)
  return launch_gather_explicit(a, true, true);
}

namespace {
template <typename T>
void run_tile_nonlocal(const AttnArgs& a, int64_t g, float* partials, int32_t* n_chunks) {
  constexpr int kPipe = DtypeOf<T>::code == SGA_F16 ? kPipeLdsK : kPipeRegK;
  const T* Q = static_cast<const T*>(a.Q);
  const T* K = static_cast<const T*>(a.K);
  const T* V = static_cast<const T*>(a.V);
  const int acc = a.accumulate ? 1 : 0;
  const int64_t first_tile = g / kTile, n_tiles = (a.L + kTile - 1) / kTile;
  if (n_tiles > first_tile && a.L > g) {
    profile_mark_begin(a.stream, "tile_nonlocal_cols_kernel");
    hipLaunchKernelGGL((tile_nonlocal_cols_kernel<T, kPipe>), dim3((unsigned)((n_tiles - first_tile + 3) / 4), (unsigned)a.H),
                       dim3(256), 0, a.stream, Q, K, V, static_cast<T*>(a.O), a.lse, a.L, (int64_t)a.window, g,
                       a.scale, acc);
    profile_mark_end(a.stream);
  }
  *n_chunks = 0;
  if (g > 0) {
    // ranges of at least 8 key blocks, as many as the partial states of the workspace allow
    // (kMaxImplicitGlobal rows x kMaxSplit ranges in all: fewer global rows, more ranges each)
    const int64_t g_rows = (g + kTile - 1) / kTile * kTile;
    int64_t max_ranges = (int64_t)kMaxImplicitGlobal * kMaxSplit / g_rows;
    if (max_ranges > 256) max_ranges = 256;
    int64_t per = (n_tiles + max_ranges - 1) / max_ranges;
    if (per < 8) per = 8;
    const int64_t ranges = (n_tiles + per - 1) / per;
    *n_chunks = (int32_t)ranges;
    hipLaunchKernelGGL((tile_nonlocal_rows_kernel<T, kPipe>),
                       dim3((unsigned)ranges, (unsigned)((g + kTile - 1) / kTile), (unsigned)a.H), dim3(64), 0, a.stream,
                       Q, K, V, a.L, (int64_t)a.window, g, per, a.scale, partials);
  }
}
}  // namespace

namespace {
template <typename T, int kD>
void run_tile_nonlocal_wide(const AttnArgs& a, int64_t g, float* partials, int32_t* n_chunks) {
  constexpr int kPipe = DtypeOf<T>::code == SGA_F16 ? kPipeLdsK : kPipeRegK;
  const T* Q = static_cast<const T*>(a.Q);
  const T* K = static_cast<const T*>(a.K);
  const T* V = static_cast<const T*>(a.V);
  const int acc = a.accumulate ? 1 : 0;
  const int64_t first_tile = g / kTile, n_tiles = (a.L + kTile - 1) / kTile;
  if (n_tiles > first_tile && a.L > g) {
    profile_mark_begin(a.stream, "tile_nonlocal_cols_wide_kernel");
    hipLaunchKernelGGL((tile_nonlocal_cols_wide_kernel<T, kD, kPipe>), dim3((unsigned)(n_tiles - first_tile), (unsigned)a.H),
                       dim3(kD), 0, a.stream, Q, K, V, static_cast<T*>(a.O), a.lse, a.L, (int64_t)a.window, g, a.scale,
                       acc);
    profile_mark_end(a.stream);
  }
  *n_chunks = 0;
  if (g > 0) {
    const int64_t g_rows = (g + kTile - 1) / kTile * kTile;
    int64_t max_ranges = (int64_t)kMaxImplicitGlobal * kMaxSplit / g_rows;
    if (max_ranges > 256) max_ranges = 256;
    int64_t per = (n_tiles + max_ranges - 1) / max_ranges;
    if (per < 8) per = 8;
    const int64_t ranges = (n_tiles + per - 1) / per;
    *n_chunks = (int32_t)ranges;
    hipLaunchKernelGGL((tile_nonlocal_rows_wide_kernel<T, kD, kPipe>),
                       dim3((unsigned)ranges, (unsigned)((g + kTile - 1) / kTile), (unsigned)a.H), dim3(kD), 0, a.stream,
                       Q, K, V, a.L, (int64_t)a.window, g, per, a.scale, partials);
  }
}
}  // namespace

void launch_tile_nonlocal(const AttnArgs& a, int64_t g, float* partials, int32_t* n_chunks) {
  if (a.d == 128) {
    if (a.dtype == SGA_F32) run_tile_nonlocal_wide<float, 128>(a, g, partials, n_chunks);
    else run_tile_nonlocal_wide<__half, 128>(a, g, partials, n_chunks);
  } else if (a.d == 256) {
    if (a.dtype == SGA_F32) run_tile_nonlocal_wide<float, 256>(a, g, partials, n_chunks);
    else run_tile_nonlocal_wide<__half, 256>(a, g, partials, n_chunks);
  } else {
    if (a.dtype == SGA_F32) run_tile_nonlocal<float>(a, g, partials, n_chunks);
    else run_tile_nonlocal<__half>(a, g, partials, n_chunks);
  }
}

sga_status launch_tile_implicit(const AttnArgs& a) {
  // (the tile kernels keep per-lane byte offsets of up to 31 keys in 32 bits, which bounds the
  // distance between consecutive keys of a class to 2^27 bytes)
  const int64_t key_bytes = (int64_t)a.stride * a.d * (a.dtype == SGA_F32 ? 4 : 2);
  if (a.H > 65535 || key_bytes > (int64_t(1) << 27)) return launch_gather_implicit(a);
  return run_tile_implicit(a);
}

}  // namespace sga
