/*
 * sga -- sparse graph attention for AMD MI355X (gfx950).  C ABI of libsga.so.
 *
 * The library computes masked attention as a graph computation (Section IV of
 * "Longer Attention Span: Increasing Transformer Context Length with Sparse
 * Graph Processing Techniques"): tokens are vertices carrying (Q_i, K_i, V_i),
 * the 0/1 attention mask A (rows = queries, columns = keys) is the edge set,
 * and for every query row i only the edges (i, j) with A_ij = 1 are visited
 * (Algorithm 1): W = scale * (Q_i . K_j), a numerically stable running softmax
 * over the row's neighbours, and the softmax-weighted sum of the V_j rows.
 *
 * Conventions that hold for every entry point
 *   - Pointers marked "device" are device (HBM) addresses owned by the caller;
 *     pointers marked "host" are ordinary host addresses.  The library never
 *     allocates, frees or retains memory and keeps no state between calls (the
 *     benchmark hook sga_profile_* at the end of this header is the one exception).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work on it and return without synchronising the host.
 *   - Argument errors are detected on the host before anything is enqueued and
 *     reported as a negative sga_status; nothing is thrown.  HIP launch errors
 *     map to SGA_ERR_HIP.
 *   - Tensors Q, K, V, O are [H][L][d] row-major (one contiguous L x d matrix per
 *     head: the single-head problem of Algorithm 1 repeated H times with one
 *     shared mask).  Storage is fp32 or IEEE fp16; all arithmetic accumulates in
 *     fp32; an fp16 output is rounded once (to nearest even) at the store.
 *   - CSR: row_ptr is int64 [L+1] (edge counts can pass 2^31), col_idx is int32
 *     [nnz] (L < 2^31).  row_ptr[0] = 0, non-decreasing; within a row col_idx is
 *     strictly increasing and in [0, L).  Duplicate or out-of-range columns are
 *     undefined behaviour of the forward.
 *   - A row with no neighbour yields O_i = 0 and lse_i = -inf (the initial state
 *     of Algorithm 1: O = 0, l = 0, m = -inf).
 *   - Supported head dimensions: d = 64, 128 and 256 on every path (the sizes of the paper's
 *     microbenchmark runs, Section V-C; the MFMA tile kernels work on 64-channel slices, one
 *     wavefront per slice), and d = 32 (the size of the verification runs, Section V-A) on the
 *     per-row kernels only (SGA_PATH_AUTO selects them; SGA_PATH_TILE returns
 *     SGA_ERR_UNSUPPORTED).  SGA_PATH_TILE_SPLIT: d = 64.
 */
#ifndef SGA_H_
#define SGA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SGA_OK = 0,
  SGA_ERR_INVALID_ARG = -1,
  SGA_ERR_UNSUPPORTED = -2,
  SGA_ERR_WORKSPACE = -3,
  SGA_ERR_OVERFLOW = -4,
  SGA_ERR_HIP = -5
} sga_status;

/* Storage type of Q, K, V and O.  Accumulation is always fp32. */
typedef enum { SGA_F32 = 0, SGA_F16 = 1 } sga_dtype;

/* Mask families of Section II-C. */
typedef enum {
  SGA_MASK_SLIDING = 0,      /* local window:   |i-j| <= window                          */
  SGA_MASK_DILATED = 1,      /* 1-D dilated:    (i-j) mod stride == 0, |i-j| <= window*stride
                                (the paper's dilation factor r is stride-1)               */
  SGA_MASK_GLOBAL_LOCAL = 2, /* local window plus global tokens 0..n_global-1, symmetric:
                                |i-j| <= window  or  i < n_global  or  j < n_global       */
  SGA_MASK_BIGBIRD = 3,      /* block mask (block x block tiles, L % block == 0):
                                query blocks 0..n_global_blocks-1 attend every key block;
                                every other query block b attends the global key blocks,
                                key blocks b-window_blocks..b+window_blocks, and
                                n_random_blocks further distinct key blocks chosen by the
                                counter-based generator described at sga_build_mask      */
  SGA_MASK_NONLOCAL = 4,     /* "global (non-local)" of Section IV-B: the global mask with the
                                local window taken out, (i < n_global or j < n_global) and
                                |i-j| > window; together with SGA_MASK_SLIDING it partitions
                                SGA_MASK_GLOBAL_LOCAL (see sga_attention_accumulate)       */
  SGA_MASK_DILATED_2D = 5    /* 2-D dilated blocks (Section II-C): i and j in the same block of
                                `block` consecutive tokens, and both in-block indices
                                multiples of stride (the paper's r is stride-1); rows whose
                                in-block index is no multiple of stride have no neighbour  */
} sga_mask_kind;

/* Attention-specific parameters P_a of Algorithm 1.  Plain data, host memory. */
typedef struct {
  uint32_t struct_bytes;     /* = sizeof(sga_mask_desc); rejects mismatched layouts       */
  int32_t kind;              /* sga_mask_kind                                             */
  int64_t L;                 /* context length, 1 <= L < 2^31                             */
  int32_t window;            /* half-width in steps, >= 0                                 */
  int32_t stride;            /* >= 1; DILATED and DILATED_2D read it (others: stride 1)   */
  int32_t n_global;          /* GLOBAL_LOCAL, NONLOCAL: 0 <= n_global <= L                */
  int32_t block;             /* BIGBIRD: block edge in tokens, 1..1024; DILATED_2D: >= 1  */
  int32_t window_blocks;     /* BIGBIRD                                                   */
  int32_t n_global_blocks;   /* BIGBIRD                                                   */
  int32_t n_random_blocks;   /* BIGBIRD: 0..16; needs L/block >= 2*window_blocks+1
                                + n_global_blocks + n_random_blocks                       */
  uint64_t seed;             /* BIGBIRD                                                   */
} sga_mask_desc;

/* Which kernels the forward may use (tests pin one; callers pass SGA_PATH_AUTO). */
typedef enum {
  SGA_PATH_AUTO = 0,    /* tile path where the mask is block-dense enough, gather elsewhere */
  SGA_PATH_GATHER = 1,  /* one wavefront per query row, per-edge K/V row gathers           */
  SGA_PATH_TILE = 2,    /* 32x32 MFMA tiles with per-tile bit masks; rows whose tile does
                           not qualify still go through the gather kernels                */
  SGA_PATH_TILE_SPLIT = 3 /* SGA_PATH_TILE for fp32 storage with the products evaluated on the
                           fp16 matrix cores: every fp32 operand x is split into fp16(x) and an
                           fp16 remainder, and a.b becomes three fp16 products accumulated in
                           fp32 (the "tensor cores" direction named under Limitations and Future Directions, kept
                           at fp32 accuracy: the dropped terms are below 2^-23 |a.b|).  Opt-in:
                           inputs must lie inside the fp16 range, |x| < 65504; SGA_F32 and
                           d = 64 only (else SGA_ERR_UNSUPPORTED)                          */
} sga_path;

const char* sga_status_string(sga_status s);

/*
 * Edge count of a mask in closed form (NNZ of the sparsity factor S_f = NNZ/L^2,
 * Section II-D).  desc: host.  nnz_out: host.  No device work.
 * Errors: SGA_ERR_INVALID_ARG for a null pointer, wrong struct_bytes or parameters
 * outside the ranges stated at sga_mask_desc.
 */
sga_status sga_mask_nnz(const sga_mask_desc* desc, int64_t* nnz_out);

/*
 * Mask -> graph (explicit form of Get_Neighbors, Section IV-B "CSR"): writes
 * the CSR of the mask, row offsets and sorted column indices; the mask is
 * binary so no values vector exists.
 *   row_ptr  device, int64 [L+1], written
 *   col_idx  device, int32 [col_capacity], the first nnz entries are written
 *   col_capacity must be >= the count sga_mask_nnz returns (else SGA_ERR_WORKSPACE).
 * Random key blocks of SGA_MASK_BIGBIRD: with mix64 the splitmix64 output
 * function and GOLD = 0x9E3779B97F4A7C15, query block b owns the stream key
 * mix64(seed + GOLD*(b+1)); attempts a = 0, 1, 2, ... propose key block
 * mix64(key + GOLD*(a+1)) mod (L/block), rejected when that block is already
 * attended (window, global or an earlier pick), until n_random_blocks are taken.
 * The result is bit-reproducible: one correct byte image per desc.
 */
sga_status sga_build_mask(const sga_mask_desc* desc, int64_t* row_ptr, int32_t* col_idx,
                          int64_t col_capacity, void* stream);

/*
 * Checks what the forward calls assume of an explicit mask (Section IV-B "CSR": row offsets
 * and sorted column indices of a binary mask) and do not check themselves: row_ptr[0] = 0,
 * row_ptr non-decreasing, row_ptr[L] <= col_capacity, every column in [0, L), the columns of a
 * row strictly increasing (no duplicates).  A forward call on arrays that break this reads
 * outside K and V or counts an edge twice.
 *   row_ptr       device, int64 [L+1], read
 *   col_idx       device, int32 [col_capacity], the first row_ptr[L] entries are read
 *   scratch       device, at least 16 bytes, 8-byte aligned, overwritten (the start of a
 *                 workspace will do; its contents are lost)
 *   bad_row_out   host, may be null: -1 if the arrays are valid, else the smallest row that
 *                 breaks the contract (L if row_ptr[0] or row_ptr[L] does)
 * Enqueues three small kernels on `stream` and waits for them (it returns a verdict).
 * Returns SGA_OK (valid), SGA_ERR_INVALID_ARG (null pointer, L < 1 or >= 2^31, negative
 * capacity, or the contract is broken), SGA_ERR_HIP.
 */
sga_status sga_validate_csr(const int64_t* row_ptr, const int32_t* col_idx, int64_t L,
                            int64_t col_capacity, void* scratch, int64_t* bad_row_out, void* stream);

/*
 * Workspace size the forward calls can use for the given problem.
 *   nnz: edge count of the explicit mask, or -1 for the implicit entry point.
 * bytes_out (host) receives a size that is sufficient for every path; a smaller
 * (or null) workspace is legal and only disables the split-row and tile paths.
 */
sga_status sga_workspace_bytes(int64_t L, int32_t H, int32_t d, int32_t dtype, int64_t nnz,
                               size_t* bytes_out);

/*
 * Algorithm 1 over an explicit CSR mask (Section IV-B): for every head h and row i
 *   O[h][i] = sum_j softmax_j( scale * Q[h][i].K[h][j] ) V[h][j],  j in col_idx[row_ptr[i]..row_ptr[i+1])
 * with the running-max / running-sum recurrence of Algorithm 1 (any evaluation
 * order of the recurrence gives the same real number; results are deterministic
 * run to run for a given workspace size).
 *   Q, K, V   device, [H][L][d], dtype storage, read only
 *   row_ptr   device, int64 [L+1];  col_idx  device, int32 [row_ptr[L]]
 *   O         device, [H][L][d], dtype storage, written
 *   scale     multiplies the fp32 dot product (Eq. 1 uses 1/sqrt(d_k))
 *   dtype     sga_dtype
 *   lse       device, float [H][L], optional (NULL): m_i + ln l_i of the row
 *   workspace device, 256-byte aligned, optional (NULL): partial states of split
 *             high-degree rows and per-tile block lists.  Its contents need not be
 *             preserved between calls; concurrent calls need separate workspaces.
 *   path      sga_path
 * Errors: SGA_ERR_INVALID_ARG (null pointer, L < 1 or >= 2^31, H < 1 or > 65535 (heads are a
 * grid dimension), unknown dtype/path, misaligned pointers), SGA_ERR_UNSUPPORTED (d not in {32, 64, 128, 256}, or
 * SGA_PATH_TILE with d != 64),
 * SGA_ERR_WORKSPACE (path = SGA_PATH_TILE without a sufficient workspace).
 */
sga_status sga_attention_forward(const void* Q, const void* K, const void* V,
                                 const int64_t* row_ptr, const int32_t* col_idx, void* O,
                                 int64_t L, int32_t H, int32_t d, float scale, void* stream,
                                 int32_t dtype, float* lse, void* workspace,
                                 size_t workspace_bytes, int32_t path);

/*
 * Algorithm 1 with an implicit mask (Section IV-B "Local", "1D Dilation"): the
 * neighbours of row i are computed from desc inside the kernel (index
 * arithmetic, no stored graph), so memory stays O(L) and L is bounded only by
 * Q, K, V, O themselves.  Supports SGA_MASK_SLIDING and SGA_MASK_DILATED (tile and
 * gather kernels), SGA_MASK_DILATED_2D ("2D Dilation") and SGA_MASK_NONLOCAL ("Global
 * (non-local)"; n_global <= 64 and a workspace of sga_workspace_bytes(..., nnz = -1) are
 * required: the global rows are split over the key range) through the per-row kernels;
 * other kinds return SGA_ERR_UNSUPPORTED (build their CSR instead).
 * The workspace is optional for the window masks; with one of sga_workspace_bytes(..., nnz = -1)
 * bytes, calls with few query tiles and wide windows (short sequences; fp32 at d = 64, both
 * types at d = 128 and 256) split each tile's key range over several wavefronts and merge the
 * partial states in key order.
 * Arguments as in sga_attention_forward; desc: host; desc->L must equal L.
 * Element offsets are 64-bit (L*d may pass 2^31).
 */
sga_status sga_attention_forward_implicit(const void* Q, const void* K, const void* V,
                                          const sga_mask_desc* desc, void* O, int64_t L,
                                          int32_t H, int32_t d, float scale, void* stream,
                                          int32_t dtype, float* lse, void* workspace,
                                          size_t workspace_bytes, int32_t path);

/*
 * Sequential composition on one shared state (Section V-F: a local, a global and a CSR kernel run
 * one after another on the same O, l, m of Algorithm 1).  These two entry points visit the
 * edges of their mask like the forward calls, but start from the state already held in O and
 * lse instead of Algorithm 1's initial state, and leave the continued state there:
 *   O    device, [H][L][d], read and written: the normalised output over the edges visited so far
 *   lse  device, float [H][L], required, read and written: m_i + ln l_i over those edges (the
 *        two statistics vectors of Algorithm 1 enter the recurrence only through this sum);
 *        -inf with O_i = 0 is the initial state, which sga_attention_forward* also leaves for
 *        rows without neighbours.
 * A sequence  forward(mask_1), accumulate(mask_2), ...  over pairwise disjoint masks equals one
 * forward over their union (an edge present in two of the masks would be counted twice: this
 * is why the global kernel of Section IV-B subtracts the local window, SGA_MASK_NONLOCAL).
 * With fp16 storage O is rounded to fp16 after every call.  All other arguments, errors and
 * the supported implicit kinds are those of the forward calls.
 */
sga_status sga_attention_accumulate(const void* Q, const void* K, const void* V,
                                    const int64_t* row_ptr, const int32_t* col_idx, void* O,
                                    int64_t L, int32_t H, int32_t d, float scale, void* stream,
                                    int32_t dtype, float* lse, void* workspace,
                                    size_t workspace_bytes, int32_t path);
sga_status sga_attention_accumulate_implicit(const void* Q, const void* K, const void* V,
                                             const sga_mask_desc* desc, void* O, int64_t L,
                                             int32_t H, int32_t d, float scale, void* stream,
                                             int32_t dtype, float* lse, void* workspace,
                                             size_t workspace_bytes, int32_t path);

/*
 * Prepared graphs: Get_Neighbors of an explicit mask evaluated once for many forward calls.
 *
 * The masks of Section II-C are fixed patterns: the same CSR serves every layer and every step,
 * while sga_attention_forward regroups it into 32 x 32 tiles (and sizes the split of its dense
 * rows) on every call.  sga_graph_prepare does that regrouping once, leaves the result in the
 * caller's workspace and describes it in a small host record; the *_prepared calls then launch
 * only the kernels that this graph needs (for a mask whose tiles all qualify: the fused
 * attention kernel alone, plus one merge kernel if some tiles are cut into segments).
 *
 *   sga_graph_prepare   row_ptr, col_idx, L, H, d, dtype: as in sga_attention_forward (d >= 64).
 *                       workspace: device, 256-byte aligned, at least sga_workspace_bytes(...)
 *                       bytes for the true edge count (else SGA_ERR_WORKSPACE).
 *                       plan_out: host, written.  Unlike every other entry point this call
 *                       WAITS for the stream (it reads the edge count and the analysis counters
 *                       back), so it cannot be captured into a HIP graph.
 *   *_prepared          arguments as in sga_attention_forward / sga_attention_accumulate, plus
 *                       the plan.  path: SGA_PATH_AUTO, SGA_PATH_TILE or SGA_PATH_TILE_SPLIT.
 *                       They enqueue kernels only (no wait, no allocation, capturable) and give
 *                       bit-identical results to the unprepared calls on the same workspace size.
 * Contract: between sga_graph_prepare and the last *_prepared call that uses its plan, the
 * workspace must not be written by anyone else (no unprepared call on it, no other graph), and
 * row_ptr / col_idx must keep their contents; Q, K, V, O, lse, scale and the stream may change
 * from call to call.  Calls that overlap in time need separate workspaces (and plans).
 * Errors: SGA_ERR_INVALID_ARG when the plan does not belong to these arguments (other L, H, d,
 * dtype, row_ptr, col_idx, workspace or size, or a foreign struct), otherwise as the forward.
 */
typedef struct {
  uint32_t struct_bytes;    /* = sizeof(sga_graph_plan)                                      */
  uint32_t magic;           /* set by sga_graph_prepare                                      */
  int64_t L, nnz;           /* nnz = row_ptr[L] as read from the device                      */
  int32_t H, d, dtype;
  uint32_t tiles_left;      /* tiles whose block lists did not fit (their rows run per row)  */
  uint32_t multi_tiles;     /* tiles cut into segments (partial states + merge)              */
  uint32_t tile_parts;      /* partial states those tiles need                               */
  uint32_t long_rows;       /* rows left to the per-row kernels that are split into chunks   */
  uint32_t row_chunks;      /* chunk work items of those rows                                */
  uint32_t flags;           /* SGA_GRAPH_* bits below                                        */
  const void* row_ptr;      /* the buffers the plan was prepared for (identity check only)   */
  const void* col_idx;
  const void* workspace;
  size_t workspace_bytes;
} sga_graph_plan;

enum {
  SGA_GRAPH_TILES_COVER_ALL = 1,   /* every row is produced by the tile kernels               */
  SGA_GRAPH_TILE_PARTS_FIT = 2,    /* the partial states of the multi-segment tiles fit       */
  SGA_GRAPH_ROW_CHUNKS_FIT = 4     /* the chunk items of the split rows fit                   */
};

sga_status sga_graph_prepare(const int64_t* row_ptr, const int32_t* col_idx, int64_t L, int32_t H,
                             int32_t d, int32_t dtype, void* workspace, size_t workspace_bytes,
                             void* stream, sga_graph_plan* plan_out);
sga_status sga_attention_forward_prepared(const void* Q, const void* K, const void* V,
                                          const int64_t* row_ptr, const int32_t* col_idx, void* O,
                                          int64_t L, int32_t H, int32_t d, float scale, void* stream,
                                          int32_t dtype, float* lse, void* workspace,
                                          size_t workspace_bytes, int32_t path,
                                          const sga_graph_plan* plan);
sga_status sga_attention_accumulate_prepared(const void* Q, const void* K, const void* V,
                                             const int64_t* row_ptr, const int32_t* col_idx, void* O,
                                             int64_t L, int32_t H, int32_t d, float scale,
                                             void* stream, int32_t dtype, float* lse,
                                             void* workspace, size_t workspace_bytes, int32_t path,
                                             const sga_graph_plan* plan);

/*
 * sga_attention_forward for callers that cannot allocate device memory or size a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  It is
 * sga_attention_forward with the workspace replaced by an array that lives in the library's own
 * device image (64 MiB per device, held from the first use of the library on that device until the
 * process ends); the call itself allocates nothing and frees nothing.
 *   nnz   host value: the edge count of the mask (row_ptr[L]) or an upper bound of it.  The call
 *         is refused with SGA_ERR_WORKSPACE when sga_workspace_bytes(L, H, d, dtype, nnz) exceeds
 *         sga_static_scratch_bytes() (a mask with more edges than stated still gives correct
 *         results, on the slower kernels that need no workspace).
 *   All other arguments, results and errors are those of sga_attention_forward; results are
 *   bit-identical to it with a workspace of sga_workspace_bytes(L, H, d, dtype, row_ptr[L]) bytes.
 * Every call on a device uses that device's one array (the current device's, which must be the
 * stream's), so calls that overlap in time on one device race: serialise them (one stream).
 * The array keeps the last call's contents; the call clears what it needs with a kernel.
 * sga_static_scratch_init resolves the array's address on the current device ahead of time (the
 * first forward on a device does it otherwise): call it once per device before capturing a graph.
 */
sga_status sga_static_scratch_init(void);
size_t sga_static_scratch_bytes(void);
sga_status sga_attention_forward_static(const void* Q, const void* K, const void* V,
                                        const int64_t* row_ptr, const int32_t* col_idx, void* O,
                                        int64_t L, int32_t H, int32_t d, float scale, void* stream,
                                        int32_t dtype, float* lse, int64_t nnz, int32_t path);

/*
 * Benchmark hook: timing of the dominant attention kernel of each forward call.
 * For callers that measure kernel time on the launch stream (a benchmark computing a
 * roofline); it is the one piece of process-wide state in the library and is not
 * thread-safe.  While enabled, every forward call records a pair of HIP events around the
 * launch of its main attention kernel (the fused SDDMM -> softmax -> SpMM kernel of
 * Algorithm 1; helper kernels such as mask analysis and partial merges are outside the
 * pair) on the call's stream.
 *   sga_profile_enable(on)   on != 0 starts a fresh recording, 0 stops it and releases its events.
 *   sga_profile_collect      waits for the recorded calls, writes the durations of the first
 *                            `capacity` of them in milliseconds (oldest first) to ms_out (host),
 *                            the number of calls recorded to n_out (host; a count above
 *                            `capacity` means the rest were not written), and clears the recording.
 *   sga_profile_last_kernel  name of the kernel inside the most recently recorded pair ("" if
 *                            none): a static string.
 * Errors: SGA_ERR_INVALID_ARG for null outputs or negative capacity, SGA_ERR_HIP if an event
 * could not be created or read (the recording is then incomplete and should be discarded).
 * No forward call may run on another thread while the hook is enabled, collected or disabled.
 */
sga_status sga_profile_enable(int32_t on);
sga_status sga_profile_collect(float* ms_out, int32_t capacity, int32_t* n_out);
const char* sga_profile_last_kernel(void);

#ifdef __cplusplus
}
#endif
#endif /* SGA_H_ */
