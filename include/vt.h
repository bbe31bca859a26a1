/*
 * vt.h - C ABI of the virtual-tensor library for MI355X (gfx950).
 *
 * A virtual tensor (paper, Sec. 4.1, Def. 3) is a pair (F, {P_1..P_n}): a mapping function
 * from the index of a tensor that is never stored to (physical tensor, physical index).
 * A chain of data-movement operators (Sec. 2.2, Def. 2) between a producer and a consumer
 * is composed on the host into one such map (Sec. 4.1, "mapping function composition")
 * and the consumer kernels apply it in their load stage (Sec. 4.2, virtual tensor I/O),
 * so the intermediates of the chain are never written to memory.
 *
 * Conventions
 *   - Every function returns a vt_status; vt_last_error() gives a thread-local message.
 *   - "device pointer": memory of the current HIP device, owned by the caller, which must
 *     stay valid until the work queued on `stream` has finished.  "host pointer": ordinary
 *     process memory, read during the call only, unless stated otherwise.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Kernels are
 *     queued asynchronously; the library never synchronises and allocates no device memory.
 *     A launch that the runtime rejects returns VT_ERR_DEVICE; a fault while a kernel runs
 *     surfaces at the caller's next synchronisation.
 *   - Tensors are row-major; strides are in elements; dense outputs are contiguous.
 *   - Invalid chains fail in vt_build and never reach a kernel.
 */
#ifndef VT_H_
#define VT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VT_MAX_DIMS 8

typedef enum {
  VT_OK = 0,
  VT_ERR_INVALID_ARG = 1,   /* null pointer, bad enum, bad value id */
  VT_ERR_SHAPE = 2,         /* shapes do not fit the operator or the consumer */
  VT_ERR_RANGE = 3,         /* slice / split / index out of range */
  VT_ERR_NOT_ONE_TO_ONE = 4,/* a map used as a store target sends two indices to one element (Sec. 4.1) */
  VT_ERR_UNSUPPORTED = 5,   /* valid, but outside what the descriptor or the kernel can express */
  VT_ERR_DEVICE = 6         /* the HIP runtime refused a launch */
} vt_status;

typedef enum { VT_F32 = 0, VT_F16 = 1, VT_BF16 = 2 } vt_dtype;

/* Data-movement operators that a chain may contain (Sec. 2.2; ONNX semantics). */
typedef enum {
  VT_OP_RESHAPE = 0,      /* a[0..ndim) = new shape; row-major order of elements is kept */
  VT_OP_PERMUTE = 1,      /* a[0..ndim) = perm; out.shape[i] = in.shape[perm[i]] */
  VT_OP_SLICE = 2,        /* a[0]=dim, a[1]=start, a[2]=stop, a[3]=step (>=1) */
  VT_OP_SPLIT = 3,        /* a[0]=dim, b[0..ndim) = sizes (ndim = number of outputs), out_index = which output */
  VT_OP_CONCAT = 4,       /* a[0]=dim; inputs in[0..n_in) */
  VT_OP_EXPAND = 5,       /* a[0..ndim) = new shape, same rank; size-1 dims broadcast */
  VT_OP_UNSQUEEZE = 6,    /* a[0]=dim of the inserted size-1 axis */
  VT_OP_INDEX_SELECT = 7  /* a[0]=dim; index/index_host/n_index */
} vt_op_kind;

/* A physical tensor: the producer's buffer (Def. 3's P_j).  Graph inputs and outputs
 * stay physical (Alg. 1), so the leaves of every chain are sources. */
typedef struct {
  void* ptr;                       /* device pointer to element (0,..,0); may be NULL for host-only use of the descriptor */
  int32_t dtype;                   /* vt_dtype */
  int32_t ndim;                    /* 1..VT_MAX_DIMS */
  int64_t shape[VT_MAX_DIMS];
  int64_t stride[VT_MAX_DIMS];     /* elements; all zero = dense row-major */
} vt_source;

#define VT_MAX_OP_INPUTS 8

/* One statement of a chain.  Value ids: v < 0 names source number (-1 - v); v >= 0 names the
 * result of statement v (which must come earlier). */
typedef struct {
  int32_t kind;                    /* vt_op_kind */
  int32_t n_in;                    /* 1, or the number of concat inputs (<= VT_MAX_OP_INPUTS) */
  int32_t in[VT_MAX_OP_INPUTS];
  int32_t out_index;               /* SPLIT: which output this statement denotes */
  int32_t ndim;                    /* number of valid entries of a (RESHAPE/PERMUTE/EXPAND) or b (SPLIT) */
  int64_t a[VT_MAX_DIMS];
  int64_t b[VT_MAX_DIMS];
  const int32_t* index;            /* INDEX_SELECT: device pointer to n_index int32 entries; read by kernels,
                                      must outlive every launch that uses the descriptor; may be NULL if the
                                      descriptor is only evaluated on the host */
  const int32_t* index_host;       /* INDEX_SELECT: host copy of the same table (required; validated and
                                      copied into the descriptor during vt_build) */
  int64_t n_index;
} vt_op;

typedef struct vt_desc vt_desc;    /* opaque; host memory owned by the library; immutable; reusable */

/* ---- descriptor builder (Sec. 4.1 composition, Sec. 4.3 Eq. 1 form, Def. 4/5 contiguity) ----
 * Composes statements ops[0..n_ops) over src[0..n_src) and returns the map of value
 * `result_value` as a descriptor: per piece (one per region served by one source, arising
 * from CONCAT) a stack of mixed-radix strided stages plus optional index tables, i.e.
 * f(I) = S.I + b(I) of Eq. 1 with b piecewise / table driven.  src and ops are host
 * pointers, copied.  Errors: INVALID_ARG, SHAPE, RANGE, UNSUPPORTED (more pieces, stages
 * or digits than the descriptor holds; index_select along a concatenated dim). */
int vt_build(const vt_source* src, int n_src, const vt_op* ops, int n_ops, int result_value,
             vt_desc** out);
int vt_free(vt_desc* d);

/* Shape, dtype, number of pieces and the contiguous run in elements (Def. 4/5 evaluated on
 * the refined index space: the number of consecutive virtual elements, counted from any
 * index whose trailing refined digits are zero, that are consecutive in one source;
 * minimum over pieces).  Any output pointer may be NULL.  shape must hold VT_MAX_DIMS. */
int vt_desc_info(const vt_desc* d, int* ndim, int64_t* shape, int* dtype,
                 int64_t* contiguous_run, int* n_pieces);
/* Profitability class of reading through the descriptor instead of a dense copy (Sec. 4.3,
 * Def. 5 and Theorem 1).  FULL: the whole virtual tensor is one contiguous range of one source,
 * i.e. the map is the original access pattern plus a constant bias: always profitable (Type I),
 * no measurement needed.  PARTIAL: not FULL, but every run of consecutive elements is at least
 * unit_bytes long (the minimal memory transfer unit; 0 selects 128 bytes, one cache line of the
 * target): likely profitable.  SCATTERED: some run is shorter; profitability is uncertain
 * (Type II) and is decided by timing both paths.  min_run_bytes (may be NULL) receives the
 * shortest run in bytes.  Host only. */
typedef enum { VT_ACCESS_FULL = 0, VT_ACCESS_PARTIAL = 1, VT_ACCESS_SCATTERED = 2 } vt_access_class;
int vt_classify(const vt_desc* d, int64_t unit_bytes, int* access_class, int64_t* min_run_bytes);

/* Block form of the contiguity analysis (Sec. 4.2, block-wise virtual tensor I/O; Sec. 4.3 Def. 4):
 * the largest power of two c <= cap_elems such that EVERY aligned group of c consecutive elements
 * of the virtual tensor, in row-major order, lies in one piece and is one contiguous range of its
 * source.  The copy kernels and the elementwise consumer apply the map once per such block.
 * Host only; c = 1 always holds. */
int vt_desc_block(const vt_desc* d, int64_t cap_elems, int64_t* block_elems);

/* Is the map an ordinary strided view of one tensor (one stride per dim, one offset: what a
 * framework's tensor object can hold without copying)?  is_strided receives 1 or 0; if 1, stride
 * (VT_MAX_DIMS entries, elements; 0 for a broadcast or size-1 dim) and offset (elements from the
 * source's ptr) are filled when non-NULL.  Used to tell the operators a stride-aware framework
 * executes as views from those it must execute as copies (the lean materialized comparison
 * path).  Host only. */
int vt_desc_as_strided(const vt_desc* d, int* is_strided, int64_t* stride, int64_t* offset);

/* Block-wise form of a two-dimensional map (Sec. 4.2: the index computation is done once per block
 * and simplified on the host): d virtual [R, C], read in aligned blocks of block_elems columns.
 * If every piece of the map is affine in the row and in at most two levels of the block index,
 * *n_segments receives the number of segments (at most 4) and segments[9*k .. 9*k+8] = row_lo,
 * row_hi, blk_lo, blk_hi (the blocks [blk_lo, blk_hi) of the rows [row_lo, row_hi)), the address
 * of the segment's first block, the distance in bytes to the next row, blk_stride, blk_group and
 * group_stride: block blk_lo + j lies (j % blk_group) * blk_stride + (j / blk_group) *
 * group_stride bytes from the first (blk_group = 0: j * blk_stride).  *n_segments = 0 if the map
 * has another form (tables, more than one stage, digits that do not collapse) or if aligned blocks
 * of that size are not contiguous ranges of a source (vt_desc_block).  `segments` has room for 36
 * values (host memory).  The add + row-sum consumer reads its operands through these segments
 * when both resolve, and through the evaluator otherwise. */
int vt_desc_row_walk(const vt_desc* d, int64_t block_elems, int* n_segments, int64_t* segments);

/* The general block-wise form (Sec. 4.2): the virtual tensor, in row-major order, is cut into
 * units of unit_elems elements (unit_elems divides the element count: the blocks of a copy, the
 * rows of a row-wise consumer).  If the map is a single index stage without tables, the address of
 * unit u is base + sum_t ((u / div_t) % mod_t) * coef_t in the piece that holds it, with at most
 * five terms per piece and four pieces; the copy kernels compute block addresses from these
 * terms when the map resolves (*resolved = 1), and through the evaluator otherwise.  This call resolves the map and evaluates the resolved form, on the host,
 * with the routine the kernels use: addresses[k] receives the address of the first element of
 * unit first + k, k in [0, count) (count may be 0: only *resolved is set).  Host only; the
 * sources need non-NULL pointers, which are never dereferenced. */
int vt_desc_walk_addresses(const vt_desc* d, int64_t unit_elems, int64_t first, int64_t count, int* resolved,
                           uint64_t* addresses);

/* Piece p: its box [lo,hi) in virtual index space, its source number and its own run. */
int vt_desc_piece(const vt_desc* d, int p, int64_t* lo, int64_t* hi, int* src_id, int64_t* run);
/* CPU evaluation of the map at one virtual index (host logic; used by tests).  vindex holds
 * ndim entries.  Returns the source number and the element offset from its ptr. */
int vt_eval_host(const vt_desc* d, const int64_t* vindex, int* src_id, int64_t* elem_offset);
/* The same, evaluated by the kernels' own routine over the device form of the descriptor
 * (run on the CPU): a pre-launch check of what the generic kernels will walk.  Returns the
 * piece number instead of the source number. */
int vt_eval_device_form(const vt_desc* d, const int64_t* vindex, int* piece, int64_t* elem_offset);
/* Human-readable dump (pieces, stages, digits) into buf (NUL-terminated, truncated to cap). */
int vt_desc_dump(const vt_desc* d, char* buf, size_t cap);

/* ---- pure data movement --------------------------------------------------------------
 * vt_materialize: gather-copy of the whole virtual tensor into dense row-major dst (device
 * pointer, same dtype).  Bit-exact.  vt_copy_op: ONE operator executed as an explicit copy
 * kernel from dense/strided inputs into dense dst: the building block of the materialized
 * comparison path (Sec. 3.1 counts six such kernels between the two compute kernels). */
int vt_materialize(const vt_desc* d, void* dst, void* stream);
int vt_copy_op(const vt_source* in, int n_in, const vt_op* op, void* dst, void* stream);

/* ---- consumers (stage 1 reads through the map; stage 2 and 3 are ordinary, Sec. 4.2) ----
 * VT_EW_ADD_ROWSUM: x, y virtual [R,C] f32; out[r] = sum_c (x[r,c] + y[r,c]), out = R floats
 *   (device).  Summation order is fixed: column c goes to partial sum c mod 64 in ascending
 *   c, the 64 partial sums are combined by the butterfly p[l] += p[l xor s], s = 32..1.
 * VT_EW_LAYERNORM: x virtual [..., C] (f16/bf16/f32), y must be NULL; per-row LayerNorm over
 *   the last dim with gamma = 1, beta = 0, biased variance, fp32 arithmetic, out dense, same
 *   dtype and shape as x. */
typedef enum { VT_EW_ADD_ROWSUM = 0, VT_EW_LAYERNORM = 1 } vt_ew_kind;
int vt_elementwise(int kind, const vt_desc* x, const vt_desc* y, float eps, void* out, void* stream);

/* Weighted sum of two virtual tensors, the combine step after a mixture-of-experts layer
 * (the consumer that reads the expert outputs back in token order; the gathers are index_select
 * operators in the chains of x and y and are never executed): out[r,:] = w[r][0] x[r,:] +
 * w[r][1] y[r,:].  x, y virtual [R,C], f16 or bf16; weights dense device [R,2] fp32; out dense
 * [R,C] of the operands' dtype; fp32 arithmetic, one rounding.  Asynchronous on `stream`. */
int vt_weighted_sum(const vt_desc* x, const vt_desc* y, const float* weights, void* out, void* stream);

/* GEMM consumer on the matrix cores (Sec. 2.3 Listing 1's three stages with a virtual stage
 * 1): C[g] = A[g] . B[g] for g in [0, n_groups).  A[g] virtual [M_g, K] (trailing dims may be
 * folded: [.., K] counts as rows x K), B[g] virtual [K, N]; f16 or bf16 operands, fp32
 * accumulation, C[g] dense [M_g, N] row-major device pointers of dtype c_dtype (same as the
 * operands, or VT_F32).  One launch covers all groups.
 * Operand forms: the tiled kernel (256 x 256 tiles) takes maps that separate into a row part plus
 * a column part with runs of 8 contiguous, 16-byte aligned elements along K for A (rows through
 * any mixed-radix map or an index table: permuted, gathered, broadcast rows) and along N or
 * along K for B (a [K,N] weight, or an [N,K] weight seen through a Permute); an A that a Concat
 * stacked along its outermost dim runs as one group per piece.  Every other representable map
 * (pieces along K, stacked index stages, tables on columns, no alignment at all) runs on a generic
 * kernel that applies the whole map per element: same results, far slower.
 * prologue = VT_GEMM_LAYERNORM applies per-row LayerNorm (gamma 1, beta 0, eps) over K to A,
 * rounded to the operand dtype, before the product, inside the load stage (the normalised
 * tensor is never stored).  The fused kernel is built for K = 64 or 128, N <= 384 and contiguous
 * rows of A; other shapes and maps run on the generic kernel with the same prologue (far slower).
 * A, B, C are host arrays of n_groups pointers. */
typedef enum { VT_GEMM_PLAIN = 0, VT_GEMM_LAYERNORM = 1 } vt_gemm_prologue;
int vt_gemm(const vt_desc* const* A, const vt_desc* const* B, void* const* C, int n_groups,
            int c_dtype, int prologue, float eps, void* stream);

/* Split-K flash-decoding attention with grouped queries (Sec. 3.1: the attention kernel
 * reads the un-expanded cache).  Q virtual [B,Hq,1,D], K and V virtual [B,Hq,S,D]
 * (f16/bf16; the planned kernel is built for D = 128).  out dense [B,Hq,D], same dtype, 8-byte aligned.  softmax(scale * q.k) in fp32.
 * Query heads whose K/V rows coincide (a broadcast digit in the map) share one read.
 * K and V may be split into pieces along the context (Concat), and a piece may reach its rows
 * through a page table: an index_select over a pool of pages of 32 k rows, in context order
 * after the usual reshape / permute (a paged KV cache); the kernel then looks up the page of
 * every 32-row tile.  Anything else that a descriptor can hold (another head dim up to 1024, more
 * index stages, tables elsewhere, rows that are not contiguous along D, pieces along other dims)
 * runs on a generic kernel that applies the whole map per element: same result to rounding,
 * far slower, no context splits; vt_decode_attn_plan reports VT_ERR_UNSUPPORTED for such operands.
 * workspace: device pointer (16-byte aligned) of at least vt_decode_attn_workspace(...) bytes,
 * holding arrival counters and the per-split partial results, prepared once with
 * vt_decode_attn_workspace_init; the split that finishes last for a (batch, kv head) merges
 * the partial results inside the same launch, in split order: results are bitwise reproducible
 * from launch to launch.  n_splits = 0 lets the library choose.  lse (device, B*Hq floats,
 * may be NULL) receives the log-sum-exp of the scaled scores. */
int vt_decode_attn(const vt_desc* Q, const vt_desc* K, const vt_desc* V, float scale, void* out,
                   float* lse, void* workspace, size_t workspace_bytes, int n_splits, void* stream);

/* What vt_decode_attn would decide for these operands, without launching anything (host only; the
 * sources need non-NULL, suitably aligned pointers but nothing is dereferenced): the number of
 * query heads served by one read of K/V, the context segments, the context splits, and how many
 * segments read an operand through a page table.  Same errors as vt_decode_attn.  Any output
 * pointer may be NULL. */
int vt_decode_attn_plan(const vt_desc* Q, const vt_desc* K, const vt_desc* V, int n_splits, int* group_size,
                        int* n_segments, int* splits, int* paged_segments);
/* Bytes of workspace vt_decode_attn needs for this problem (S = context length: the number of
 * splits the library picks for n_splits = 0, and with it the size of the partial results, depends
 * on it).  Host only. */
size_t vt_decode_attn_workspace(int B, int Hq, int D, int S, int n_splits);
/* Clears a freshly allocated workspace (its first bytes hold one arrival counter per (batch,
 * kv head), which must be zero when vt_decode_attn starts and which vt_decode_attn leaves at
 * zero).  Call once after allocating, on the stream of the first vt_decode_attn, or clear
 * the buffer yourself.  Launches that share a workspace must not overlap in time. */
int vt_decode_attn_workspace_init(void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): vt_decode_attn without the workspace argument.  The
 * partial results and arrival counters live in a fixed array inside the library's own device
 * memory, vt_decode_attn_static_capacity() bytes (4 MiB) per GPU, held until the process ends.
 * The call allocates nothing and frees nothing; it queues a small fill kernel that clears the
 * arrival counters, then the same kernel as vt_decode_attn, and gives the same bits.  Problems
 * whose workspace (vt_decode_attn_workspace) exceeds the capacity return VT_ERR_INVALID_ARG with a
 * message naming both sizes; all other arguments and errors are those of vt_decode_attn.  All
 * calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams,
 * two threads) race and give wrong results. */
size_t vt_decode_attn_static_capacity(void);
int vt_decode_attn_static(const vt_desc* Q, const vt_desc* K, const vt_desc* V, float scale, void* out,
                          float* lse, int n_splits, void* stream);

/* Copy kernel in the store direction: every element of the virtual tensor src is written to the
 * physical place that dst's map names; other elements of dst's tensors are left alone.  This is
 * the explicit Split / Reshape / ScatterND of the materialized comparison path.  src and dst have
 * the same shape and dtype; dst must be one to one (as for vt_gemm_store) and its sources must
 * carry writable device pointers.  Asynchronous on `stream`. */
int vt_scatter(const vt_desc* src, const vt_desc* dst, void* stream);

/* Producer-side virtual store (Sec. 3.1 and Fig. 4; Sec. 4.2, stage 3 through the map):
 * C = A . B, fp32 accumulation, each element rounded to the operands' 16-bit type and written to
 * the physical tensor and offset that the OUTPUT descriptor C names; nothing else is written, so
 * the tensors behind C keep all other contents (what Split + Reshape + ScatterND would produce
 * from the dense product, without executing them).
 *   A  [M,K]: single piece, rows through its map, K contiguous, 8-byte aligned rows.
 *   B  [K,N]: a row-major matrix (constant row stride, multiple of 8 elements, 16-byte aligned).
 *   C  [M,N]: its pieces split the columns only (at most 4); every source carries a writable
 *      device pointer.  The map must be one to one: a broadcast digit or pieces whose ranges in
 *      one tensor may overlap give VT_ERR_NOT_ONE_TO_ONE; index tables and stacked stages on
 *      the output give VT_ERR_UNSUPPORTED.
 * N and K are multiples of 8.  Up to 128 rows run on a kernel built for a handful of rows (a
 * decode step: M = batch; rows are processed 16 at a time and B is read once per 16 rows); more
 * rows run on the tiled kernel of vt_gemm with the map applied in its store stage (A and B then
 * obey vt_gemm's layout rules; the workspace is not used).
 * workspace: device pointer (16-byte aligned), at least vt_gemm_store_workspace(M, N, K) bytes,
 * cleared once with vt_gemm_store_workspace_init (arrival counters, left at zero by every call,
 * and the partial sums of the K slices); calls that share a workspace must not overlap in time.
 * Results are bitwise reproducible from call to call.  Asynchronous on `stream`. */
size_t vt_gemm_store_workspace(int64_t M, int64_t N, int64_t K);
int vt_gemm_store_workspace_init(void* workspace, size_t workspace_bytes, void* stream);
int vt_gemm_store(const vt_desc* A, const vt_desc* B, const vt_desc* C, void* workspace,
                  size_t workspace_bytes, void* stream);

/* ---- which tensors to make virtual (Sec. 5) -------------------------------------------------
 * The virtual tensor opportunity graph of a computation graph (Sec. 5.1, Def. 6, Alg. 1) and the
 * global greedy choice of a points-to graph (Sec. 5.2, Alg. 2).  Host only.
 * A graph is n_tensors tensors (numbers 0 .. n_tensors-1) and a list of statements; kind is a
 * vt_op_kind, VT_OP_SCATTER_ND (inputs: data, indices, updates) or VT_OP_COMPUTE (any operator
 * that is not data movement: creates no opportunity).  pinned[t] != 0 marks the inputs and outputs
 * of the graph, which stay physical.  A *bundle* says: `tensor` can become a virtual tensor of
 * `targets` by eliminating statement `stmt`, reading through the map (VT_DIR_READ: the tensor is
 * an output of the operator) or storing through it (VT_DIR_STORE: the tensor is an input that
 * lives inside the operator's output).  The bundles of one tensor exclude each other (the conflict
 * set).  A strategy is an array bundle_of_tensor[n_tensors]: a bundle number, or -1 = physical. */
#define VT_OP_SCATTER_ND 8
#define VT_OP_COMPUTE (-1)
#define VT_DIR_READ 1
#define VT_DIR_STORE 2
typedef struct {
  int32_t kind;
  int32_t n_in;
  int32_t in[VT_MAX_OP_INPUTS];
  int32_t n_out;                   /* 1, or the number of outputs of a SPLIT */
  int32_t out[VT_MAX_OP_INPUTS];
} vt_graph_stmt;
typedef struct vt_vtog vt_vtog;    /* opaque; host memory owned by the library */
/* Alg. 1.  directions: VT_DIR_READ | VT_DIR_STORE or one of them.  Errors: INVALID_ARG. */
int vt_vtog_build(const vt_graph_stmt* stmts, int n_stmts, int n_tensors, const uint8_t* pinned, int directions,
                  vt_vtog** out);
int vt_vtog_free(vt_vtog* g);
int vt_vtog_size(const vt_vtog* g, int* n_tensors, int* n_bundles);
/* Bundle b (in statement order); targets must hold VT_MAX_OP_INPUTS entries.  Outputs may be NULL. */
int vt_vtog_bundle(const vt_vtog* g, int b, int* tensor, int* n_targets, int* targets, int* stmt, int* direction);
/* ok = 1 if every chosen bundle belongs to its tensor and following the edges always ends at a
 * physical tensor (no cycle): a points-to graph (Sec. 5.2). */
int vt_vtog_is_points_to_graph(const vt_vtog* g, const int* bundle_of_tensor, int* ok);
/* Alg. 2.  saving(user, b, bundle_of_tensor) returns the latency saving w of adding bundle b to the
 * strategy built so far (measured by the caller, e.g. by timing both variants on the GPU); it is
 * called once per bundle at the start and again for the bundles that point to a tensor that has
 * just joined.  Every iteration anchors one tensor: the one whose best ready bundle (targets all
 * anchored, saving >= 0) saves most, with that bundle; if no bundle is ready, the unanchored tensor
 * nearest the graph's outputs, as a physical tensor.  bundle_of_tensor (n_tensors entries)
 * receives the strategy, total the sum of the savings taken; order (may be NULL, n_tensors
 * entries) the bundles in the order they were taken, n_order their number. */
typedef double (*vt_saving_fn)(void* user, int bundle, const int* bundle_of_tensor);
int vt_vtog_greedy(const vt_vtog* g, vt_saving_fn saving, void* user, int* bundle_of_tensor, double* total,
                   int* order, int* n_order);

const char* vt_last_error(void);
const char* vt_version(void);

#ifdef __cplusplus
}
#endif
#endif /* VT_H_ */
