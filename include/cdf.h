/*
 * libcdf - the per-partition layer step of cache-based distributed full-batch GCN
 * training (CDFGNN), for one AMD MI355X (gfx950).
 *
 * One partition owns n_loc vertices ("local rows") and reads n_halo remote
 * neighbours ("halo rows"). Feature matrices are row-major with local rows first:
 * Xfull = [ local rows ; halo rows ], (n_loc + n_halo) x dim.
 *
 * Conventions for every entry point
 *  - C ABI. Every pointer is a DEVICE pointer owned by the caller unless the
 *    parameter comment says "host". The library never allocates or frees device
 *    memory; scratch comes from the caller's workspace `ws` (size it with
 *    cdf_workspace_bytes; 256-byte aligned).
 *  - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the null
 *    stream) and the call returns without synchronising. Counts produced on the
 *    device (n_sent) stay on the device; consumers read them there.
 *  - Row-major matrices carry a leading dimension `ld` in ELEMENTS (ld >= dim).
 *  - Element type cdf_dtype: fp32, or bf16 storage with fp32 arithmetic.
 *  - Return value: CDF_OK or a negative cdf_status. Invalid arguments are rejected
 *    on the host before anything is launched. cdf_last_error() gives a host string.
 *  - Inputs are assumed finite. What a NaN does is nevertheless defined: the row maxima and
 *    minima of the cache test (LINF) and of the quantiser drop NaN elements (IEEE maxNum / minNum),
 *    so such a row is judged and scaled by its other elements, a NaN element gets code 0, and a row
 *    that holds only NaN is never sent; with CDF_NORM_L2 a NaN makes both sums NaN and the row is
 *    not sent (comparisons with NaN are false).
 *  - Calls sharing a workspace must be ordered on one stream; distinct workspaces may run
 *    concurrently.
 *  - n_rows == 0, max_sent == 0 and *n_sent == 0 are valid and do nothing.
 */
#ifndef CDF_H
#define CDF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CDF_OK = 0,
  CDF_ERR_INVALID_ARG = -1, /* null / negative / misaligned / ld < dim / non-finite eps */
  CDF_ERR_UNSUPPORTED = -2, /* dtype, bits, norm or scheme combination not provided */
  CDF_ERR_WORKSPACE = -3,   /* workspace missing or too small */
  CDF_ERR_HIP = -4          /* a launch failed; see cdf_last_error() */
} cdf_status;

typedef enum { CDF_F32 = 0, CDF_BF16 = 1 } cdf_dtype;

/* Row norm of the cache test. LINF is the paper's (Alg. 2, Sec. 4.1). L2 compares
 * squared sums in fp32 with a fixed summation order: 256 interleaved chains (chain c
 * takes elements c, c+256, ... in ascending order, one fused multiply-add each), then a
 * radix-2 butterfly over the chain index with strides 1, 2, ..., 128. */
typedef enum { CDF_NORM_LINF = 0, CDF_NORM_L2 = 1 } cdf_norm;

/* Message coding (Sec. 5). MINMAX is the paper's linear quantiser with 2^B - 1 levels;
 * SYMMETRIC is a zero-centred variant; NONE sends the fp32 row unchanged. */
typedef enum { CDF_Q_MINMAX = 0, CDF_Q_SYMMETRIC = 1, CDF_Q_NONE = 2 } cdf_qscheme;

/* What the sender does to its cache after a row is sent (Alg. 2: cached <- current). */
typedef enum { CDF_COMMIT_NONE = 0, CDF_COMMIT_CUR = 1, CDF_COMMIT_DEQ = 2 } cdf_commit;

/* CSR matrix, column indices ascending within a row. */
typedef struct {
  int32_t n_rows, n_cols;
  int64_t nnz;
  const int64_t* rowptr; /* [n_rows + 1], rowptr[0] = 0, rowptr[n_rows] = nnz */
  const int32_t* colidx; /* [nnz], each in [0, n_cols) */
  const float* vals;     /* [nnz] */
  const int32_t* plan;   /* NULL, or the table cdf_spmm_plan built for exactly these row pointers */
} cdf_csr;

/* Host-side text of the last error raised on the calling thread ("" if none). */
const char* cdf_last_error(void);

/*
 * Optional per-kernel timing for benchmarks (host functions, not thread safe). While
 * enabled, every kernel launch of the library is bracketed by a pair of HIP events on the
 * launch stream (default-priority events, no device memory). cdf_profile_enable(1) clears
 * earlier records; cdf_profile_read() waits for the recorded launches of one kernel id
 * (0 .. cdf_profile_kernels()-1) and writes their durations in milliseconds, in launch order,
 * to the HOST array ms[cap]; it returns the number of launches recorded (may exceed cap),
 * or a negative status. At most 8192 launches are kept per session.
 */
int cdf_profile_enable(int on);
int cdf_profile_kernels(void);
const char* cdf_profile_kernel_name(int kernel);
int cdf_profile_read(int kernel, float* ms /* host */, int cap);
/* All recorded launches in launch order: kernel id and duration (ms) of launch i go to the HOST arrays
 * kernel[i], ms[i] for i < cap (either may be NULL); returns the number recorded or a negative status. */
int cdf_profile_read_all(int32_t* kernel /* host */, float* ms /* host */, int cap);

/* A plain device-to-device copy kernel (16 bytes per lane, grid-stride) of `bytes` bytes
 * (multiple of 16, both pointers 16-byte aligned). It exists so that hardware counter
 * readings of the other kernels can be scaled by what the same counters report for a
 * transfer of known size. */
int cdf_profile_copy(void* dst, const void* src, size_t bytes, void* stream);

/* Bytes of workspace that cover any call on matrices of at most max_rows rows (of a
 * feature matrix or of a CSR operand, whichever is larger), max_dim columns and
 * max_nnz stored entries. Host function, no device work. The figure includes the
 * row-indexed scratch (max_rows * (max_dim + 8) bytes) with which the layer steps test
 * and code the halo rows in one pass; a layer step given less than that, but at least its
 * own minimum, runs the two-pass route and produces the same bits. */
size_t cdf_workspace_bytes(int64_t max_rows, int32_t max_dim, int64_t max_nnz);

/* Bytes of one packed message row: dim*4 for CDF_Q_NONE, else ceil(dim*bits/8). The
 * paper's message size B*L + 2T bits (Sec. 5) is this plus the 8 bytes of `meta`. */
size_t cdf_code_row_bytes(int32_t dim, int bits, cdf_qscheme qs);

/*
 * Adaptive cache test (Alg. 2, the condition of the mirror loop).
 *   mask[r] = ( ||cur[r] - cached[r]|| > eps * ||cached[r]|| ), strict, product form, so a
 *   zero cached row is sent on any non-zero difference and an unchanged row never is.
 *   idx     = ascending list of the rows with mask 1;  *n_sent = their number.
 * cur, cached : n_rows x dim, leading dimension ld, type dt (read only here).
 * mask [n_rows] bytes, idx [n_rows] int32 (entries past *n_sent are not written), n_sent [1].
 * eps must be finite and >= 0.
 */
int cdf_cache_filter(const void* cur, const void* cached, int32_t n_rows, int32_t dim, int64_t ld,
                     cdf_dtype dt, float eps, cdf_norm norm, uint8_t* mask, int32_t* idx,
                     int32_t* n_sent, void* ws, size_t ws_bytes, void* stream);

/*
 * cdf_cache_filter for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc. Same
 * arguments and results as cdf_cache_filter, minus ws / ws_bytes: the per-block counts and offsets
 * (the only scratch the test needs) live in a static device array inside the library, about 1 MiB,
 * one copy per GPU, held until the process ends. The call allocates and frees nothing; its first
 * call on a device looks the array's address up (a host-side query). The device that owns the
 * buffers must be the current device.
 *  - n_rows above 8 388 608 (8 Mi) is rejected with CDF_ERR_UNSUPPORTED.
 *  - Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU (different
 *    streams or threads) race; order them on one stream. The array keeps the last call's contents;
 *    each call overwrites the part it reads, so nothing needs clearing in between.
 */
int cdf_cache_filter_static(const void* cur, const void* cached, int32_t n_rows, int32_t dim, int64_t ld,
                            cdf_dtype dt, float eps, cdf_norm norm, uint8_t* mask, int32_t* idx,
                            int32_t* n_sent, void* stream);

/*
 * Message build for the listed rows (Alg. 2 "send the difference"; Sec. 5, first equation)
 * followed by the cache commit. For k < *n_sent, r = idx[k]:
 *   m = cur[r] - cached[r]  (delta != 0, the paper)   or   m = cur[r]  (delta == 0)
 *   MINMAX   : lo = min m, hi = max m, Lv = 2^bits - 1, inv = Lv / (hi - lo) (0 if hi == lo),
 *              q_j = clamp(floor((m_j - lo) * inv + 0.5), 0, Lv)   [fused multiply-add, fp32]
 *              meta[k] = (lo, hi)
 *   SYMMETRIC: a = max |m|, Qm = 2^(bits-1) - 1, inv = Qm / a (0 if a == 0),
 *              q_j = clamp(floor(m_j * inv + 0.5), -Qm, Qm), two's complement in `bits` bits
 *              meta[k] = (a / Qm, 0)
 *   NONE     : the fp32 values of m; meta[k] = (0, 0)
 *   codes row k = cdf_code_row_bytes() bytes; 8 bits: one code per byte; 4 bits: even element
 *   in the low nibble, odd element in the high nibble, unused tail nibble zero.
 *   commit: CUR cached[r] <- cur[r];  DEQ cached[r] <- (delta ? cached[r] : 0) + recovered m;
 *   NONE leaves the cache.
 * cached may be NULL only if delta == 0 and commit == CDF_COMMIT_NONE.
 * max_sent bounds *n_sent (capacity of idx / codes / meta); bits is 8 or 4.
 * Width limit (cdf_quantize, cdf_dequantize, cdf_cache_filter_quantize and the layer steps, which
 * call them): a row is held in registers, 512 lane-vectors at most, so dim <= 512 * v where v is the
 * number of elements per lane-vector: 4 if dim and ld are multiples of 4 and every row pointer is
 * aligned to 4 elements, else 2 under the same conditions for 2, else 1 - dim <= 2048, 1024 or 512.
 * Wider rows are refused with CDF_ERR_UNSUPPORTED before anything is launched; cdf_max_message_dim
 * gives the limit for a width, pitch and type (base pointers taken as aligned). cdf_cache_filter and
 * the aggregation have no such limit.
 */
int32_t cdf_max_message_dim(int32_t dim, int64_t ld, cdf_dtype dt);

int cdf_quantize(const void* cur, void* cached, const int32_t* idx, const int32_t* n_sent,
                 int32_t max_sent, int32_t dim, int64_t ld, cdf_dtype dt, int bits, cdf_qscheme qs,
                 cdf_commit commit, int delta, uint8_t* codes, float* meta, void* stream);

/* Host-side test hook: the number of polls after which a workgroup of the look-back route above gives
 * up waiting for its predecessors (polls <= 0 restores the default of about a million). */
int cdf_set_message_wait_limit(int polls);

/*
 * Message recovery (Sec. 5, second equation) and the receiver's cache update (Alg. 2,
 * message loop: cached_total <- cached_total + delta). For k < *n_sent:
 *   MINMAX   : scale = (hi - lo) / Lv,  m~_j = q_j * scale + lo   [fused, fp32]
 *   SYMMETRIC: m~_j = q_j * meta[k][0]
 *   NONE     : m~_j = stored fp32 value
 *   accumulate != 0: dst[idx[k]][j] += m~_j    else: dst[idx[k]][j] = m~_j
 * dst : rows of leading dimension ld and type dt (bf16: the fp32 result is rounded to
 * nearest even). Rows listed twice in idx race; idx from cdf_cache_filter has none.
 */
int cdf_dequantize(const uint8_t* codes, const float* meta, const int32_t* idx, const int32_t* n_sent,
                   int32_t max_sent, int32_t dim, int bits, cdf_qscheme qs, void* dst, int64_t ld,
                   cdf_dtype dt, int accumulate, void* stream);

/*
 * cdf_cache_filter followed by cdf_quantize on the same rows, in one pass over them where that is
 * possible (quantised messages, ws of cdf_workspace_bytes(n_rows, dim, 0) or more):
 * a row is read once, tested, and - if it fails - coded and committed from the same registers.
 * Small inputs (all workgroups resident at once, some ten thousand rows) write every message
 * straight to its place: a workgroup learns the number of sent rows before its own from its
 * predecessors through status words in the workspace (single-pass scan with look-back; a workgroup
 * publishes its count before it waits, the wait is bounded). Larger inputs stage the messages by row
 * and move them into rank order with a second small kernel. In every other case the two calls run one
 * after the other. mask, idx, *n_sent, codes, meta and the committed cache are bit-identical to the
 * two calls on every route. Arguments as for those calls; capacity of idx / codes / meta = n_rows.
 * Should the bounded wait ever expire (never seen; it needs a workgroup that is not scheduled for
 * about a second), *n_sent is -1, which every consumer in this library treats as "no messages".
 */
int cdf_cache_filter_quantize(const void* cur, void* cached, int32_t n_rows, int32_t dim, int64_t ld,
                              cdf_dtype dt, float eps, cdf_norm norm, int bits, cdf_qscheme qs,
                              cdf_commit commit, int delta, uint8_t* mask, int32_t* idx, int32_t* n_sent,
                              uint8_t* codes, float* meta, void* ws, size_t ws_bytes, void* stream);

/*
 * Work split of the aggregation, computed once per matrix (the adjacency of a partition never changes
 * during training, Sec. 3.1): the aggregation kernels cut the stored entries into equal chunks, one per
 * wavefront, and need the row in which each chunk starts. With A->plan == NULL every cdf_spmm_* call
 * (and every layer step) recomputes that table in its workspace; cdf_spmm_plan writes it to the caller's
 * buffer `plan` (device memory, cdf_spmm_plan_bytes(A->nnz) bytes, 4-byte aligned) so that the caller can
 * store the pointer in A->plan and skip that launch from then on. The table depends on rowptr and nnz only.
 */
size_t cdf_spmm_plan_bytes(int64_t nnz);
int cdf_spmm_plan(const cdf_csr* A /* host */, int32_t* plan, size_t plan_bytes, void* stream);

/*
 * Aggregation over the normalised adjacency (Sec. 3.1, the product A^_i H of the forward
 * equation): Y[n_rows x dim] = A * X[n_cols x dim], fp32 accumulation in an order fixed by
 * the matrix shape alone (no atomics): bit-reproducible from run to run. `A` is a HOST pointer
 * to a struct of device arrays whose row pointers must be consistent (rowptr[n_rows] == nnz).
 * X and Y must not overlap. Empty rows give zero rows.
 */
int cdf_spmm_fwd(const cdf_csr* A, const void* X, int64_t ldx, void* Y, int64_t ldy, int32_t dim,
                 cdf_dtype dt, void* ws, size_t ws_bytes, void* stream);

/*
 * The transposed product of back-propagation (Sec. 3.1, gradient w.r.t. the layer input):
 * dX[(n_loc + n_halo) x dim] = A^T * dY[n_loc x dim], computed as a row-gather over `At`,
 * the CSR of A^T built once by the caller, so it needs no atomics either.
 */
int cdf_spmm_bwd(const cdf_csr* At, const void* dY, int64_t ldy, void* dX, int64_t ldx, int32_t dim,
                 cdf_dtype dt, void* ws, size_t ws_bytes, void* stream);

/*
 * Aggregation and dense transform of a layer in one call (Sec. 3.1, first equation:
 * H' = sigma(A^ H W)):  M = A X,  Z = M W,  H = sigma(Z).
 * When the output is narrow (f_out <= 64), the rows are fp32 with 16-byte aligned pitch and W plus
 * four row buffers fit 64 KB of LDS, the transform runs in the row epilogue of the aggregation kernel:
 * a finished row of M is stored (the backward step needs it) and multiplied with W from LDS straight
 * away, so M is not read back and the dense kernel is not launched. Otherwise the call is
 * cdf_spmm_fwd followed by cdf_dense_fwd. Same results within fp32 rounding either way; each route is
 * bit-reproducible. The layer steps keep the two launches: the one-kernel route has to give a whole
 * wavefront to every stored entry and measured slower on every benchmark workload (the column-sliced
 * aggregation plus the matrix-core kernel wins even where a step is launch-bound). M [n_rows x f_in] type dt with pitch ldm, Z (nullable) and H (nullable) [n_rows x
 * f_out] fp32 contiguous; ws as for cdf_spmm_fwd.
 */
int cdf_spmm_dense_fwd(const cdf_csr* A /* host */, const void* X, int64_t ldx, cdf_dtype dt, const float* W,
                       int32_t f_in, int32_t f_out, int relu, void* M, int64_t ldm, float* Z, float* H, void* ws,
                       size_t ws_bytes, void* stream);

/*
 * Dense transform (Sec. 3.1: Z = (A^ H) W, H' = sigma(Z), sigma = ReLU or identity) on
 * the matrix cores. M [n x f_in] type dt, W [f_in x f_out] fp32 row-major,
 * Z (nullable), H (nullable) [n x f_out] fp32 row-major, contiguous.
 * fp32 M: fp32 matrix instructions. bf16 M with 16-byte aligned rows: bf16 matrix
 * instructions with W split into a bf16 high and low part (W = hi + lo up to 2^-17 |W|),
 * fp32 accumulation; other bf16 layouts widen M to fp32 on load.
 */
int cdf_dense_fwd(const void* M, int64_t ldm, cdf_dtype dt, const float* W, int32_t n, int32_t f_in,
                  int32_t f_out, int relu, float* Z, float* H, void* stream);

/*
 * Gradients of the dense transform (chain rule of Sec. 3.1 with sigma'(z) = [z > 0]):
 *   dZ = relu ? dH * [Zs > 0] : dH      (Zs: Z or H of the forward pass - same sign test)
 *   dW [f_in x f_out] fp32 = M^T dZ     (row blocks reduced in a fixed order: reproducible)
 *   dM [n x f_in] type dt  = dZ W^T     (skipped when dM is NULL)
 * fp32 matrix instructions, except for bf16 activations with 16-byte aligned W, dH, Zs: dM (f_out % 8
 * == 0) on the bf16 matrix instructions with dZ and W each split into a bf16 high and low part (three
 * products, the low x low one dropped), fp32 accumulation, bf16 result; dW (f_in % 128 == 0, f_out %
 * 64 == 0, 16-byte aligned rows of M) likewise with dZ split in two (M is bf16 already).
 */
int cdf_dense_bwd(const void* M, int64_t ldm, cdf_dtype dt, const float* W, const float* Zs,
                  const float* dH, int32_t n, int32_t f_in, int32_t f_out, int relu, float* dW,
                  void* dM, int64_t lddm, void* ws, size_t ws_bytes, void* stream);

/*
 * Forward step of one layer on one partition (Alg. 1 forward line with Alg. 2 and Sec. 5
 * applied to the rows that cross the partition boundary):
 *   1. cache test of halo_fresh (what the halo rows' owners hold now) against cache_sent
 *      (what they last sent)                                   -> mask, idx, n_sent
 *   2. message build + commit of cache_sent                    -> codes, meta
 *   3. recovery and update of the halo rows of xfull (+= when delta, = otherwise)
 *   4. M = A * xfull                 5. Z = M W, H = sigma(Z)
 * `A` is a host pointer; all other pointers are device pointers.
 */
typedef struct {
  const cdf_csr* A;       /* host pointer; n_rows = n_loc, n_cols = n_loc + n_halo */
  int32_t n_loc, n_halo, f_in, f_out;
  cdf_dtype dt;           /* type of xfull, halo_fresh, cache_sent, M */
  int relu;
  void* xfull;            /* (n_loc+n_halo) x f_in, ld = f_in; halo rows updated in place */
  const void* halo_fresh; /* n_halo x f_in */
  void* cache_sent;       /* n_halo x f_in, updated in place by the commit */
  const float* W;         /* f_in x f_out */
  float eps;
  cdf_norm norm;
  int bits;
  cdf_qscheme qs;
  cdf_commit commit;
  int delta;              /* 1: difference messages, receiver adds (the paper); 0: value messages */
  void* M;                /* out: n_loc x f_in, type dt (kept for the backward step) */
  float* Z;               /* out, nullable: n_loc x f_out */
  float* H;               /* out: n_loc x f_out */
  uint8_t* mask;          /* out: [n_halo] */
  int32_t* idx;           /* out: [n_halo] */
  int32_t* n_sent;        /* out: [1] */
  uint8_t* codes;         /* out: [n_halo * cdf_code_row_bytes(f_in, bits, qs)] */
  float* meta;            /* out: [n_halo * 2] */
} cdf_layer_fwd_args;

int cdf_gcn_layer_fwd(const cdf_layer_fwd_args* args /* host */, void* ws, size_t ws_bytes, void* stream);

/*
 * Backward step of one layer on one partition (Alg. 1 backward lines; the cache and the
 * quantiser applied to gradients exactly as to features, Sec. 4.1):
 *   1. dZ = dH * sigma'(Zs);  dW = M^T dZ;  dM = dZ W^T
 *   2. dxfull = A^T dM : rows [0, n_loc) local input gradients, rows [n_loc, n_loc+n_halo)
 *      partial gradients owed to the owners of the halo rows
 *   3. cache test of those halo gradient rows against gcache_sent -> mask, idx, n_sent
 *   4. message build + commit of gcache_sent                     -> codes, meta
 * Steps 2-4 are skipped when need_dx == 0 (first layer: inputs need no gradient).
 */
typedef struct {
  const cdf_csr* At;      /* host pointer; n_rows = n_loc + n_halo, n_cols = n_loc */
  int32_t n_loc, n_halo, f_in, f_out;
  cdf_dtype dt;           /* type of M, dM, dxfull, gcache_sent */
  int relu, need_dx;
  const float* dH;        /* n_loc x f_out */
  const float* Zs;        /* n_loc x f_out: Z or H of the forward step (unused if !relu) */
  const void* M;          /* n_loc x f_in */
  const float* W;         /* f_in x f_out */
  float* dW;              /* out: f_in x f_out */
  void* dM;               /* out / scratch: n_loc x f_in, type dt */
  void* dxfull;           /* out: (n_loc+n_halo) x f_in, type dt */
  void* gcache_sent;      /* n_halo x f_in, updated in place by the commit */
  float eps;
  cdf_norm norm;
  int bits;
  cdf_qscheme qs;
  cdf_commit commit;
  int delta;
  uint8_t* mask;
  int32_t* idx;
  int32_t* n_sent;
  uint8_t* codes;
  float* meta;
} cdf_layer_bwd_args;

int cdf_gcn_layer_bwd(const cdf_layer_bwd_args* args /* host */, void* ws, size_t ws_bytes, void* stream);

/*
 * Transform-first variant of the layer step: Z = A^ (X W) instead of (A^ X) W (Sec. 3.1 writes
 * the product A^ H W without fixing the order). The rows that cross the partition boundary are
 * then rows of T = X W, f_out wide, so this order moves fewer bytes whenever f_out < f_in -
 * in the messages and in the aggregation alike. fp32 only.
 *
 * Forward:
 *   1. tfull[0:n_loc] = x_local W                                    (dense transform)
 *   2. cache test of halo_fresh (the owners' current T rows) against cache_sent, message build
 *      and commit, recovery into tfull[n_loc:]                       (Alg. 2, Sec. 5; f_out wide)
 *   3. Z = A tfull (optional), H = sigma(Z)                          (aggregation, ReLU fused)
 */
typedef struct {
  const cdf_csr* A;       /* host pointer; n_loc x (n_loc + n_halo) */
  int32_t n_loc, n_halo, f_in, f_out;
  int relu;
  const float* x_local;   /* n_loc x f_in */
  const float* W;         /* f_in x f_out */
  float* tfull;           /* (n_loc+n_halo) x f_out: local rows written, halo rows updated in place */
  const float* halo_fresh; /* n_halo x f_out */
  float* cache_sent;      /* n_halo x f_out */
  float eps;
  cdf_norm norm;
  int bits;
  cdf_qscheme qs;
  cdf_commit commit;
  int delta;
  float* Z;               /* out, nullable: n_loc x f_out */
  float* H;               /* out: n_loc x f_out */
  uint8_t* mask;          /* out: [n_halo] */
  int32_t* idx;           /* out: [n_halo] */
  int32_t* n_sent;        /* out: [1] */
  uint8_t* codes;         /* out: [n_halo * cdf_code_row_bytes(f_out, bits, qs)] */
  float* meta;            /* out: [n_halo * 2] */
} cdf_layer_tf_fwd_args;

int cdf_gcn_layer_tf_fwd(const cdf_layer_tf_fwd_args* args /* host */, void* ws, size_t ws_bytes, void* stream);

/*
 * Backward of the transform-first step:
 *   1. dZ = dH * sigma'(Zs)                                          (kept in the caller's dZ buffer)
 *   2. dtfull = A^T dZ : rows [0, n_loc) are dT of the local rows, rows [n_loc, ..) the partial
 *      gradients owed to the halo rows' owners
 *   3. cache test + message build on those halo gradient rows against gcache_sent
 *   4. dW = x_local^T dT_local ;  dx_local = dT_local W^T (skipped when dx_local is NULL)
 */
typedef struct {
  const cdf_csr* At;      /* host pointer; (n_loc + n_halo) x n_loc */
  int32_t n_loc, n_halo, f_in, f_out;
  int relu;
  const float* dH;        /* n_loc x f_out */
  const float* Zs;        /* n_loc x f_out: Z or H of the forward step (unused if !relu) */
  const float* x_local;   /* n_loc x f_in */
  const float* W;         /* f_in x f_out */
  float* dZ;              /* scratch: n_loc x f_out (unused if !relu) */
  float* dtfull;          /* out: (n_loc+n_halo) x f_out */
  float* dW;              /* out: f_in x f_out */
  float* dx_local;        /* out, nullable: n_loc x f_in */
  float* gcache_sent;     /* n_halo x f_out, updated in place by the commit */
  float eps;
  cdf_norm norm;
  int bits;
  cdf_qscheme qs;
  cdf_commit commit;
  int delta;
  uint8_t* mask;
  int32_t* idx;
  int32_t* n_sent;
  uint8_t* codes;
  float* meta;
} cdf_layer_tf_bwd_args;

int cdf_gcn_layer_tf_bwd(const cdf_layer_tf_bwd_args* args /* host */, void* ws, size_t ws_bytes, void* stream);

/*
 * ---- Pieces of the training loop around the layer step ----
 *
 * Softmax cross-entropy (the loss of Sec. 7.1) over the rows with 0 <= labels[r] < classes; the
 * other rows are outside the loss (Sec. 3.1: only owned vertices contribute) and get a zero gradient.
 *   *loss_sum = sum_r -log softmax(logits[r])[labels[r]]
 *   dlogits[r] = scale * (softmax(logits[r]) - onehot(labels[r]))
 *   counts[0] = rows whose largest logit (lowest index on ties) is the label, counts[1] = rows used
 * logits, dlogits: n x classes fp32 contiguous; labels int32 [n]; loss_sum [1], counts [2] device.
 * ws: cdf_workspace_bytes(n, classes, 0) is enough. Sums are taken in a fixed order.
 */
int cdf_softmax_xent(const float* logits, const int32_t* labels, int32_t n, int32_t classes, float scale,
                     float* dlogits, float* loss_sum, int32_t* counts, void* ws, size_t ws_bytes, void* stream);

/*
 * One Adam step (the optimiser of Sec. 7.1), t = 1, 2, ...:
 *   m <- beta1 m + (1-beta1) dW ; v <- beta2 v + (1-beta2) dW^2 ;
 *   W <- W - lr (m / (1-beta1^t)) / (sqrt(v / (1-beta2^t)) + eps)
 */
int cdf_adam_step(float* W, const float* dW, float* m, float* v, int64_t count, float lr, float beta1,
                  float beta2, float eps, int32_t t, void* stream);

/* dst[i] += src[i] (the owner's "sum with its own value" of Sec. 3.2, and the sum of the
 * partitions' parameter gradients when several partitions are stepped on one device). */
int cdf_accumulate(float* dst, const float* src, int64_t count, void* stream);

/*
 * Row exchange between partitions that are stepped on one device (stands in for the gather /
 * scatter messages of Sec. 3.2): dst row r = src row idx[r], r < n. idx on the device, every
 * idx[r] a valid row of src; rows of `dim` elements of type dt; src and dst must not overlap.
 */
int cdf_gather_rows(const void* src, int64_t ld_src, const int32_t* idx, int32_t n, int32_t dim,
                    cdf_dtype dt, void* dst, int64_t ld_dst, void* stream);

/* out[k] = map[idx[k]] for k < min(*n_sent, max_sent): turns the halo-local row list of a
 * message into the receiver's row numbers before cdf_dequantize applies it there. */
int cdf_map_index(const int32_t* idx, const int32_t* n_sent, int32_t max_sent, const int32_t* map,
                  int32_t* out, void* stream);

/*
 * ---- Pieces of the master / mirror exchange of the vertex-cut framing (Sec. 3.2, Alg. 2 in full) ----
 *
 * "active vertex u" (Alg. 2): flags[(map ? map[idx[k]] : idx[k]) + offset] = 1 for k < min(*n_sent, max_sent).
 * flags is a byte array the caller cleared; map may be NULL.
 */
int cdf_mark_rows(const int32_t* idx, const int32_t* n_sent, int32_t max_sent, const int32_t* map,
                  int32_t offset, uint8_t* flags, void* stream);

/*
 * The mirrors of active vertices (Alg. 2, last loop: the cached total of every active vertex goes to
 * its mirrors): mask[r] = flags[map[r]] != 0 for r < n_rows, idx = the ascending list of such r,
 * *n_sent their number. map[r] is the flag position of the master of mirror row r.
 * ws as for cdf_cache_filter.
 */
int cdf_active_rows(const uint8_t* flags, const int32_t* map, int32_t n_rows, uint8_t* mask, int32_t* idx,
                    int32_t* n_sent, void* ws, size_t ws_bytes, void* stream);

/* h[i] = max(z[i], 0): the activation applied after the exchange has combined the partial sums
 * (Sec. 3.1, H = sigma(Z), with Z only complete once Alg. 2 has run). */
int cdf_relu_fwd(const float* z, float* h, int64_t count, void* stream);

/*
 * Threshold controller (Sec. 4.1, the case equation and the moving average). Host function.
 *   acc < mean - mu1 and eps < nu1 :  eps <- min(lambda1 eps, eps + xi)
 *   acc > mean + mu2 and eps > nu2 :  eps <- max(lambda2 eps, eps - xi)
 *   then *mean_acc <- 0.8 *mean_acc + 0.2 acc   (the accuracy is compared with the average of the
 *   epochs before it). swap_conditions != 0 exchanges the two conditions, which is what the prose
 *   of Sec. 4.1 describes. p == NULL: the paper's defaults (0.001, 0.02, 0.3, 0.001, 0.01, 1.05, 0.9).
 */
typedef struct {
  float mu1, mu2, nu1, nu2, xi, lambda1, lambda2;
  int swap_conditions;
} cdf_eps_params;
float cdf_eps_update(float eps, float acc, float* mean_acc /* host, in/out */, const cdf_eps_params* p /* host */);

/*
 * ---- Graph partitioning (host functions, host pointers, no GPU involved) ----
 *
 * Hierarchical EBV vertex-cut (Sec. 6): the undirected edges (eu[e], ev[e]), each listed once,
 * no self pairs, are assigned one after another; edge (u, v) goes to the device i with the
 * smallest
 *   (1-gamma) ([i not in d_rep_u] + [i not in d_rep_v]) + gamma ([host_i not in h_rep_u] + [host_i not in h_rep_v])
 *   + alpha e_count[i] / (|E|/p) + beta v_count[i] / (|V|/p)                       (double arithmetic,
 * terms added left to right; the lowest i wins ties), host_i = i / devices_per_host. d_rep / h_rep are
 * the devices / hosts a vertex already has a replica on, e_count / v_count the edges / vertex replicas
 * assigned to a device so far. sort_edges != 0 processes the edges by ascending sum of their end
 * vertices' degrees (stable; the order of the EBV algorithm the section builds on), otherwise as given.
 * gamma = 0 is plain EBV. part [n_edges] receives the device of every edge. p <= 64.
 */
typedef struct {
  int32_t p, devices_per_host;
  double alpha, beta, gamma;
  int sort_edges;
} cdf_ebv_params;
int cdf_ebv_partition(int64_t n_vertices, int64_t n_edges, const int64_t* eu, const int64_t* ev,
                      const cdf_ebv_params* prm, int32_t* part);

/*
 * Statistics of a vertex-cut (Sec. 6: replication factor sum|V_i| / |V|, edge imbalance
 * max|E_i| / (|E|/p), vertex imbalance max|V_i| / (sum|V_i|/p); Sec. 7 ablation: the largest number of
 * messages one device sends inside its host / across hosts per exchange, counting one gather message per
 * mirror and one scatter message per mirror of each of its masters). The master of a vertex is the replica
 * holding most of its edges (lowest device on ties; a vertex without edges lives on device v mod p);
 * master [n_vertices] is written when not NULL.
 */
typedef struct {
  double replication_factor, edge_imbalance, vertex_imbalance;
  int64_t max_inner, max_outer, replicas_total;
} cdf_cut_stats;
int cdf_cut_statistics(int64_t n_vertices, int64_t n_edges, const int64_t* eu, const int64_t* ev,
                       const int32_t* part, int32_t p, int32_t devices_per_host, int32_t* master,
                       cdf_cut_stats* out);

#ifdef __cplusplus
}
#endif
#endif /* CDF_H */
