/*
 * basa.h — C ABI of the MI355X (gfx950) Block Approximate Sparse Attention library.
 *
 * The library implements the operator of the paper's Alg. 1 ("Norm-Rank Attention
 * with Covariance Compensation") in three stages plus a dense baseline:
 *   1. norm ranking and block pooling      (Sec. 3.3 Eq. 9-10; Sec. 3.1; Sec. 3.4)
 *   2. compensated block-score map, row distribution and top-kappa block selection
 *                                           (Eq. 2, Eq. 13-14, Alg. 1 steps 5-11)
 *   3. bidirectional block-sparse attention over the kept blocks
 *                                           (Sec. 2, Alg. 1 step 12)
 *
 * General rules
 *   - Every data pointer is a DEVICE pointer unless a comment says "host".
 *     Descriptor structs (basa_tensor, basa_params) are read on the HOST.
 *   - The caller owns every buffer, including workspaces.  The library never
 *     allocates or frees device memory and never synchronises: all work is
 *     enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream).
 *   - Functions return a basa_status.  Arguments are validated on the host before
 *     any kernel is launched; on error nothing has been enqueued.  A human-readable
 *     reason is kept per thread and returned by basa_last_error().
 *   - Tensors are [batch, heads, L, d] with d contiguous; strides are in elements.
 *     Supported: d in {64, 128}; dtype f32 or bf16; block B in {64, 128}.
 *     Query head h reads KV head h / (heads_q / heads_kv).
 *   - Blocks: block g of a sorted sequence holds sorted positions
 *     [g*B, min((g+1)*B, L)); N = ceil(L/B); a ragged last block is allowed.
 *   - Permutations and block lists passed IN are device data the host cannot check.
 *     A permutation entry outside [0, L) is replaced by its own position and a list
 *     entry outside [0, N_k) is skipped: malformed input gives wrong rows, never an
 *     access outside the caller's tensors.
 */
#ifndef BASA_H
#define BASA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  BASA_OK = 0,
  BASA_ERR_INVALID_ARG = 1,  /* null pointer, bad shape, bad parameter value            */
  BASA_ERR_UNSUPPORTED = 2,  /* legal request this build has no kernel for               */
  BASA_ERR_WORKSPACE = 3,    /* workspace pointer null or smaller than required          */
  BASA_ERR_HIP = 4           /* a HIP runtime call failed; see basa_last_error()         */
} basa_status;

typedef enum { BASA_F32 = 0, BASA_BF16 = 1 } basa_dtype;

/* Which sequences are norm-sorted before blocking (the four rows of Tab. 7). */
typedef enum { BASA_SORT_NONE = 0, BASA_SORT_Q = 1, BASA_SORT_K = 2, BASA_SORT_QK = 3 } basa_sort;

typedef struct {
  const void* ptr;           /* device                                                    */
  int32_t dtype;             /* basa_dtype                                                */
  int32_t batch, heads, L, d;
  int64_t stride_b, stride_h, stride_l;   /* in elements; the d axis has stride 1        */
} basa_tensor;

typedef struct {
  int32_t block;             /* B: 64 or 128 (Tab. 1 caption; Sec. 4.1 uses 128)          */
  int32_t sort;              /* basa_sort; the full method is BASA_SORT_QK                */
  int32_t window;            /* 0: one sort per head (Sec. 3.3); W>0: every run of W
                                consecutive tokens is sorted by itself (Alg. 1 step 1,
                                "(windowed) sort"); W must be a multiple of B             */
  float beta;                /* compensation weight of Eq. 13 (default 1; 0 = plain Eq. 2) */
  double sparsity;           /* s in [0,1): every query block keeps
                                kappa = max(1, N_k - floor(s*N_k + 1e-9)) key blocks       */
  double mass_target;        /* 0: keep exactly kappa blocks per row (Alg. 1 step 10).
                                p in (0,1]: keep, in order of decreasing m', the FEWEST
                                blocks whose m' sum to at least p ("the mask is built from
                                m under a computational budget", Sec. 3.1 after Eq. 2, read
                                as a mass budget), at least min_keep and at most kappa    */
  int32_t min_keep;          /* floor on the per-row count when mass_target > 0; 0 means 1 */
  int32_t attn_shape;        /* basa_sparse_attn, bf16 only: shape of the attention workgroup.
                              * 0 = chosen by the library (on the device, between 3 and 2, from
                              * how much the lists of neighbouring query blocks overlap),
                              * 1 = 256 queries sharing every K/V tile, 2 = 128 queries,
                              * 3 = 512 queries (64 per wave).  1 and 2 give identical bits;
                              * 3 runs the online softmax against a reference that is raised only
                              * when the row sums ask for it, not against the running maximum, and
                              * repeats with running maxima the workgroups whose row sums left the
                              * range in which that is exact; 4 = shape 3 with running maxima from
                              * the start (for comparison).  3 and 4 agree with 1 and 2 within the
                              * output tolerance.  The causal variant always runs shape 3 (4 if
                              * asked for); other entry points ignore the field */
  int32_t n_segments;        /* 0: none.  1..BASA_MAX_SEGMENTS: the sort is segment-aware (the
                                windowed sort of Alg. 1 step 1 with runs of unequal length, e.g.
                                one run per modality or frame): tokens segment_starts[j] ..
                                segment_starts[j+1]-1 (the last segment ends at L) are sorted
                                among themselves and keep their range of positions.  Excludes
                                window > 0; with two tensors (basa_select) L_q must equal L_k  */
  int32_t budget_total;      /* 0: none.  G > 0: the rows of one (batch, head) keep at most G key
                                blocks together.  The rows that ask for the most are trimmed
                                first, to a common cap t: the largest t in [max(1, min_keep),
                                kappa] with sum_r min(count_r, t) <= G (if even the smallest t
                                does not fit, the per-row minimum wins); a trimmed row keeps its
                                t blocks of largest m'.  With mass_target = 0 every row asks for
                                kappa, so G lowers the common count to G / N_q                 */
  const int32_t* segment_starts;   /* HOST array of n_segments token indices: first 0, strictly
                                ascending, last < L; read during the call only (NULL if none) */
  int32_t causal;            /* 0: bidirectional attention, the paper's method.  1: the autoregressive
                                variant the paper names as future work (Sec. 6), under this
                                library's own reading: the query at ORIGINAL index i may attend to
                                the key at original index j iff j <= i + (L_k - L_q), whatever the
                                sorting did to their positions.  basa_select then drops every block
                                pair without a visible token pair before the row softmax and the
                                ranking, and a row keeps min(kappa, its live blocks) (row_count may
                                be 0 when L_q > L_k); basa_sparse_attn / basa_dense_attn mask token
                                by token, and a query none of whose visible keys lie in the listed
                                blocks gets a zero output row and lse = -inf.  The `scores` output
                                of basa_select stays unmasked                                   */
  int32_t select_path;       /* basa_select: how the score map of Eq. 2 / Eq. 14 reaches the row
                                selection of Alg. 1 steps 9-11.  1 = through the map in the workspace
                                (one kernel writes it, one reads it).  2 = in one kernel that
                                keeps the map on chip; possible when nobody needs the map in
                                memory (fixed count per row, no `scores` output, no total budget,
                                not causal, at most 1024 key blocks per row), else
                                BASA_ERR_UNSUPPORTED.  0 = the library's choice: the faster of the
                                two where both apply, which on MI355X is 1.  Logits, kept sets
                                and lists are the same either way; row_mass may differ in its
                                last bits (another order of summation)                          */
} basa_params;
#define BASA_MAX_SEGMENTS 63

/* Host helper: the per-query-block budget kappa (Alg. 1 input) for n_k key blocks at
 * sparsity s, by the formula above.  Returns -1 if s is outside [0,1) or n_k < 1. */
int32_t basa_kappa(int32_t n_k, double sparsity);

/* Bytes of workspace basa_select needs for these shapes (0 on invalid arguments).  Each stage has
 * its own size call, so that a caller who runs one stage does not reserve the others' scratch. */
size_t basa_select_workspace_size(const basa_tensor* q, const basa_tensor* k, const basa_params* p);
/* Bytes of workspace basa_sparse_attn / basa_dense_attn need (0 on invalid arguments). */
size_t basa_attn_workspace_size(const basa_tensor* q, const basa_tensor* k, const basa_params* p);
/* Bytes of workspace basa_norm_sort needs for x. */
size_t basa_sort_workspace_size(const basa_tensor* x, const basa_params* p);

/*
 * Norm ranking of one tensor (Sec. 3.3, Eq. 9-10; Alg. 1 steps 1-2).
 * The sort key of a token is its squared L2 norm, accumulated in fp64 and rounded
 * once to fp32; tokens are ordered by non-decreasing key, equal keys by original
 * index; p->window selects windowed sorting.
 *   perm      out [batch, heads, L] int32: perm[i] = original index of the token at
 *             sorted position i.
 *   keys_out  out, nullable, [batch, heads, L] float: the fp32 keys, original order.
 *   ws        workspace of basa_sort_workspace_size() bytes.
 */
basa_status basa_norm_sort(const basa_tensor* x, const basa_params* p, int32_t* perm,
                           float* keys_out, void* ws, size_t ws_bytes, void* stream);

/*
 * basa_norm_sort for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs,
 * outputs and results as basa_norm_sort; the two buffers of packed sort words live in a device
 * array of BASA_STATIC_SCRATCH_BYTES that is part of the library image (every GPU the library
 * runs on holds one copy until the process ends).  The call allocates and frees nothing, creates
 * no events (the basa_profile_* timing aid does not see it) and does not synchronise.
 *   - batch * heads * L above BASA_STATIC_SCRATCH_BYTES / 16 tokens (2 Mi with the default size):
 *     BASA_ERR_WORKSPACE, nothing enqueued.
 *   - Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (two streams,
 *     two threads) race; serialise them.  Nothing has to start at zero, so no clearing is done.
 *   - The array's address is resolved once per device, at the first call made with that device
 *     current, or by basa_static_init(); a caller that records a graph calls basa_static_init()
 *     before the capture begins.
 */
#define BASA_STATIC_SCRATCH_BYTES (32u << 20)
size_t basa_static_scratch_size(void);
basa_status basa_static_init(void);
basa_status basa_norm_sort_static(const basa_tensor* x, const basa_params* p, int32_t* perm,
                                  float* keys_out, void* stream);

/*
 * Block pooling (Sec. 3.1 mean pooling; Sec. 3.4 "blockwise first/second moments";
 * Alg. 1 steps 3-4): per block of the ordered sequence x[perm], the mean and the
 * per-dimension population variance (divide by the block's token count).
 *   perm      nullable [batch, heads, L] int32; NULL = original order.
 *   mean      out [batch, heads, N, d] float.
 *   var       out, nullable, [batch, heads, N, d] float.
 *   x_sorted  out, nullable: the ordered sequence itself, x_sorted[b, h, i, :] = x[b, h, perm[i], :],
 *             contiguous [batch, heads, L, d] in the dtype of x, 16-byte aligned, not aliasing x
 *             (the pooling pass holds every row anyway; materialising it costs the write only).
 */
basa_status basa_downsample(const basa_tensor* x, const int32_t* perm, const basa_params* p,
                            float* mean, float* var, void* x_sorted, void* stream);

/*
 * Block selection (Alg. 1 steps 1-11): norm ranking of Q and/or K (p->sort), block
 * statistics, compensated block logits l' = Qbar.Kbar/sqrt(d) + beta*Delta^ with
 * Delta^ of Eq. 14, row softmax m' (Eq. 2) and the kappa largest m' per row (equal
 * values: lower key-block index first).  With p->mass_target > 0 the number kept varies by
 * row: the fewest of the largest m' that sum to at least mass_target, clamped to
 * [min_keep, kappa]; the sums are formed in fp32, so a row whose cumulative mass comes
 * within rounding (about 1e-6 relative) of the target may keep one block more or fewer
 * than exact arithmetic would.
 *   mask_bits  out, nullable, [batch, heads_q, N_q, ceil(N_k/32)] uint32, bit (g_k%32)
 *              of word g_k/32 set iff block pair (g_q, g_k) is kept.
 *   row_count  out [batch, heads_q, N_q] int32: number of kept key blocks (= kappa, or the
 *              row's own count when mass_target > 0).
 *   row_cols   out [batch, heads_q, N_q, kappa] int32: kept key blocks, ascending, in the
 *              first row_count entries of each row (the rest is left untouched).
 *   perm_q     out [batch, heads_q, L_q] int32 (identity when Q is not sorted).
 *   perm_k     out [batch, heads_kv, L_k] int32 (identity when K is not sorted).
 *   row_mass   out, nullable, [batch, heads_q, N_q] float: sum of kept m'.
 *   scores     out, nullable, [batch, heads_q, N_q, N_k] float: the logits l'.
 *   ws         workspace of basa_select_workspace_size() bytes.
 */
basa_status basa_select(const basa_tensor* q, const basa_tensor* k, const basa_params* p,
                        uint32_t* mask_bits, int32_t* row_count, int32_t* row_cols,
                        int32_t* perm_q, int32_t* perm_k, float* row_mass, float* scores,
                        void* ws, size_t ws_bytes, void* stream);

/*
 * Block-sparse attention (Sec. 2; Alg. 1 step 12).  For every query block g_q of the
 * ordered queries Q' = Q[perm_q], softmax attention (Eq. 1) restricted to the tokens
 * of the listed key blocks of K' = K[perm_k], V' = V[perm_k], normalised over those
 * tokens; the row of sorted position i is written to out row perm_q[i].
 * bf16 tensors: bf16 MFMA with fp32 accumulation and fp32 softmax state (d = 64 or 128);
 * f32 tensors: fp32 throughout.
 *   row_count    [batch, heads_q, N_q] int32, each in [1, N_k].
 *   row_cols     [batch, heads_q, N_q, cols_stride] int32, ascending, each in [0, N_k).
 *                NULL means every key block for every row (dense).  The lists are device
 *                data the host cannot check: an entry outside [0, N_k) is ignored, a count
 *                above cols_stride is cut to it, and a query block left without any valid
 *                key block gets zero output rows (lse -inf).  Entries must not repeat.
 *   perm_q/_k    nullable (NULL = identity).
 *   out          [batch, heads_q, L_q, d], dtype of q, 16-byte aligned.
 *   out_strides  nullable HOST array of 3: strides of out's batch, head and token axes in
 *                elements (each a multiple of 16 bytes, token stride >= d; the d axis has
 *                stride 1).  NULL = contiguous.  A token-major [batch, L_q, heads_q, d]
 *                buffer, which a following projection reads directly, is {L*H*d, d, H*d}.
 *                Rows of out must not alias each other or the inputs.
 *   lse          out, nullable, [batch, heads_q, L_q] float: log-sum-exp of the kept
 *                logits of every query (original order).
 *   ws           workspace of basa_attn_workspace_size() bytes.
 *   p            block and attn_shape are read.
 */
basa_status basa_sparse_attn(const basa_tensor* q, const basa_tensor* k, const basa_tensor* v,
                             const int32_t* row_count, const int32_t* row_cols,
                             int32_t cols_stride, const int32_t* perm_q, const int32_t* perm_k,
                             const basa_params* p, void* out, const int64_t* out_strides,
                             float* lse, void* ws, size_t ws_bytes, void* stream);

/*
 * Dense bidirectional attention (Eq. 1) through the same kernels with every key
 * block listed and no permutation: the baseline sparse runs are compared with.
 * Only p->block is read.
 */
basa_status basa_dense_attn(const basa_tensor* q, const basa_tensor* k, const basa_tensor* v,
                            const basa_params* p, void* out, const int64_t* out_strides,
                            float* lse, void* ws, size_t ws_bytes, void* stream);

const char* basa_status_string(basa_status s);
/* Reason of the last non-OK status returned on this thread (host string, owned by the
 * library, valid until the next failing call on the thread). */
const char* basa_last_error(void);
/*
 * Per-kernel timing aid for benchmarks.  While enabled, every kernel launch of the
 * entry points above is bracketed by a pair of HIP events recorded on the caller's
 * stream (events are created per launch; nothing else changes).  basa_profile_read
 * waits for the recorded events, adds the elapsed milliseconds and launch counts per
 * kernel id into the host arrays total_ms[n] / launches[n] (n >= basa_profile_kernel_count()),
 * and forgets the records.  Kernel ids are 0 .. count-1; basa_profile_kernel_name(id)
 * names them.  Not for use under stream capture.
 */
basa_status basa_profile_enable(int on);
int32_t basa_profile_kernel_count(void);
const char* basa_profile_kernel_name(int32_t id);
basa_status basa_profile_read(double* total_ms /*host*/, int32_t* launches /*host*/, int32_t n);

/*
 * ---- Selection-fidelity diagnostics (off the hot path; cost of a dense attention) ----
 *
 * Oracle block distribution (Sec. 3.1, Eq. 3): m_hat[g_q, g_k] = mean over the query
 * tokens of block g_q of the dense attention weight (Eq. 1) that falls on the key tokens
 * of block g_k, for the ordered sequences Q[perm_q], K[perm_k] (NULL: original order).
 * bf16 tensors run on the matrix cores (d = 64 or 128; with max_dev at most 8192 / (128 / B) key
 * blocks, BASA_ERR_UNSUPPORTED beyond), f32 tensors on an exact-arithmetic kernel that is not tuned.
 *   base_logits  nullable [batch, heads_q, N_q, N_k] float: block logits l of Eq. 2
 *                (basa_select's `scores` with beta = 0); needed for max_dev.
 *   m_hat        out [batch, heads_q, N_q, N_k] float; every row sums to 1.
 *   max_dev      out, nullable, same shape: max over the token pairs (i, j) of the block pair
 *                of |Q_i.K_j/sqrt(d) - base_logits[g_q, g_k]|, the observed deviation that
 *                Sec. 3.2 bounds by U (Eq. 8) and Fig. 2 correlates with it.
 *   lse          out, nullable, [batch, heads_q, L_q] float, original token order:
 *                log-sum-exp of every query's scaled logits over all keys.
 *   ws           workspace of basa_block_mass_workspace_size() bytes (0 on invalid arguments).
 */
size_t basa_block_mass_workspace_size(const basa_tensor* q, const basa_tensor* k);
basa_status basa_block_mass(const basa_tensor* q, const basa_tensor* k, const int32_t* perm_q,
                            const int32_t* perm_k, const basa_params* p, const float* base_logits,
                            float* m_hat, float* max_dev, float* lse, void* ws, size_t ws_bytes,
                            void* stream);
/*
 * Block-wise norm metrics (Sec. 3.2, Eq. 7) of the ordered sequence x[perm]: per block the
 * radius R = max_i ||x_i - mean|| and the maximum norm M = max_i ||x_i||.
 *   radius, max_norm  out [batch, heads, N] float.
 */
basa_status basa_block_radius(const basa_tensor* x, const int32_t* perm, const basa_params* p,
                              float* radius, float* max_norm, void* stream);
/*
 * Deviation bound (Eq. 8): bound[bh, g_q, g_k] = (R^Q M^K + M^Q R^K + R^Q R^K) / sqrt(d) from the
 * outputs of basa_block_radius for Q ([bh_q, n_q]) and K ([bh_kv, n_k]); query head bh reads
 * KV head bh / (bh_q / bh_kv).   bound: out [bh_q, n_q, n_k] float.
 */
basa_status basa_deviation_bound(const float* radius_q, const float* max_norm_q, const float* radius_k,
                                 const float* max_norm_k, int32_t bh_q, int32_t bh_kv, int32_t n_q,
                                 int32_t n_k, int32_t d, float* bound, void* stream);
/*
 * Per row of the block map (rows = batch * heads_q * N_q, n_k columns): recall = sum of m_hat
 * over the blocks kept in mask_bits (the dense attention mass the selection retains), and
 * l1 = || softmax(scores) - m_hat ||_1, the distance the analysis of Sec. 3.2 is about.
 * All device pointers; recall and l1 are [rows] float, either may be NULL (not both).
 */
basa_status basa_selection_fidelity(const float* scores, const uint32_t* mask_bits, const float* m_hat,
                                    int64_t rows, int32_t n_k, float* recall, float* l1, void* stream);
/*
 * The sums a Pearson correlation coefficient (R of Fig. 2) is made of, over n pairs of device
 * floats: sums[0..5] = n, sum x, sum y, sum x^2, sum y^2, sum xy (device, fp64, overwritten).
 * Accumulated with fp64 atomics: the last bits depend on the order of arrival.
 */
basa_status basa_pearson_sums(const float* x, const float* y, int64_t n, double* sums, void* stream);

/*
 * Calibration aid for benchmarks (no part of the method): enqueues a kernel that issues
 * `iters` x 32 independent bf16 32x32x16 matrix-core instructions per wave on register
 * operands, 8 waves per compute unit, and nothing else.  random_operands != 0: the operand
 * fragments hold pseudo-random values and change from one instruction to the next, as they
 * do in real work; 0: one constant everywhere.  The rate this loop reaches is the rate the
 * chip sustains for such operands (its power management included).
 *   out        device, at least 131072 floats (scratch the kernel writes its sums to)
 *   out_elems  floats `out` holds; too few: BASA_ERR_WORKSPACE
 *   flops      host, nullable: receives the floating-point operations of the launch
 * Time it with events on `stream`.
 */
basa_status basa_calibrate_mfma(int32_t random_operands, int32_t iters, float* out, size_t out_elems,
                                double* flops /*host*/, void* stream);

/*
 * Calibration aid: enqueues one read-only pass over `bytes` bytes of device memory at `buf`
 * (16-byte aligned, at least 1 MiB; a tail of up to 32 KiB may be left unread), 16-byte loads,
 * nothing written but possibly the word at `out` (device).  bytes / elapsed time is the
 * read-only stream rate the memory system sustains.
 */
basa_status basa_calibrate_read(const void* buf, size_t bytes, uint32_t* out, void* stream);

/* Library version, e.g. "basa 0.1 gfx950". */
const char* basa_version(void);

#ifdef __cplusplus
}
#endif
#endif /* BASA_H */
