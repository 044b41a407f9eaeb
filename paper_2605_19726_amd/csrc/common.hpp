// Shared host/device declarations of the basa library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "basa.h"

namespace basa {

constexpr int kWave = 64;

// A [batch, heads, L, d] tensor as the kernels see it (passed by value).
struct TensorView {
  const void* ptr;
  int32_t dtype;  // basa_dtype
  int32_t batch, heads, L, d;
  int64_t stride_b, stride_h, stride_l;
  __host__ __device__ inline int64_t head_offset(int bh) const {
    int b = bh / heads, h = bh - b * heads;
    return (int64_t)b * stride_b + (int64_t)h * stride_h;
  }
};

inline TensorView view_of(const basa_tensor& t) {
  return TensorView{t.ptr, t.dtype, t.batch, t.heads, t.L, t.d, t.stride_b, t.stride_h, t.stride_l};
}

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Thread-local error text behind basa_last_error().
void set_error(const char* fmt, ...);
basa_status hip_fail(hipError_t e, const char* what);

#define BASA_HIP_CHECK_LAUNCH(what)                          \
  do {                                                       \
    hipError_t e__ = hipGetLastError();                      \
    if (e__ != hipSuccess) return ::basa::hip_fail(e__, what); \
  } while (0)

// ---- optional per-kernel timing (basa_profile_*): a scope object brackets one launch
// with a pair of HIP events on the launch stream when profiling is enabled.
enum KernelId {
  K_NORM_TILE_SORT = 0, K_MERGE, K_STATS, K_SCORES, K_ROW_SELECT, K_GATHER, K_ATTN,
  K_ATTN_SIMPLE, K_BLOCK_MASS, K_DIAG_SMALL, K_SCORES_SELECT, K_COUNT
};
struct ProfScope {
  ProfScope(int id, hipStream_t st);
  ~ProfScope();
  int slot_;
  hipStream_t st_;
};

// ---- stage launchers (each validates nothing: the C entry points do) -------------

// Sort keys + segmented sort.  Writes perm[bh][L]; optional keys_out[bh][L].
size_t sort_workspace_bytes(int BH, int L);
constexpr int kMaxSortLen = 1 << 27;      // token indices take 27 bits of a packed sort word
// Segment starts of a segment-aware sort, passed to kernels by value: bound[0] = 0 < bound[1] <
// ... < bound[n-1] < bound[n] = L; n <= 1 means one segment.
struct SegList {
  int n;
  int bound[BASA_MAX_SEGMENTS + 1];
};
basa_status launch_norm_sort(const TensorView& x, int window, const SegList& segs, int32_t* perm, float* keys_out,
                             void* ws, hipStream_t st);
// Two tensors of identical L, d and dtype through the same launches (ws sized for both).
basa_status launch_norm_sort2(const TensorView& q, const TensorView& k, int window, const SegList& segs, int32_t* perm_q,
                              int32_t* perm_k, void* ws, hipStream_t st);
basa_status launch_iota_perm(int32_t* perm, int BH, int L, hipStream_t st);

// Block statistics.  Any of the outputs may be null.
//   mean/var : [BH][N][d]
//   feat     : selection features as three bf16 parts whose sum is the fp32 value (part 0 its bf16
//              rounding, part 1 the rounding of the rest, part 2 of what is left: 24 bits together),
//              [BH][part 3][3d/8][N][8] bf16: feature k of block g at [part][k/8][g][k%8]; feat_bytes_per_block(d)
//              bytes per block
//              (content depends on `feat_is_query`):
//              query side (Qbar/sqrt(d), beta*VarQ/d, beta*Qbar^2/d),
//              key side   (Kbar, Kbar^2+VarK, VarK)
//   x_sorted : the ordered sequence x[perm] itself, contiguous [BH][L][d] in the dtype of x
basa_status launch_block_stats(const TensorView& x, const int32_t* perm, int B, float* mean,
                               float* var, void* feat, int feat_is_query, float beta, void* x_sorted,
                               hipStream_t st);

// Selection features of Q (query side) and K (key side), identical L / d / dtype, in one launch.
basa_status launch_select_features(const TensorView& q, const int32_t* perm_q, void* feat_q,
                                   const TensorView& k, const int32_t* perm_k, void* feat_k, int B,
                                   float beta, hipStream_t st);

// Block logits: scores[BHq][Nq][Nk] = featQ . featK over `kdim` features.
inline size_t feat_bytes_per_block(int d) { return (size_t)3 * 3 * d * 2; }
basa_status launch_block_scores(const void* featQ, const void* featK, float* scores, int BHq,
                                int group, int Nq, int Nk, int kdim_used, int feat_stride,
                                hipStream_t st);

// Score map and fixed-count selection in one launch, the map kept on chip (at most 1024 key blocks
// per row, whole k-steps of 16): same logits, same kept sets and lists as launch_block_scores followed by
// launch_row_select with mass_target = 0.  scores_select_supported says whether a shape qualifies.
bool scores_select_supported(int Nk, int kdim_used, int feat_stride);
basa_status launch_scores_select(const void* featQ, const void* featK, int BHq, int group, int Nq, int Nk,
                                 int kdim_used, int feat_stride, int kappa, uint32_t* mask_bits,
                                 int32_t* row_count, int32_t* row_cols, float* row_mass, hipStream_t st);

// Row softmax mass + top-kappa selection from a score map; mass_target > 0 switches to the
// cumulative-mass count per row (floor min_keep, cap kappa).  row_cols rows are kappa apart.
// keep_in (nullable): per-row count that replaces both rules (used after launch_budget_cap).
// live (nullable): causal liveness of block pairs, see launch_block_index_range; a row then keeps
// at most as many blocks as are live for it (possibly none).
struct LiveBlocks {
  const int32_t* q_max;       // [BHq][Nq] largest original index among the queries of a block, or null
  const int32_t* k_min;       // [BHkv][Nk] smallest original index among the keys of a block
  int Nq, group, offset;      // rows per head, query heads per KV head, L_k - L_q
};
basa_status launch_row_select(const float* scores, int rows_total, int Nk, int kappa,
                              float mass_target, int min_keep, const int32_t* keep_in, const LiveBlocks& live,
                              uint32_t* mask_bits, int32_t* row_count, int32_t* row_cols, float* row_mass,
                              hipStream_t st);
// Per block of a permutation: out[bh][g] = max (want_max) or min of perm[bh][g*B .. min((g+1)*B, L)).
basa_status launch_block_index_range(const int32_t* perm, int BH, int L, int B, int want_max, int32_t* out,
                                     hipStream_t st);

// Total budget per (batch, head): keep_out[r] = min(row_count[r], t), t the largest cap in
// [max(1, floor_keep), kappa] with sum_r min(row_count[r], t) <= budget (else the smallest cap).
basa_status launch_budget_cap(const int32_t* row_count, int BHq, int Nq, int kappa, int floor_keep,
                              int budget, int32_t* keep_out, hipStream_t st);

// Attention.
struct AttnArgs {
  TensorView q, k, v;
  const int32_t* row_count;   // [BHq][Nq]
  const int32_t* row_cols;    // [BHq][Nq][cols_stride] or null (= all blocks)
  int32_t cols_stride;
  const int32_t* perm_q;      // [BHq][Lq] or null
  const int32_t* perm_k;      // [BHkv][Lk] or null
  int B;
  void* out;                  // [batch][heads_q][Lq][d], dtype of q, strides below (elements; d has stride 1)
  int64_t out_sb, out_sh, out_sl;
  __host__ __device__ inline int64_t out_offset(int bh, int64_t row) const {
    const int b = bh / q.heads, h = bh - b * q.heads;
    return (int64_t)b * out_sb + (int64_t)h * out_sh + row * out_sl;
  }
  float* lse;                 // [BHq][Lq] or null
  void* ws;
  size_t ws_bytes;
  int variant;                // matrix-core path: 0 = library's choice, 1 = 256 queries per workgroup, 2 = 128, 3 = 512
  int causal;                 // 1: key at original index j is visible to the query at original index i iff j <= i + causal_off
  int causal_off;             // L_k - L_q
};
size_t attn_mfma_workspace_bytes(int BHq, int BHkv, int Lq, int Lk, int d, int B);
basa_status launch_attn_simple(const AttnArgs& a, hipStream_t st);
basa_status launch_attn_mfma(const AttnArgs& a, hipStream_t st);

// Selection-fidelity diagnostics (diag.hip).  block mass: bf16 on the matrix cores, f32 on a plain kernel.
size_t block_mass_workspace_bytes(int BHq, int BHkv, int Lq, int Lk, int d);
basa_status launch_block_mass(const TensorView& q, const TensorView& k, const int32_t* perm_q,
                              const int32_t* perm_k, int B, const float* base_logits, float* m_hat,
                              float* max_dev, float* lse, void* ws, hipStream_t st);
basa_status launch_block_radius(const TensorView& x, const int32_t* perm, int B, float* radius,
                                float* max_norm, hipStream_t st);
basa_status launch_deviation_bound(const float* rq, const float* mq, const float* rk, const float* mk,
                                   int BHq, int group, int Nq, int Nk, int d, float* U, hipStream_t st);
basa_status launch_fidelity_rows(const float* scores, const uint32_t* mask_bits, const float* m_hat,
                                 int rows, int Nk, float* recall, float* l1, hipStream_t st);
basa_status launch_pearson_sums(const float* x, const float* y, int64_t n, double* sums, hipStream_t st);

// calibration (calib.hip): a loop of independent bf16 MFMAs on register operands
size_t calib_mfma_out_elems();
double calib_mfma_flops(int iters);
hipError_t launch_calib_mfma(bool random_operands, int iters, float* out, hipStream_t stream);
hipError_t launch_calib_read(const void* buf, size_t bytes, uint32_t* out, hipStream_t stream);

// ---- device helpers ------------------------------------------------------------
#if defined(__HIPCC__)
// Entry `pos` of a permutation of 0..L-1 (null = identity).  Permutations are device data the
// host cannot check: a value that is no index falls back to `pos`, so that a malformed
// permutation gives wrong rows, never an access outside the tensor.
__device__ __forceinline__ int perm_at(const int32_t* __restrict__ pm, int64_t offset, int pos, int L) {
  if (!pm) return pos;
  const int r = pm[offset + pos];
  return (unsigned)r < (unsigned)L ? r : pos;
}
__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}
// Chunk `sub` of the rows at sorted positions pos0, pos0 + step, ... (zeros past L).  All loads are
// unconditional with clamped indices and issued back to back (first the permutation entries, then
// the rows): a load inside a divergent branch is followed by a full wait, which serialises them.
template <int ITERS>
__device__ __forceinline__ void gather_chunks(uint4 (&v)[ITERS], const int32_t* pm, const char* base, int L,
                                              int64_t row_bytes, int pos0, int step, int sub) {
  int row[ITERS];
  if (pm) {
#pragma unroll
    for (int it = 0; it < ITERS; ++it) row[it] = pm[min(pos0 + it * step, L - 1)];
  } else {
#pragma unroll
    for (int it = 0; it < ITERS; ++it) row[it] = min(pos0 + it * step, L - 1);
  }
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int r = (unsigned)row[it] < (unsigned)L ? row[it] : min(pos0 + it * step, L - 1);   // malformed entry
    v[it] = reinterpret_cast<const uint4*>(base + r * row_bytes)[sub];
  }
#pragma unroll
  for (int it = 0; it < ITERS; ++it)
    if (pos0 + it * step >= L) v[it] = make_uint4(0u, 0u, 0u, 0u);
}

// 16 bytes of a row as floats: 8 bf16 or 4 f32 values.
template <bool kBf16>
struct Chunk16 {
  static constexpr int kElems = kBf16 ? 8 : 4;
  float v[kElems];
  __device__ __forceinline__ void load(const void* row_base, int chunk) {
    set(reinterpret_cast<const uint4*>(row_base)[chunk]);
  }
  __device__ __forceinline__ void set(const uint4& raw) {
    if constexpr (kBf16) {
      uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        v[2 * i] = __uint_as_float(w[i] << 16);
        v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
      }
    } else {
      v[0] = __uint_as_float(raw.x); v[1] = __uint_as_float(raw.y);
      v[2] = __uint_as_float(raw.z); v[3] = __uint_as_float(raw.w);
    }
  }
  __device__ __forceinline__ void zero() {
#pragma unroll
    for (int i = 0; i < kElems; ++i) v[i] = 0.f;
  }
};
#endif

}  // namespace basa
