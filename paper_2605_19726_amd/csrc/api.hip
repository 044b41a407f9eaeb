// extern "C" boundary of the basa library: host-side validation, workspace carving and
// the order in which the stage kernels are enqueued.  Nothing here allocates device
// memory or synchronises.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <mutex>
#include <vector>
#include "common.hpp"

namespace basa {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

basa_status hip_fail(hipError_t e, const char* what) {
  set_error("%s: %s", what, hipGetErrorString(e));
  return BASA_ERR_HIP;
}

// ---- profiling records -------------------------------------------------------------
namespace {
struct ProfRec { int id; hipEvent_t start, stop; };
std::mutex g_prof_mu;
bool g_prof_on = false;
thread_local bool t_prof_off = false;      // set around calls that must not create events
std::vector<ProfRec> g_prof_recs;
const char* const kKernelNames[K_COUNT] = {
    "norm_tile_sort_kernel", "merge_pass_kernel", "block_stats_kernel",
    "block_scores_kernel", "row_select_kernel", "gather_kernels", "attn_mfma_kernel",
    "attn_simple_kernel", "block_mass_kernel", "diagnostic_small_kernels", "scores_select_kernel"};
}  // namespace

ProfScope::ProfScope(int id, hipStream_t st) : slot_(-1), st_(st) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  if (!g_prof_on || t_prof_off) return;
  ProfRec r;
  r.id = id;
  if (hipEventCreate(&r.start) != hipSuccess) return;
  if (hipEventCreate(&r.stop) != hipSuccess) { (void)hipEventDestroy(r.start); return; }
  (void)hipEventRecord(r.start, st);
  g_prof_recs.push_back(r);
  slot_ = (int)g_prof_recs.size() - 1;
}

ProfScope::~ProfScope() {
  if (slot_ < 0) return;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  if (slot_ < (int)g_prof_recs.size()) (void)hipEventRecord(g_prof_recs[slot_].stop, st_);
}

namespace {

int kappa_of(int n_k, double s) {
  if (!(s >= 0.0 && s < 1.0) || n_k < 1) return -1;
  const int dropped = (int)std::floor(s * (double)n_k + 1e-9);
  const int k = n_k - dropped;
  return k < 1 ? 1 : k;
}

basa_status check_tensor(const basa_tensor* t, const char* name) {
  if (!t) { set_error("%s: null tensor descriptor", name); return BASA_ERR_INVALID_ARG; }
  if (!t->ptr) { set_error("%s: null data pointer", name); return BASA_ERR_INVALID_ARG; }
  if (t->dtype != BASA_F32 && t->dtype != BASA_BF16) {
    set_error("%s: dtype %d is neither f32 nor bf16", name, t->dtype); return BASA_ERR_INVALID_ARG;
  }
  if (t->batch < 1 || t->heads < 1 || t->L < 1) {
    set_error("%s: batch, heads and L must be >= 1 (got %d, %d, %d)", name, t->batch, t->heads, t->L);
    return BASA_ERR_INVALID_ARG;
  }
  if (t->d != 64 && t->d != 128) {
    set_error("%s: head dimension %d not supported (64 or 128)", name, t->d); return BASA_ERR_UNSUPPORTED;
  }
  const int per16 = t->dtype == BASA_BF16 ? 8 : 4;
  if (t->stride_l < t->d || t->stride_l % per16 || t->stride_h % per16 || t->stride_b % per16 ||
      t->stride_h < 0 || t->stride_b < 0) {
    set_error("%s: strides must be non-negative multiples of 16 bytes with stride_l >= d", name);
    return BASA_ERR_INVALID_ARG;
  }
  if (reinterpret_cast<uintptr_t>(t->ptr) % 16) {
    set_error("%s: data pointer must be 16-byte aligned", name); return BASA_ERR_INVALID_ARG;
  }
  if ((int64_t)t->batch * t->heads > 65535) {
    set_error("%s: batch*heads exceeds 65535", name); return BASA_ERR_UNSUPPORTED;
  }
  return BASA_OK;
}

basa_status check_params(const basa_params* p, bool need_sparsity) {
  if (!p) { set_error("null basa_params"); return BASA_ERR_INVALID_ARG; }
  if (p->block != 64 && p->block != 128) {
    set_error("block size %d not supported (64 or 128)", p->block); return BASA_ERR_UNSUPPORTED;
  }
  if (p->sort < BASA_SORT_NONE || p->sort > BASA_SORT_QK) {
    set_error("sort mode %d out of range", p->sort); return BASA_ERR_INVALID_ARG;
  }
  if (p->window < 0 || (p->window % p->block) != 0) {
    set_error("window %d must be 0 or a positive multiple of the block size", p->window);
    return BASA_ERR_INVALID_ARG;
  }
  if (p->n_segments < 0 || p->n_segments > BASA_MAX_SEGMENTS) {
    set_error("n_segments %d outside [0, %d]", p->n_segments, BASA_MAX_SEGMENTS); return BASA_ERR_INVALID_ARG;
  }
  if (p->n_segments > 0) {
    if (!p->segment_starts) { set_error("n_segments > 0 with a null segment_starts"); return BASA_ERR_INVALID_ARG; }
    if (p->window != 0) { set_error("window and segments exclude each other"); return BASA_ERR_INVALID_ARG; }
    if (p->segment_starts[0] != 0) { set_error("segment_starts[0] must be 0"); return BASA_ERR_INVALID_ARG; }
    for (int j = 1; j < p->n_segments; ++j)
      if (p->segment_starts[j] <= p->segment_starts[j - 1]) {
        set_error("segment_starts must ascend strictly (entry %d)", j); return BASA_ERR_INVALID_ARG;
      }
  }
  if (need_sparsity && !(p->sparsity >= 0.0 && p->sparsity < 1.0)) {
    set_error("sparsity %g outside [0, 1)", p->sparsity); return BASA_ERR_INVALID_ARG;
  }
  if (!(p->beta == p->beta) || std::isinf(p->beta)) {
    set_error("beta must be finite"); return BASA_ERR_INVALID_ARG;
  }
  if (need_sparsity && !(p->mass_target >= 0.0 && p->mass_target <= 1.0)) {
    set_error("mass_target %g outside [0, 1]", p->mass_target); return BASA_ERR_INVALID_ARG;
  }
  if (need_sparsity && p->budget_total < 0) {
    set_error("budget_total %d is negative", p->budget_total); return BASA_ERR_INVALID_ARG;
  }
  if (need_sparsity && p->min_keep < 0) {
    set_error("min_keep %d is negative", p->min_keep); return BASA_ERR_INVALID_ARG;
  }
  if (p->causal != 0 && p->causal != 1) { set_error("causal must be 0 or 1"); return BASA_ERR_INVALID_ARG; }
  if (p->select_path < 0 || p->select_path > 2) { set_error("select_path must be 0, 1 or 2"); return BASA_ERR_INVALID_ARG; }
  return BASA_OK;
}

// The segment list of p for a sequence of L tokens, in the form the kernels take.
basa_status seg_list(const basa_params* p, int L, SegList* out) {
  out->n = p->n_segments;
  for (int j = 0; j < p->n_segments; ++j) out->bound[j] = p->segment_starts[j];
  for (int j = p->n_segments; j <= BASA_MAX_SEGMENTS; ++j) out->bound[j] = L;
  if (p->n_segments > 0 && p->segment_starts[p->n_segments - 1] >= L) {
    set_error("last segment start %d is not below L = %d", p->segment_starts[p->n_segments - 1], L);
    return BASA_ERR_INVALID_ARG;
  }
  return BASA_OK;
}

basa_status check_qk(const basa_tensor* q, const basa_tensor* k) {
  basa_status s;
  if ((s = check_tensor(q, "q")) != BASA_OK) return s;
  if ((s = check_tensor(k, "k")) != BASA_OK) return s;
  if (q->dtype != k->dtype || q->d != k->d || q->batch != k->batch) {
    set_error("q and k must agree in dtype, head dimension and batch"); return BASA_ERR_INVALID_ARG;
  }
  if (q->heads % k->heads != 0) {
    set_error("query heads (%d) must be a multiple of kv heads (%d)", q->heads, k->heads);
    return BASA_ERR_INVALID_ARG;
  }
  return BASA_OK;
}

basa_status check_qkv(const basa_tensor* q, const basa_tensor* k, const basa_tensor* v) {
  basa_status s;
  if ((s = check_qk(q, k)) != BASA_OK) return s;
  if ((s = check_tensor(v, "v")) != BASA_OK) return s;
  if (v->dtype != k->dtype || v->d != k->d || v->batch != k->batch || v->heads != k->heads || v->L != k->L) {
    set_error("v must have the shape and dtype of k"); return BASA_ERR_INVALID_ARG;
  }
  return BASA_OK;
}

struct SelectWs {
  size_t sort_off, featq_off, featk_off, scores_off, range_off, total;
};

SelectWs carve_select(const basa_tensor* q, const basa_tensor* k, const basa_params* p) {
  const int BHq = q->batch * q->heads, BHk = k->batch * k->heads;
  const int Nq = ceil_div(q->L, p->block), Nk = ceil_div(k->L, p->block);
  SelectWs w;
  size_t o = 0;
  w.sort_off = o;
  o += sort_workspace_bytes(BHq + BHk, q->L > k->L ? q->L : k->L);   // Q and K may be sorted together
  w.featq_off = o; o += align_up((size_t)BHq * Nq * feat_bytes_per_block(q->d), 256);
  w.featk_off = o; o += align_up((size_t)BHk * Nk * feat_bytes_per_block(k->d), 256);
  w.scores_off = o; o += align_up((size_t)BHq * Nq * Nk * sizeof(float), 256);
  w.range_off = o; o += align_up(((size_t)BHq * Nq + (size_t)BHk * Nk) * sizeof(int32_t), 256);   // causal: block index ranges
  w.total = o;
  return w;
}

bool use_mfma(const basa_tensor* q) { return q->dtype == BASA_BF16; }   // d is 64 or 128 (check_tensor)

basa_status attn_common(const basa_tensor* q, const basa_tensor* k, const basa_tensor* v,
                        const int32_t* row_count, const int32_t* row_cols, int32_t cols_stride,
                        const int32_t* perm_q, const int32_t* perm_k, int B, int variant, int causal, void* out,
                        const int64_t* out_strides, float* lse, void* ws, size_t ws_bytes, void* stream) {
  if (!out) { set_error("null output pointer"); return BASA_ERR_INVALID_ARG; }
  if (reinterpret_cast<uintptr_t>(out) % 16) { set_error("out must be 16-byte aligned"); return BASA_ERR_INVALID_ARG; }
  AttnArgs a;
  a.out_sl = q->d; a.out_sh = (int64_t)q->L * q->d; a.out_sb = (int64_t)q->heads * q->L * q->d;
  if (out_strides) {
    const int64_t per16 = q->dtype == BASA_BF16 ? 8 : 4;
    a.out_sb = out_strides[0]; a.out_sh = out_strides[1]; a.out_sl = out_strides[2];
    if (a.out_sl < q->d || a.out_sl % per16 || a.out_sh % per16 || a.out_sb % per16 || a.out_sh < 0 || a.out_sb < 0) {
      set_error("out_strides must be non-negative multiples of 16 bytes with the token stride >= d");
      return BASA_ERR_INVALID_ARG;
    }
  }
  a.q = view_of(*q); a.k = view_of(*k); a.v = view_of(*v);
  a.row_count = row_count; a.row_cols = row_cols; a.cols_stride = cols_stride;
  a.perm_q = perm_q; a.perm_k = perm_k; a.B = B; a.out = out; a.lse = lse; a.ws = ws; a.ws_bytes = ws_bytes;
  a.variant = variant;
  a.causal = causal; a.causal_off = k->L - q->L;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (use_mfma(q)) {
    const size_t need = attn_mfma_workspace_bytes(q->batch * q->heads, k->batch * k->heads, q->L, k->L, q->d, B);
    if (!ws || ws_bytes < need) {
      set_error("attention workspace too small: need %zu bytes, got %zu", need, ws ? ws_bytes : (size_t)0);
      return BASA_ERR_WORKSPACE;
    }
    if (reinterpret_cast<uintptr_t>(ws) % 256) { set_error("workspace must be 256-byte aligned"); return BASA_ERR_INVALID_ARG; }
    return launch_attn_mfma(a, st);
  }
  return launch_attn_simple(a, st);
}

}  // namespace
}  // namespace basa

using namespace basa;

extern "C" {

int32_t basa_kappa(int32_t n_k, double sparsity) { return kappa_of(n_k, sparsity); }

size_t basa_sort_workspace_size(const basa_tensor* x, const basa_params* p) {
  if (check_tensor(x, "x") != BASA_OK || check_params(p, false) != BASA_OK) return 0;
  return sort_workspace_bytes(x->batch * x->heads, x->L);
}

size_t basa_select_workspace_size(const basa_tensor* q, const basa_tensor* k, const basa_params* p) {
  if (check_qk(q, k) != BASA_OK || check_params(p, true) != BASA_OK) return 0;
  return carve_select(q, k, p).total;
}

size_t basa_attn_workspace_size(const basa_tensor* q, const basa_tensor* k, const basa_params* p) {
  if (check_qk(q, k) != BASA_OK || check_params(p, false) != BASA_OK) return 0;
  if (!use_mfma(q)) return 256;   // the fp32 path needs none; keep the size non-zero for callers
  return attn_mfma_workspace_bytes(q->batch * q->heads, k->batch * k->heads, q->L, k->L, q->d, p->block);
}

basa_status basa_norm_sort(const basa_tensor* x, const basa_params* p, int32_t* perm, float* keys_out,
                           void* ws, size_t ws_bytes, void* stream) {
  basa_status s;
  if ((s = check_tensor(x, "x")) != BASA_OK) return s;
  if ((s = check_params(p, false)) != BASA_OK) return s;
  if (!perm) { set_error("null perm output"); return BASA_ERR_INVALID_ARG; }
  const size_t need = sort_workspace_bytes(x->batch * x->heads, x->L);
  if (!ws || ws_bytes < need) {
    set_error("sort workspace too small: need %zu bytes, got %zu", need, ws ? ws_bytes : (size_t)0);
    return BASA_ERR_WORKSPACE;
  }
  if (reinterpret_cast<uintptr_t>(ws) % 256) { set_error("workspace must be 256-byte aligned"); return BASA_ERR_INVALID_ARG; }
  SegList segs;
  if ((s = seg_list(p, x->L, &segs)) != BASA_OK) return s;
  if (x->L > kMaxSortLen) { set_error("sequences beyond %d tokens not supported", kMaxSortLen); return BASA_ERR_UNSUPPORTED; }
  return launch_norm_sort(view_of(*x), p->window, segs, perm, keys_out, ws, reinterpret_cast<hipStream_t>(stream));
}

basa_status basa_downsample(const basa_tensor* x, const int32_t* perm, const basa_params* p, float* mean,
                            float* var, void* x_sorted, void* stream) {
  basa_status s;
  if ((s = check_tensor(x, "x")) != BASA_OK) return s;
  if ((s = check_params(p, false)) != BASA_OK) return s;
  if (!mean) { set_error("null mean output"); return BASA_ERR_INVALID_ARG; }
  if (x_sorted && reinterpret_cast<uintptr_t>(x_sorted) % 16) {
    set_error("x_sorted must be 16-byte aligned"); return BASA_ERR_INVALID_ARG;
  }
  if (x_sorted && x_sorted == x->ptr) { set_error("x_sorted must not alias x"); return BASA_ERR_INVALID_ARG; }
  return launch_block_stats(view_of(*x), perm, p->block, mean, var, nullptr, 0, 0.f, x_sorted,
                            reinterpret_cast<hipStream_t>(stream));
}

basa_status basa_select(const basa_tensor* q, const basa_tensor* k, const basa_params* p,
                        uint32_t* mask_bits, int32_t* row_count, int32_t* row_cols, int32_t* perm_q,
                        int32_t* perm_k, float* row_mass, float* scores, void* ws, size_t ws_bytes,
                        void* stream) {
  basa_status s;
  if ((s = check_qk(q, k)) != BASA_OK) return s;
  if ((s = check_params(p, true)) != BASA_OK) return s;
  if (!row_count || !row_cols || !perm_q || !perm_k) {
    set_error("row_count, row_cols, perm_q and perm_k outputs are required"); return BASA_ERR_INVALID_ARG;
  }
  const SelectWs w = carve_select(q, k, p);
  if (!ws || ws_bytes < w.total) {
    set_error("select workspace too small: need %zu bytes, got %zu", w.total, ws ? ws_bytes : (size_t)0);
    return BASA_ERR_WORKSPACE;
  }
  if (reinterpret_cast<uintptr_t>(ws) % 256) { set_error("workspace must be 256-byte aligned"); return BASA_ERR_INVALID_ARG; }
  const int B = p->block;
  const int BHq = q->batch * q->heads, BHk = k->batch * k->heads;
  const int Nq = ceil_div(q->L, B), Nk = ceil_div(k->L, B);
  if (Nk > 4096) { set_error("more than 4096 key blocks per row (%d) not supported", Nk); return BASA_ERR_UNSUPPORTED; }
  if (q->L > kMaxSortLen) { set_error("sequences beyond %d tokens not supported", kMaxSortLen); return BASA_ERR_UNSUPPORTED; }
  const int kappa = kappa_of(Nk, p->sparsity);
  SegList segs;
  if (p->n_segments > 0 && q->L != k->L) {
    set_error("a segment-aware sort needs L_q == L_k (%d, %d)", q->L, k->L); return BASA_ERR_INVALID_ARG;
  }
  if ((s = seg_list(p, q->L, &segs)) != BASA_OK) return s;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  char* base = reinterpret_cast<char*>(ws);
  void* sort_ws = base + w.sort_off;
  void* featq = base + w.featq_off;
  void* featk = base + w.featk_off;
  float* sc = scores ? scores : reinterpret_cast<float*>(base + w.scores_off);
  const TensorView qv = view_of(*q), kv = view_of(*k);

  const bool sort_q = p->sort == BASA_SORT_Q || p->sort == BASA_SORT_QK;
  const bool sort_k = p->sort == BASA_SORT_K || p->sort == BASA_SORT_QK;
  const bool same_len = q->L == k->L;       // then Q and K share every launch
  if (sort_q && sort_k && same_len) {
    s = launch_norm_sort2(qv, kv, p->window, segs, perm_q, perm_k, sort_ws, st);
    if (s != BASA_OK) return s;
  } else {
    if (sort_q) s = launch_norm_sort(qv, p->window, segs, perm_q, nullptr, sort_ws, st);
    else s = launch_iota_perm(perm_q, BHq, q->L, st);
    if (s != BASA_OK) return s;
    if (sort_k) s = launch_norm_sort(kv, p->window, segs, perm_k, nullptr, sort_ws, st);
    else s = launch_iota_perm(perm_k, BHk, k->L, st);
    if (s != BASA_OK) return s;
  }
  const int32_t* pq = sort_q ? perm_q : nullptr;
  const int32_t* pk = sort_k ? perm_k : nullptr;
  if (same_len) {
    if ((s = launch_select_features(qv, pq, featq, kv, pk, featk, B, p->beta, st)) != BASA_OK) return s;
  } else {
    if ((s = launch_block_stats(qv, pq, B, nullptr, nullptr, featq, 1, p->beta, nullptr, st)) != BASA_OK) return s;
    if ((s = launch_block_stats(kv, pk, B, nullptr, nullptr, featk, 0, p->beta, nullptr, st)) != BASA_OK) return s;
  }
  const int kdim = (p->beta == 0.f) ? q->d : 3 * q->d;
  // fixed count per row, nobody asks for the map, no second pass over it: the map stays on chip
  const bool fusable = !scores && !p->causal && p->mass_target == 0.0 && p->budget_total == 0 &&
                       scores_select_supported(Nk, kdim, 3 * q->d);
  if (p->select_path == 2 && !fusable) {
    set_error("select_path = 2 needs a fixed count per row, no scores output, no causal mask, no total budget "
              "and at most 1024 key blocks per row");
    return BASA_ERR_UNSUPPORTED;
  }
  // (the two-kernel path below is the faster one on this part, 0.21 against 0.30 ms at 128K, so the
  //  library's own choice, select_path = 0, is that one)
  if (fusable && p->select_path == 2)
    return launch_scores_select(featq, featk, BHq, q->heads / k->heads, Nq, Nk, kdim, 3 * q->d, kappa, mask_bits,
                                row_count, row_cols, row_mass, st);
  if ((s = launch_block_scores(featq, featk, sc, BHq, q->heads / k->heads, Nq, Nk, kdim, 3 * q->d, st)) != BASA_OK) return s;
  LiveBlocks live{nullptr, nullptr, Nq, q->heads / k->heads, k->L - q->L};
  if (p->causal) {
    int32_t* q_max = reinterpret_cast<int32_t*>(base + w.range_off);
    int32_t* k_min = q_max + (size_t)BHq * Nq;
    if ((s = launch_block_index_range(perm_q, BHq, q->L, B, 1, q_max, st)) != BASA_OK) return s;
    if ((s = launch_block_index_range(perm_k, BHk, k->L, B, 0, k_min, st)) != BASA_OK) return s;
    live.q_max = q_max; live.k_min = k_min;
  }
  if ((s = launch_row_select(sc, BHq * Nq, Nk, kappa, (float)p->mass_target, p->min_keep, nullptr, live, mask_bits,
                             row_count, row_cols, row_mass, st)) != BASA_OK) return s;
  if (p->budget_total > 0) {
    // the sort buffers are free by now: the trimmed per-row counts live there
    int32_t* keep = reinterpret_cast<int32_t*>(sort_ws);
    const int floor_keep = p->mass_target > 0.0 ? p->min_keep : 1;
    if ((s = launch_budget_cap(row_count, BHq, Nq, kappa, floor_keep, p->budget_total, keep, st)) != BASA_OK) return s;
    s = launch_row_select(sc, BHq * Nq, Nk, kappa, 0.f, 0, keep, live, mask_bits, row_count, row_cols, row_mass, st);
  }
  return s;
}

basa_status basa_sparse_attn(const basa_tensor* q, const basa_tensor* k, const basa_tensor* v,
                             const int32_t* row_count, const int32_t* row_cols, int32_t cols_stride,
                             const int32_t* perm_q, const int32_t* perm_k, const basa_params* p, void* out,
                             const int64_t* out_strides, float* lse, void* ws, size_t ws_bytes, void* stream) {
  basa_status s;
  if ((s = check_qkv(q, k, v)) != BASA_OK) return s;
  if ((s = check_params(p, false)) != BASA_OK) return s;
  if (row_cols && !row_count) { set_error("row_cols given without row_count"); return BASA_ERR_INVALID_ARG; }
  if (row_cols && cols_stride < 1) { set_error("cols_stride must be >= 1"); return BASA_ERR_INVALID_ARG; }
  if (p->attn_shape < 0 || p->attn_shape > 4) { set_error("attn_shape must be 0, 1, 2, 3 or 4"); return BASA_ERR_INVALID_ARG; }
  return attn_common(q, k, v, row_count, row_cols, cols_stride, perm_q, perm_k, p->block, p->attn_shape, p->causal, out,
                     out_strides, lse, ws, ws_bytes, stream);
}

basa_status basa_dense_attn(const basa_tensor* q, const basa_tensor* k, const basa_tensor* v,
                            const basa_params* p, void* out, const int64_t* out_strides, float* lse, void* ws,
                            size_t ws_bytes, void* stream) {
  basa_status s;
  if ((s = check_qkv(q, k, v)) != BASA_OK) return s;
  if ((s = check_params(p, false)) != BASA_OK) return s;
  return attn_common(q, k, v, nullptr, nullptr, 0, nullptr, nullptr, p->block, 3, p->causal, out, out_strides, lse, ws,
                     ws_bytes, stream);
}


}  // extern "C"

// ---- the entry point that allocates nothing ------------------------------------------------
// Scratch of the norm ranking (the two buffers of packed sort words) as a device array owned by
// the library image: every GPU the library runs on holds its own copy, at its own address, until
// the process ends.  `scratch` is a host-side stand-in for that array, never a device address:
// host code uses the pointer that hipGetSymbolAddress returned for the current device.
namespace basa {
namespace {
constexpr size_t kStaticScratchBytes = (size_t)BASA_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};      // per device, resolved at the first use on that device

basa_status static_scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) { set_error("device ordinal %d outside [0, %d)", dev, kMaxDevices); return BASA_ERR_UNSUPPORTED; }
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(static scratch)");
    if (!ptr || reinterpret_cast<uintptr_t>(ptr) % 256) { set_error("static scratch resolved to a misaligned address"); return BASA_ERR_HIP; }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return BASA_OK;
}
}  // namespace
}  // namespace basa

extern "C" {

size_t basa_static_scratch_size(void) { return kStaticScratchBytes; }

basa_status basa_static_init(void) {
  void* ptr = nullptr;
  return static_scratch_of_current_device(&ptr);
}

basa_status basa_norm_sort_static(const basa_tensor* x, const basa_params* p, int32_t* perm, float* keys_out,
                                  void* stream) {
  basa_status s;
  if ((s = check_tensor(x, "x")) != BASA_OK) return s;
  if ((s = check_params(p, false)) != BASA_OK) return s;
  if (!perm) { set_error("null perm output"); return BASA_ERR_INVALID_ARG; }
  SegList segs;
  if ((s = seg_list(p, x->L, &segs)) != BASA_OK) return s;
  if (x->L > kMaxSortLen) { set_error("sequences beyond %d tokens not supported", kMaxSortLen); return BASA_ERR_UNSUPPORTED; }
  const size_t need = sort_workspace_bytes(x->batch * x->heads, x->L);
  if (need > kStaticScratchBytes) {
    set_error("basa_norm_sort_static: batch*heads*L = %lld tokens need %zu bytes of scratch, the static array holds %zu "
              "(at most %zu tokens); use basa_norm_sort with a caller workspace",
              (long long)x->batch * x->heads * x->L, need, kStaticScratchBytes, kStaticScratchBytes / 16);
    return BASA_ERR_WORKSPACE;
  }
  void* ptr = nullptr;
  if ((s = static_scratch_of_current_device(&ptr)) != BASA_OK) return s;
  // nothing in the scratch has to start at zero: the tile pass writes every word the merges read
  t_prof_off = true;                       // the timing aid creates events; this call creates nothing
  s = launch_norm_sort(view_of(*x), p->window, segs, perm, keys_out, ptr, reinterpret_cast<hipStream_t>(stream));
  t_prof_off = false;
  return s;
}

}  // extern "C"

extern "C" {

const char* basa_status_string(basa_status s) {
  switch (s) {
    case BASA_OK: return "BASA_OK";
    case BASA_ERR_INVALID_ARG: return "BASA_ERR_INVALID_ARG";
    case BASA_ERR_UNSUPPORTED: return "BASA_ERR_UNSUPPORTED";
    case BASA_ERR_WORKSPACE: return "BASA_ERR_WORKSPACE";
    case BASA_ERR_HIP: return "BASA_ERR_HIP";
  }
  return "BASA_ERR_UNKNOWN";
}

const char* basa_last_error(void) { return g_err; }

basa_status basa_profile_enable(int on) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  g_prof_on = on != 0;
  return BASA_OK;
}

int32_t basa_profile_kernel_count(void) { return K_COUNT; }

const char* basa_profile_kernel_name(int32_t id) {
  return (id >= 0 && id < K_COUNT) ? kKernelNames[id] : "";
}

basa_status basa_profile_read(double* total_ms, int32_t* launches, int32_t n) {
  if (!total_ms || !launches || n < K_COUNT) {
    set_error("basa_profile_read needs arrays of at least %d entries", (int)K_COUNT);
    return BASA_ERR_INVALID_ARG;
  }
  std::lock_guard<std::mutex> lk(g_prof_mu);
  for (int i = 0; i < n; ++i) { total_ms[i] = 0.0; launches[i] = 0; }
  basa_status rc = BASA_OK;
  for (ProfRec& r : g_prof_recs) {
    float ms = 0.f;
    hipError_t e = hipEventSynchronize(r.stop);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.start, r.stop);
    if (e == hipSuccess) { total_ms[r.id] += ms; launches[r.id] += 1; }
    else rc = hip_fail(e, "basa_profile_read");
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  g_prof_recs.clear();
  return rc;
}
const char* basa_version(void) { return "basa 0.1 gfx950"; }

size_t basa_block_mass_workspace_size(const basa_tensor* q, const basa_tensor* k) {
  if (check_qk(q, k) != BASA_OK) return 0;
  if (q->dtype != BASA_BF16) return 256;      // the f32 kernel needs none; non-zero for callers
  return block_mass_workspace_bytes(q->batch * q->heads, k->batch * k->heads, q->L, k->L, q->d);
}

basa_status basa_block_mass(const basa_tensor* q, const basa_tensor* k, const int32_t* perm_q,
                            const int32_t* perm_k, const basa_params* p, const float* base_logits,
                            float* m_hat, float* max_dev, float* lse, void* ws, size_t ws_bytes,
                            void* stream) {
  basa_status s;
  if ((s = check_qk(q, k)) != BASA_OK) return s;
  if ((s = check_params(p, false)) != BASA_OK) return s;
  if (!m_hat) { set_error("basa_block_mass: m_hat output is required"); return BASA_ERR_INVALID_ARG; }
  if (max_dev && !base_logits) {
    set_error("basa_block_mass: max_dev needs base_logits"); return BASA_ERR_INVALID_ARG;
  }
  const size_t need = basa_block_mass_workspace_size(q, k);
  if (!ws || ws_bytes < need) {
    set_error("block mass workspace too small: need %zu bytes, got %zu", need, ws ? ws_bytes : (size_t)0);
    return BASA_ERR_WORKSPACE;
  }
  if (reinterpret_cast<uintptr_t>(ws) % 256) { set_error("workspace must be 256-byte aligned"); return BASA_ERR_INVALID_ARG; }
  return launch_block_mass(view_of(*q), view_of(*k), perm_q, perm_k, p->block, base_logits, m_hat, max_dev, lse,
                           ws, reinterpret_cast<hipStream_t>(stream));
}

basa_status basa_block_radius(const basa_tensor* x, const int32_t* perm, const basa_params* p, float* radius,
                              float* max_norm, void* stream) {
  basa_status s;
  if ((s = check_tensor(x, "x")) != BASA_OK) return s;
  if ((s = check_params(p, false)) != BASA_OK) return s;
  if (!radius || !max_norm) { set_error("basa_block_radius: both outputs are required"); return BASA_ERR_INVALID_ARG; }
  return launch_block_radius(view_of(*x), perm, p->block, radius, max_norm, reinterpret_cast<hipStream_t>(stream));
}

basa_status basa_deviation_bound(const float* radius_q, const float* max_norm_q, const float* radius_k,
                                 const float* max_norm_k, int32_t bh_q, int32_t bh_kv, int32_t n_q, int32_t n_k,
                                 int32_t d, float* bound, void* stream) {
  if (!radius_q || !max_norm_q || !radius_k || !max_norm_k || !bound) {
    set_error("basa_deviation_bound: null argument"); return BASA_ERR_INVALID_ARG;
  }
  if (bh_q < 0 || bh_kv < 1 || bh_q % bh_kv != 0 || n_q < 0 || n_k < 0 || d < 1 || bh_q > 65535 || n_q > 65535) {
    set_error("basa_deviation_bound: bad sizes"); return BASA_ERR_INVALID_ARG;
  }
  return launch_deviation_bound(radius_q, max_norm_q, radius_k, max_norm_k, bh_q, bh_q / bh_kv, n_q, n_k, d, bound,
                                reinterpret_cast<hipStream_t>(stream));
}

basa_status basa_selection_fidelity(const float* scores, const uint32_t* mask_bits, const float* m_hat,
                                    int64_t rows, int32_t n_k, float* recall, float* l1, void* stream) {
  if (!scores || !mask_bits || !m_hat || (!recall && !l1)) {
    set_error("basa_selection_fidelity: null argument"); return BASA_ERR_INVALID_ARG;
  }
  if (rows < 0 || rows > (int64_t)1 << 30 || n_k < 1) {
    set_error("basa_selection_fidelity: bad sizes"); return BASA_ERR_INVALID_ARG;
  }
  return launch_fidelity_rows(scores, mask_bits, m_hat, (int)rows, n_k, recall, l1, reinterpret_cast<hipStream_t>(stream));
}

basa_status basa_pearson_sums(const float* x, const float* y, int64_t n, double* sums, void* stream) {
  if (!x || !y || !sums || n < 0) { set_error("basa_pearson_sums: null argument or negative n"); return BASA_ERR_INVALID_ARG; }
  return launch_pearson_sums(x, y, n, sums, reinterpret_cast<hipStream_t>(stream));
}

basa_status basa_calibrate_read(const void* buf, size_t bytes, uint32_t* out, void* stream) {
  if (!buf || !out || bytes < (1u << 20) || (reinterpret_cast<uintptr_t>(buf) & 15)) {
    set_error("basa_calibrate_read: needs a 16-byte aligned device buffer of at least 1 MiB and an output word");
    return BASA_ERR_INVALID_ARG;
  }
  const hipError_t e = launch_calib_read(buf, bytes, out, (hipStream_t)stream);
  return e == hipSuccess ? BASA_OK : hip_fail(e, "basa_calibrate_read");
}

basa_status basa_calibrate_mfma(int32_t random_operands, int32_t iters, float* out, size_t out_elems,
                                double* flops, void* stream) {
  if (!out || iters < 1 || iters > (1 << 24)) {
    set_error("basa_calibrate_mfma: out must be a device buffer and 1 <= iters <= 2^24");
    return BASA_ERR_INVALID_ARG;
  }
  if (out_elems < calib_mfma_out_elems()) {
    set_error("basa_calibrate_mfma: out holds %zu floats, needs %zu", out_elems, calib_mfma_out_elems());
    return BASA_ERR_WORKSPACE;
  }
  if (flops) *flops = calib_mfma_flops(iters);
  const hipError_t e = launch_calib_mfma(random_operands != 0, iters, out, (hipStream_t)stream);
  return e == hipSuccess ? BASA_OK : hip_fail(e, "basa_calibrate_mfma");
}

}  // extern "C"
