// Block pooling (Sec. 3.1 mean pooling; Sec. 3.4 per-dimension variances; Alg. 1
// steps 3-4).  One workgroup gathers the B rows of one block of the ordered sequence
// x[perm], keeps them in registers, and reduces twice: sum -> mean, then centred
// squares -> population variance (two-pass, so no cancellation).
//
// Besides mean/var it can emit the block's selection features, with which the
// compensated logit of Eq. 2 + Eq. 14 is ONE dot product of length 3d:
//   l' = [Qbar/sqrt(d), beta*VarQ/d, beta*Qbar^2/d] . [Kbar, Kbar^2 + VarK, VarK]
#include "common.hpp"

namespace basa {
namespace {

// One tensor's share of a launch.  Up to two tensors of identical L, d and dtype go through the
// same launch: rows blockIdx.y < BH0 belong to job 0, the rest to job 1.
struct StatsJob {
  TensorView x;
  const int32_t* perm;
  float* mean_out;
  float* var_out;
  float* feat_out;
  int feat_is_query;
};

template <bool kBf16, int kD, int kB>
__global__ __launch_bounds__(256) void block_stats_kernel(StatsJob j0, StatsJob j1, int BH0, float beta) {
  constexpr int kElem = kBf16 ? 2 : 4;
  constexpr int LPR = kD * kElem / 16;       // lanes per row
  constexpr int RPI = 256 / LPR;             // rows per iteration
  constexpr int ITERS = kB / RPI;
  constexpr int E = Chunk16<kBf16>::kElems;
  static_assert(ITERS >= 1, "block too small for this tiling");
  __shared__ float red[RPI][kD];
  __shared__ float mean_s[kD];

  const bool second = (int)blockIdx.y >= BH0;
  const StatsJob& job = second ? j1 : j0;
  const TensorView& x = job.x;
  const int32_t* perm = job.perm;
  float* mean_out = job.mean_out;
  float* var_out = job.var_out;
  float* feat_out = job.feat_out;
  const int feat_is_query = job.feat_is_query;
  const int bh = second ? blockIdx.y - BH0 : blockIdx.y, g = blockIdx.x;
  const int L = x.L;
  const int N = (L + kB - 1) / kB;
  const int sub = threadIdx.x % LPR, rig = threadIdx.x / LPR;
  const char* base = reinterpret_cast<const char*>(x.ptr) + x.head_offset(bh) * kElem;
  const int32_t* pm = perm ? perm + (int64_t)bh * L : nullptr;
  const int n_valid = min(kB, L - g * kB);

  Chunk16<kBf16> c[ITERS];
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    int pos = g * kB + it * RPI + rig;
    if (pos < L) {
      const int row = perm_at(pm, 0, pos, L);
      c[it].load(base + (int64_t)row * x.stride_l * kElem, sub);
    } else {
      c[it].zero();
    }
  }
  float s[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    float a = 0.f;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) a += c[it].v[e];
    s[e] = a;
  }
#pragma unroll
  for (int e = 0; e < E; ++e) red[rig][sub * E + e] = s[e];
  __syncthreads();
  const float inv_n = 1.0f / (float)n_valid;
  float mean_c = 0.f;
  if (threadIdx.x < kD) {
    float a = 0.f;
#pragma unroll
    for (int r = 0; r < RPI; ++r) a += red[r][threadIdx.x];
    mean_c = a * inv_n;
    mean_s[threadIdx.x] = mean_c;
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const float m = mean_s[sub * E + e];
    float a = 0.f;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      int pos = g * kB + it * RPI + rig;
      float dv = c[it].v[e] - m;
      a += (pos < L) ? dv * dv : 0.f;
    }
    red[rig][sub * E + e] = a;
  }
  __syncthreads();
  if (threadIdx.x < kD) {
    float a = 0.f;
#pragma unroll
    for (int r = 0; r < RPI; ++r) a += red[r][threadIdx.x];
    const float var_c = a * inv_n;
    const int64_t o = ((int64_t)bh * N + g) * kD + threadIdx.x;
    if (mean_out) mean_out[o] = mean_c;
    if (var_out) var_out[o] = var_c;
    if (feat_out) {
      // feature k of block g lives at [k / 4][g][k % 4]: the score kernel reads 16-byte groups of
      // 32 consecutive blocks with one coalesced load
      float* f = feat_out + (int64_t)bh * N * (3 * kD) + (int64_t)g * 4 + (threadIdx.x & 3);
      const int64_t c0 = (int64_t)(threadIdx.x >> 2) * N * 4, third = (int64_t)(kD / 4) * N * 4;
      if (feat_is_query) {
        f[c0] = mean_c * (1.0f / sqrtf((float)kD));
        f[third + c0] = beta * var_c * (1.0f / (float)kD);
        f[2 * third + c0] = beta * (mean_c * mean_c) * (1.0f / (float)kD);
      } else {
        f[c0] = mean_c;
        f[third + c0] = mean_c * mean_c + var_c;
        f[2 * third + c0] = var_c;
      }
    }
  }
}

}  // namespace

static basa_status block_stats_impl(const StatsJob& j0, const StatsJob* j1, int B, float beta, hipStream_t st) {
  const TensorView& x = j0.x;
  const int BH0 = x.batch * x.heads;
  const int BH1 = j1 ? j1->x.batch * j1->x.heads : 0;
  const int N = ceil_div(x.L, B);
  if (BH0 + BH1 == 0 || N == 0) return BASA_OK;
  dim3 grid(N, BH0 + BH1);
  ProfScope prof(K_STATS, st);
  const bool bf = x.dtype == BASA_BF16;
  const StatsJob& jb = j1 ? *j1 : j0;
#define BASA_STATS(BF, D, BB) \
  hipLaunchKernelGGL((block_stats_kernel<BF, D, BB>), grid, dim3(256), 0, st, j0, jb, BH0, beta)
  if (bf && x.d == 128 && B == 128) BASA_STATS(true, 128, 128);
  else if (bf && x.d == 128 && B == 64) BASA_STATS(true, 128, 64);
  else if (bf && x.d == 64 && B == 128) BASA_STATS(true, 64, 128);
  else if (bf && x.d == 64 && B == 64) BASA_STATS(true, 64, 64);
  else if (!bf && x.d == 128 && B == 128) BASA_STATS(false, 128, 128);
  else if (!bf && x.d == 128 && B == 64) BASA_STATS(false, 128, 64);
  else if (!bf && x.d == 64 && B == 128) BASA_STATS(false, 64, 128);
  else BASA_STATS(false, 64, 64);
#undef BASA_STATS
  BASA_HIP_CHECK_LAUNCH("block_stats_kernel");
  return BASA_OK;
}

basa_status launch_block_stats(const TensorView& x, const int32_t* perm, int B, float* mean,
                               float* var, float* feat, int feat_is_query, float beta,
                               hipStream_t st) {
  const StatsJob j{x, perm, mean, var, feat, feat_is_query};
  return block_stats_impl(j, nullptr, B, beta, st);
}

basa_status launch_select_features(const TensorView& q, const int32_t* perm_q, float* feat_q,
                                   const TensorView& k, const int32_t* perm_k, float* feat_k, int B,
                                   float beta, hipStream_t st) {
  const StatsJob jq{q, perm_q, nullptr, nullptr, feat_q, 1};
  const StatsJob jk{k, perm_k, nullptr, nullptr, feat_k, 0};
  return block_stats_impl(jq, &jk, B, beta, st);
}

}  // namespace basa
