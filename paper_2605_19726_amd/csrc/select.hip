// Compensated block-score map and per-row top-kappa selection
// (Eq. 2, Eq. 13-14; Alg. 1 steps 5-11).
//
// Scores: with the per-block features written by the pooling kernel the logit l' of a
// block pair is a dot product, so the N_q x N_k map of a head is a small fp32 GEMM.
// It runs on the fp32 matrix cores (v_mfma_f32_32x32x2_f32), the features staged through
// LDS (they are stored four to a group, groups of consecutive blocks adjacent, so that every
// load of a wave is one contiguous run).
//
// Selection: one wave per row of the map.  The kappa-th largest logit is found by a
// 32-step bisection on an order-preserving integer image of the floats (ballot +
// popcount per step), then the kept columns are compacted in ascending order; among
// logits equal to the threshold the lower block indices win.  Softmax is monotone, so
// ranking by l' is ranking by m'; the softmax is evaluated only for the kept mass.
#include "common.hpp"

namespace basa {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* gbl_ptr_t;

// ---------------------------------------------------------------------------------
// scores[bhq][gq][gk] = sum_k featQ[bhq][gq][k] * featK[bhq/group][gk][k], k < K
// MFMA 32x32x2 operand roles: A[i][kk] lives in lane (i, kk), kk = lane/32; the k range
// is split in halves, lanes 0-31 walk k in [0, K/2), lanes 32-63 walk [K/2, K).
//
// A workgroup of four waves owns a 128 x 256 tile of the map, a wave 64 x 128 of it (eight 32x32
// accumulators).  The features of the tile's 128 + 256 blocks travel through LDS in stages of 16
// k per half (48 KB, double buffered, filled with direct-to-LDS loads one stage ahead), so that
// every feature is fetched once per workgroup: with each wave streaming its own operands from L2
// the kernel was bound by L2 bandwidth (16 bytes per CU cycle), not by the matrix cores.
// ---------------------------------------------------------------------------------
constexpr int kTQ = 128, kTK = 256;       // tile of the map per workgroup
constexpr int kKS = 2;                    // feature groups (of 4) per half of the k range per stage
constexpr int kQStage = 2 * kKS * kTQ;    // float4 per stage: [half][group][block]
constexpr int kKStage = 2 * kKS * kTK;
constexpr int kStage = kQStage + kKStage;
constexpr int kScoresLdsBytes = 2 * kStage * 16;
constexpr int kChunks = kStage / 64;      // direct-to-LDS loads of one wave-width (64 x 16 B) per stage

__global__ __launch_bounds__(256, 2) void block_scores_kernel(const float* __restrict__ featQ,
                                                              const float* __restrict__ featK,
                                                              float* __restrict__ scores, int group,
                                                              int Nq, int Nk, int K, int S) {
  extern __shared__ __attribute__((aligned(16))) float4 stage_buf[];
  // consecutive workgroup ids go round-robin over the 8 XCDs: hand each XCD a contiguous range
  // of (head, tile) so that a head's features are pulled into one L2 only
  const int total = gridDim.x, tiles_x = (Nk + kTK - 1) / kTK, tiles_y = (Nq + kTQ - 1) / kTQ;
  int logical = blockIdx.x;
  if ((total & 7) == 0) logical = (blockIdx.x & 7) * (total >> 3) + (blockIdx.x >> 3);
  const int bhq = logical / (tiles_x * tiles_y);
  const int rem = logical - bhq * (tiles_x * tiles_y);
  const int ty = rem / tiles_x, tx = rem - ty * tiles_x;
  const int bhk = bhq / group;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int li = lane & 31, h = lane >> 5;
  const int row_base = ty * kTQ, col_base = tx * kTK;
  const int wq = wave >> 1, wk = wave & 1;       // this wave: rows wq*64.., columns wk*128..

  // features are stored [K/4][N][4] floats: one 16-byte group per block, blocks adjacent
  const int half = K >> 1;
  const int n_stages = half / (4 * kKS);
  const int64_t gq = (int64_t)Nq * 4, gk = (int64_t)Nk * 4;      // floats per group of 4 features
  const float* fq = featQ + (int64_t)bhq * Nq * S;
  const float* fk = featK + (int64_t)bhk * Nk * S;

  // stage s into buffer buf: chunk c = 64 consecutive blocks of one feature group; blocks past
  // the end of the map read the last block (their outputs are never stored)
  auto issue_stage = [&](int s, int buf) {
    float4* dst = stage_buf + buf * kStage;
#pragma unroll
    for (int i = 0; i < kChunks / 4; ++i) {
      const int c = i * 4 + wave;                 // wave-uniform
      const float* src;
      int off;
      if (c < kQStage / 64) {
        const int hh = c / (kKS * 2), j = (c >> 1) % kKS, part = c & 1;
        const int grp = ((hh * half) >> 2) + s * kKS + j;
        src = fq + grp * gq + (int64_t)min(row_base + part * 64 + lane, Nq - 1) * 4;
        off = (hh * kKS + j) * kTQ + part * 64;
      } else {
        const int cc = c - kQStage / 64;
        const int hh = cc / (kKS * 4), j = (cc >> 2) % kKS, part = cc & 3;
        const int grp = ((hh * half) >> 2) + s * kKS + j;
        src = fk + grp * gk + (int64_t)min(col_base + part * 64 + lane, Nk - 1) * 4;
        off = kQStage + (hh * kKS + j) * kTK + part * 64;
      }
      __builtin_amdgcn_global_load_lds((gbl_ptr_t)src, (lds_ptr_t)(dst + off), 16, 0, 0);
    }
  };

  floatx16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = floatx16{0};
  issue_stage(0, 0);
  for (int s = 0; s < n_stages; ++s) {
    // my loads of stage s have landed; after the barrier everyone's have, and everyone is done
    // with the other buffer (stage s-1), which the next loads overwrite
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (s + 1 < n_stages) issue_stage(s + 1, (s + 1) & 1);
    const float4* Qs = stage_buf + (s & 1) * kStage;
    const float4* Ks = Qs + kQStage;
#pragma unroll
    for (int j = 0; j < kKS; ++j) {
      const float4 a0 = Qs[(h * kKS + j) * kTQ + wq * 64 + li];
      const float4 a1 = Qs[(h * kKS + j) * kTQ + wq * 64 + 32 + li];
      float4 b[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) b[t] = Ks[(h * kKS + j) * kTK + wk * 128 + 32 * t + li];
      const float xa0[4] = {a0.x, a0.y, a0.z, a0.w};
      const float xa1[4] = {a1.x, a1.y, a1.z, a1.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const float xb = e == 0 ? b[t].x : e == 1 ? b[t].y : e == 2 ? b[t].z : b[t].w;
          acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa0[e], xb, acc[t], 0, 0, 0);
          acc[4 + t] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa1[e], xb, acc[4 + t], 0, 0, 0);
        }
      }
    }
  }
  // accumulator register r of lane (j, h) holds row 8*(r/4) + 4*h + r%4, column j
  float* out = scores + (int64_t)bhq * Nq * Nk;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int col = col_base + wk * 128 + 32 * t + li;
    if (col >= Nk) continue;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int ri = 8 * (r >> 2) + 4 * h + (r & 3);
      const int rA = row_base + wq * 64 + ri, rB = rA + 32;
      if (rA < Nq) out[(int64_t)rA * Nk + col] = acc[t][r];
      if (rB < Nq) out[(int64_t)rB * Nk + col] = acc[4 + t][r];
    }
  }
}

// ---------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t ordered_bits(float f) {
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// mass_target == 0: every row keeps `kappa` blocks.  mass_target > 0: a row keeps the fewest of
// its largest m' that sum to at least mass_target, at least min_keep and at most kappa; the
// count is found first (a second bisection, on "mass of the logits >= T"), then the same
// top-count machinery runs with the row's own count.
template <int MAXI>
__global__ __launch_bounds__(256) void row_select_kernel(const float* __restrict__ scores,
                                                         int rows_total, int Nk, int kappa,
                                                         float mass_target, int min_keep,
                                                         uint32_t* __restrict__ mask_bits,
                                                         int32_t* __restrict__ row_count,
                                                         int32_t* __restrict__ row_cols,
                                                         float* __restrict__ row_mass) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + wave;
  if (row >= rows_total) return;
  const float* src = scores + (int64_t)row * Nk;
  float e[MAXI];                        // logits first, then exp(l - max)
  uint32_t u[MAXI];
  float mx = -INFINITY;
  // all loads first, unconditional with the index clamped into the row: a load inside a divergent
  // branch is followed by a full wait, which would serialise the MAXI loads of a lane
#pragma unroll
  for (int i = 0; i < MAXI; ++i) e[i] = src[min(i * 64 + lane, Nk - 1)];
#pragma unroll
  for (int i = 0; i < MAXI; ++i) {
    const bool in_row = i * 64 + lane < Nk;
    e[i] = in_row ? e[i] + 0.0f : -INFINITY;        // -0 -> +0 so that equal values have equal images
    u[i] = in_row ? ordered_bits(e[i]) : 0u;        // 0 is below the image of every float
    mx = fmaxf(mx, e[i]);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  float sum_all = 0.f;
#pragma unroll
  for (int i = 0; i < MAXI; ++i) {
    e[i] = (i * 64 + lane < Nk) ? expf(e[i] - mx) : 0.f;
    sum_all += e[i];
  }
  sum_all = wave_sum(sum_all);

  int keep = kappa;
  if (mass_target > 0.f) {
    const float need = mass_target * sum_all;
    // T2 = largest image T such that the logits with image >= T carry at least the target
    uint32_t T2 = 0;
    for (int bit = 31; bit >= 0; --bit) {
      const uint32_t cand = T2 | (1u << bit);
      float sm = 0.f;
#pragma unroll
      for (int i = 0; i < MAXI; ++i) sm += (u[i] >= cand) ? e[i] : 0.f;
      if (wave_sum(sm) >= need) T2 = cand;
    }
    // everything above T2 is needed; of the logits equal to T2, as many as close the gap
    int n_gt = 0, n_eq = 0;
    float m_gt = 0.f, e_eq = 0.f;
#pragma unroll
    for (int i = 0; i < MAXI; ++i) {
      n_gt += __popcll(__ballot(u[i] > T2));
      n_eq += __popcll(__ballot(u[i] == T2));
      m_gt += (u[i] > T2) ? e[i] : 0.f;
      e_eq = fmaxf(e_eq, (u[i] == T2) ? e[i] : 0.f);
    }
    m_gt = wave_sum(m_gt);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) e_eq = fmaxf(e_eq, __shfl_xor(e_eq, off));
    int r = n_eq;
    if (e_eq > 0.f) r = min(n_eq, max(1, (int)ceilf((need - m_gt) / e_eq)));
    keep = min(kappa, max(max(1, min_keep), n_gt + r));
  }

  // T = keep-th largest image
  uint32_t T = 0;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cand = T | (1u << bit);
    int cnt = 0;
#pragma unroll
    for (int i = 0; i < MAXI; ++i) cnt += __popcll(__ballot(u[i] >= cand));
    if (cnt >= keep) T = cand;
  }
  int n_gt = 0;
#pragma unroll
  for (int i = 0; i < MAXI; ++i) n_gt += __popcll(__ballot(u[i] > T));
  const int need_eq = keep - n_gt;       // >= 1 by construction of T

  const uint64_t lt_mask = (1ull << lane) - 1ull;
  const int words = (Nk + 31) >> 5;
  int32_t* cols = row_cols ? row_cols + (int64_t)row * kappa : nullptr;
  uint32_t* mrow = mask_bits ? mask_bits + (int64_t)row * words : nullptr;
  int emitted = 0, eq_seen = 0;
  float sum_sel = 0.f;
#pragma unroll
  for (int i = 0; i < MAXI; ++i) {
    if (i * 64 < Nk) {
      const bool eq = (u[i] == T);
      const uint64_t beq = __ballot(eq);
      const int eq_rank = eq_seen + __popcll(beq & lt_mask);
      const bool sel = (u[i] > T) || (eq && eq_rank < need_eq);
      const uint64_t bsel = __ballot(sel);
      if (sel) {
        sum_sel += e[i];
        if (cols) cols[emitted + __popcll(bsel & lt_mask)] = i * 64 + lane;
      }
      if (mrow && lane < 2 && 2 * i + lane < words)
        mrow[2 * i + lane] = (uint32_t)(bsel >> (32 * lane));
      emitted += __popcll(bsel);
      eq_seen += __popcll(beq);
    }
  }
  sum_sel = wave_sum(sum_sel);
  if (lane == 0) {
    if (row_count) row_count[row] = emitted;
    if (row_mass) row_mass[row] = sum_sel / sum_all;
  }
}

}  // namespace

basa_status launch_block_scores(const float* featQ, const float* featK, float* scores, int BHq,
                                int group, int Nq, int Nk, int kdim_used, int feat_stride,
                                hipStream_t st) {
  if (BHq == 0 || Nq == 0 || Nk == 0) return BASA_OK;
  if (kdim_used % (8 * kKS) != 0) {        // whole stages: 16 k per half
    set_error("score map: contraction length %d is not a multiple of %d", kdim_used, 8 * kKS);
    return BASA_ERR_UNSUPPORTED;
  }
  const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&block_scores_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kScoresLdsBytes);
  if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(dynamic LDS)");
  dim3 grid(ceil_div(Nk, kTK) * ceil_div(Nq, kTQ) * BHq);
  ProfScope prof(K_SCORES, st);
  hipLaunchKernelGGL(block_scores_kernel, grid, dim3(256), kScoresLdsBytes, st, featQ, featK, scores, group, Nq,
                     Nk, kdim_used, feat_stride);
  BASA_HIP_CHECK_LAUNCH("block_scores_kernel");
  return BASA_OK;
}

basa_status launch_row_select(const float* scores, int rows_total, int Nk, int kappa,
                              float mass_target, int min_keep, uint32_t* mask_bits,
                              int32_t* row_count, int32_t* row_cols, float* row_mass,
                              hipStream_t st) {
  if (rows_total == 0) return BASA_OK;
  dim3 grid(ceil_div(rows_total, 4));
  ProfScope prof(K_ROW_SELECT, st);
#define BASA_SEL(M)                                                                            \
  hipLaunchKernelGGL((row_select_kernel<M>), grid, dim3(256), 0, st, scores, rows_total, Nk,   \
                     kappa, mass_target, min_keep, mask_bits, row_count, row_cols, row_mass)
  if (Nk <= 256) BASA_SEL(4);
  else if (Nk <= 1024) BASA_SEL(16);
  else if (Nk <= 2048) BASA_SEL(32);
  else if (Nk <= 4096) BASA_SEL(64);
  else {
    set_error("row selection supports at most 4096 key blocks per row (got %d)", Nk);
    return BASA_ERR_UNSUPPORTED;
  }
#undef BASA_SEL
  BASA_HIP_CHECK_LAUNCH("row_select_kernel");
  return BASA_OK;
}

}  // namespace basa
