// Compensated block-score map and per-row top-kappa selection
// (Eq. 2, Eq. 13-14; Alg. 1 steps 5-11).
//
// Scores: with the per-block features written by the pooling kernel the logit l' of a
// block pair is a dot product, so the N_q x N_k map of a head is a small GEMM of fp32
// accuracy.  It runs on the bf16 matrix cores over three-part splits of the features, which
// are staged through LDS (eight to a group, groups of consecutive blocks adjacent, so that
// every load of a wave is one contiguous run).
//
// Selection: one wave per row of the map.  The kappa-th largest logit is found by a
// 32-step bisection on an order-preserving integer image of the floats (ballot +
// popcount per step), then the kept columns are compacted in ascending order; among
// logits equal to the threshold the lower block indices win.  Softmax is monotone, so
// ranking by l' is ranking by m'; the softmax is evaluated only for the kept mass.
#include <climits>
#include "common.hpp"

namespace basa {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* gbl_ptr_t;

// ---------------------------------------------------------------------------------
// scores[bhq][gq][gk] = sum_k featQ[bhq][gq][k] * featK[bhq/group][gk][k], k < K
//
// Every feature arrives as three bf16 parts q = q0 + q1 + q2 (8 + 8 + 8 mantissa bits; the
// pooling kernel splits them), and the fp32 product q*k is rebuilt from the six part products
// that matter: q0k0 + (q0k1 + q1k0) + (q0k2 + q1k1 + q2k0); the three left out are below 2^-24
// of |q k|, the size of an fp32 rounding.  bf16 products are exact in the fp32 accumulator, so
// the map has fp32 accuracy at six bf16 MFMAs (32 cycles each, 16 k) where the fp32 matrix
// instruction needs eight of 64 cycles: 2.7 times fewer matrix-core cycles.
//
// MFMA 32x32x16 operand roles: lane (i, h) holds A[i][8h .. 8h+7], and B likewise by column.
// A workgroup of four waves owns a 128 x 256 tile of the map, a wave 64 x 128 of it (eight
// 32x32 accumulators).  The parts of the tile's 128 + 256 blocks travel through LDS one k-step
// (16 k: 36 KB) at a time, double buffered and filled with direct-to-LDS loads one step ahead,
// so that every feature is fetched once per workgroup.
// ---------------------------------------------------------------------------------
constexpr int kTQ = 128, kTK = 256;       // tile of the map per workgroup
constexpr int kQStage = 3 * 2 * kTQ;      // 16-byte groups per step: [part][k-half of the step][block]
constexpr int kKStage = 3 * 2 * kTK;
constexpr int kStage = kQStage + kKStage;
constexpr int kScoresLdsBytes = 2 * kStage * 16;
constexpr int kChunks = kStage / 64;      // direct-to-LDS loads of one wave-width (64 x 16 B) per step
static_assert(kChunks % 4 == 0 && (kQStage / 64) % 4 == 0, "chunks are dealt to the four waves in rounds");

__global__ __launch_bounds__(256, 2) void block_scores_kernel(const uint4* __restrict__ featQ,
                                                              const uint4* __restrict__ featK,
                                                              float* __restrict__ scores, int group,
                                                              int Nq, int Nk, int K, int S) {
  extern __shared__ __attribute__((aligned(16))) uint4 stage_buf[];
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

  // features: [part][S/8][N] groups of 8 bf16 (16 bytes); k-step s uses groups 2s and 2s+1
  const int n_steps = K >> 4;
  const int groups = S >> 3;
  const uint4* fq = featQ + (int64_t)bhq * 3 * groups * Nq;
  const uint4* fk = featK + (int64_t)bhk * 3 * groups * Nk;

  // step s into buffer buf: chunk c = 64 consecutive blocks of one group of one part; blocks
  // past the end of the map read the last block (their outputs are never stored)
  auto issue_step = [&](int s, int buf) {
    uint4* dst = stage_buf + buf * kStage;
#pragma unroll
    for (int i = 0; i < kChunks / 4; ++i) {
      const int c = i * 4 + wave;                 // wave-uniform
      const uint4* src;
      int off;
      if (i < kQStage / 256) {                    // c = part*4 + khalf*2 + which 64 of the 128 rows
        const int part = c >> 2, kh = (c >> 1) & 1, sub = c & 1;
        src = fq + ((int64_t)part * groups + 2 * s + kh) * Nq + min(row_base + sub * 64 + lane, Nq - 1);
        off = (part * 2 + kh) * kTQ + sub * 64;
      } else {                                    // cc = part*8 + khalf*4 + which 64 of the 256 columns
        const int cc = c - kQStage / 64;
        const int part = cc >> 3, kh = (cc >> 2) & 1, sub = cc & 3;
        src = fk + ((int64_t)part * groups + 2 * s + kh) * Nk + min(col_base + sub * 64 + lane, Nk - 1);
        off = kQStage + (part * 2 + kh) * kTK + sub * 64;
      }
      __builtin_amdgcn_global_load_lds((gbl_ptr_t)src, (lds_ptr_t)(dst + off), 16, 0, 0);
    }
  };

  floatx16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = floatx16{0};
  issue_step(0, 0);
  for (int s = 0; s < n_steps; ++s) {
    // my loads of step s have landed; after the barrier everyone's have, and everyone is done
    // with the other buffer (step s-1), which the next loads overwrite
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (s + 1 < n_steps) issue_step(s + 1, (s + 1) & 1);
    const uint4* Qs = stage_buf + (s & 1) * kStage;
    const uint4* Ks = Qs + kQStage;
    bf16x8 a[3][2], b[3][4];
#pragma unroll
    for (int part = 0; part < 3; ++part) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const uint4 v = Qs[(part * 2 + h) * kTQ + wq * 64 + 32 * u + li];
        a[part][u] = __builtin_bit_cast(bf16x8, v);
      }
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const uint4 v = Ks[(part * 2 + h) * kTK + wk * 128 + 32 * t + li];
        b[part][t] = __builtin_bit_cast(bf16x8, v);
      }
    }
    // by key part, the smallest first (the order in which the fused kernel below receives them)
    constexpr int PQ[6] = {0, 1, 0, 2, 1, 0};
    constexpr int PK[6] = {2, 1, 1, 0, 0, 0};
#pragma unroll
    for (int pr = 0; pr < 6; ++pr) {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[PQ[pr]][0], b[PK[pr]][t], acc[t], 0, 0, 0);
        acc[4 + t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[PQ[pr]][1], b[PK[pr]][t], acc[4 + t], 0, 0, 0);
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

__device__ __forceinline__ float float_of_ordered(uint32_t u) {
  return __uint_as_float((u & 0x80000000u) ? (u ^ 0x80000000u) : ~u);
}

// mass_target == 0: every row keeps `kappa` blocks.  mass_target > 0: a row keeps the fewest of
// its largest m' that sum to at least mass_target, at least min_keep and at most kappa; the
// count is found first (a second bisection, on "mass of the logits >= T"), then the same
// top-count machinery runs with the row's own count.
template <int MAXI, bool kLive>
__global__ __launch_bounds__(256) void row_select_kernel(const float* __restrict__ scores,
                                                         int rows_total, int Nk, int kappa,
                                                         float mass_target, int min_keep,
                                                         const int32_t* __restrict__ keep_in, LiveBlocks live,
                                                         uint32_t* __restrict__ mask_bits,
                                                         int32_t* __restrict__ row_count,
                                                         int32_t* __restrict__ row_cols,
                                                         float* __restrict__ row_mass) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + wave;
  if (row >= rows_total) return;
  const float* src = scores + (int64_t)row * Nk;
  // causal variant: a key block is live for this row iff its smallest original key index does not
  // exceed the row's largest original query index (+ offset); dead blocks take no part below
  const int32_t* kmin = kLive ? live.k_min + (int64_t)(row / live.Nq / live.group) * Nk : nullptr;
  const int q_lim = kLive ? live.q_max[row] + live.offset : 0;
  float e[MAXI];                        // logits first, then exp(l - max)
  uint32_t u[MAXI];
  float mx = -INFINITY;
  // all loads first, unconditional with the index clamped into the row: a load inside a divergent
  // branch is followed by a full wait, which would serialise the MAXI loads of a lane
#pragma unroll
  for (int i = 0; i < MAXI; ++i) e[i] = src[min(i * 64 + lane, Nk - 1)];
  int n_live = Nk;
  if constexpr (kLive) {
    int km[MAXI];
#pragma unroll
    for (int i = 0; i < MAXI; ++i) km[i] = kmin[min(i * 64 + lane, Nk - 1)];
    n_live = 0;
#pragma unroll
    for (int i = 0; i < MAXI; ++i) {
      const bool alive = i * 64 + lane < Nk && km[i] <= q_lim;
      n_live += __popcll(__ballot(alive));
      if (!alive) e[i] = __uint_as_float(0x7fc00000u);      // marked; replaced below
    }
    if (n_live == 0) {                                      // every key lies after every query of the block
      if (lane == 0) {
        if (row_count) row_count[row] = 0;
        if (row_mass) row_mass[row] = 0.f;
      }
      if (mask_bits)
        for (int w = lane; w < (Nk + 31) >> 5; w += 64) mask_bits[(int64_t)row * ((Nk + 31) >> 5) + w] = 0u;
      return;
    }
  }
#pragma unroll
  for (int i = 0; i < MAXI; ++i) {
    const bool in_row = i * 64 + lane < Nk && !(kLive && e[i] != e[i]);
    e[i] = in_row ? e[i] + 0.0f : -INFINITY;        // -0 -> +0 so that equal values have equal images
    u[i] = in_row ? ordered_bits(e[i]) : 0u;        // 0 is below the image of every float
    mx = fmaxf(mx, e[i]);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  float sum_all = 0.f;
#pragma unroll
  for (int i = 0; i < MAXI; ++i) {
    // (image 0: past the row, or a dead block)
    e[i] = (kLive ? u[i] != 0u : i * 64 + lane < Nk) ? __expf(e[i] - mx) : 0.f;
    sum_all += e[i];
  }
  sum_all = wave_sum(sum_all);

  int keep = keep_in ? max(1, min(keep_in[row], kappa)) : kappa;
  if (kLive) keep = min(keep, n_live);
  if (!keep_in && mass_target > 0.f) {
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
    keep = min(kLive ? min(kappa, n_live) : kappa, max(max(1, min_keep), n_gt + r));
  }

  // T = keep-th largest image
  uint32_t T = 0;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cand = T | (1u << bit);
    int cnt = 0;
#pragma unroll
    for (int i = 0; i < MAXI; ++i) cnt += __popcll(__ballot(u[i] >= cand));
    if (cnt >= keep) T = cand;
    // exactly `keep` images at or above cand: they are the kept set, whatever the lower bits of
    // the keep-th largest are (typically after about 8 + log2 N_k of the 32 steps)
    if (cnt == keep) break;
  }
  int n_gt = 0;
#pragma unroll
  for (int i = 0; i < MAXI; ++i) n_gt += __popcll(__ballot(u[i] > T));
  const int need_eq = keep - n_gt;       // how many of the images equal to T are kept

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

// ---------------------------------------------------------------------------------
// Score map and fixed-count row selection in ONE kernel: the map never leaves the chip
// (Alg. 1 steps 5-11 with the logits kept where they are produced).
//
// A workgroup of eight waves owns 64 rows of a head's map and ALL its columns (at most 128 NT):
// wave (rh, cq) holds rows 32 rh .. +31 against columns 32 NT cq .. +32 NT - 1 as NT transposed
// 32x32 accumulators (A = key features, B = query features), so lane (j, h) owns row j: register r
// of accumulator t is column 32 t + 8 (r / 4) + 4 h + r % 4 of the wave's range, and the lane and
// its partner (h ^ 1) together hold the wave's whole share of that row.  The same six part
// products as block_scores_kernel are accumulated in the same order, so the logits are the same
// bits.  Features stream through a ring of four LDS buffers in units of one k-step of ONE key
// part (all columns, both k-halves) plus the matching query part; a unit is requested three
// units before its use, and the unit of key part kp is multiplied with the query parts 0 .. 2-kp,
// which are in registers by then.
//
// Selection works on the accumulators in place (as order-preserving integer images): the
// bisection of row_select_kernel with per-lane counts, summed over the 8 lanes of a row through
// LDS, one barrier per step.  The kept set goes through per-row bitmaps in LDS (one word per
// accumulator: no atomics), from which one wave per row writes the bitmap, the ascending column
// list and the kept mass.
// ---------------------------------------------------------------------------------
constexpr int kFR = 64;                    // rows of the map per workgroup
template <int NT>
struct FusedGeo {
  static constexpr int kCols = 128 * NT;               // columns covered: 4 column waves x NT blocks of 32
  static constexpr int kUnit = 2 * kCols + 2 * kFR;    // 16-byte groups per unit: K [k-half][column], Q [k-half][row]
  static constexpr int kLoads = 2 * kCols / 64 / 8;    // direct-to-LDS loads of K groups per wave and unit
  static constexpr int kWords = 4 * NT;                // bitmap words per row
  static constexpr int kWStride = kWords + 1;          // padded: the lanes of a wave write one word of 32 rows at once
  static constexpr int kRingBytes = 4 * kUnit * 16;
  // after the map is complete the ring is reused: counters, partial sums, bitmaps, one list per wave
  static constexpr int kPostBytes = (3 * 64 + 4 + 64 * 4 + 2 * 4 * 64 + 2 * 64 * kWStride + 8 * kCols) * 4;
  static_assert(kPostBytes <= kRingBytes, "the selection scratch must fit into the ring");
};

__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int o = __shfl_up(v, off);
    if (lane >= off) v += o;
  }
  return v;
}

template <int NT>
__global__ __launch_bounds__(512, 1) void scores_select_kernel(const uint4* __restrict__ featQ,
                                                               const uint4* __restrict__ featK, int group,
                                                               int Nq, int Nk, int K, int S, int kappa,
                                                               uint32_t* __restrict__ mask_bits,
                                                               int32_t* __restrict__ row_count,
                                                               int32_t* __restrict__ row_cols,
                                                               float* __restrict__ row_mass) {
  using G = FusedGeo<NT>;
  extern __shared__ __attribute__((aligned(16))) uint4 fbuf[];
  const int strips = (Nq + kFR - 1) / kFR, total = gridDim.x;
  int logical = blockIdx.x;
  if ((total & 7) == 0) logical = (blockIdx.x & 7) * (total >> 3) + (blockIdx.x >> 3);   // one XCD, one range of heads
  const int bhq = logical / strips, strip = logical - bhq * strips;
  const int bhk = bhq / group;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 31, h = lane >> 5;
  const int rh = wave >> 2, cq = wave & 3;
  const int row_local = rh * 32 + li;
  const int n_steps = K >> 4, groups = S >> 3, units = 3 * n_steps;
  const uint4* fq = featQ + (int64_t)bhq * 3 * groups * Nq;
  const uint4* fk = featK + (int64_t)bhk * 3 * groups * Nk;

  // unit v = (k-step v / 3, key part 2 - v % 3, query part v % 3) into ring buffer v % 4; rows and
  // columns past the end of the map read the last one (their results are never used).  Every
  // wave issues kLoads + 1 loads per unit (the 2 x 64 query groups are requested by four waves
  // each, same bytes to the same place), so that one wait count fits all.
  auto issue_unit = [&](int v, int buf) {
    const int s = v / 3, j = v - 3 * s, kp = 2 - j;
    uint4* dst = fbuf + buf * G::kUnit;
#pragma unroll
    for (int i = 0; i < G::kLoads; ++i) {
      const int c = i * 8 + wave;                            // wave-uniform chunk of 64 columns
      const int kh = c / (G::kCols / 64), sub = c - kh * (G::kCols / 64);
      const uint4* src = fk + ((int64_t)kp * groups + 2 * s + kh) * Nk + min(sub * 64 + lane, Nk - 1);
      __builtin_amdgcn_global_load_lds((gbl_ptr_t)src, (lds_ptr_t)(dst + kh * G::kCols + sub * 64), 16, 0, 0);
    }
    const int kh = wave & 1;
    const uint4* src = fq + ((int64_t)j * groups + 2 * s + kh) * Nq + min(strip * kFR + lane, Nq - 1);
    __builtin_amdgcn_global_load_lds((gbl_ptr_t)src, (lds_ptr_t)(dst + 2 * G::kCols + kh * kFR), 16, 0, 0);
  };

  floatx16 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) acc[t] = floatx16{0};
  issue_unit(0, 0);
  issue_unit(1, 1);
  issue_unit(2, 2);
#pragma nounroll
  for (int s = 0; s < n_steps; ++s) {
    bf16x8 qreg[3];
#pragma unroll
    for (int j = 0; j < 3; ++j) {
      const int v = 3 * s + j;
      // all but my two youngest batches have landed: unit v is among them.  After the barrier
      // everyone's part of it has, and everyone is done with unit v - 1, whose buffer the next
      // request overwrites (past the last unit: the last one again, into that same dead buffer,
      // so that the count of outstanding loads stays what the wait assumes).
      if (G::kLoads == 1) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
      else if (G::kLoads == 2) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
      else asm volatile("s_waitcnt vmcnt(10)" ::: "memory");
      __syncthreads();
      issue_unit(min(v + 3, units - 1), (v + 3) & 3);
      const uint4* U = fbuf + (v & 3) * G::kUnit;
      qreg[j] = __builtin_bit_cast(bf16x8, U[2 * G::kCols + h * kFR + row_local]);
      bf16x8 a[NT];
#pragma unroll
      for (int t = 0; t < NT; ++t) a[t] = __builtin_bit_cast(bf16x8, U[h * G::kCols + cq * 32 * NT + 32 * t + li]);
      // (query parts outermost: neighbouring matrix instructions are independent; every accumulator
      //  still receives its products in the order stated above)
#pragma unroll
      for (int qp = j; qp >= 0; --qp)
#pragma unroll
        for (int t = 0; t < NT; ++t)
          acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[t], qreg[qp], acc[t], 0, 0, 0);
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // the trailing requests still write into the ring
  __syncthreads();

  // ---------------- selection, on the accumulators in place
  uint32_t* cnt = reinterpret_cast<uint32_t*>(fbuf);            // [3][64] counts of one bisection step
  uint32_t* nd = cnt + 3 * 64;                                  // [3] (+1): "a row is still searching"
  uint32_t* mximg = nd + 4;                                     // [64] image of the row maximum
  uint32_t* cgt = mximg + 64;                                   // [64] entries above the threshold
  int32_t* needeq = reinterpret_cast<int32_t*>(cgt + 64);       // [64] ties to keep
  float* e_thr = reinterpret_cast<float*>(needeq + 64);         // [64] exp(threshold - max)
  float* part = e_thr + 64;                                     // [2][4][64] partial sums per column wave
  uint32_t* gtw = reinterpret_cast<uint32_t*>(part + 2 * 4 * 64);   // [64][kWStride] bits above the threshold
  uint32_t* eqw = gtw + 64 * G::kWStride;                       // [64][kWStride] bits equal to it
  int32_t* stage = reinterpret_cast<int32_t*>(eqw + 64 * G::kWStride);   // [8][kCols] one column list per wave
  if (tid < 3 * 64) cnt[tid] = 0u;
  if (tid < 4) nd[tid] = 0u;
  if (tid < 64) { mximg[tid] = 0u; cgt[tid] = 0u; }

  uint32_t u[NT][16];
  uint32_t mxl = 0u;
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int col = cq * 32 * NT + 32 * t + 8 * (r >> 2) + 4 * h + (r & 3);
      u[t][r] = col < Nk ? ordered_bits(acc[t][r] + 0.0f) : 0u;      // -0 -> +0; 0 is below the image of every float
      mxl = max(mxl, u[t][r]);
    }
  __syncthreads();
  const int keep = kappa;
  float mx = 0.f;
  if (row_mass) {
    mxl = max(mxl, (uint32_t)__shfl_xor((int)mxl, 32));
    if (h == 0) atomicMax(&mximg[row_local], mxl);
    __syncthreads();
    mx = float_of_ordered(mximg[row_local]);
    float sum = 0.f;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) sum += __expf(u[t][r] != 0u ? float_of_ordered(u[t][r]) - mx : -INFINITY);
    sum += __shfl_xor(sum, 32);
    if (h == 0) part[cq * 64 + row_local] = sum;
  }

  // T = keep-th largest image of the row
  uint32_t T = 0u;
  bool done = false;
  for (int k = 0; k < 32; ++k) {
    const int b0 = k % 3;
    const uint32_t cand = T | (0x80000000u >> k);
    int c = 0;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) c += u[t][r] >= cand ? 1 : 0;
    c += __shfl_xor(c, 32);
    if (h == 0 && !done) atomicAdd(&cnt[b0 * 64 + row_local], (uint32_t)c);
    __syncthreads();
    if (k > 0 && nd[(k - 1) % 3] == 0u) break;          // no row was still searching after the step before
    const int tot = (int)cnt[b0 * 64 + row_local];
    if (!done) {
      if (tot >= keep) T = cand;
      // exactly `keep` images at or above cand: they are the kept set, whatever the lower bits are
      if (tot == keep) done = true;
    }
    if (!done) nd[b0] = 1u;
    if (tid < 64) cnt[((k + 2) % 3) * 64 + tid] = 0u;
    if (tid == 0) nd[(k + 1) % 3] = 0u;
  }
  {
    int c = 0;
    float sg = 0.f;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) c += u[t][r] > T ? 1 : 0;
    if (row_mass) {
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) sg += __expf(u[t][r] > T ? float_of_ordered(u[t][r]) - mx : -INFINITY);
    }
    c += __shfl_xor(c, 32);
    sg += __shfl_xor(sg, 32);
    if (h == 0) {
      atomicAdd(&cgt[row_local], (uint32_t)c);
      if (row_mass) part[(4 + cq) * 64 + row_local] = sg;
    }
  }
  // one bitmap word per accumulator: the lane's 16 columns and its partner's interleave in fours
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    uint32_t g = 0u, e = 0u;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const uint32_t bit = 1u << (8 * (r >> 2) + (r & 3));
      g |= u[t][r] > T ? bit : 0u;
      e |= u[t][r] == T ? bit : 0u;
    }
    g <<= 4 * h; e <<= 4 * h;
    g |= (uint32_t)__shfl_xor((int)g, 32);
    e |= (uint32_t)__shfl_xor((int)e, 32);
    if (h == 0) gtw[row_local * G::kWStride + cq * NT + t] = g;
    else eqw[row_local * G::kWStride + cq * NT + t] = e;
  }
  __syncthreads();
  if (cq == 0 && h == 0) {
    needeq[row_local] = keep - (int)cgt[row_local];
    e_thr[row_local] = row_mass ? __expf(float_of_ordered(T) - mx) : 0.f;
  }
  __syncthreads();

  // ---------------- one wave per row: bitmap, ascending column list, count, mass
  const int words = (Nk + 31) >> 5;
  const int wd = lane >> 1, half = lane & 1;
  int32_t* stg = stage + wave * G::kCols;
  for (int i = 0; i < 8; ++i) {
    const int rl = wave * 8 + i;
    const int64_t grow = (int64_t)bhq * Nq + strip * kFR + rl;
    if (strip * kFR + rl >= Nq) break;                  // wave-uniform: the rows of a wave ascend
    const uint32_t g = wd < G::kWords ? gtw[rl * G::kWStride + wd] : 0u;
    const uint32_t e = wd < G::kWords ? eqw[rl * G::kWStride + wd] : 0u;
    const int ne = needeq[rl];
    // of the entries equal to the threshold the lowest columns are kept
    const int pe = __popc(e);
    const int eq_before = wave_incl_scan(half == 0 ? pe : 0, lane) - pe;     // both lanes of a word: words below it
    const int take = min(max(ne - eq_before, 0), pe);
    uint32_t ek = e;
    while (__popc(ek) > take) ek &= ~(0x80000000u >> __clz(ek));
    const uint32_t f = g | ek;
    if (mask_bits && half == 0 && wd < words) mask_bits[grow * words + wd] = f;
    const int pf = __popc(f);
    const int incl = wave_incl_scan(half == 0 ? pf : 0, lane);
    const int n_kept = __builtin_amdgcn_readlane(incl, 63);
    int start = incl - pf + (half ? __popc(f & 0xffffu) : 0);
    uint32_t my = (f >> (16 * half)) & 0xffffu;
    while (my) {
      stg[start++] = wd * 32 + 16 * half + (__ffs(my) - 1);
      my &= my - 1u;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the wave's own LDS writes, before its reads
    if (row_cols)
      for (int k = lane; k < n_kept; k += 64) row_cols[grow * kappa + k] = stg[k];
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // ... and the reads before the next row's writes
    if (lane == 0) {
      if (row_count) row_count[grow] = n_kept;
      if (row_mass) {
        const float sa = (part[0 * 64 + rl] + part[1 * 64 + rl]) + (part[2 * 64 + rl] + part[3 * 64 + rl]);
        const float sg = (part[4 * 64 + rl] + part[5 * 64 + rl]) + (part[6 * 64 + rl] + part[7 * 64 + rl]);
        row_mass[grow] = (sg + (ne > 0 ? (float)ne * e_thr[rl] : 0.f)) / sa;
      }
    }
  }
}

// ---------------------------------------------------------------------------------
// Total budget of kept blocks per (batch, head): one workgroup per head builds the histogram of
// the rows' counts and walks the caps t = lo .. kappa: total(t) = sum_{c <= t} c*hist[c] +
// t * #{rows with c > t} never decreases with t, so the last t that fits is the answer.
// ---------------------------------------------------------------------------------
constexpr int kMaxCount = 4096;
__global__ __launch_bounds__(256) void budget_cap_kernel(const int32_t* __restrict__ row_count, int Nq, int kappa,
                                                         int floor_keep, int budget, int32_t* __restrict__ keep_out) {
  __shared__ int hist[kMaxCount + 1];
  __shared__ int cap_s;
  const int32_t* cnt = row_count + (int64_t)blockIdx.x * Nq;
  for (int i = threadIdx.x; i <= kappa; i += 256) hist[i] = 0;
  __syncthreads();
  for (int r = threadIdx.x; r < Nq; r += 256) atomicAdd(&hist[max(0, min(cnt[r], kappa))], 1);
  __syncthreads();
  if (threadIdx.x == 0) {
    const int lo = max(1, min(floor_keep, kappa));
    int64_t below = 0;           // sum of the counts <= t
    int rows_below = 0;          // rows with count <= t
    for (int c = 0; c < lo; ++c) { below += (int64_t)c * hist[c]; rows_below += hist[c]; }
    int cap = lo;
    for (int t = lo; t <= kappa; ++t) {
      below += (int64_t)t * hist[t];
      rows_below += hist[t];
      if (below + (int64_t)t * (Nq - rows_below) <= (int64_t)budget) cap = t;
    }
    cap_s = cap;
  }
  __syncthreads();
  const int cap = cap_s;
  for (int r = threadIdx.x; r < Nq; r += 256) keep_out[(int64_t)blockIdx.x * Nq + r] = min(cnt[r], cap);
}

}  // namespace

basa_status launch_budget_cap(const int32_t* row_count, int BHq, int Nq, int kappa, int floor_keep,
                              int budget, int32_t* keep_out, hipStream_t st) {
  if (BHq == 0 || Nq == 0) return BASA_OK;
  if (kappa > kMaxCount) {
    set_error("a total budget supports at most %d key blocks per row (got %d)", kMaxCount, kappa);
    return BASA_ERR_UNSUPPORTED;
  }
  ProfScope prof(K_ROW_SELECT, st);
  hipLaunchKernelGGL(budget_cap_kernel, dim3(BHq), dim3(256), 0, st, row_count, Nq, kappa, floor_keep, budget,
                     keep_out);
  BASA_HIP_CHECK_LAUNCH("budget_cap_kernel");
  return BASA_OK;
}

basa_status launch_block_scores(const void* featQ, const void* featK, float* scores, int BHq,
                                int group, int Nq, int Nk, int kdim_used, int feat_stride,
                                hipStream_t st) {
  if (BHq == 0 || Nq == 0 || Nk == 0) return BASA_OK;
  if (kdim_used % 16 != 0 || feat_stride % 8 != 0) {        // whole k-steps of 16
    set_error("score map: contraction length %d is not a multiple of 16", kdim_used);
    return BASA_ERR_UNSUPPORTED;
  }
  const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&block_scores_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kScoresLdsBytes);
  if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(dynamic LDS)");
  dim3 grid(ceil_div(Nk, kTK) * ceil_div(Nq, kTQ) * BHq);
  ProfScope prof(K_SCORES, st);
  hipLaunchKernelGGL(block_scores_kernel, grid, dim3(256), kScoresLdsBytes, st, reinterpret_cast<const uint4*>(featQ),
                     reinterpret_cast<const uint4*>(featK), scores, group, Nq, Nk, kdim_used, feat_stride);
  BASA_HIP_CHECK_LAUNCH("block_scores_kernel");
  return BASA_OK;
}

bool scores_select_supported(int Nk, int kdim_used, int feat_stride) {
  return Nk >= 1 && Nk <= 1024 && kdim_used >= 16 && kdim_used % 16 == 0 && feat_stride % 8 == 0;
}

basa_status launch_scores_select(const void* featQ, const void* featK, int BHq, int group, int Nq, int Nk,
                                 int kdim_used, int feat_stride, int kappa, uint32_t* mask_bits,
                                 int32_t* row_count, int32_t* row_cols, float* row_mass, hipStream_t st) {
  if (BHq == 0 || Nq == 0 || Nk == 0) return BASA_OK;
  if (!scores_select_supported(Nk, kdim_used, feat_stride)) {
    set_error("fused score map and selection: %d key blocks per row (at most 1024), contraction length %d "
              "(a multiple of 16)", Nk, kdim_used);
    return BASA_ERR_UNSUPPORTED;
  }
  dim3 grid(ceil_div(Nq, kFR) * BHq);
  ProfScope prof(K_SCORES_SELECT, st);
#define BASA_FUSED(NT)                                                                                    \
  do {                                                                                                    \
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&scores_select_kernel<NT>),    \
                                             hipFuncAttributeMaxDynamicSharedMemorySize,                  \
                                             FusedGeo<NT>::kRingBytes);                                   \
    if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(dynamic LDS)");                          \
    hipLaunchKernelGGL((scores_select_kernel<NT>), grid, dim3(512), FusedGeo<NT>::kRingBytes, st,         \
                       reinterpret_cast<const uint4*>(featQ), reinterpret_cast<const uint4*>(featK),      \
                       group, Nq, Nk, kdim_used, feat_stride, kappa, mask_bits, row_count, row_cols,      \
                       row_mass);                                                                         \
  } while (0)
  if (Nk <= 256) BASA_FUSED(2);
  else if (Nk <= 512) BASA_FUSED(4);
  else BASA_FUSED(8);
#undef BASA_FUSED
  BASA_HIP_CHECK_LAUNCH("scores_select_kernel");
  return BASA_OK;
}

namespace {
// One wave per block of a permutation: the largest (or smallest) original index in the block.
__global__ __launch_bounds__(256) void block_index_range_kernel(const int32_t* __restrict__ perm, int L, int B, int N,
                                                                int64_t blocks_total, int want_max,
                                                                int32_t* __restrict__ out) {
  const int64_t blk = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (blk >= blocks_total) return;
  const int lane = threadIdx.x & 63;
  const int64_t bh = blk / N;
  const int g = (int)(blk - bh * N);
  const int n = min(B, L - g * B);
  int v = want_max ? INT_MIN : INT_MAX;
  for (int i = lane; i < n; i += 64) {
    const int pos = g * B + i;
    const int r = perm_at(perm, bh * L, pos, L);
    v = want_max ? max(v, r) : min(v, r);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const int o = __shfl_xor(v, off);
    v = want_max ? max(v, o) : min(v, o);
  }
  if (lane == 0) out[blk] = v;
}

}  // namespace

basa_status launch_block_index_range(const int32_t* perm, int BH, int L, int B, int want_max, int32_t* out,
                                     hipStream_t st) {
  const int N = ceil_div(L, B);
  const int64_t total = (int64_t)BH * N;
  if (total == 0) return BASA_OK;
  ProfScope prof(K_ROW_SELECT, st);
  hipLaunchKernelGGL(block_index_range_kernel, dim3((unsigned)((total + 3) / 4)), dim3(256), 0, st, perm, L, B, N, total,
                     want_max, out);
  BASA_HIP_CHECK_LAUNCH("block_index_range_kernel");
  return BASA_OK;
}

basa_status launch_row_select(const float* scores, int rows_total, int Nk, int kappa,
                              float mass_target, int min_keep, const int32_t* keep_in, const LiveBlocks& live,
                              uint32_t* mask_bits, int32_t* row_count, int32_t* row_cols, float* row_mass,
                              hipStream_t st) {
  if (rows_total == 0) return BASA_OK;
  dim3 grid(ceil_div(rows_total, 4));
  ProfScope prof(K_ROW_SELECT, st);
#define BASA_SEL(M)                                                                                      \
  do {                                                                                                   \
    if (live.q_max)                                                                                      \
      hipLaunchKernelGGL((row_select_kernel<M, true>), grid, dim3(256), 0, st, scores, rows_total, Nk,   \
                         kappa, mass_target, min_keep, keep_in, live, mask_bits, row_count, row_cols, row_mass); \
    else                                                                                                 \
      hipLaunchKernelGGL((row_select_kernel<M, false>), grid, dim3(256), 0, st, scores, rows_total, Nk,  \
                         kappa, mass_target, min_keep, keep_in, live, mask_bits, row_count, row_cols, row_mass); \
  } while (0)
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
