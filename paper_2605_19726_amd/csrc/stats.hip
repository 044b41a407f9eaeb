// Block pooling (Sec. 3.1 mean pooling; Sec. 3.4 per-dimension variances; Alg. 1
// steps 3-4).  A workgroup gathers the B rows of a block of the ordered sequence
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
  uint16_t* feat_out;        // bf16 parts, [3][3d/8][N][8]
  int feat_is_query;
  void* sorted_out;          // nullable: the ordered sequence x[perm], contiguous [BH][L][d], dtype of x
};

constexpr int kGroup = 8;      // consecutive blocks per workgroup

// Element e of a 16-byte chunk as a float.
template <bool kBf16>
__device__ __forceinline__ float chunk_elem(const uint4& r, int e) {
  const uint32_t w[4] = {r.x, r.y, r.z, r.w};
  if constexpr (kBf16) return __uint_as_float((e & 1) ? (w[e >> 1] & 0xffff0000u) : (w[e >> 1] << 16));
  else return __uint_as_float(w[e]);
}

// A workgroup pools kGroup consecutive blocks of the ordered sequence, one after the other.  A row
// is 16-byte chunks spread over LPR adjacent lanes; a thread holds chunk `sub` of ITERS rows.  The
// rows of block b+1 (and the permutation entries of block b+2) are requested before block b is
// reduced, so the workgroup has loads in flight all the time: the gather is bound by the number of
// bytes in flight, and a kernel that loads, reduces and retires one block at a time has none in
// flight for half of its life.  Sums over the rows held by a wave are taken with lane exchanges,
// over the four waves through LDS.  The features of the kGroup blocks are collected in LDS and
// written at the end as 128-byte runs (in the [part][k/8][g][k%8] layout one block's features are
// 16-byte pieces 16 KB apart, which cost a fifth of the kernel when every block wrote its own).
template <bool kBf16, int kD, int kB>
__global__ __launch_bounds__(256) void block_stats_kernel(StatsJob j0, StatsJob j1, int BH0, float beta) {
  constexpr int kElem = kBf16 ? 2 : 4;
  constexpr int LPR = kD * kElem / 16;       // lanes per row
  constexpr int RPI = 256 / LPR;             // rows per iteration
  constexpr int ITERS = kB / RPI;
  constexpr int E = kBf16 ? 8 : 4;           // elements per chunk
  static_assert(ITERS >= 1 && LPR <= 64, "block too small for this tiling");
  __shared__ float red[2][2][4][kD];         // [block parity][mean | centred squares][wave][column]
  __shared__ __attribute__((aligned(16))) uint16_t stage[3][3 * kD / 8][kGroup][8];   // [part][k/8][block][k%8]

  const bool second = (int)blockIdx.y >= BH0;
  const StatsJob& job = second ? j1 : j0;
  const TensorView& x = job.x;
  float* mean_out = job.mean_out;
  float* var_out = job.var_out;
  uint16_t* feat_out = job.feat_out;
  const int feat_is_query = job.feat_is_query;
  uint4* sorted_out = reinterpret_cast<uint4*>(job.sorted_out);
  const int bh = second ? blockIdx.y - BH0 : blockIdx.y;
  const int L = x.L;
  const int N = (L + kB - 1) / kB;
  const int g0 = blockIdx.x * kGroup;
  const int nb = min(kGroup, N - g0);        // blocks of this workgroup that exist (>= 1 by the grid)
  const int sub = threadIdx.x % LPR, rig = threadIdx.x / LPR;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const char* base = reinterpret_cast<const char*>(x.ptr) + x.head_offset(bh) * kElem;
  const int32_t* pm = job.perm ? job.perm + (int64_t)bh * L : nullptr;
  const int64_t row_bytes = x.stride_l * kElem;

  // Token rows of block b for this thread.  Every load below is unconditional, with its index
  // clamped into the sequence (a position past L reads row L-1 and is masked out where it is
  // used): a load inside
  // a divergent branch is followed by a full wait, which serialises the eight loads of a thread.
  auto load_rows = [&](int b, int (&rows)[ITERS]) {             // entries as stored, checked at use
    const int p0 = (g0 + min(b, nb - 1)) * kB + rig;
    if (pm) {
#pragma unroll
      for (int it = 0; it < ITERS; ++it) rows[it] = pm[min(p0 + it * RPI, L - 1)];
    } else {
#pragma unroll
      for (int it = 0; it < ITERS; ++it) rows[it] = min(p0 + it * RPI, L - 1);
    }
  };
  auto load_chunks = [&](int b, const int (&rows)[ITERS], uint4 (&raw)[ITERS]) {
    const int p0 = (g0 + min(b, nb - 1)) * kB + rig;
    // a block past the workgroup's last has every lane read the head's first 16 bytes instead (one
    // cache line per instruction): streaming loads are not cached, a repeated block would be paid for
    const bool live = b < nb;                    // uniform over the workgroup
    const int sub_l = live ? sub : 0;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      // a malformed permutation entry falls back to the position itself
      const int row = (unsigned)rows[it] < (unsigned)L ? rows[it] : min(p0 + it * RPI, L - 1);
      // (streaming loads, as in the key pass: every row is read once)
      // (bit-cast into uint4, not held as the builtin's vector type: the compiler moves such vectors from
      //  buffer to buffer as whole registers, copies that count as uses of loads still in flight)
      typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
      raw[it] = __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + (live ? row : 0) * row_bytes) + sub_l));
    }
  };

  // Order of issue matters: loads return in order, so the permutation entries of block b+2 are
  // requested BEFORE the rows of block b+1; waiting for them later (to form the addresses of
  // block b+2) then leaves the rows of block b+1 in flight instead of draining the queue.
  int rows[ITERS], rows_after[ITERS];
  uint4 cur[ITERS], nxt[ITERS];
  load_rows(0, rows);
  load_chunks(0, rows, cur);
  load_rows(1, rows);
  for (int b = 0; b < nb; ++b) {
    load_rows(b + 2, rows_after);
    load_chunks(b + 1, rows, nxt);
    const int g = g0 + b;
    const int n_valid = min(kB, L - g * kB);
    const float inv_n = 1.0f / (float)n_valid;
    if (sorted_out) {
      // the rows are in registers exactly as loaded: the materialised ordered sequence is a copy
#pragma unroll
      for (int it = 0; it < ITERS; ++it) {
        const int pos = g * kB + it * RPI + rig;
        if (pos < L) sorted_out[((int64_t)bh * L + pos) * LPR + sub] = cur[it];
      }
    }

    // ---- per wave: mean and centred squares of the rows it holds (two passes over registers,
    // lane exchanges only, so the four waves run through both without meeting)
    constexpr int RPW = 64 / LPR;            // rows of one iteration held by a wave
    int n_w = 0;                             // valid rows of this wave's share of the block
#pragma unroll
    for (int it = 0; it < ITERS; ++it) n_w += max(0, min(RPW, n_valid - it * RPI - wave * RPW));
    const float inv_nw = n_w > 0 ? 1.0f / (float)n_w : 0.f;
    float mean_w[E], m2_w[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
      float a = 0.f;
      if (n_valid == kB) {                     // every block but a ragged last one
#pragma unroll
        for (int it = 0; it < ITERS; ++it) a += chunk_elem<kBf16>(cur[it], e);
      } else {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
          const int pos = g * kB + it * RPI + rig;
          a += (pos < L) ? chunk_elem<kBf16>(cur[it], e) : 0.f;
        }
      }
#pragma unroll
      for (int off = LPR; off < 64; off <<= 1) a += __shfl_xor(a, off);
      mean_w[e] = a * inv_nw;
    }
    // (the raw chunks are made opaque so that the floats of the first pass are converted again,
    // two integer ops each, rather than kept: 64 registers that the loads in flight need more)
#pragma unroll
    for (int it = 0; it < ITERS; ++it)
      asm volatile("" : "+v"(cur[it].x), "+v"(cur[it].y), "+v"(cur[it].z), "+v"(cur[it].w));
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const float m = mean_w[e];
      float a = 0.f;
      if (n_valid == kB) {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
          const float dv = chunk_elem<kBf16>(cur[it], e) - m;
          a = fmaf(dv, dv, a);
        }
      } else {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
          const int pos = g * kB + it * RPI + rig;
          const float dv = chunk_elem<kBf16>(cur[it], e) - m;
          a += (pos < L) ? dv * dv : 0.f;
        }
      }
#pragma unroll
      for (int off = LPR; off < 64; off <<= 1) a += __shfl_xor(a, off);
      m2_w[e] = a;
    }
    float (*rd)[4][kD] = red[b & 1];         // [0] wave means, [1] wave sums of centred squares
    if (lane < LPR) {
#pragma unroll
      for (int e = 0; e < E; ++e) {
        rd[0][wave][sub * E + e] = mean_w[e];
        rd[1][wave][sub * E + e] = m2_w[e];
      }
    }
    __syncthreads();
    // the other half of red is written before the next barrier, this half after it: every read
    // below is over by then
    if (threadIdx.x < kD) {
      // ---- the four waves' shares combined exactly: mean = sum n_w mean_w / n,
      //      M2 = sum M2_w + sum n_w (mean_w - mean)^2   (no cancellation either)
      const int c = threadIdx.x;
      float nw[4], mw[4];
      float acc = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        int cnt = 0;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) cnt += max(0, min(RPW, n_valid - it * RPI - w * RPW));
        nw[w] = (float)cnt;
        mw[w] = rd[0][w][c];
        acc = fmaf(nw[w], mw[w], acc);
      }
      const float mean_c = acc * inv_n;
      float m2 = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float dm = mw[w] - mean_c;
        m2 += rd[1][w][c] + nw[w] * dm * dm;
      }
      const float var_c = m2 * inv_n;
      const int64_t o = ((int64_t)bh * N + g) * kD + c;
      if (mean_out) mean_out[o] = mean_c;
      if (var_out) var_out[o] = var_c;
      if (feat_out) {
        float f[3];
        if (feat_is_query) {
          f[0] = mean_c * (1.0f / sqrtf((float)kD));
          f[1] = beta * var_c * (1.0f / (float)kD);
          f[2] = beta * (mean_c * mean_c) * (1.0f / (float)kD);
        } else {
          f[0] = mean_c;
          f[1] = mean_c * mean_c + var_c;
          f[2] = var_c;
        }
#pragma unroll
        for (int i = 0; i < 3; ++i) {
          // feature k = i*kD + c as three bf16 parts: each part is the rounding of what the parts
          // before it left (the subtractions are exact in fp32)
          const int k = i * kD + c;
          float rest = f[i];
#pragma unroll
          for (int part = 0; part < 3; ++part) {
            const __bf16 hi = (__bf16)rest;
            stage[part][k >> 3][b][k & 7] = __builtin_bit_cast(uint16_t, hi);
            rest -= (float)hi;
          }
        }
      }
    }
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      cur[it] = nxt[it];
      rows[it] = rows_after[it];
    }
  }
  if (feat_out) {
    // feature k of block g lives at [part][k / 8][g][k % 8]: the score kernel fetches 16-byte groups
    // of 64 consecutive blocks with one coalesced load
    __syncthreads();
    uint4* f4 = reinterpret_cast<uint4*>(feat_out + (int64_t)bh * N * (3 * 3 * kD));
    const uint4* st4 = reinterpret_cast<const uint4*>(&stage[0][0][0][0]);
    for (int i = threadIdx.x; i < 3 * (3 * kD / 8) * kGroup; i += 256) {
      const int pg = i / kGroup, gi = i % kGroup;         // pg = part * (3d/8) + k/8
      // (streaming stores: 151 MB of features written among 2.2 GB of reads; without the hint they cost
      //  2 % more of this kernel, and the score kernel that reads them next is none the slower)
      typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
      if (gi < nb)
        __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(&st4[i]),
                                    reinterpret_cast<u32x4*>(&f4[(int64_t)pg * N + g0 + gi]));
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
  dim3 grid(ceil_div(N, kGroup), BH0 + BH1);
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
                               float* var, void* feat, int feat_is_query, float beta, void* x_sorted,
                               hipStream_t st) {
  const StatsJob j{x, perm, mean, var, reinterpret_cast<uint16_t*>(feat), feat_is_query, x_sorted};
  return block_stats_impl(j, nullptr, B, beta, st);
}

basa_status launch_select_features(const TensorView& q, const int32_t* perm_q, void* feat_q,
                                   const TensorView& k, const int32_t* perm_k, void* feat_k, int B,
                                   float beta, hipStream_t st) {
  const StatsJob jq{q, perm_q, nullptr, nullptr, reinterpret_cast<uint16_t*>(feat_q), 1, nullptr};
  const StatsJob jk{k, perm_k, nullptr, nullptr, reinterpret_cast<uint16_t*>(feat_k), 0, nullptr};
  return block_stats_impl(jq, &jk, B, beta, st);
}

}  // namespace basa
