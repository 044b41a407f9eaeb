// Selection-fidelity diagnostics (Sec. 3.1 "oracle block distribution", Eq. 3; Sec. 3.2,
// Eq. 7-8 and the correlation study of Fig. 2).  They measure how well the cheap block
// distribution m' tracks the block masses of the dense attention map, and need the dense
// map: cost O(L^2 d), like dense attention.  None of this is on the selection / attention
// path.
//
//   block_mass_kernel   m_hat[g_q, g_k] = (1/|I(g_q)|) sum_{i in g_q} sum_{j in g_k} A_ij
//                       (Eq. 3) for the ordered sequences Q[perm_q], K[perm_k], and optionally
//                       max_{i,j} |l^_ij - l_{g_q,g_k}| per block pair (the observed logit
//                       deviation of Fig. 2).  bf16, d = 128, on the matrix cores: a workgroup
//                       of 4 waves owns 128 ordered queries (one wave per 32) and walks ALL key
//                       tiles twice: pass 0 finds every query's log-sum-exp with an online
//                       softmax, pass 1 exponentiates against it and adds up each tile.
//   block_radius_kernel R_g = max_i ||x_i - mean_g||, M_g = max_i ||x_i|| per block (Eq. 7)
//   deviation_bound_kernel  U = (R^Q M^K + M^Q R^K + R^Q R^K) / sqrt(d)   (Eq. 8)
//   fidelity_rows_kernel    per row of the block map: sum of m_hat over the kept blocks
//                       (recall) and || softmax(l') - m_hat ||_1
//   pearson_sums_kernel     the six sums a Pearson correlation coefficient is made of
#include <type_traits>
#include "common.hpp"

namespace basa {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kTileKeys = 64;
constexpr int kQueriesPerWg = 128;
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* gbl_ptr_t;

// Sizes that follow from the head dimension D (64 or 128).
template <int D>
struct MGeo {
  static constexpr int kRowBytes = D * 2;
  static constexpr int kCPR = D / 8;                          // 16-byte chunks per row
  static constexpr int kTileBytes = kTileKeys * kRowBytes;    // 16 KB or 8 KB
  static constexpr int kKSteps = D / 16;
  static constexpr int kChunksPerTile = kTileBytes / 1024;    // 1 KB direct-to-LDS loads per tile
};

struct MassArgs {
  const uint4* Qs;           // [BHq][rows_q][D/8 chunks]   ordered queries, zero rows past L_q
  const char* Kt;            // [BHkv][tiles][64 rows][D/8 chunks], chunk c of row r at c ^ (r & (D/8 - 1))
  const int32_t* perm_q;     // nullable
  const float* base_logits;  // nullable [BHq][Nq][Nk]: l of Eq. 2
  float* m_hat;              // [BHq][Nq][Nk]
  float* max_dev;            // nullable [BHq][Nq][Nk]
  float* lse;                // nullable [BHq][Lq], original token order
  int Nq, Nk, Lq, Lk, group, rows_q, tiles;
  float scale_log2e, inv_sqrt_d;
};

// Wave-wide sum / max with the result in lane 63, by data-parallel-primitive moves between lanes
// (no trip through the LDS crossbar): quads, half rows, rows of 16, then the row totals.
template <int kCtrl, int kRowMask, bool kMax>
__device__ __forceinline__ float dpp_step(float v) {
  const float o = __int_as_float(__builtin_amdgcn_update_dpp(kMax ? (int)0xff800000 : 0, __float_as_int(v), kCtrl, kRowMask, 0xf, !kMax));
  return kMax ? fmaxf(v, o) : v + o;
}
template <bool kMax>
__device__ __forceinline__ float wave_reduce_to_lane63(float v) {
  v = dpp_step<0xB1, 0xf, kMax>(v);     // quad_perm [1,0,3,2]
  v = dpp_step<0x4E, 0xf, kMax>(v);     // quad_perm [2,3,0,1]
  v = dpp_step<0x141, 0xf, kMax>(v);    // row_half_mirror
  v = dpp_step<0x140, 0xf, kMax>(v);    // row_mirror
  v = dpp_step<0x142, 0xa, kMax>(v);    // row_bcast:15 into rows 1 and 3
  v = dpp_step<0x143, 0xc, kMax>(v);    // row_bcast:31 into rows 2 and 3
  return v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}
__device__ __forceinline__ float max3f(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

// S^T = K Q^T of one 64-key tile in LDS for this wave's 32 queries: two 32-key row blocks.
template <int D>
__device__ __forceinline__ void mass_scores(const char* ks, const bf16x8 (&qf)[MGeo<D>::kKSteps], int kaddr0,
                                            floatx16& s0, floatx16& s1) {
  s0 = floatx16{0}; s1 = floatx16{0};
#pragma unroll
  for (int s = 0; s < MGeo<D>::kKSteps; ++s) {
    const int ka = kaddr0 ^ (s << 5);
    const bf16x8 k0 = *reinterpret_cast<const bf16x8*>(ks + ka);
    const bf16x8 k1 = *reinterpret_cast<const bf16x8*>(ks + ka + 32 * MGeo<D>::kRowBytes);
    s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0, qf[s], s0, 0, 0, 0);
    s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1, qf[s], s1, 0, 0, 0);
  }
}

// Dynamic LDS: [ring: 2 K tiles][logit rows: NQB x Nk floats (kDev)].  K tiles arrive by direct-to-LDS
// loads one tile ahead, one workgroup barrier per tile; the ragged last tile is peeled so that the
// masking code stays out of the loop; the running maximum of pass 0 is refreshed lazily; the tile
// sums of pass 1 are kept per lane over the tiles of a key block and reduced once per key block.
template <int kB, int D, bool kDev>      // kDev: also the observed logit deviation (needs base_logits)
__global__ __launch_bounds__(256, 2) void block_mass_kernel(MassArgs a) {
  using G = MGeo<D>;
  constexpr int NQB = kQueriesPerWg / kB;   // query blocks per workgroup: 1 or 2
  constexpr int WPG = kB / 32;              // waves per query block: 4 or 2
  constexpr int TPB = kB / kTileKeys;       // key tiles per key block: 2 or 1
  constexpr int kLoadsPerWave = G::kChunksPerTile / 4;
  constexpr float kLazyTau = 8.0f;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  __shared__ float part_mass[2][4], part_dev[2][4];
  float* lrow = reinterpret_cast<float*>(smem + 2 * G::kTileBytes);      // [NQB][Nk] (kDev)

  const int bhq = blockIdx.y, bhk = bhq / a.group, wg = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 31, h = lane >> 5;
  const int grp = wave / WPG;                            // query block of this wave inside the workgroup
  const int qpos = wg * kQueriesPerWg + wave * 32 + li;  // ordered position of this lane's query
  const bool q_valid = qpos < a.Lq;

  // Q^T operand: lane (query li, half h) holds Q[q][16 s + 8 h .. +7] for every k-step s
  bf16x8 qf[G::kKSteps];
  {
    const uint4* qp = a.Qs + ((int64_t)bhq * a.rows_q + qpos) * G::kCPR;
#pragma unroll
    for (int s = 0; s < G::kKSteps; ++s) {
      uint4 t4 = qp[2 * s + h];
      qf[s] = *reinterpret_cast<bf16x8*>(&t4);
    }
  }
  if (kDev) {
    for (int i = tid; i < NQB * a.Nk; i += 256) {
      const int gqb = min(wg * NQB + i / a.Nk, a.Nq - 1);
      lrow[i] = a.base_logits[((int64_t)bhq * a.Nq + gqb) * a.Nk + i % a.Nk];
    }
  }
  const char* Kh = a.Kt + (int64_t)bhk * a.tiles * G::kTileBytes;
  const int kaddr0 = li * G::kRowBytes + ((h ^ (li & (G::kCPR - 1))) << 4);
  const float c = a.scale_log2e;
  const int T = a.tiles;
  auto issue_tile = [&](int tile, int stage) {
#pragma unroll
    for (int j = 0; j < kLoadsPerWave; ++j) {
      const int cb = j * 4 + wave;
      const char* src = Kh + (int64_t)tile * G::kTileBytes + cb * 1024 + (uint32_t)(lane * 16);
      __builtin_amdgcn_global_load_lds((gbl_ptr_t)src, (lds_ptr_t)(smem + stage * G::kTileBytes + cb * 1024), 16, 0, 0);
    }
  };

  // ---- pass 0: log-sum-exp of every query over all keys (online softmax, lazy running maximum)
  float m_run = -INFINITY, l_run = 0.f;
  auto lse_tile = [&](auto masked, int t) {
    floatx16 s0, s1;
    mass_scores<D>(smem + (t & 1) * G::kTileBytes, qf, kaddr0, s0, s1);
    if (decltype(masked)::value) {
      const int nvalid = a.Lk - t * kTileKeys;          // >= 1
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int kk = 8 * (q >> 2) + 4 * h + (q & 3);
        if (kk >= nvalid) s0[q] = -INFINITY;
        if (32 + kk >= nvalid) s1[q] = -INFINITY;
      }
    }
    float mx = max3f(s0[0], s1[0], s0[1]);
#pragma unroll
    for (int q = 1; q < 15; ++q) mx = max3f(mx, s1[q], s0[q + 1]);
    mx = fmaxf(mx, s1[15]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float mc = mx * c;
    if (__builtin_amdgcn_ballot_w64(mc > m_run + kLazyTau) != 0) {
      const float m_new = fmaxf(m_run, mc);
      l_run *= __builtin_amdgcn_exp2f(m_run - m_new);
      m_run = m_new;
    }
    float sum = 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q)
      sum += __builtin_amdgcn_exp2f(fmaf(s0[q], c, -m_run)) + __builtin_amdgcn_exp2f(fmaf(s1[q], c, -m_run));
    l_run += sum;
  };
  issue_tile(0, 0);
  for (int t = 0; t + 1 < T; ++t) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    issue_tile(t + 1, (t + 1) & 1);
    lse_tile(std::false_type{}, t);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  lse_tile(std::true_type{}, T - 1);
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float lse2 = m_run + __log2f(l_tot);
  if (a.lse && q_valid && h == 0) {
    const int orow = perm_at(a.perm_q, (int64_t)bhq * a.Lq, qpos, a.Lq);
    a.lse[(int64_t)bhq * a.Lq + orow] = lse2 * 0.6931471805599453f;
  }
  __syncthreads();               // every wave is done with the ring before tile 0 lands in it again

  // ---- pass 1: exponentiate against the log-sum-exp, add up every key block
  float acc_sum = 0.f, acc_dev = 0.f;      // this lane's share of the current key block
  auto mass_tile = [&](auto masked, int t) {
    floatx16 s0, s1;
    mass_scores<D>(smem + (t & 1) * G::kTileBytes, qf, kaddr0, s0, s1);
    float lblk = 0.f;
    if (kDev) lblk = lrow[grp * a.Nk + t / TPB];
    float sum = 0.f, dev = 0.f;
    if (decltype(masked)::value) {
      const int nvalid = a.Lk - t * kTileKeys;
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int kk = 8 * (q >> 2) + 4 * h + (q & 3);
        if (kk < nvalid) {
          sum += __builtin_amdgcn_exp2f(fmaf(s0[q], c, -lse2));
          if (kDev) dev = fmaxf(dev, fabsf(fmaf(s0[q], a.inv_sqrt_d, -lblk)));
        }
        if (32 + kk < nvalid) {
          sum += __builtin_amdgcn_exp2f(fmaf(s1[q], c, -lse2));
          if (kDev) dev = fmaxf(dev, fabsf(fmaf(s1[q], a.inv_sqrt_d, -lblk)));
        }
      }
    } else {
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        sum += __builtin_amdgcn_exp2f(fmaf(s0[q], c, -lse2)) + __builtin_amdgcn_exp2f(fmaf(s1[q], c, -lse2));
        if (kDev) dev = max3f(dev, fabsf(fmaf(s0[q], a.inv_sqrt_d, -lblk)), fabsf(fmaf(s1[q], a.inv_sqrt_d, -lblk)));
      }
    }
    if (q_valid) { acc_sum += sum; acc_dev = fmaxf(acc_dev, dev); }
    if ((t % TPB) == TPB - 1 || t == T - 1) {
      // end of a key block: this wave's total to LDS (lane 63 holds it); combined after the next barrier
      const float ws = wave_reduce_to_lane63<false>(acc_sum);
      const float wd = kDev ? wave_reduce_to_lane63<true>(acc_dev) : 0.f;
      if (lane == 63) { part_mass[(t / TPB) & 1][wave] = ws; part_dev[(t / TPB) & 1][wave] = wd; }
      acc_sum = 0.f; acc_dev = 0.f;
    }
  };
  // thread b < NQB adds up, in a fixed order, the waves of query block b for key block kb
  auto combine = [&](int kb) {
    if (tid < NQB) {
      const int gqb = wg * NQB + tid;
      if (gqb < a.Nq) {
        float m = 0.f, dv = 0.f;
#pragma unroll
        for (int w = 0; w < WPG; ++w) {
          m += part_mass[kb & 1][tid * WPG + w];
          dv = fmaxf(dv, part_dev[kb & 1][tid * WPG + w]);
        }
        const int n_q = min(kB, a.Lq - gqb * kB);
        const int64_t o = ((int64_t)bhq * a.Nq + gqb) * a.Nk + kb;
        a.m_hat[o] = m / (float)n_q;
        if (kDev) a.max_dev[o] = dv;
      }
    }
  };
  issue_tile(0, 0);
  for (int t = 0; t + 1 < T; ++t) {
    // lgkmcnt too: the wave's own store of its block total (end of the tile before) has to be in LDS
    // before the barrier lets another wave read it.  The fence inside __syncthreads() is supposed to
    // see to that, but in this loop the compiler's wait-count pass was found to drop the LDS part
    // (rare stale totals, different from run to run), so the wait is spelt out.
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __syncthreads();
    if (t > 0 && (t % TPB) == 0) combine(t / TPB - 1);      // the key block that ended with tile t-1
    issue_tile(t + 1, (t + 1) & 1);
    mass_tile(std::false_type{}, t);
  }
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  __syncthreads();
  if (T > 1 && ((T - 1) % TPB) == 0) combine((T - 1) / TPB - 1);
  mass_tile(std::true_type{}, T - 1);
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __syncthreads();
  combine((T - 1) / TPB);
}

// Exact-arithmetic variant for f32 tensors (any supported d and B): one thread per query of a query
// block, keys staged through LDS 16 at a time; pass 0 the log-sum-exp, pass 1 the block masses and
// deviations, reduced over the block's threads in a fixed order.  Not tuned: fp32 inputs are the
// small parity workloads.
template <int kDim, int kB>
__global__ __launch_bounds__(kB) void block_mass_simple_kernel(TensorView q, TensorView k, const int32_t* __restrict__ perm_q,
                                                               const int32_t* __restrict__ perm_k,
                                                               const float* __restrict__ base_logits,
                                                               float* __restrict__ m_hat, float* __restrict__ max_dev,
                                                               float* __restrict__ lse_out, int Nq, int Nk) {
  constexpr int kTK = 16;
  __shared__ __attribute__((aligned(16))) float Ks[kTK][kDim];
  __shared__ float red_s[kB], red_d[kB];
  const int gq = blockIdx.x, bhq = blockIdx.y, bhk = bhq / (q.heads / k.heads);
  const int Lq = q.L, Lk = k.L;
  const int pos = gq * kB + threadIdx.x;
  const bool active = pos < Lq;
  const int qrow = active ? perm_at(perm_q, (int64_t)bhq * Lq, pos, Lq) : 0;
  float qv[kDim];
  {
    const float4* qp = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(q.ptr) + q.head_offset(bhq) +
                                                       (int64_t)qrow * q.stride_l);
#pragma unroll
    for (int t = 0; t < kDim / 4; ++t) {
      const float4 v = qp[t];
      qv[4 * t] = v.x; qv[4 * t + 1] = v.y; qv[4 * t + 2] = v.z; qv[4 * t + 3] = v.w;
    }
  }
  const float* kbase = reinterpret_cast<const float*>(k.ptr) + k.head_offset(bhk);
  const float scale = 1.0f / sqrtf((float)kDim);
  const int n_q = min(kB, Lq - gq * kB);
  float m = -INFINITY, l = 0.f, lse = 0.f;
  for (int pass = 0; pass < 2; ++pass) {
    for (int gk = 0; gk < Nk; ++gk) {
      const int kvalid = min(kB, Lk - gk * kB);
      float bsum = 0.f, bdev = 0.f;
      const float lblk = (pass == 1 && max_dev) ? base_logits[((int64_t)bhq * Nq + gq) * Nk + gk] : 0.f;
      for (int t0 = 0; t0 < kvalid; t0 += kTK) {
        const int nk = min(kTK, kvalid - t0);
        __syncthreads();
        for (int w = threadIdx.x; w < kTK * (kDim / 4); w += kB) {
          const int j = w / (kDim / 4), c4 = w - j * (kDim / 4);
          float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
          if (j < nk) {
            const int krow = perm_at(perm_k, (int64_t)bhk * Lk, gk * kB + t0 + j, Lk);
            v = reinterpret_cast<const float4*>(kbase + (int64_t)krow * k.stride_l)[c4];
          }
          *reinterpret_cast<float4*>(&Ks[j][4 * c4]) = v;
        }
        __syncthreads();
        float s[kTK], tmax = -INFINITY;
#pragma unroll
        for (int j = 0; j < kTK; ++j) {
          float d0 = 0.f;
#pragma unroll
          for (int t = 0; t < kDim; ++t) d0 = fmaf(qv[t], Ks[j][t], d0);
          s[j] = (j < nk) ? d0 * scale : -INFINITY;
          tmax = fmaxf(tmax, s[j]);
        }
        if (pass == 0) {
          const float m_new = fmaxf(m, tmax);
          l *= expf(m - m_new);
#pragma unroll
          for (int j = 0; j < kTK; ++j) l += expf(s[j] - m_new);
          m = m_new;
        } else {
#pragma unroll
          for (int j = 0; j < kTK; ++j) {
            bsum += expf(s[j] - lse);                         // keys past the block: exp(-inf) = 0
            if (j < nk) bdev = fmaxf(bdev, fabsf(s[j] - lblk));
          }
        }
      }
      if (pass == 1) {
        // the block's queries added up in a fixed order (tree over the threads)
        __syncthreads();
        red_s[threadIdx.x] = active ? bsum : 0.f;
        red_d[threadIdx.x] = active ? bdev : 0.f;
        __syncthreads();
        for (int off = kB / 2; off > 0; off >>= 1) {
          if ((int)threadIdx.x < off) {
            red_s[threadIdx.x] += red_s[threadIdx.x + off];
            red_d[threadIdx.x] = fmaxf(red_d[threadIdx.x], red_d[threadIdx.x + off]);
          }
          __syncthreads();
        }
        if (threadIdx.x == 0) {
          const int64_t o = ((int64_t)bhq * Nq + gq) * Nk + gk;
          m_hat[o] = red_s[0] / (float)n_q;
          if (max_dev) max_dev[o] = red_d[0];
        }
      }
    }
    if (pass == 0) {
      lse = m + logf(l);
      if (lse_out && active) lse_out[(int64_t)bhq * Lq + qrow] = lse;
    }
  }
}

// Rows of a bf16 tensor in the given order, zero rows up to rows_padded; swizzle = 1 writes
// the K-tile image (chunk c of row r at chunk position c ^ (r & (chunks per row - 1))).
template <int D>
__global__ __launch_bounds__(256) void diag_gather_rows_kernel(TensorView x, const int32_t* __restrict__ perm,
                                                               uint4* __restrict__ dst, int rows_padded,
                                                               int swizzle) {
  constexpr int CPR = D / 8, RPI = 256 / CPR, ITERS = 64 / RPI;
  const int bh = blockIdx.y;
  const int sub = threadIdx.x % CPR, rig = threadIdx.x / CPR;
  const int32_t* pm = perm ? perm + (int64_t)bh * x.L : nullptr;
  const char* base = reinterpret_cast<const char*>(x.ptr) + x.head_offset(bh) * 2;
  uint4 v[ITERS];
  gather_chunks<ITERS>(v, pm, base, x.L, (int64_t)x.stride_l * 2, blockIdx.x * 64 + rig, RPI, sub);
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int pos = blockIdx.x * 64 + it * RPI + rig;
    const int cpos = swizzle ? (sub ^ (pos & (CPR - 1))) : sub;
    if (pos < rows_padded) dst[((int64_t)bh * rows_padded + pos) * CPR + cpos] = v[it];
  }
}

// ---------------------------------------------------------------------------------
// Eq. 7: per block of the ordered sequence, R = max_i ||x_i - mean||, M = max_i ||x_i||
// ---------------------------------------------------------------------------------
template <bool kBf16, int kDim, int kB>
__global__ __launch_bounds__(256) void block_radius_kernel(TensorView x, const int32_t* __restrict__ perm,
                                                           float* __restrict__ radius,
                                                           float* __restrict__ max_norm) {
  constexpr int kElem = kBf16 ? 2 : 4;
  constexpr int LPR = kDim * kElem / 16;     // lanes per row
  constexpr int RPI = 256 / LPR;             // rows per iteration
  constexpr int ITERS = kB / RPI;
  constexpr int E = Chunk16<kBf16>::kElems;
  __shared__ float red[RPI][kDim];
  __shared__ float mean_s[kDim];
  __shared__ float wmax[2][4];

  const int bh = blockIdx.y, g = blockIdx.x;
  const int L = x.L, N = (L + kB - 1) / kB;
  const int sub = threadIdx.x % LPR, rig = threadIdx.x / LPR;
  const char* base = reinterpret_cast<const char*>(x.ptr) + x.head_offset(bh) * kElem;
  const int32_t* pm = perm ? perm + (int64_t)bh * L : nullptr;
  const int n_valid = min(kB, L - g * kB);

  Chunk16<kBf16> c[ITERS];
  {
    uint4 raw[ITERS];
    gather_chunks<ITERS>(raw, pm, base, L, (int64_t)x.stride_l * kElem, g * kB + rig, RPI, sub);
#pragma unroll
    for (int it = 0; it < ITERS; ++it) c[it].set(raw[it]);       // rows past L are zeros
  }
#pragma unroll
  for (int e = 0; e < E; ++e) {
    float s = 0.f;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) s += c[it].v[e];
    red[rig][sub * E + e] = s;
  }
  __syncthreads();
  if (threadIdx.x < kDim) {
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < RPI; ++r) s += red[r][threadIdx.x];
    mean_s[threadIdx.x] = s / (float)n_valid;
  }
  __syncthreads();
  float best_r = 0.f, best_m = 0.f;
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    float dr = 0.f, dm = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const float v = c[it].v[e], dv = v - mean_s[sub * E + e];
      dr += dv * dv;
      dm += v * v;
    }
#pragma unroll
    for (int off = LPR / 2; off > 0; off >>= 1) {
      dr += __shfl_xor(dr, off, LPR);
      dm += __shfl_xor(dm, off, LPR);
    }
    if (g * kB + it * RPI + rig < L) { best_r = fmaxf(best_r, dr); best_m = fmaxf(best_m, dm); }
  }
  best_r = wave_max(best_r);
  best_m = wave_max(best_m);
  if ((threadIdx.x & 63) == 0) { wmax[0][threadIdx.x >> 6] = best_r; wmax[1][threadIdx.x >> 6] = best_m; }
  __syncthreads();
  if (threadIdx.x == 0) {
    const float r2 = fmaxf(fmaxf(wmax[0][0], wmax[0][1]), fmaxf(wmax[0][2], wmax[0][3]));
    const float m2 = fmaxf(fmaxf(wmax[1][0], wmax[1][1]), fmaxf(wmax[1][2], wmax[1][3]));
    radius[(int64_t)bh * N + g] = sqrtf(r2);
    max_norm[(int64_t)bh * N + g] = sqrtf(m2);
  }
}

// Eq. 8, one thread per block pair.
__global__ __launch_bounds__(256) void deviation_bound_kernel(const float* __restrict__ rq,
                                                              const float* __restrict__ mq,
                                                              const float* __restrict__ rk,
                                                              const float* __restrict__ mk,
                                                              float* __restrict__ U, int group, int Nq,
                                                              int Nk, float inv_sqrt_d) {
  const int bhq = blockIdx.z, gq = blockIdx.y, gk = blockIdx.x * 256 + threadIdx.x;
  if (gk >= Nk) return;
  const int bhk = bhq / group;
  const float Rq = rq[(int64_t)bhq * Nq + gq], Mq = mq[(int64_t)bhq * Nq + gq];
  const float Rk = rk[(int64_t)bhk * Nk + gk], Mk = mk[(int64_t)bhk * Nk + gk];
  U[((int64_t)bhq * Nq + gq) * Nk + gk] = (Rq * Mk + Mq * Rk + Rq * Rk) * inv_sqrt_d;
}

// One wave per row of the block map: recall = sum of m_hat over the kept blocks,
// l1 = sum_k | softmax(l')_k - m_hat_k |.
__global__ __launch_bounds__(256) void fidelity_rows_kernel(const float* __restrict__ scores,
                                                            const uint32_t* __restrict__ mask_bits,
                                                            const float* __restrict__ m_hat, int rows,
                                                            int Nk, float* __restrict__ recall,
                                                            float* __restrict__ l1) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  const float* sc = scores + (int64_t)row * Nk;
  const float* mh = m_hat + (int64_t)row * Nk;
  const uint32_t* mb = mask_bits + (int64_t)row * ((Nk + 31) >> 5);
  float mx = -INFINITY;
  for (int k = lane; k < Nk; k += 64) mx = fmaxf(mx, sc[k]);
  mx = wave_max(mx);
  float z = 0.f;
  for (int k = lane; k < Nk; k += 64) z += expf(sc[k] - mx);
  z = wave_sum(z);
  float rec = 0.f, dist = 0.f;
  for (int k = lane; k < Nk; k += 64) {
    const float mp = expf(sc[k] - mx) / z, t = mh[k];
    dist += fabsf(mp - t);
    if ((mb[k >> 5] >> (k & 31)) & 1u) rec += t;
  }
  rec = wave_sum(rec);
  dist = wave_sum(dist);
  if (lane == 0) {
    if (recall) recall[row] = rec;
    if (l1) l1[row] = dist;
  }
}

// sums[0..5] += n, sum x, sum y, sum x^2, sum y^2, sum x y   (fp64)
__global__ __launch_bounds__(256) void pearson_sums_kernel(const float* __restrict__ x,
                                                           const float* __restrict__ y, int64_t n,
                                                           double* __restrict__ sums) {
  __shared__ double red[5][4];
  double sx = 0, sy = 0, sxx = 0, syy = 0, sxy = 0;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const double a = x[i], b = y[i];
    sx += a; sy += b; sxx += a * a; syy += b * b; sxy += a * b;
  }
  double v[5] = {sx, sy, sxx, syy, sxy};
#pragma unroll
  for (int j = 0; j < 5; ++j) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v[j] += __shfl_xor(v[j], off);
    if ((threadIdx.x & 63) == 0) red[j][threadIdx.x >> 6] = v[j];
  }
  __syncthreads();
  if (threadIdx.x < 5) {
    const int j = threadIdx.x;
    atomicAdd(&sums[1 + j], red[j][0] + red[j][1] + red[j][2] + red[j][3]);
  }
  if (threadIdx.x == 5 && blockIdx.x == 0) atomicAdd(&sums[0], (double)n);
}

__global__ void zero_doubles_kernel(double* p, int n) {
  if ((int)threadIdx.x < n) p[threadIdx.x] = 0.0;
}

size_t q_bytes(int BHq, int Lq, int d) { return align_up((size_t)BHq * ceil_div(Lq, kQueriesPerWg) * kQueriesPerWg * d * 2, 256); }
size_t k_bytes(int BHkv, int Lk, int d) { return align_up((size_t)BHkv * ceil_div(Lk, kTileKeys) * kTileKeys * d * 2, 256); }

template <int D>
basa_status launch_block_mass_mfma(const TensorView& q, const TensorView& k, const int32_t* perm_q,
                                   const int32_t* perm_k, int B, const float* base_logits, float* m_hat,
                                   float* max_dev, float* lse, void* ws, hipStream_t st) {
  const int BHq = q.batch * q.heads, BHkv = k.batch * k.heads;
  const int rows_q = ceil_div(q.L, kQueriesPerWg) * kQueriesPerWg, tiles = ceil_div(k.L, kTileKeys);
  uint4* Qs = reinterpret_cast<uint4*>(ws);
  uint4* Kt = reinterpret_cast<uint4*>(reinterpret_cast<char*>(ws) + q_bytes(BHq, q.L, D));
  {
    ProfScope prof(K_GATHER, st);
    hipLaunchKernelGGL(diag_gather_rows_kernel<D>, dim3(rows_q / 64, BHq), dim3(256), 0, st, q, perm_q, Qs, rows_q, 0);
    BASA_HIP_CHECK_LAUNCH("diag_gather_rows_kernel(Q)");
    hipLaunchKernelGGL(diag_gather_rows_kernel<D>, dim3(tiles, BHkv), dim3(256), 0, st, k, perm_k, Kt, tiles * kTileKeys, 1);
    BASA_HIP_CHECK_LAUNCH("diag_gather_rows_kernel(K)");
  }
  MassArgs a;
  a.Qs = Qs; a.Kt = reinterpret_cast<const char*>(Kt); a.perm_q = perm_q; a.base_logits = base_logits;
  a.m_hat = m_hat; a.max_dev = max_dev; a.lse = lse;
  a.Nq = ceil_div(q.L, B); a.Nk = ceil_div(k.L, B); a.Lq = q.L; a.Lk = k.L;
  a.group = q.heads / k.heads; a.rows_q = rows_q; a.tiles = tiles;
  a.scale_log2e = 1.4426950408889634f / sqrtf((float)D);
  a.inv_sqrt_d = 1.0f / sqrtf((float)D);
  const bool want_dev = max_dev != nullptr && base_logits != nullptr;
  const size_t lds = 2 * MGeo<D>::kTileBytes + (want_dev ? (size_t)(kQueriesPerWg / B) * a.Nk * sizeof(float) : 0);
  if (lds > 64 * 1024) {
    set_error("block mass: %d key blocks need %zu bytes of LDS per workgroup (limit 65536)", a.Nk, lds);
    return BASA_ERR_UNSUPPORTED;
  }
  ProfScope prof(K_BLOCK_MASS, st);
  const dim3 grid(rows_q / kQueriesPerWg, BHq);
#define BASA_MASS(BB, DEV)                                                                                     \
  do {                                                                                                         \
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&block_mass_kernel<BB, D, DEV>),    \
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);           \
    if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(dynamic LDS)");                               \
    hipLaunchKernelGGL((block_mass_kernel<BB, D, DEV>), grid, dim3(256), lds, st, a);                          \
  } while (0)
  if (B == 128 && want_dev) BASA_MASS(128, true);
  else if (B == 128) BASA_MASS(128, false);
  else if (want_dev) BASA_MASS(64, true);
  else BASA_MASS(64, false);
#undef BASA_MASS
  BASA_HIP_CHECK_LAUNCH("block_mass_kernel");
  return BASA_OK;
}

}  // namespace

size_t block_mass_workspace_bytes(int BHq, int BHkv, int Lq, int Lk, int d) {
  return q_bytes(BHq, Lq, d) + k_bytes(BHkv, Lk, d);
}

basa_status launch_block_mass(const TensorView& q, const TensorView& k, const int32_t* perm_q,
                              const int32_t* perm_k, int B, const float* base_logits, float* m_hat,
                              float* max_dev, float* lse, void* ws, hipStream_t st) {
  const int BHq = q.batch * q.heads;
  if (BHq == 0 || q.L == 0 || k.L == 0) return BASA_OK;
  if (q.dtype == BASA_BF16) {
    return q.d == 128 ? launch_block_mass_mfma<128>(q, k, perm_q, perm_k, B, base_logits, m_hat, max_dev, lse, ws, st)
                      : launch_block_mass_mfma<64>(q, k, perm_q, perm_k, B, base_logits, m_hat, max_dev, lse, ws, st);
  }
  // f32 tensors: the exact-arithmetic kernel, no workspace
  const int Nq = ceil_div(q.L, B), Nk = ceil_div(k.L, B);
  float* dev_out = (max_dev && base_logits) ? max_dev : nullptr;
  ProfScope prof(K_BLOCK_MASS, st);
  const dim3 grid(Nq, BHq);
#define BASA_MS(DD, BB) \
  hipLaunchKernelGGL((block_mass_simple_kernel<DD, BB>), grid, dim3(BB), 0, st, q, k, perm_q, perm_k, base_logits, m_hat, dev_out, lse, Nq, Nk)
  if (q.d == 128 && B == 128) BASA_MS(128, 128);
  else if (q.d == 128) BASA_MS(128, 64);
  else if (B == 128) BASA_MS(64, 128);
  else BASA_MS(64, 64);
#undef BASA_MS
  BASA_HIP_CHECK_LAUNCH("block_mass_simple_kernel");
  return BASA_OK;
}

basa_status launch_block_radius(const TensorView& x, const int32_t* perm, int B, float* radius,
                                float* max_norm, hipStream_t st) {
  const int BH = x.batch * x.heads, N = ceil_div(x.L, B);
  if (BH == 0 || N == 0) return BASA_OK;
  const dim3 grid(N, BH);
  const bool bf = x.dtype == BASA_BF16;
  ProfScope prof(K_DIAG_SMALL, st);
#define BASA_RAD(BF, D, BB) \
  hipLaunchKernelGGL((block_radius_kernel<BF, D, BB>), grid, dim3(256), 0, st, x, perm, radius, max_norm)
  if (bf && x.d == 128 && B == 128) BASA_RAD(true, 128, 128);
  else if (bf && x.d == 128 && B == 64) BASA_RAD(true, 128, 64);
  else if (bf && x.d == 64 && B == 128) BASA_RAD(true, 64, 128);
  else if (bf && x.d == 64 && B == 64) BASA_RAD(true, 64, 64);
  else if (!bf && x.d == 128 && B == 128) BASA_RAD(false, 128, 128);
  else if (!bf && x.d == 128 && B == 64) BASA_RAD(false, 128, 64);
  else if (!bf && x.d == 64 && B == 128) BASA_RAD(false, 64, 128);
  else BASA_RAD(false, 64, 64);
#undef BASA_RAD
  BASA_HIP_CHECK_LAUNCH("block_radius_kernel");
  return BASA_OK;
}

basa_status launch_deviation_bound(const float* rq, const float* mq, const float* rk, const float* mk,
                                   int BHq, int group, int Nq, int Nk, int d, float* U, hipStream_t st) {
  if (BHq == 0 || Nq == 0 || Nk == 0) return BASA_OK;
  ProfScope prof(K_DIAG_SMALL, st);
  hipLaunchKernelGGL(deviation_bound_kernel, dim3(ceil_div(Nk, 256), Nq, BHq), dim3(256), 0, st, rq, mq, rk, mk,
                     U, group, Nq, Nk, 1.0f / sqrtf((float)d));
  BASA_HIP_CHECK_LAUNCH("deviation_bound_kernel");
  return BASA_OK;
}

basa_status launch_fidelity_rows(const float* scores, const uint32_t* mask_bits, const float* m_hat,
                                 int rows, int Nk, float* recall, float* l1, hipStream_t st) {
  if (rows == 0) return BASA_OK;
  ProfScope prof(K_DIAG_SMALL, st);
  hipLaunchKernelGGL(fidelity_rows_kernel, dim3(ceil_div(rows, 4)), dim3(256), 0, st, scores, mask_bits, m_hat,
                     rows, Nk, recall, l1);
  BASA_HIP_CHECK_LAUNCH("fidelity_rows_kernel");
  return BASA_OK;
}

basa_status launch_pearson_sums(const float* x, const float* y, int64_t n, double* sums, hipStream_t st) {
  ProfScope prof(K_DIAG_SMALL, st);
  hipLaunchKernelGGL(zero_doubles_kernel, dim3(1), dim3(64), 0, st, sums, 6);
  BASA_HIP_CHECK_LAUNCH("zero_doubles_kernel");
  if (n > 0) {
    const int grid = (int)((n + 256 * 64 - 1) / (256 * 64));
    hipLaunchKernelGGL(pearson_sums_kernel, dim3(grid > 1024 ? 1024 : grid), dim3(256), 0, st, x, y, n, sums);
    BASA_HIP_CHECK_LAUNCH("pearson_sums_kernel");
  }
  return BASA_OK;
}

}  // namespace basa
