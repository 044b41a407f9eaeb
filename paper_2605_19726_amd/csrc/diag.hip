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
#include "common.hpp"

namespace basa {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kD = 128;
constexpr int kTileKeys = 64;
constexpr int kTileChunks = 1024;          // 16-byte chunks of one 64-key tile
constexpr int kQueriesPerWg = 128;

struct MassArgs {
  const uint4* Qs;           // [BHq][rows_q][16 chunks]   ordered queries, zero rows past L_q
  const uint4* Kt;           // [BHkv][tiles][64 rows][16 chunks], chunk c of row r at c ^ (r & 15)
  const int32_t* perm_q;     // nullable
  const float* base_logits;  // nullable [BHq][Nq][Nk]: l of Eq. 2
  float* m_hat;              // [BHq][Nq][Nk]
  float* max_dev;            // nullable [BHq][Nq][Nk]
  float* lse;                // nullable [BHq][Lq], original token order
  int Nq, Nk, Lq, Lk, group, rows_q, tiles;
  float scale_log2e, inv_sqrt_d;
};

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

template <int kB, bool kDev>      // kDev: also the observed logit deviation (needs base_logits)
__global__ __launch_bounds__(256) void block_mass_kernel(MassArgs a) {
  constexpr int NQB = kQueriesPerWg / kB;   // query blocks per workgroup: 1 or 2
  constexpr int WPG = kB / 32;              // waves per query block: 4 or 2
  constexpr int TPB = kB / kTileKeys;       // key tiles per key block: 2 or 1
  __shared__ uint4 kbuf[2][kTileChunks];
  __shared__ float part_mass[2][4], part_dev[2][4];

  const int bhq = blockIdx.y, bhk = bhq / a.group, wg = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 31, h = lane >> 5;
  const int gq = wg * NQB + wave / WPG;                 // may be >= Nq in the last workgroup
  const int qpos = wg * kQueriesPerWg + wave * 32 + li; // ordered position of this lane's query
  const bool q_valid = qpos < a.Lq;

  // Q^T operand: lane (query li, half h) holds Q[q][16 s + 8 h .. +7] for s = 0..7
  bf16x8 qf[8];
  {
    const uint4* qp = a.Qs + ((int64_t)bhq * a.rows_q + qpos) * 16;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      uint4 t4 = qp[2 * s + h];
      qf[s] = *reinterpret_cast<bf16x8*>(&t4);
    }
  }
  const uint4* Kh = a.Kt + (int64_t)bhk * a.tiles * kTileChunks;
  const int kaddr0 = li * 256 + ((h ^ (li & 15)) << 4);
  const float c = a.scale_log2e;
  const int T = a.tiles;

  float m_run = -INFINITY, l_run = 0.f, lse2 = 0.f;
  for (int pass = 0; pass < 2; ++pass) {
    uint4 r[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) kbuf[0][i * 256 + tid] = Kh[i * 256 + tid];
    __syncthreads();
    float acc_mass = 0.f, acc_dev = 0.f;     // used by threads tid < NQB in pass 1
    for (int t = 0; t < T; ++t) {
      // next tile into registers (past the end: the last tile again, stored but never used;
      // kept unconditional so that r stays in registers and the loads stay in flight)
      {
        const int tn = min(t + 1, T - 1);
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = Kh[(int64_t)tn * kTileChunks + i * 256 + tid];
      }
      const char* ks = reinterpret_cast<const char*>(kbuf[t & 1]);
      floatx16 s0 = {0}, s1 = {0};
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const int ka = kaddr0 ^ (s << 5);
        const bf16x8 k0 = *reinterpret_cast<const bf16x8*>(ks + ka);
        const bf16x8 k1 = *reinterpret_cast<const bf16x8*>(ks + ka + 32 * 256);
        s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0, qf[s], s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1, qf[s], s1, 0, 0, 0);
      }
      // register r of lane half h holds key 8*(r/4) + 4h + r%4 of its 32-key half
      const int nvalid = a.Lk - t * kTileKeys;          // >= 1
      if (pass == 0) {
        float mx = -INFINITY;
#pragma unroll
        for (int q = 0; q < 16; ++q) {
          const int kk = 8 * (q >> 2) + 4 * h + (q & 3);
          if (kk >= nvalid) s0[q] = -INFINITY;
          if (32 + kk >= nvalid) s1[q] = -INFINITY;
          mx = fmaxf(mx, fmaxf(s0[q], s1[q]));
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx * c);
        float sum = 0.f;
#pragma unroll
        for (int q = 0; q < 16; ++q)
          sum += __builtin_amdgcn_exp2f(fmaf(s0[q], c, -m_new)) + __builtin_amdgcn_exp2f(fmaf(s1[q], c, -m_new));
        l_run = l_run * __builtin_amdgcn_exp2f(m_run - m_new) + sum;
        m_run = m_new;
      } else {
        float lblk = 0.f;
        if (kDev && gq < a.Nq) lblk = a.base_logits[((int64_t)bhq * a.Nq + gq) * a.Nk + t / TPB];
        float sum = 0.f, dev = 0.f;
#pragma unroll
        for (int q = 0; q < 16; ++q) {
          const int kk = 8 * (q >> 2) + 4 * h + (q & 3);
          if (kk < nvalid) {
            sum += __builtin_amdgcn_exp2f(fmaf(s0[q], c, -lse2));
            if (kDev) dev = fmaxf(dev, fabsf(s0[q] * a.inv_sqrt_d - lblk));
          }
          if (32 + kk < nvalid) {
            sum += __builtin_amdgcn_exp2f(fmaf(s1[q], c, -lse2));
            if (kDev) dev = fmaxf(dev, fabsf(s1[q] * a.inv_sqrt_d - lblk));
          }
        }
        if (!q_valid) { sum = 0.f; dev = 0.f; }
        sum = wave_sum(sum);
        if (kDev) dev = wave_max(dev);
        if (lane == 0) { part_mass[t & 1][wave] = sum; part_dev[t & 1][wave] = dev; }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) kbuf[(t + 1) & 1][i * 256 + tid] = r[i];
      __syncthreads();
      if (pass == 1 && tid < NQB) {
        // thread b adds up, in a fixed order, the waves of query block b and the tiles of a key block
        const int gqb = wg * NQB + tid;
        if (gqb < a.Nq) {
#pragma unroll
          for (int w = 0; w < WPG; ++w) {
            acc_mass += part_mass[t & 1][tid * WPG + w];
            acc_dev = fmaxf(acc_dev, part_dev[t & 1][tid * WPG + w]);
          }
          if ((t % TPB) == TPB - 1 || t == T - 1) {
            const int n_q = min(kB, a.Lq - gqb * kB);
            const int64_t o = ((int64_t)bhq * a.Nq + gqb) * a.Nk + t / TPB;
            a.m_hat[o] = acc_mass / (float)n_q;
            if (kDev) a.max_dev[o] = acc_dev;
            acc_mass = 0.f;
            acc_dev = 0.f;
          }
        }
      }
    }
    if (pass == 0) {
      const float l_tot = l_run + __shfl_xor(l_run, 32);
      lse2 = m_run + __log2f(l_tot);
      if (a.lse && q_valid && h == 0) {
        const int orow = perm_at(a.perm_q, (int64_t)bhq * a.Lq, qpos, a.Lq);
        a.lse[(int64_t)bhq * a.Lq + orow] = lse2 * 0.6931471805599453f;
      }
    }
    // the last iteration ended with a barrier: kbuf[0] may be refilled
  }
}

// Rows of a bf16 tensor in the given order, zero rows up to rows_padded; swizzle = 1 writes
// the K-tile image (chunk c of row r at chunk position c ^ (r & 15)).
__global__ __launch_bounds__(256) void diag_gather_rows_kernel(TensorView x, const int32_t* __restrict__ perm,
                                                               uint4* __restrict__ dst, int rows_padded,
                                                               int swizzle) {
  const int bh = blockIdx.y;
  const int sub = threadIdx.x & 15, rig = threadIdx.x >> 4;
  const int32_t* pm = perm ? perm + (int64_t)bh * x.L : nullptr;
  const char* base = reinterpret_cast<const char*>(x.ptr) + x.head_offset(bh) * 2;
  uint4 v[4];
  gather_chunks<4>(v, pm, base, x.L, (int64_t)x.stride_l * 2, blockIdx.x * 64 + rig, 16, sub);
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int pos = blockIdx.x * 64 + it * 16 + rig;
    const int cpos = swizzle ? (sub ^ (pos & 15)) : sub;
    if (pos < rows_padded) dst[((int64_t)bh * rows_padded + pos) * 16 + cpos] = v[it];
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

size_t q_bytes(int BHq, int Lq) { return align_up((size_t)BHq * ceil_div(Lq, kQueriesPerWg) * kQueriesPerWg * kD * 2, 256); }
size_t k_bytes(int BHkv, int Lk) { return align_up((size_t)BHkv * ceil_div(Lk, kTileKeys) * kTileKeys * kD * 2, 256); }

}  // namespace

size_t block_mass_workspace_bytes(int BHq, int BHkv, int Lq, int Lk) { return q_bytes(BHq, Lq) + k_bytes(BHkv, Lk); }

basa_status launch_block_mass(const TensorView& q, const TensorView& k, const int32_t* perm_q,
                              const int32_t* perm_k, int B, const float* base_logits, float* m_hat,
                              float* max_dev, float* lse, void* ws, hipStream_t st) {
  const int BHq = q.batch * q.heads, BHkv = k.batch * k.heads;
  if (BHq == 0 || q.L == 0 || k.L == 0) return BASA_OK;
  const int rows_q = ceil_div(q.L, kQueriesPerWg) * kQueriesPerWg, tiles = ceil_div(k.L, kTileKeys);
  uint4* Qs = reinterpret_cast<uint4*>(ws);
  uint4* Kt = reinterpret_cast<uint4*>(reinterpret_cast<char*>(ws) + q_bytes(BHq, q.L));
  {
    ProfScope prof(K_GATHER, st);
    hipLaunchKernelGGL(diag_gather_rows_kernel, dim3(rows_q / 64, BHq), dim3(256), 0, st, q, perm_q, Qs, rows_q, 0);
    BASA_HIP_CHECK_LAUNCH("diag_gather_rows_kernel(Q)");
    hipLaunchKernelGGL(diag_gather_rows_kernel, dim3(tiles, BHkv), dim3(256), 0, st, k, perm_k, Kt, tiles * kTileKeys, 1);
    BASA_HIP_CHECK_LAUNCH("diag_gather_rows_kernel(K)");
  }
  MassArgs a;
  a.Qs = Qs; a.Kt = Kt; a.perm_q = perm_q; a.base_logits = base_logits;
  a.m_hat = m_hat; a.max_dev = max_dev; a.lse = lse;
  a.Nq = ceil_div(q.L, B); a.Nk = ceil_div(k.L, B); a.Lq = q.L; a.Lk = k.L;
  a.group = q.heads / k.heads; a.rows_q = rows_q; a.tiles = tiles;
  a.scale_log2e = 1.4426950408889634f / sqrtf((float)kD);
  a.inv_sqrt_d = 1.0f / sqrtf((float)kD);
  ProfScope prof(K_BLOCK_MASS, st);
  const dim3 grid(rows_q / kQueriesPerWg, BHq);
  const bool want_dev = max_dev != nullptr && base_logits != nullptr;
  if (B == 128 && want_dev) hipLaunchKernelGGL((block_mass_kernel<128, true>), grid, dim3(256), 0, st, a);
  else if (B == 128) hipLaunchKernelGGL((block_mass_kernel<128, false>), grid, dim3(256), 0, st, a);
  else if (want_dev) hipLaunchKernelGGL((block_mass_kernel<64, true>), grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL((block_mass_kernel<64, false>), grid, dim3(256), 0, st, a);
  BASA_HIP_CHECK_LAUNCH("block_mass_kernel");
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
