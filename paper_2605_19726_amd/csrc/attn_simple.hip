// Block-sparse attention, plain fp32 arithmetic (Sec. 2; Eq. 1; Alg. 1 step 12).
// One thread owns one query of the block: its Q row and output accumulator live in
// registers, K/V rows of the kept key blocks are gathered through perm_k into LDS
// 16 keys at a time, softmax is the online (running max / running sum) form.
// This is the exact-arithmetic path for f32 tensors (bf16 tensors always take the matrix-core
// kernel); it is not tuned for speed.
#include <climits>
#include "common.hpp"

namespace basa {
namespace {

constexpr int kTK = 16;   // keys staged per step

template <bool kBf16, int kD, int kB>
__global__ __launch_bounds__(kB) void attn_simple_kernel(AttnArgs a, int Nq, int Nk, float scale) {
  constexpr int kElem = kBf16 ? 2 : 4;
  constexpr int LPR = kD * kElem / 16;
  constexpr int E = Chunk16<kBf16>::kElems;
  __shared__ __attribute__((aligned(16))) float Ks[kTK][kD];
  __shared__ __attribute__((aligned(16))) float Vs[kTK][kD];
  __shared__ int Kidx[kTK];      // original index of every staged key (causal variant)

  const int gq = blockIdx.x, bhq = blockIdx.y;
  const int group = a.q.heads / a.k.heads;
  const int bhk = bhq / group;
  const int Lq = a.q.L, Lk = a.k.L;
  const int pos = gq * kB + threadIdx.x;
  const bool active = pos < Lq;
  const int32_t* pq = a.perm_q ? a.perm_q + (int64_t)bhq * Lq : nullptr;
  const int32_t* pk = a.perm_k ? a.perm_k + (int64_t)bhk * Lk : nullptr;
  const int qrow = active ? perm_at(pq, 0, pos, Lq) : 0;
  // causal variant: keys whose original index exceeds q_lim are invisible to this query
  const int q_lim = a.causal ? qrow + a.causal_off : INT_MAX;

  float q[kD], acc[kD];
  {
    const char* qb = reinterpret_cast<const char*>(a.q.ptr) +
                     (a.q.head_offset(bhq) + (int64_t)qrow * a.q.stride_l) * kElem;
#pragma unroll
    for (int c = 0; c < LPR; ++c) {
      Chunk16<kBf16> ch;
      ch.load(qb, c);
#pragma unroll
      for (int e = 0; e < E; ++e) q[c * E + e] = ch.v[e];
    }
#pragma unroll
    for (int t = 0; t < kD; ++t) acc[t] = 0.f;
  }
  float m = -INFINITY, l = 0.f;

  const char* kbase = reinterpret_cast<const char*>(a.k.ptr) + a.k.head_offset(bhk) * kElem;
  const char* vbase = reinterpret_cast<const char*>(a.v.ptr) + a.v.head_offset(bhk) * kElem;
  const int64_t rowid = (int64_t)bhq * Nq + gq;
  const int count = a.row_cols ? min(a.row_count[rowid], a.cols_stride) : Nk;
  const int32_t* cols = a.row_cols ? a.row_cols + rowid * a.cols_stride : nullptr;

  for (int ci = 0; ci < count; ++ci) {
    const int gk = cols ? cols[ci] : ci;
    if ((unsigned)gk >= (unsigned)Nk) continue;       // not a key block: ignored (uniform over the workgroup)
    const int kstart = gk * kB;
    const int kvalid = min(kB, Lk - kstart);
    for (int t0 = 0; t0 < kvalid; t0 += kTK) {
      const int nk = min(kTK, kvalid - t0);
      __syncthreads();
      for (int w = threadIdx.x; w < 2 * kTK * LPR; w += kB) {
        const int which = w / (kTK * LPR);
        const int rem = w - which * (kTK * LPR);
        const int j = rem / LPR, c = rem - j * LPR;
        Chunk16<kBf16> ch;
        if (j < nk) {
          const int kp = kstart + t0 + j;
          const int krow = perm_at(pk, 0, kp, Lk);
          const char* src = which ? vbase + (int64_t)krow * a.v.stride_l * kElem
                                  : kbase + (int64_t)krow * a.k.stride_l * kElem;
          ch.load(src, c);
        } else {
          ch.zero();
        }
        float* dst = which ? &Vs[j][c * E] : &Ks[j][c * E];
#pragma unroll
        for (int e = 0; e < E; ++e) dst[e] = ch.v[e];
        if (which == 0 && c == 0) Kidx[j] = j < nk ? perm_at(pk, 0, kstart + t0 + j, Lk) : INT_MAX;
      }
      __syncthreads();
      float s[kTK];
      float tmax = -INFINITY;
#pragma unroll
      for (int j = 0; j < kTK; ++j) {
        float d0 = 0.f;
#pragma unroll
        for (int t = 0; t < kD; t += 4) {
          const float4 kv = *reinterpret_cast<const float4*>(&Ks[j][t]);
          d0 = fmaf(q[t], kv.x, d0); d0 = fmaf(q[t + 1], kv.y, d0);
          d0 = fmaf(q[t + 2], kv.z, d0); d0 = fmaf(q[t + 3], kv.w, d0);
        }
        s[j] = (j < nk && Kidx[j] <= q_lim) ? d0 * scale : -INFINITY;
        tmax = fmaxf(tmax, s[j]);
      }
      const float m_new = fmaxf(m, tmax);
      // (nothing visible so far: subtract 0 instead of -inf, so that exp sees -inf and never inf - inf)
      const float m_sub = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = expf(m - m_sub);      // m = -inf on the first step gives 0
      l *= alpha;
#pragma unroll
      for (int t = 0; t < kD; ++t) acc[t] *= alpha;
#pragma unroll
      for (int j = 0; j < kTK; ++j) {
        const float p = expf(s[j] - m_sub);     // masked keys: exp(-inf) = 0
        l += p;
#pragma unroll
        for (int t = 0; t < kD; t += 4) {
          const float4 vv = *reinterpret_cast<const float4*>(&Vs[j][t]);
          acc[t] = fmaf(p, vv.x, acc[t]); acc[t + 1] = fmaf(p, vv.y, acc[t + 1]);
          acc[t + 2] = fmaf(p, vv.z, acc[t + 2]); acc[t + 3] = fmaf(p, vv.w, acc[t + 3]);
        }
      }
      m = m_new;
    }
  }
  if (!active) return;
  const float inv_l = l > 0.f ? 1.0f / l : 0.f;       // a row without any valid key block: zeros
  const int64_t orow = (int64_t)bhq * Lq + qrow;
  const int64_t ooff = a.out_offset(bhq, qrow);
  if constexpr (kBf16) {
    __bf16* o = reinterpret_cast<__bf16*>(a.out) + ooff;
#pragma unroll
    for (int t = 0; t < kD; ++t) o[t] = (__bf16)(acc[t] * inv_l);
  } else {
    float4* o = reinterpret_cast<float4*>(reinterpret_cast<float*>(a.out) + ooff);
#pragma unroll
    for (int t = 0; t < kD; t += 4)
      o[t / 4] = make_float4(acc[t] * inv_l, acc[t + 1] * inv_l, acc[t + 2] * inv_l, acc[t + 3] * inv_l);
  }
  if (a.lse) a.lse[orow] = m + logf(l);
}

}  // namespace

basa_status launch_attn_simple(const AttnArgs& a, hipStream_t st) {
  const int BHq = a.q.batch * a.q.heads;
  const int Nq = ceil_div(a.q.L, a.B), Nk = ceil_div(a.k.L, a.B);
  if (BHq == 0 || Nq == 0) return BASA_OK;
  const float scale = 1.0f / sqrtf((float)a.q.d);
  dim3 grid(Nq, BHq);
  ProfScope prof(K_ATTN_SIMPLE, st);
  const bool bf = a.q.dtype == BASA_BF16;
#define BASA_AS(BF, D, BB) \
  hipLaunchKernelGGL((attn_simple_kernel<BF, D, BB>), grid, dim3(BB), 0, st, a, Nq, Nk, scale)
  if (bf && a.q.d == 128 && a.B == 128) BASA_AS(true, 128, 128);
  else if (bf && a.q.d == 128 && a.B == 64) BASA_AS(true, 128, 64);
  else if (bf && a.q.d == 64 && a.B == 128) BASA_AS(true, 64, 128);
  else if (bf && a.q.d == 64 && a.B == 64) BASA_AS(true, 64, 64);
  else if (!bf && a.q.d == 128 && a.B == 128) BASA_AS(false, 128, 128);
  else if (!bf && a.q.d == 128 && a.B == 64) BASA_AS(false, 128, 64);
  else if (!bf && a.q.d == 64 && a.B == 128) BASA_AS(false, 64, 128);
  else BASA_AS(false, 64, 64);
#undef BASA_AS
  BASA_HIP_CHECK_LAUNCH("attn_simple_kernel");
  return BASA_OK;
}

}  // namespace basa
