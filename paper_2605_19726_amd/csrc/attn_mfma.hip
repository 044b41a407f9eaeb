// Block-sparse attention on the bf16 matrix cores of gfx950 (Sec. 2; Eq. 1; Alg. 1
// step 12), head dimension 128.
//
// Layout prepared once per call by the gather kernels below (workspace):
//   Qs [BHq ][Nq*B][128] bf16   rows of Q in sorted order, zero rows past L_q
//   Ks [BHkv][Nk*B][128] bf16   rows of K in sorted order, zero rows past L_k
//   Vt [BHkv][Nk*B/64][128][64] bf16   V in sorted order, transposed per 64-key tile
//                                      (d major), keys of every 16-group stored in the
//                                      order the MFMA B/A operand slots consume them.
//
// Main kernel: one workgroup per query block, one wave per 32 queries.  Scores are
// computed TRANSPOSED, S^T = K Q^T with v_mfma_f32_32x32x16_bf16 (A = K tile rows from
// LDS, B = Q^T held in registers), so that every lane owns ONE query: the running max,
// running sum and the rescale factor of the online softmax are per-lane scalars, the
// row max needs a single exchange between lanes l and l+32, and the exponentiated
// accumulator registers are, after packing to bf16, already the B operand of the
// second product O^T = V^T P^T (A = V^T tile rows from LDS).  K/V tiles of 64 keys are
// double-buffered in LDS: global loads of tile t+1 are in flight while tile t is used.
#include "common.hpp"

namespace basa {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kD = 128;
constexpr int kTileKeys = 64;
constexpr int kKStride = 136;   // bf16 elements per K row in LDS (256 B + 16 B pad)
constexpr int kVStride = 72;    // bf16 elements per V^T row in LDS (128 B + 16 B pad)
constexpr int kKTileElems = kTileKeys * kKStride;
constexpr int kVTileElems = kD * kVStride;
constexpr int kStageElems = kKTileElems + kVTileElems;

// Key order inside a 16-key group of Vt: the accumulator of a 32x32 MFMA holds, in lane
// half h, rows 4h+{0..3} and 8+4h+{0..3} of each 16-row group; packing those 8 values
// gives operand slot 8h+e <-> key 8*(e/4) + 4h + e%4, and Vt stores keys in slot order.

// ---------------------------------------------------------------------------------
// Gather rows of a bf16 tensor in sorted order into a dense, zero-padded buffer.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gather_rows_kernel(TensorView x, const int32_t* __restrict__ perm,
                                                          uint4* __restrict__ dst, int rows_padded) {
  const int bh = blockIdx.y;
  const int sub = threadIdx.x & 15, rig = threadIdx.x >> 4;
  const int32_t* pm = perm ? perm + (int64_t)bh * x.L : nullptr;
  const char* base = reinterpret_cast<const char*>(x.ptr) + x.head_offset(bh) * 2;
  uint4 v[4];
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int pos = blockIdx.x * 64 + it * 16 + rig;
    v[it] = make_uint4(0, 0, 0, 0);
    if (pos < x.L) {
      const int row = pm ? pm[pos] : pos;
      v[it] = reinterpret_cast<const uint4*>(base + (int64_t)row * x.stride_l * 2)[sub];
    }
  }
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int pos = blockIdx.x * 64 + it * 16 + rig;
    if (pos < rows_padded) dst[((int64_t)bh * rows_padded + pos) * 16 + sub] = v[it];
  }
}

// V: gather 64 sorted rows, transpose through LDS, write the [128][64] tile.
__global__ __launch_bounds__(256) void gather_vt_kernel(TensorView v, const int32_t* __restrict__ perm,
                                                        uint4* __restrict__ dst, int tiles_per_head) {
  __shared__ __attribute__((aligned(16))) uint16_t rows[kTileKeys][kKStride];
  const int bh = blockIdx.y, tile = blockIdx.x;
  const int sub = threadIdx.x & 15, rig = threadIdx.x >> 4;
  const int32_t* pm = perm ? perm + (int64_t)bh * v.L : nullptr;
  const char* base = reinterpret_cast<const char*>(v.ptr) + v.head_offset(bh) * 2;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int kk = it * 16 + rig;
    const int pos = tile * kTileKeys + kk;
    uint4 val = make_uint4(0, 0, 0, 0);
    if (pos < v.L) {
      const int row = pm ? pm[pos] : pos;
      val = reinterpret_cast<const uint4*>(base + (int64_t)row * v.stride_l * 2)[sub];
    }
    *reinterpret_cast<uint4*>(&rows[kk][sub * 8]) = val;
  }
  __syncthreads();
  // 1024 output chunks of 8 slots; thread handles chunk (d = id/8, s8 = id%8)
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int id = it * 256 + threadIdx.x;
    const int dd = id >> 3, s8 = id & 7;
    const int g16 = s8 >> 1, hh = s8 & 1;
    uint16_t e[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int key = 16 * g16 + 8 * (j >> 2) + 4 * hh + (j & 3);
      e[j] = rows[key][dd];
    }
    uint4 o;
    o.x = e[0] | ((uint32_t)e[1] << 16); o.y = e[2] | ((uint32_t)e[3] << 16);
    o.z = e[4] | ((uint32_t)e[5] << 16); o.w = e[6] | ((uint32_t)e[7] << 16);
    dst[(((int64_t)bh * tiles_per_head + tile) * kD + dd) * 8 + s8] = o;
  }
}

// ---------------------------------------------------------------------------------
// Main kernel.
// ---------------------------------------------------------------------------------
struct MfmaArgs {
  const uint4* Qs; const uint4* Ks; const uint4* Vt;
  const int32_t* row_count; const int32_t* row_cols; int32_t cols_stride;
  const int32_t* perm_q;
  __bf16* out; float* lse;
  int Nq, Nk, Lq, Lk, group, total_blocks;
  float scale_log2e;
};

template <int kB>
__global__ __launch_bounds__(kB * 2, 2) void attn_mfma_kernel(MfmaArgs a) {
  constexpr int NT = kB * 2;                 // threads
  constexpr int TPB = kB / kTileKeys;        // key tiles per block
  constexpr int CPT = 1024 / NT;             // 16-byte chunks per thread per tile (K and V each)
  extern __shared__ __attribute__((aligned(16))) __bf16 smem[];

  // XCD-aware order: consecutive workgroup ids go round-robin over the 8 XCDs; give each
  // XCD a contiguous range of (head, query block) so that its L2 sees one head at a time.
  int logical = blockIdx.x;
  if ((a.total_blocks & 7) == 0) logical = (blockIdx.x & 7) * (a.total_blocks >> 3) + (blockIdx.x >> 3);
  const int bhq = logical / a.Nq, gq = logical - bhq * a.Nq;
  const int bhk = bhq / a.group;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int li = lane & 31, h = lane >> 5;

  const int64_t rowid = (int64_t)bhq * a.Nq + gq;
  const int count = a.row_cols ? a.row_count[rowid] : a.Nk;
  const int32_t* cols = a.row_cols ? a.row_cols + rowid * a.cols_stride : nullptr;
  int n_iter = count * TPB;
  {
    // a ragged last key block may leave its trailing tile without any valid key
    const int last_col = cols ? cols[count - 1] : a.Nk - 1;
    if (TPB == 2 && last_col * kB + kTileKeys >= a.Lk) n_iter -= 1;
  }
  const int tiles_per_head = a.Nk * TPB;
  const uint4* Kh = a.Ks + (int64_t)bhk * tiles_per_head * 1024;
  const uint4* Vh = a.Vt + (int64_t)bhk * tiles_per_head * 1024;

  // Q^T operand: lane (query li, half h) holds Q[q][16 s + 8 h .. +7] for s = 0..7
  bf16x8 qf[8];
  {
    const int64_t qrow = ((int64_t)bhq * a.Nq + gq) * kB + wave * 32 + li;
    const uint4* qp = a.Qs + qrow * 16;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      uint4 t = qp[2 * s + h];
      qf[s] = *reinterpret_cast<bf16x8*>(&t);
    }
  }

  floatx16 o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) o[i] = floatx16{0};
  float m_run = -INFINITY, l_run = 0.f;

  auto tile_of = [&](int it) -> int {
    const int c = cols ? cols[it / TPB] : it / TPB;
    return c * TPB + (it % TPB);
  };
  // Staging registers of the tile in flight.  The prefetch is unconditional (the last
  // iteration re-fetches its own tile) so that these stay in registers.
  uint4 kreg[CPT], vreg[CPT];
  int t_cur = tile_of(0);
  {
    const uint4* kp = Kh + (int64_t)t_cur * 1024;
    const uint4* vp = Vh + (int64_t)t_cur * 1024;
#pragma unroll
    for (int i = 0; i < CPT; ++i) { kreg[i] = kp[i * NT + tid]; vreg[i] = vp[i * NT + tid]; }
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int id = i * NT + tid;
      *reinterpret_cast<uint4*>(smem + (id >> 4) * kKStride + (id & 15) * 8) = kreg[i];
      *reinterpret_cast<uint4*>(smem + kKTileElems + (id >> 3) * kVStride + (id & 7) * 8) = vreg[i];
    }
  }
  __syncthreads();

  for (int it = 0; it < n_iter; ++it) {
    const int buf = it & 1;
    const int t_next = tile_of(min(it + 1, n_iter - 1));
    {
      const uint4* kp = Kh + (int64_t)t_next * 1024;
      const uint4* vp = Vh + (int64_t)t_next * 1024;
#pragma unroll
      for (int i = 0; i < CPT; ++i) { kreg[i] = kp[i * NT + tid]; vreg[i] = vp[i * NT + tid]; }
    }
    const __bf16* ks = smem + buf * kStageElems;
    const __bf16* vs = ks + kKTileElems;

    // ---- S^T = K Q^T : two 32-key row blocks
    floatx16 s0 = {0}, s1 = {0};
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const bf16x8 k0 = *reinterpret_cast<const bf16x8*>(ks + li * kKStride + 16 * s + 8 * h);
      const bf16x8 k1 = *reinterpret_cast<const bf16x8*>(ks + (32 + li) * kKStride + 16 * s + 8 * h);
      s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0, qf[s], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1, qf[s], s1, 0, 0, 0);
    }
    // ---- mask keys past L_k (only the last tile of a ragged sequence)
    const int key0 = t_cur * kTileKeys;
    if (key0 + kTileKeys > a.Lk) {
      const int nvalid = a.Lk - key0;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int kk = 8 * (r >> 2) + 4 * h + (r & 3);
        if (kk >= nvalid) s0[r] = -INFINITY;
        if (32 + kk >= nvalid) s1[r] = -INFINITY;
      }
    }
    // ---- online softmax in the log2 domain
    float mx = s0[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s0[r]);
#pragma unroll
    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s1[r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx * a.scale_log2e);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    float psum = 0.f;
    bf16x8 pb[4];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float p0 = __builtin_amdgcn_exp2f(fmaf(s0[r], a.scale_log2e, -m_new));
      const float p1 = __builtin_amdgcn_exp2f(fmaf(s1[r], a.scale_log2e, -m_new));
      psum += p0 + p1;
      pb[r >> 3][r & 7] = (__bf16)p0;
      pb[2 + (r >> 3)][r & 7] = (__bf16)p1;
    }
    l_run = l_run * alpha + psum;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[i][r] *= alpha;

    // ---- O^T += V^T P^T
#pragma unroll
    for (int g = 0; g < 4; ++g) {         // 16-key group of the tile
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const bf16x8 vv = *reinterpret_cast<const bf16x8*>(vs + (32 * db + li) * kVStride + 16 * g + 8 * h);
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vv, pb[g], o[db], 0, 0, 0);
      }
    }
    {
      __bf16* kd = smem + (buf ^ 1) * kStageElems;
      __bf16* vd = kd + kKTileElems;
#pragma unroll
      for (int i = 0; i < CPT; ++i) {
        const int id = i * NT + tid;
        *reinterpret_cast<uint4*>(kd + (id >> 4) * kKStride + (id & 15) * 8) = kreg[i];
        *reinterpret_cast<uint4*>(vd + (id >> 3) * kVStride + (id & 7) * 8) = vreg[i];
      }
    }
    t_cur = t_next;
    __syncthreads();
  }

  // ---- epilogue: normalise, scatter rows to their original positions
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv_l = 1.0f / l_tot;
  const int pos = gq * kB + wave * 32 + li;
  if (pos < a.Lq) {
    const int orow = a.perm_q ? a.perm_q[(int64_t)bhq * a.Lq + pos] : pos;
    __bf16* op = a.out + ((int64_t)bhq * a.Lq + orow) * kD;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        bf16x4 pk;
#pragma unroll
        for (int e = 0; e < 4; ++e) pk[e] = (__bf16)(o[db][4 * r4 + e] * inv_l);
        *reinterpret_cast<bf16x4*>(op + 32 * db + 8 * r4 + 4 * h) = pk;
      }
    if (a.lse && h == 0)
      a.lse[(int64_t)bhq * a.Lq + orow] = (m_run + __log2f(l_tot)) * 0.6931471805599453f;
  }
}

size_t off_k(int BHq, int Nq, int B) { return align_up((size_t)BHq * Nq * B * kD * 2, 256); }
size_t sz_kv(int BHkv, int Nk, int B) { return align_up((size_t)BHkv * Nk * B * kD * 2, 256); }

}  // namespace

size_t attn_mfma_workspace_bytes(int BHq, int BHkv, int Lq, int Lk, int d, int B) {
  (void)d;
  const int Nq = ceil_div(Lq, B), Nk = ceil_div(Lk, B);
  return off_k(BHq, Nq, B) + 2 * sz_kv(BHkv, Nk, B);
}

basa_status launch_attn_mfma(const AttnArgs& a, hipStream_t st) {
  const int BHq = a.q.batch * a.q.heads, BHkv = a.k.batch * a.k.heads;
  const int B = a.B;
  const int Nq = ceil_div(a.q.L, B), Nk = ceil_div(a.k.L, B);
  if (BHq == 0 || Nq == 0) return BASA_OK;
  char* ws = reinterpret_cast<char*>(a.ws);
  uint4* Qs = reinterpret_cast<uint4*>(ws);
  uint4* Ks = reinterpret_cast<uint4*>(ws + off_k(BHq, Nq, B));
  uint4* Vt = reinterpret_cast<uint4*>(ws + off_k(BHq, Nq, B) + sz_kv(BHkv, Nk, B));

  {
  ProfScope prof(K_GATHER, st);
  hipLaunchKernelGGL(gather_rows_kernel, dim3(Nq * B / 64, BHq), dim3(256), 0, st, a.q, a.perm_q, Qs, Nq * B);
  BASA_HIP_CHECK_LAUNCH("gather_rows_kernel(Q)");
  hipLaunchKernelGGL(gather_rows_kernel, dim3(Nk * B / 64, BHkv), dim3(256), 0, st, a.k, a.perm_k, Ks, Nk * B);
  BASA_HIP_CHECK_LAUNCH("gather_rows_kernel(K)");
  hipLaunchKernelGGL(gather_vt_kernel, dim3(Nk * B / 64, BHkv), dim3(256), 0, st, a.v, a.perm_k, Vt, Nk * B / 64);
  BASA_HIP_CHECK_LAUNCH("gather_vt_kernel");
  }

  MfmaArgs m;
  m.Qs = Qs; m.Ks = Ks; m.Vt = Vt;
  m.row_count = a.row_count; m.row_cols = a.row_cols; m.cols_stride = a.cols_stride;
  m.perm_q = a.perm_q;
  m.out = reinterpret_cast<__bf16*>(a.out); m.lse = a.lse;
  m.Nq = Nq; m.Nk = Nk; m.Lq = a.q.L; m.Lk = a.k.L;
  m.group = a.q.heads / a.k.heads;
  m.total_blocks = BHq * Nq;
  m.scale_log2e = 1.4426950408889634f / sqrtf((float)kD);
  const size_t lds = 2 * kStageElems * sizeof(__bf16);
  ProfScope prof(K_ATTN, st);
  if (B == 128) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_mfma_kernel<128>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute");
    hipLaunchKernelGGL((attn_mfma_kernel<128>), dim3(m.total_blocks), dim3(256), lds, st, m);
  } else {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_mfma_kernel<64>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute");
    hipLaunchKernelGGL((attn_mfma_kernel<64>), dim3(m.total_blocks), dim3(128), lds, st, m);
  }
  BASA_HIP_CHECK_LAUNCH("attn_mfma_kernel");
  return BASA_OK;
}

}  // namespace basa
