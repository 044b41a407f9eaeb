// Block-sparse attention on the bf16 matrix cores of gfx950 (Sec. 2; Eq. 1; Alg. 1
// step 12), head dimension D = 128 (the shapes below) or 64 (rows, tiles and accumulators
// half as large: 8 chunks per row, K swizzle by row & 7, 8 KB tiles).
//
// Layout prepared once per call by the gather kernels below (workspace).  K and V are
// stored as 64-key tiles that are byte-for-byte the LDS image the main kernel wants, so
// the global -> LDS copy is a linear 16 KB copy done with direct-to-LDS loads:
//   (Q needs no copy: every wave reads the rows of its 32 queries once, through perm_q)
//   Kt [BHkv][tiles][64 rows][16 chunks of 8 bf16]   rows of K in sorted order; chunk c
//        of row r sits at chunk position c ^ (r & 15)                (XOR swizzle)
//   Vt [BHkv][tiles][128 d-rows][8 chunks of 8 keys] V in sorted order, transposed per
//        tile (d major); the 8 keys of a chunk are in MFMA operand-slot order (below);
//        chunk c of d-row r sits at chunk position c ^ ((r >> 1) & 7)
// The swizzles make every ds_read_b128 of 16 consecutive lanes hit 16 distinct 16-byte
// bank groups.
//
// Main kernel: one workgroup of 8 waves owns 256 consecutive sorted queries, i.e. 2 query
// blocks of 128 (4 of 64), one wave per 32 queries.  Streaming K/V tiles from L2 into LDS is
// the costly part beside the MFMAs themselves (with 128 queries per tile fetch the kernel was
// 12 % slower: 8 TB/s of L2 -> LDS traffic), so the query blocks of a workgroup share every tile,
// and 256 queries are what the register file holds (64 accumulator registers per 32 queries,
// two waves per SIMD): the workgroup walks the UNION
// of their block lists in ascending order, each tile is fetched once, and only the waves
// whose query block lists the tile's key block compute on it.  Scores are computed
// TRANSPOSED, S^T = K Q^T with v_mfma_f32_32x32x16_bf16 (A = K tile rows from
// LDS, B = Q^T held in registers), so that every lane owns ONE query: the running max,
// running sum and the rescale factor of the online softmax are per-lane scalars, the
// row max needs a single exchange between lanes l and l+32, and the exponentiated
// accumulator registers are, after packing to bf16, already the B operand of the
// second product O^T = V^T P^T (A = V^T tile rows from LDS).
// The accumulator of a 32x32 MFMA holds, in lane half h, rows 4h+{0..3} and 8+4h+{0..3}
// of each 16-row group; packing those 8 values gives operand slot 8h+e <-> key
// 8*(e/4) + 4h + e%4 of the group, which is the key order inside a Vt chunk pair.
// The running max is refreshed lazily: the accumulators are rescaled only when some
// query's tile max exceeds its running max by more than 2^8, so the common iteration
// touches O only through MFMA.  K/V tiles go through a 4-stage LDS ring used as two slots of
// two tiles: one pair is computed while the next pair lands; one workgroup barrier per pair.
#include <algorithm>
#include <climits>
#include <type_traits>
#include "common.hpp"

namespace basa {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kTileKeys = 64;
constexpr int kIxStride = kTileKeys + 4;    // causal: ints per tile of the key-index array (64 indices, min, max, 2 unused)
#ifndef BASA_ATTN_QR
#define BASA_ATTN_QR 7
#endif
constexpr float kLazyTau = 8.0f;            // log2 of the largest exponentiated score kept
// The pass without running maxima (64 queries per wave): a query's reference moves up by kShiftLog2
// once the probabilities of half a tile add up to more than kSafeSum; a row whose final sum lies
// outside [kMinSum, kMaxSum] (or is not a number) has left the range in which that pass is exact.
constexpr float kSafeSum = 1.0995116e12f;   // 2^40
constexpr float kShiftLog2 = 40.0f;
constexpr float kShiftMul = 9.094947e-13f;  // 2^-40
constexpr float kMinSum = 8.6736174e-19f;   // 2^-60
constexpr float kMaxSum = 1.2676506e30f;    // 2^100
// Two shapes of workgroup.  SHARED: 8 waves own 256 queries = two (four) neighbouring query blocks
// that share every K/V tile; best when their lists overlap, which they do for the full method.
// SOLO: 4 waves own 128 queries = one query block of 128 (two of 64), two workgroups per compute
// unit; every tile is fetched per 128 queries, but no wave ever waits for a tile that only its
// neighbour lists - best when neighbouring lists have little in common.
constexpr int kSharedQueries = 256, kSoloQueries = 128, kWideQueries = 512;
#ifndef BASA_ATTN_DEFAULT_LISTS
#define BASA_ATTN_DEFAULT_LISTS 3      // shape taken for block lists the overlap probe does not cover
#endif

// Sizes that follow from the head dimension D.
template <int D>
struct Geo {
  static constexpr int kRowBytes = D * 2;                    // one row of Q or K
  static constexpr int kChunksPerRow = kRowBytes / 16;       // 16-byte chunks per row: 16 or 8
  static constexpr int kTileBytes = kTileKeys * kRowBytes;   // one K tile; a V^T tile (D rows of 128 B) is as large
  static constexpr int kStageBytes = 2 * kTileBytes;         // K tile then V^T tile
  static constexpr int kKSteps = D / 16;                     // MFMA k-steps of S^T = K Q^T
  static constexpr int kDBlocks = D / 32;                    // 32-row blocks of O^T
  static constexpr int kChunksPerTile = kTileBytes / 1024;   // 1 KB direct-to-LDS loads per K (or V^T) tile
};
// Ring stages of a workgroup: one of 512 threads has the compute unit to itself and walks tiles in
// pairs (two slots of two); two workgroups of 256 threads share a compute unit and walk one by one.
// With 64 queries per wave a tile keeps the workgroup busy twice as long, and one tile of prefetch
// distance (two stages) covers the load.
#ifndef BASA_ATTN_ST64
#define BASA_ATTN_ST64 2
#endif
constexpr int stages_of(int threads, int qpw) { return threads == 512 ? (qpw == 32 ? 4 : BASA_ATTN_ST64) : 2; }
// k-steps of Q^T a wave of 64 queries keeps in registers (the rest is parked in LDS): all for D = 64
// (the causal variant of the 64-queries-per-wave kernel carries the two visibility limits and the
//  key indices of the half-tile on top: one more k-step of Q^T is parked)
// (the pass without running maxima needs no registers for them and keeps all of Q^T, 117.6-119.1 ms
//  against 119.7-120.5 with one k-step parked; its causal variant does better with two parked as before:
//  139-140 ms against 147 with one)
#ifndef BASA_ATTN_QR_FAST
#define BASA_ATTN_QR_FAST 8
#endif
constexpr int q_reg_steps(int d, int qpw, bool causal = false, bool fast = false) {
  return (qpw == 64 && d == 128) ? (fast && !causal ? BASA_ATTN_QR_FAST : BASA_ATTN_QR - (causal ? 1 : 0)) : d / 16;
}

// ---------------------------------------------------------------------------------
// Gather kernels
// ---------------------------------------------------------------------------------
// Rows of a bf16 tensor in sorted order, zero-padded; swizzle = 1 writes K-tile order.
template <int D>
__global__ __launch_bounds__(256) void gather_rows_kernel(TensorView x, const int32_t* __restrict__ perm,
                                                          uint4* __restrict__ dst, int rows_padded,
                                                          int swizzle) {
  constexpr int CPR = Geo<D>::kChunksPerRow, RPI = 256 / CPR, ITERS = 64 / RPI;
  const int bh = blockIdx.y;
  const int sub = threadIdx.x % CPR, rig = threadIdx.x / CPR;
  const int32_t* pm = perm ? perm + (int64_t)bh * x.L : nullptr;
  const char* base = reinterpret_cast<const char*>(x.ptr) + x.head_offset(bh) * 2;
  uint4 v[ITERS];
  gather_chunks<ITERS>(v, pm, base, x.L, (int64_t)x.stride_l * 2, blockIdx.x * 64 + rig, RPI, sub);
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int pos = blockIdx.x * 64 + it * RPI + rig;
    const int c = swizzle ? (sub ^ (pos & (CPR - 1))) : sub;
    if (pos < rows_padded) dst[((int64_t)bh * rows_padded + pos) * CPR + c] = v[it];
  }
}

// V: gather 64 sorted rows, transpose through LDS, write the swizzled [D][64] tile.
template <int D>
__global__ __launch_bounds__(256) void gather_vt_kernel(TensorView v, const int32_t* __restrict__ perm,
                                                        uint4* __restrict__ dst, int tiles_per_head) {
  constexpr int CPR = Geo<D>::kChunksPerRow, RPI = 256 / CPR, ITERS = 64 / RPI;
  constexpr int kRowStride = D + 8;   // one row + 16 B pad
  __shared__ __attribute__((aligned(16))) uint16_t rows[kTileKeys][kRowStride];
  const int bh = blockIdx.y, tile = blockIdx.x;
  const int sub = threadIdx.x % CPR, rig = threadIdx.x / CPR;
  const int32_t* pm = perm ? perm + (int64_t)bh * v.L : nullptr;
  const char* base = reinterpret_cast<const char*>(v.ptr) + v.head_offset(bh) * 2;
  uint4 val[ITERS];
  gather_chunks<ITERS>(val, pm, base, v.L, (int64_t)v.stride_l * 2, tile * kTileKeys + rig, RPI, sub);
#pragma unroll
  for (int it = 0; it < ITERS; ++it) *reinterpret_cast<uint4*>(&rows[it * RPI + rig][sub * 8]) = val[it];
  __syncthreads();
  // 8 D output chunks of 8 slots; thread handles chunk (d = id/8, s8 = id%8):
  // 16-key group g16 = s8/2, lane half hh = s8%2, slot e <-> key 16 g16 + 8(e/4) + 4 hh + e%4
#pragma unroll
  for (int it = 0; it < D * 8 / 256; ++it) {
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
    dst[(((int64_t)bh * tiles_per_head + tile) * D + dd) * 8 + (s8 ^ ((dd >> 1) & 7))] = o;
  }
}

// ---------------------------------------------------------------------------------
// Main kernel
// ---------------------------------------------------------------------------------
struct MfmaArgs {
  TensorView q; const char* Kt; const char* Vt;
  const int32_t* row_count; const int32_t* row_cols; int32_t cols_stride;
  const int32_t* perm_q;
  __bf16* out; float* lse;
  int Nq, Nk, Lq, Lk, group, wgs_per_head, total_wgs;
  float scale_log2e;
  int64_t out_sb, out_sh, out_sl;   // strides of out in elements
  int heads_q;
  const int32_t* kix;        // causal: [BHkv][tiles][kIxStride] original key indices of a tile, then their min and max
  int causal_off;            // causal: L_k - L_q
  const int32_t* probe;      // nullable: {blocks in the union of a group's lists, blocks in its lists} over sampled groups
  int run_if_solo;           // with probe: this launch runs iff (lists overlap little) == run_if_solo
  int32_t* redo;             // nullable, one word per workgroup: written by the pass without running maxima (1 = a row
                             // sum left the safe range), read by the pass with them, which skips workgroups at 0
};

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* gbl_ptr_t;

// Per-wave state of the online softmax and the output accumulator.
template <int D>
struct WaveState {
  floatx16 o[Geo<D>::kDBlocks];
  float m_run, l_run;
};

// max of three floats; this file is compiled with -fno-honor-nans (scores are finite or
// -inf), so no NaN canonicalisation is emitted and this becomes one v_max3_f32.
__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

// One 64-key tile: S^T, softmax, O^T update, reading the LDS stage at `stage`.  kMasked:
// keys at tile positions >= nvalid do not exist (ragged end of the sequence) and get -inf.
template <bool kMasked, int D>
__device__ __forceinline__ void process_tile(WaveState<D>& st, const bf16x8 (&qf)[Geo<D>::kKSteps], const char* stage,
                                             int kaddr0, int vaddr0, float c, int nvalid, int h) {
  const char* ks = stage;
  const char* vs = stage + Geo<D>::kTileBytes;

  // ---- S^T = K Q^T : two 32-key row blocks
  floatx16 s0 = {0}, s1 = {0};
#pragma unroll
  for (int s = 0; s < Geo<D>::kKSteps; ++s) {
    const int ka = kaddr0 ^ (s << 5);     // chunk 2s+h of row li at position (2s+h) ^ (li & (chunks per row - 1))
    const bf16x8 k0 = *reinterpret_cast<const bf16x8*>(ks + ka);
    const bf16x8 k1 = *reinterpret_cast<const bf16x8*>(ks + ka + 32 * Geo<D>::kRowBytes);
    s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0, qf[s], s0, 0, 0, 0);
    s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1, qf[s], s1, 0, 0, 0);
  }
  if (kMasked && nvalid < kTileKeys) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int kk = 8 * (r >> 2) + 4 * h + (r & 3);
      if (kk >= nvalid) s0[r] = -INFINITY;
      if (32 + kk >= nvalid) s1[r] = -INFINITY;
    }
  }
  // ---- online softmax in the log2 domain, lazy running max
  float mx = max3(s0[0], s1[0], s0[1]);
#pragma unroll
  for (int r = 1; r < 15; ++r) mx = max3(mx, s1[r], s0[r + 1]);
  mx = max3(mx, s1[15], __shfl_xor(max3(mx, s1[15], s1[15]), 32));
  const float mc = mx * c;
  if (__builtin_amdgcn_ballot_w64(mc > st.m_run + kLazyTau) != 0) {
    const float m_new = fmaxf(st.m_run, mc);
    const float alpha = __builtin_amdgcn_exp2f(st.m_run - m_new);
    st.m_run = m_new;
    st.l_run *= alpha;
#pragma unroll
    for (int i = 0; i < Geo<D>::kDBlocks; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.o[i][r] *= alpha;
  }
  const float m_use = st.m_run;
  bf16x8 pb[4];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    pb[r >> 3][r & 7] = (__bf16)__builtin_amdgcn_exp2f(fmaf(s0[r], c, -m_use));
    pb[2 + (r >> 3)][r & 7] = (__bf16)__builtin_amdgcn_exp2f(fmaf(s1[r], c, -m_use));
  }
  // row sum of the bf16-rounded probabilities (the values the second product consumes)
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
  float lsum = st.l_run;
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    lsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pb[g], pb[g], 0, 1), ones, lsum, false);
    lsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pb[g], pb[g], 2, 3), ones, lsum, false);
    lsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pb[g], pb[g], 4, 5), ones, lsum, false);
    lsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pb[g], pb[g], 6, 7), ones, lsum, false);
  }
  st.l_run = lsum;

  // ---- O^T += V^T P^T
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    const int va = vaddr0 ^ (g << 5);     // chunk 2g+h of d-row li at position (2g+h) ^ ((li>>1)&7)
#pragma unroll
    for (int db = 0; db < Geo<D>::kDBlocks; ++db) {
      const bf16x8 vv = *reinterpret_cast<const bf16x8*>(vs + va + db * 32 * 128);
      st.o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vv, pb[g], st.o[db], 0, 0, 0);
    }
  }
}

// LDS byte address of a pointer into the workgroup's shared memory, and a 16-byte fragment read at one.
typedef const __attribute__((address_space(3))) char* lds_cptr_t;
typedef const __attribute__((address_space(3))) bf16x8* lds_frag_ptr_t;
__device__ __forceinline__ uint32_t lds_addr(const char* p) { return (uint32_t)(uintptr_t)(lds_cptr_t)p; }
__device__ __forceinline__ bf16x8 lds_frag(uint32_t addr) { return *(lds_frag_ptr_t)(uintptr_t)addr; }

// Two query groups per wave (64 queries): the same arithmetic per query, but every K and V^T
// fragment read from LDS feeds two MFMAs (one per group), and the 64-key tile is walked as two
// 32-key halves so that only 32 score registers per group pair are live at a time.
template <int D>
struct WaveState2 {
  floatx16 o[2][Geo<D>::kDBlocks];
  float m_run[2], l_run[2];
  float lt[2];               // kFast: the row sums of the half tile before this one
};

// kQR of the k-steps take their Q^T fragments from registers; the others are read back from the
// wave's lane-private LDS area at `qs` ([group 2][k-step][lane] 16 bytes): O (128 registers) and all
// of Q (64) would leave the compiler too few of the 256 registers a wave has at two waves per SIMD.
// kCausal: kix4 points at the lane's four key indices of the tile's first group of eight keys
// (original positions, INT_MAX past the end of the sequence, which also covers the ragged tile); a
// key is visible to the query of group a / b iff its index does not exceed qla / qlb.
// kFast: no maximum is taken.  The reference m of a query only has to keep 2^(c s - m) inside the
// range of the formats (bf16 and fp32 share their exponent), it need not be the maximum: it starts at
// 0 and is raised by kShiftLog2 whenever the row sums of the half tile before, which are needed
// anyway, exceed kSafeSum.  The caller checks the final sums (kMinSum, kMaxSum) and has the rows
// computed again with running maxima if a sum has left the safe range.  Taking the maximum of every
// half tile (16 v_max3, two lane exchanges, and the wait of every exponential for the last score)
// was a quarter of the vector instructions of a tile.
template <bool kMasked, int D, int kQR, bool kCausal = false, bool kFast = false>
__device__ __forceinline__ void process_tile2(WaveState2<D>& st, const bf16x8 (&qa)[kQR], const bf16x8 (&qb)[kQR],
                                              const char* qs, const char* stage, int kaddr0, int vaddr0, float c,
                                              int nvalid, int h, const int* kix4 = nullptr, int qla = 0, int qlb = 0) {
  constexpr int kQL = Geo<D>::kKSteps - kQR;               // k-steps whose Q^T fragments live in LDS
  // One LDS address per operand and tile; the k-step (group) is folded in by an xor at the point of
  // use (ring stages start at multiples of 32 KB, so the xor of bits 5-8 commutes with adding the
  // stage).  The two bases are opaque to the compiler, which would otherwise keep all twelve xor-ed
  // addresses in registers for the whole kernel and add the stage offset to each in every tile.
  uint32_t kbase = lds_addr(stage) + (uint32_t)kaddr0;
  uint32_t vbase = lds_addr(stage) + (uint32_t)(Geo<D>::kTileBytes + vaddr0);
  asm volatile("" : "+v"(kbase), "+v"(vbase));
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    if (kMasked && half == 1 && nvalid <= 32) break;        // wave-uniform: no key in the second half
    // the parked fragments are read again in every half: kept in registers across the halves they
    // would cost the 16 registers that parking them is meant to free
    asm volatile("" ::: "memory");
    floatx16 sa = {0}, sb = {0};
#pragma unroll
    for (int s = 0; s < Geo<D>::kKSteps; ++s) {
      const bf16x8 kf = lds_frag((kbase ^ (uint32_t)(s << 5)) + half * 32 * Geo<D>::kRowBytes);
      if (s < kQR) {
        sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qa[s < kQR ? s : 0], sa, 0, 0, 0);
        sb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qb[s < kQR ? s : 0], sb, 0, 0, 0);
      } else {
        const bf16x8 fa = *reinterpret_cast<const bf16x8*>(qs + (s - kQR) * 1024);
        const bf16x8 fb = *reinterpret_cast<const bf16x8*>(qs + (kQL + s - kQR) * 1024);
        sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, fa, sa, 0, 0, 0);
        sb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, fb, sb, 0, 0, 0);
      }
    }
    if (!kCausal && kMasked && nvalid < kTileKeys) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int kk = 32 * half + 8 * (r >> 2) + 4 * h + (r & 3);
        if (kk >= nvalid) { sa[r] = -INFINITY; sb[r] = -INFINITY; }
      }
    }
    if constexpr (kCausal) {
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int4 ix = *reinterpret_cast<const int4*>(kix4 + 32 * half + 8 * g4);
        const int ia[4] = {ix.x, ix.y, ix.z, ix.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (ia[e] > qla) sa[4 * g4 + e] = -INFINITY;
          if (ia[e] > qlb) sb[4 * g4 + e] = -INFINITY;
        }
      }
    }
    if constexpr (kFast) {
      if (__builtin_amdgcn_ballot_w64(st.lt[0] > kSafeSum || st.lt[1] > kSafeSum) != 0) {
        // a query's keys are split over two lanes (lane halves), which must move its reference together
        // (the exchanges first, by every lane: inside a short-circuit `||` only the lanes that still have
        //  to ask would be active, and a lane exchange reads 0 from an inactive lane)
        const float other_a = __shfl_xor(st.lt[0], 32), other_b = __shfl_xor(st.lt[1], 32);
        const bool ua = (st.lt[0] > kSafeSum) | (other_a > kSafeSum);
        const bool ub = (st.lt[1] > kSafeSum) | (other_b > kSafeSum);
        const float aa = ua ? kShiftMul : 1.f, ab = ub ? kShiftMul : 1.f;
        st.m_run[0] += ua ? kShiftLog2 : 0.f; st.m_run[1] += ub ? kShiftLog2 : 0.f;
        st.l_run[0] *= aa; st.l_run[1] *= ab;
#pragma unroll
        for (int i = 0; i < Geo<D>::kDBlocks; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) { st.o[0][i][r] *= aa; st.o[1][i][r] *= ab; }
      }
    } else {
      float mxa = max3(sa[0], sa[1], sa[2]), mxb = max3(sb[0], sb[1], sb[2]);
#pragma unroll
      for (int r = 3; r < 15; r += 2) { mxa = max3(mxa, sa[r], sa[r + 1]); mxb = max3(mxb, sb[r], sb[r + 1]); }
      mxa = fmaxf(mxa, sa[15]); mxb = fmaxf(mxb, sb[15]);
      // (exchanging the halves with v_permlane32_swap instead of the LDS permute measured 1 % slower)
      mxa = fmaxf(mxa, __shfl_xor(mxa, 32)); mxb = fmaxf(mxb, __shfl_xor(mxb, 32));
      const float mca = mxa * c, mcb = mxb * c;
      if (__builtin_amdgcn_ballot_w64(mca > st.m_run[0] + kLazyTau || mcb > st.m_run[1] + kLazyTau) != 0) {
        const float na = fmaxf(st.m_run[0], mca), nb = fmaxf(st.m_run[1], mcb);
        // (causal: a query that still sees nothing has -inf on both sides; its state stays as it is)
        const float aa = (kCausal && na == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(st.m_run[0] - na);
        const float ab = (kCausal && nb == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(st.m_run[1] - nb);
        st.m_run[0] = na; st.m_run[1] = nb;
        st.l_run[0] *= aa; st.l_run[1] *= ab;
#pragma unroll
        for (int i = 0; i < Geo<D>::kDBlocks; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) { st.o[0][i][r] *= aa; st.o[1][i][r] *= ab; }
      }
    }
    // (causal: a query that has seen no key yet subtracts 0, so that exp2 sees -inf, never inf - inf)
    const float ma = (!kFast && kCausal && st.m_run[0] == -INFINITY) ? 0.f : st.m_run[0];
    const float mb = (!kFast && kCausal && st.m_run[1] == -INFINITY) ? 0.f : st.m_run[1];
    bf16x8 pa[2], pb[2];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      pa[r >> 3][r & 7] = (__bf16)__builtin_amdgcn_exp2f(fmaf(sa[r], c, -ma));
      pb[r >> 3][r & 7] = (__bf16)__builtin_amdgcn_exp2f(fmaf(sb[r], c, -mb));
    }
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    float la = kFast ? 0.f : st.l_run[0], lb = kFast ? 0.f : st.l_run[1];
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      la = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pa[g], pa[g], 0, 1), ones, la, false);
      la = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pa[g], pa[g], 2, 3), ones, la, false);
      la = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pa[g], pa[g], 4, 5), ones, la, false);
      la = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pa[g], pa[g], 6, 7), ones, la, false);
      lb = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pb[g], pb[g], 0, 1), ones, lb, false);
      lb = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pb[g], pb[g], 2, 3), ones, lb, false);
      lb = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pb[g], pb[g], 4, 5), ones, lb, false);
      lb = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pb[g], pb[g], 6, 7), ones, lb, false);
    }
    if constexpr (kFast) {
      st.l_run[0] += la; st.l_run[1] += lb;
      st.lt[0] = la; st.lt[1] = lb;
    } else {
      st.l_run[0] = la; st.l_run[1] = lb;
    }
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      const uint32_t va = vbase ^ (uint32_t)((2 * half + g) << 5);
#pragma unroll
      for (int db = 0; db < Geo<D>::kDBlocks; ++db) {
        const bf16x8 vv = lds_frag(va + db * 32 * 128);
        st.o[0][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vv, pa[g], st.o[0][db], 0, 0, 0);
        st.o[1][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vv, pb[g], st.o[1][db], 0, 0, 0);
      }
    }
  }
}

// State of a wave by number of query groups, with uniform accessors for prologue and epilogue.
template <int D, int NG> struct StateOf { typedef WaveState<D> type; };
template <int D> struct StateOf<D, 2> { typedef WaveState2<D> type; };
template <int D>
__device__ __forceinline__ void init_state(WaveState<D>& st, bool = false) {
#pragma unroll
  for (int i = 0; i < Geo<D>::kDBlocks; ++i) st.o[i] = floatx16{0};
  st.m_run = -INFINITY;
  st.l_run = 0.f;
}
template <int D>
__device__ __forceinline__ void init_state(WaveState2<D>& st, bool fast = false) {
#pragma unroll
  for (int r = 0; r < 2; ++r) {
#pragma unroll
    for (int i = 0; i < Geo<D>::kDBlocks; ++i) st.o[r][i] = floatx16{0};
    st.m_run[r] = fast ? 0.f : -INFINITY;
    st.l_run[r] = 0.f;
    st.lt[r] = 0.f;
  }
}
template <int D> __device__ __forceinline__ float l_of(const WaveState<D>& st, int) { return st.l_run; }
template <int D> __device__ __forceinline__ float m_of(const WaveState<D>& st, int) { return st.m_run; }
template <int D> __device__ __forceinline__ const floatx16& o_of(const WaveState<D>& st, int, int db) { return st.o[db]; }
template <int D> __device__ __forceinline__ float l_of(const WaveState2<D>& st, int r) { return st.l_run[r]; }
template <int D> __device__ __forceinline__ float m_of(const WaveState2<D>& st, int r) { return st.m_run[r]; }
template <int D> __device__ __forceinline__ const floatx16& o_of(const WaveState2<D>& st, int r, int db) { return st.o[r][db]; }

__device__ __forceinline__ int64_t out_off(const MfmaArgs& a, int bhq, int row) {
  const int b = bhq / a.heads_q, hh = bhq - b * a.heads_q;
  return (int64_t)b * a.out_sb + (int64_t)hh * a.out_sh + (int64_t)row * a.out_sl;
}

// Dynamic LDS: [ring: kStages x 32 KB][parked Q^T fragments][seq: Nk words][wave_counts: kWaves words].
// seq[i] = key block of the i-th entry of the union list | (bit 24+g set iff query block g of
// this workgroup lists it).  While seq is being built the ring area holds the per-key-block
// membership flags.
// kCausal (512-query shape only): the ring is followed by the original key indices of each stage's
// tile (with their minimum), every score is masked by original position, and a wave skips a tile
// none of whose keys is visible to any of its queries.
template <int kB, int D, int kWgQueries, int kQPW, bool kCausal = false, bool kFast = false>
__global__ __launch_bounds__(kWgQueries / kQPW * 64, kWgQueries / kQPW == 8 ? 1 : 2) void attn_mfma_kernel(MfmaArgs a) {
  using G = Geo<D>;
  static_assert(!kCausal || (kQPW == 64 && kWgQueries == kWideQueries), "the causal path is built on the 512-query shape");
  static_assert(!kFast || (kQPW == 64 && kWgQueries == kWideQueries), "the pass without running maxima is built on the 512-query shape");
  constexpr int kWaves = kWgQueries / kQPW, kThreads = kWaves * 64, kQueriesPerWg = kWgQueries;
  constexpr int kNG = kQPW / 32;             // 32-query groups per wave: 1 or 2
  constexpr int kStages = stages_of(kThreads, kQPW);
  constexpr int kQR = q_reg_steps(D, kQPW, kCausal, kFast), kQL = G::kKSteps - kQR;
  constexpr int kQParkBytes = kWaves * kNG * kQL * 1024;
  constexpr int kTileBytes = G::kTileBytes, kStageBytes = G::kStageBytes, kRingBytes = kStages * kStageBytes;
  constexpr int kLoadsPerWave = 2 * G::kChunksPerTile / kWaves;
  constexpr int NQB = kQueriesPerWg / kB;    // query blocks per workgroup: 2 or 4 (SOLO: 1 or 2)
  if (a.probe) {
    // the other shape of workgroup is launched too; exactly one of the two does the work.  A
    // 512-query workgroup walks the union of its 512 / B lists; four 128-query ones walk the
    // unions of their own 128 / B lists.  Measured break-even (wide 26.4 against 27.1 ms at a
    // ratio of 1.29, 157.7 against 143.6 ms at 1.64): the narrow shape wins once the wide union
    // exceeds about 1.35 times the average narrow one.
    const int uni = a.probe[0], uni_sub = a.probe[1];
    const bool little_overlap = 100 * (int64_t)uni * 4 > 135 * (int64_t)uni_sub;
    if ((int)little_overlap != a.run_if_solo) return;
  }
  constexpr int TPB = kB / kTileKeys;        // key tiles per key block: 2 or 1
  extern __shared__ __attribute__((aligned(16))) char smem[];
  uint32_t* flags = reinterpret_cast<uint32_t*>(smem);
  uint32_t* seq = reinterpret_cast<uint32_t*>(smem + kRingBytes + kQParkBytes);
  uint32_t* wave_counts = seq + a.Nk;
  int* kix_lds = reinterpret_cast<int*>(smem + ((kRingBytes + kQParkBytes + a.Nk * 4 + kWaves * 4 + 15) & ~15));   // kCausal

  // XCD-aware order: consecutive workgroup ids go round-robin over the 8 XCDs; give each
  // XCD a contiguous range of (head, query blocks) so that its L2 sees one head at a time.
  int logical = blockIdx.x;
  if ((a.total_wgs & 7) == 0) logical = (blockIdx.x & 7) * (a.total_wgs >> 3) + (blockIdx.x >> 3);
  // the pass with running maxima, launched behind the one without: only the workgroups that one gave up on
  if (!kFast && a.redo && a.redo[logical] == 0) return;
  const int bhq = logical / a.wgs_per_head, wg = logical - bhq * a.wgs_per_head;
  const int bhk = bhq / a.group;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 31, h = lane >> 5;
  const int grp = wave * kQPW / kB;                    // query block of this wave inside the wg
  const int nqb = min(NQB, a.Nq - wg * NQB);           // query blocks that exist
  const int pos0 = wg * kQueriesPerWg + wave * kQPW + li;   // sorted position of this lane's first query (next: +32)

  // ---- union of the block lists of this workgroup's query blocks ------------------------
  for (int c = tid; c < a.Nk; c += kThreads) flags[c] = a.row_cols ? 0u : ((1u << nqb) - 1u);
  __syncthreads();
  if (a.row_cols) {
    for (int g = 0; g < nqb; ++g) {
      const int64_t rowid = (int64_t)bhq * a.Nq + wg * NQB + g;
      const int cnt = min(a.row_count[rowid], a.cols_stride);
      const int32_t* cl = a.row_cols + rowid * a.cols_stride;
      for (int i = tid; i < cnt; i += kThreads) {
        const int col = cl[i];
        if ((unsigned)col < (unsigned)a.Nk) atomicOr(&flags[col], 1u << g);     // anything else is ignored
      }
    }
    __syncthreads();
  }
  int n_union = 0;
  for (int base = 0; base < a.Nk; base += kThreads) {
    const int cidx = base + tid;
    const uint32_t f = cidx < a.Nk ? flags[cidx] : 0u;
    const uint64_t bal = __builtin_amdgcn_ballot_w64(f != 0u);
    if (lane == 0) wave_counts[wave] = __popcll(bal);
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const int cw = wave_counts[w];
      before += (w < wave) ? cw : 0;
      total += cw;
    }
    if (f != 0u) seq[n_union + before + __popcll(bal & ((1ull << lane) - 1ull))] = (uint32_t)cidx | (f << 24);
    n_union += total;
    __syncthreads();
  }
  // every thread has passed its last read of flags (the ring area) and seq is complete

  if (n_union == 0) {
    // no valid key block in any list of this workgroup (malformed input): its rows become zeros
    for (int r = 0; r < kNG; ++r) {
      const int pos = pos0 + 32 * r;
      if (pos < a.Lq) {
        const int orow = perm_at(a.perm_q, (int64_t)bhq * a.Lq, pos, a.Lq);
        uint4* op = reinterpret_cast<uint4*>(a.out + out_off(a, bhq, orow));
        for (int i = 0; i < G::kChunksPerRow / 2; ++i) op[(G::kChunksPerRow / 2) * h + i] = make_uint4(0u, 0u, 0u, 0u);
        if (a.lse && h == 0) a.lse[(int64_t)bhq * a.Lq + orow] = -INFINITY;
      }
    }
    if (kFast && tid == 0) a.redo[logical] = 0;
    return;
  }
  int n_tiles = n_union * TPB;
  {
    // a ragged last key block may leave its trailing tile without any valid key
    const int last_col = (int)(seq[n_union - 1] & 0xffffffu);
    if (TPB == 2 && last_col * kB + kTileKeys >= a.Lk) n_tiles -= 1;
  }
  const int64_t tiles_per_head = (int64_t)a.Nk * TPB;
  const char* Kh = a.Kt + (int64_t)bhk * tiles_per_head * kTileBytes;
  const char* Vh = a.Vt + (int64_t)bhk * tiles_per_head * kTileBytes;

  // entry of union position i (wave-uniform value in an SGPR)
  auto entry_of = [&](int t) -> uint32_t {
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)seq[t / TPB]);
  };
  // direct-to-LDS copy of tile `tile` into ring stage `stage`: 32 chunks of 1 KB, chunk
  // j*kWaves+wave by this wave (16 K chunks, then 16 V chunks)
  auto issue_tile = [&](int tile, int stage) {
    const char* kp = Kh + (int64_t)tile * kTileBytes;      // wave-uniform bases
    const char* vp = Vh + (int64_t)tile * kTileBytes;
#pragma unroll
    for (int j = 0; j < kLoadsPerWave; ++j) {
      const int cb = j * kWaves + wave;                   // wave-uniform: K chunks first, then V^T chunks
      const char* src = (cb < G::kChunksPerTile ? kp : vp) + (cb % G::kChunksPerTile) * 1024 + (uint32_t)(lane * 16);
      char* dst = smem + stage * kStageBytes + cb * 1024;
      __builtin_amdgcn_global_load_lds((gbl_ptr_t)src, (lds_ptr_t)dst, 16, 0, 0);
    }
    if constexpr (kCausal) {
      // the tile's key indices, minimum and maximum: kIxStride ints = 17 lanes of 16 bytes
      if (wave == 0 && lane < kIxStride / 4) {
        const int32_t* src = a.kix + ((int64_t)bhk * tiles_per_head + tile) * kIxStride + lane * 4;
        __builtin_amdgcn_global_load_lds((gbl_ptr_t)src, (lds_ptr_t)(kix_lds + stage * kIxStride), 16, 0, 0);
      }
    }
  };
  auto tile_of = [&](int t) -> int {
    const int tt = min(t, n_tiles - 1);
    return (int)(entry_of(tt) & 0xffffffu) * TPB + (tt % TPB);
  };

  // prologue: the first tile (SHARED: the first pair; past the end: the last tile again, never read)
  issue_tile(tile_of(0), 0);
  if (kStages == 4) issue_tile(tile_of(1), 1);

  // Q^T operand: lane (query li, half h) holds Q[q][16 s + 8 h .. +7] for s = 0..7
  bf16x8 qf[kNG][kQR];
  int q_lim[kNG];               // kCausal: the largest original key index the lane's query of each group may see
#pragma unroll
  for (int r = 0; r < kNG; ++r) q_lim[r] = INT_MIN;
  char* qpark = smem + kRingBytes + (wave * kNG * kQL) * 1024 + lane * 16;    // this lane's parked fragments
#pragma unroll
  for (int r = 0; r < kNG; ++r) {
    // the query of sorted position qpos, read from the caller's tensor; positions past L_q
    // (padding of the last block, or a query block that does not exist) read row 0 and are never stored
    const int qpos = pos0 + 32 * r;
    const int qrow = qpos < a.Lq ? perm_at(a.perm_q, (int64_t)bhq * a.Lq, qpos, a.Lq) : 0;
    if (kCausal && qpos < a.Lq) q_lim[r] = qrow + a.causal_off;
    const uint4* qp = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(a.q.ptr) +
                                                     (a.q.head_offset(bhq) + (int64_t)qrow * a.q.stride_l) * 2);
#pragma unroll
    for (int s = 0; s < G::kKSteps; ++s) {
      uint4 t = qp[2 * s + h];
      if (s < kQR) qf[r][s < kQR ? s : 0] = *reinterpret_cast<bf16x8*>(&t);
      else *reinterpret_cast<uint4*>(qpark + (r * kQL + s - kQR) * 1024) = t;    // read back by this lane only
    }
  }
  // LDS byte offsets inside a stage.  K: row li (+32 for the second block), chunk 2s+h at
  // position (2s+h) ^ (li & 15).  V^T: d-row li (+32 db), chunk 2g+h at (2g+h) ^ ((li>>1)&7).
  // (step s / group g are folded in by xor with s<<5 / g<<5 at the point of use)
  const int kaddr = li * G::kRowBytes + ((h ^ (li & (G::kChunksPerRow - 1))) << 4);
  const int vaddr = li * 128 + ((h ^ ((li >> 1) & 7)) << 4);

  typename StateOf<D, kNG>::type st;
  init_state<D>(st, kFast);
  const float c = a.scale_log2e;
  // one 64-key tile of the ring, for the one or two query groups of this wave
  auto tile = [&](auto masked, int stage_no, int nvalid) {
    const char* stage = smem + stage_no * kStageBytes;
    if constexpr (kNG == 1) process_tile<decltype(masked)::value, D>(st, qf[0], stage, kaddr, vaddr, c, nvalid, h);
    else {
      // the lane half is needed by the masking code only (ragged tile, causal mask): taken from the
      // thread index there, it does not occupy a register through the main loop
      int h2 = 0;
      if (decltype(masked)::value || kCausal) {
        int t2 = threadIdx.x;
        asm volatile("" : "+v"(t2));
        h2 = (t2 >> 5) & 1;
      }
      process_tile2<decltype(masked)::value, D, kQR, kCausal, kFast>(st, qf[0], qf[kNG - 1], qpark, stage, kaddr, vaddr, c, nvalid,
                                                                     h2, kix_lds + stage_no * kIxStride + 4 * h2, q_lim[0],
                                                                     q_lim[kNG - 1]);
    }
  };
  // causal: the largest limit among this wave's queries (lanes without a query ask for nothing); a tile
  // whose smallest key index lies beyond it has nothing for the wave
  int wq_max = INT_MIN;
  if constexpr (kCausal) {
    wq_max = max(q_lim[0], q_lim[kNG - 1]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) wq_max = max(wq_max, __shfl_xor(wq_max, off));
    wq_max = __builtin_amdgcn_readfirstlane(wq_max);
  }
  auto tile_has_visible_keys = [&](int stage_no) -> bool {
    if constexpr (!kCausal) return true;
    return __builtin_amdgcn_readfirstlane(kix_lds[stage_no * kIxStride + kTileKeys]) <= wq_max;
  };
  constexpr std::false_type kFull{};
  constexpr std::true_type kRagged{};
  const uint32_t my_bit = 1u << (24 + grp);

  // All tiles but the last: never ragged.  The last tile is peeled so that the masking code
  // (and its per-lane constants) stays out of the loop.  Loads are issued in tile order, so
  // "at most 2 tiles of my loads outstanding" means my part of tile t has landed; the barrier
  // then says everyone's part has, and that everyone is done with tile t-1, whose stage the
  // next load overwrites.
  // Tiles travel in PAIRS: ring stages {0,1} and {2,3} form two slots of two tiles, and the
  // workgroup meets at one barrier per pair (half as many barriers, half the skew cost).
  // Iteration p computes tiles 2p, 2p+1 from slot p%2 while tiles 2p+2, 2p+3 land in the other
  // slot; their loads are issued right after the barrier, which also says that every wave is
  // done with that other slot (pair p-1).  The union entries of later tiles are read from LDS
  // early and turned into scalars late, so their latency hides behind the arithmetic.
  if constexpr (kNG == 2) {
    // 64 queries per wave: ONE call site for full tiles (a second inlined copy of the tile code
    // costs the register allocator its footing).  Tiles travel in rounds of R = kStages / 2; the
    // workgroup meets once per round, and round p + 1 lands in the other half of the ring while
    // round p is computed.
    constexpr int R = kStages / 2;
    uint32_t e_cur = entry_of(0);
    int t = 0;
#pragma nounroll
    for (; t + 1 < n_tiles; ++t) {
      if (t % R == 0) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        const int half_next = ((t / R) + 1) & 1;
#pragma unroll
        for (int j = 0; j < R; ++j) issue_tile(tile_of(t + R + j), half_next * R + j);
      }
      const uint32_t raw_n = seq[(t + 1) / TPB];
      if ((e_cur & my_bit) && tile_has_visible_keys(((t / R) & 1) * R + t % R)) tile(kFull, ((t / R) & 1) * R + t % R, kTileKeys);
      e_cur = (uint32_t)__builtin_amdgcn_readfirstlane((int)raw_n);
    }
    if (t % R == 0) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
    }
    const int nvalid = a.Lk - ((int)(e_cur & 0xffffffu) * TPB + (t % TPB)) * kTileKeys;
    if ((e_cur & my_bit) && tile_has_visible_keys(((t / R) & 1) * R + t % R)) tile(kRagged, ((t / R) & 1) * R + t % R, nvalid);
  } else if constexpr (kStages == 4) {
  uint32_t e_a = entry_of(0);
  uint32_t e_b = entry_of(min(1, n_tiles - 1));
  int t = 0;
  for (; t + 2 < n_tiles; t += 2) {          // pairs that do not contain the last tile
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const int tf0 = min(t + 2, n_tiles - 1), tf1 = min(t + 3, n_tiles - 1);
    const uint32_t raw_f0 = seq[tf0 / TPB], raw_f1 = seq[tf1 / TPB];
    const int slot_next = ((t >> 1) + 1) & 1;
    {
      const int b0 = __builtin_amdgcn_readfirstlane((int)raw_f0) & 0xffffff;
      const int b1 = __builtin_amdgcn_readfirstlane((int)raw_f1) & 0xffffff;
      issue_tile(b0 * TPB + (tf0 % TPB), 2 * slot_next);
      issue_tile(b1 * TPB + (tf1 % TPB), 2 * slot_next + 1);
    }
    const int slot = ((t >> 1) & 1) * 2;            // first ring stage of the pair
    if (e_a & my_bit) tile(kFull, slot, kTileKeys);
    if (e_b & my_bit) tile(kFull, slot + 1, kTileKeys);
    e_a = (uint32_t)__builtin_amdgcn_readfirstlane((int)raw_f0);
    e_b = (uint32_t)__builtin_amdgcn_readfirstlane((int)raw_f1);
  }
  {
    // the last pair: one or two tiles, the very last one possibly ragged
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const int slot = ((t >> 1) & 1) * 2;
    if (t + 1 < n_tiles) {
      if (e_a & my_bit) tile(kFull, slot, kTileKeys);
      const int nvalid = a.Lk - ((int)(e_b & 0xffffffu) * TPB + ((t + 1) % TPB)) * kTileKeys;
      if (e_b & my_bit) tile(kRagged, slot + 1, nvalid);
    } else {
      const int nvalid = a.Lk - ((int)(e_a & 0xffffffu) * TPB + (t % TPB)) * kTileKeys;
      if (e_a & my_bit) tile(kRagged, slot, nvalid);
    }
  }
  } else {
    // SOLO: two stages, one tile per barrier; tile t+1 lands while tile t is computed
    uint32_t e_cur = entry_of(0);
    int t = 0;
    for (; t + 1 < n_tiles; ++t) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      const uint32_t raw_n = seq[(t + 1) / TPB];
      const uint32_t e_nxt = (uint32_t)__builtin_amdgcn_readfirstlane((int)raw_n);
      issue_tile((int)(e_nxt & 0xffffffu) * TPB + ((t + 1) % TPB), (t + 1) & 1);
      if (e_cur & my_bit) tile(kFull, t & 1, kTileKeys);
      e_cur = e_nxt;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const int nvalid = a.Lk - ((int)(e_cur & 0xffffffu) * TPB + (t % TPB)) * kTileKeys;
    if (e_cur & my_bit) tile(kRagged, t & 1, nvalid);
  }

  // ---- epilogue: normalise, scatter rows to their original positions
  // positions and lane halves are rebuilt from the thread index (opaque to the compiler): carried
  // through the main loop they would take registers that the accumulators and Q^T fragments need
  int tid_e = threadIdx.x;
  asm volatile("" : "+v"(tid_e));
  const int h_e = (tid_e >> 5) & 1;
  const int pos_e = wg * kQueriesPerWg + (tid_e >> 6) * kQPW + (tid_e & 31);
  int unsafe = 0;                // kFast: some row of this lane has a sum outside the safe range
#pragma unroll
  for (int r = 0; r < kNG; ++r) {
    const float l_part = l_of(st, r), m_fin = m_of(st, r);
    const float l_tot = l_part + __shfl_xor(l_part, 32);
    const float inv_l = l_tot > 0.f ? 1.0f / l_tot : 0.f;    // a query block without any valid key block: zeros
    const int pos = pos_e + 32 * r;
    // (on the bit patterns, which order like the values for positive floats and put inf, NaN and anything
    //  negative above kMaxSum: this file is compiled without NaN semantics for float comparisons)
    if (kFast && pos < a.Lq && __float_as_uint(l_tot) - __float_as_uint(kMinSum) > __float_as_uint(kMaxSum) - __float_as_uint(kMinSum))
      unsafe = 1;
    const int h = h_e;
    if (pos < a.Lq) {
      const int orow = perm_at(a.perm_q, (int64_t)bhq * a.Lq, pos, a.Lq);
      __bf16* op = a.out + out_off(a, bhq, orow);
#pragma unroll
      for (int db = 0; db < G::kDBlocks; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          bf16x4 pk;
#pragma unroll
          for (int e = 0; e < 4; ++e) pk[e] = (__bf16)(o_of(st, r, db)[4 * r4 + e] * inv_l);
          *reinterpret_cast<bf16x4*>(op + 32 * db + 8 * r4 + 4 * h) = pk;
        }
      if (a.lse && h == 0)
        a.lse[(int64_t)bhq * a.Lq + orow] = (m_fin + __log2f(l_tot)) * 0.6931471805599453f;
    }
  }
  if constexpr (kFast) {
    // (a row without any visible key has the sum 0 as well and is sent round again: it comes out as zeros both times)
    const int any = __syncthreads_or(unsafe);
    if (threadIdx.x == 0) a.redo[logical] = any;
  }
}

size_t sz_kv(int BHkv, int Nk, int B, int d) { return align_up((size_t)BHkv * Nk * B * d * 2, 256); }
size_t sz_kix(int BHkv, int Nk, int B) { return align_up((size_t)BHkv * (Nk * B / kTileKeys) * kIxStride * 4, 256); }

template <int D>
size_t lds_bytes(int threads, int qpw, int Nk, bool causal = false, bool fast = false) {
  const size_t park = (size_t)(threads / 64) * (qpw / 32) * (D / 16 - q_reg_steps(D, qpw, causal, fast)) * 1024;
  const size_t base = (size_t)stages_of(threads, qpw) * Geo<D>::kStageBytes + park + (size_t)Nk * 4 + (threads / 64) * 4;
  return causal ? ((base + 15) & ~(size_t)15) + (size_t)stages_of(threads, qpw) * kIxStride * 4 : base;
}

template <int kB, int D, int kWgQueries, int kQPW, bool kCausal = false, bool kFast = false>
basa_status launch_main(MfmaArgs m, int BHq, hipStream_t st) {
  constexpr int kThreads = kWgQueries / kQPW * 64;
  const size_t lds = lds_bytes<D>(kThreads, kQPW, m.Nk, kCausal, kFast);
  // while the union list is built, the per-key-block membership flags live in the ring area
  if ((size_t)m.Nk * 4 > (size_t)stages_of(kThreads, kQPW) * Geo<D>::kStageBytes) {
    set_error("attention: %d key blocks exceed the %zu this workgroup shape can list", m.Nk,
              (size_t)stages_of(kThreads, kQPW) * Geo<D>::kStageBytes / 4);
    return BASA_ERR_UNSUPPORTED;
  }
  m.wgs_per_head = ceil_div(m.Nq * kB, kWgQueries);
  m.total_wgs = BHq * m.wgs_per_head;
  const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_mfma_kernel<kB, D, kWgQueries, kQPW, kCausal, kFast>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(dynamic LDS)");
  hipLaunchKernelGGL((attn_mfma_kernel<kB, D, kWgQueries, kQPW, kCausal, kFast>), dim3(m.total_wgs), dim3(kThreads), lds, st, m);
  BASA_HIP_CHECK_LAUNCH("attn_mfma_kernel");
  return BASA_OK;
}
// dispatch on block size and head dimension
template <int kWgQueries, int kQPW, bool kCausal = false, bool kFast = false>
basa_status launch_shape(const MfmaArgs& m, int B, int d, int BHq, hipStream_t st) {
  if (d == 128) return B == 128 ? launch_main<128, 128, kWgQueries, kQPW, kCausal, kFast>(m, BHq, st)
                                : launch_main<64, 128, kWgQueries, kQPW, kCausal, kFast>(m, BHq, st);
  return B == 128 ? launch_main<128, 64, kWgQueries, kQPW, kCausal, kFast>(m, BHq, st)
                  : launch_main<64, 64, kWgQueries, kQPW, kCausal, kFast>(m, BHq, st);
}
// The 512-query shape in two passes: without running maxima, then, for the workgroups whose row sums
// left the safe range (none on ordinary inputs: that launch returns at once), with them.
template <bool kCausal>
basa_status launch_wide(MfmaArgs m, int B, int d, int BHq, int32_t* redo, bool two_pass, hipStream_t st) {
  if (two_pass) {
    m.redo = redo;
    const basa_status s = launch_shape<kWideQueries, 64, kCausal, true>(m, B, d, BHq, st);
    if (s != BASA_OK) return s;
  } else {
    m.redo = nullptr;
  }
  return launch_shape<kWideQueries, 64, kCausal, false>(m, B, d, BHq, st);
}

// Causal variant: per 64-key tile of the ordered keys, the original index of every key (INT_MAX past
// the end of the sequence), then the smallest and the largest of the 64.
__global__ __launch_bounds__(64) void key_index_kernel(const int32_t* __restrict__ perm, int Lk, int tiles_per_head,
                                                       int32_t* __restrict__ out) {
  const int tile = blockIdx.x, bh = blockIdx.y, lane = threadIdx.x;
  const int pos = tile * kTileKeys + lane;
  const int idx = pos < Lk ? perm_at(perm, (int64_t)bh * Lk, pos, Lk) : INT_MAX;
  int lo = idx, hi = idx;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    lo = min(lo, __shfl_xor(lo, off));
    hi = max(hi, __shfl_xor(hi, off));
  }
  int32_t* o = out + ((int64_t)bh * tiles_per_head + tile) * kIxStride;
  o[lane] = idx;
  if (lane < 4) o[kTileKeys + lane] = lane == 0 ? lo : (lane == 1 ? hi : 0);
}

// How much the lists of the query blocks that would share a 512-query workgroup have in common, on
// every kProbeStride-th such group of gsz = 512 / B neighbouring blocks: probe[0] += blocks in the
// union of the group's lists (what a 512-query workgroup walks), probe[1] += the same for each of
// the group's four 128-query subgroups, added up (what four 128-query workgroups walk; for B = 128
// simply the blocks in the four lists).  One wave per group: the lists are or-ed into bitmaps in LDS.
constexpr int kProbeStride = 8, kProbeMaxBlocks = 8192;
__global__ __launch_bounds__(256) void list_overlap_kernel(const int32_t* __restrict__ row_count,
                                                           const int32_t* __restrict__ row_cols, int cols_stride,
                                                           int Nq, int Nk, int gsz, int groups_total,
                                                           int32_t* __restrict__ probe) {
  __shared__ uint32_t bits[4][kProbeMaxBlocks / 32], sub[4][kProbeMaxBlocks / 32];
  const int wv = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int group = (blockIdx.x * 4 + wv) * kProbeStride;
  const bool active = group < groups_total;             // no early exit: every wave meets the barriers
  const int groups_per_head = Nq / gsz;
  const int bh = active ? group / groups_per_head : 0, g0 = active ? (group - bh * groups_per_head) * gsz : 0;
  const unsigned limit = (unsigned)min(Nk, kProbeMaxBlocks);
  const int words = (int)((limit + 31) >> 5);
  const int rows_per_sub = gsz / 4;                     // query blocks of a 128-query subgroup: 1 or 2
  for (int w = lane; w < words; w += 64) bits[wv][w] = 0u;
  int uni_sub = 0;
  for (int sg = 0; sg < 4; ++sg) {
    for (int w = lane; w < words; w += 64) sub[wv][w] = 0u;
    __syncthreads();
    for (int r = 0; r < rows_per_sub; ++r) {
      const int64_t row = (int64_t)bh * Nq + g0 + sg * rows_per_sub + r;
      const int n = active ? max(0, min(row_count[row], cols_stride)) : 0;
      const int32_t* A = row_cols + row * cols_stride;
      for (int i = lane; i < n; i += 64) {
        const unsigned v = (unsigned)A[i];
        if (v < limit) atomicOr(&sub[wv][v >> 5], 1u << (v & 31));
      }
    }
    __syncthreads();
    for (int w = lane; w < words; w += 64) {
      const uint32_t x = sub[wv][w];
      uni_sub += __popc(x);
      bits[wv][w] |= x;                                  // word w belongs to this lane in every round
    }
  }
  int uni = 0;
  for (int w = lane; w < words; w += 64) uni += __popc(bits[wv][w]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    uni += __shfl_xor(uni, off);
    uni_sub += __shfl_xor(uni_sub, off);
  }
  if (active && lane == 0) {
    atomicAdd(&probe[0], uni);
    atomicAdd(&probe[1], uni_sub);
  }
}
__global__ void zero_probe_kernel(int32_t* probe) {
  if (threadIdx.x < 2) probe[threadIdx.x] = 0;
}

template <int D>
basa_status launch_gathers(const AttnArgs& a, uint4* Kt, uint4* Vt, int BHkv, int Nk, hipStream_t st) {
  const int B = a.B;
  hipLaunchKernelGGL(gather_rows_kernel<D>, dim3(Nk * B / 64, BHkv), dim3(256), 0, st, a.k, a.perm_k, Kt, Nk * B, 1);
  BASA_HIP_CHECK_LAUNCH("gather_rows_kernel(K)");
  hipLaunchKernelGGL(gather_vt_kernel<D>, dim3(Nk * B / 64, BHkv), dim3(256), 0, st, a.v, a.perm_k, Vt, Nk * B / 64);
  BASA_HIP_CHECK_LAUNCH("gather_vt_kernel");
  return BASA_OK;
}

}  // namespace

size_t attn_mfma_workspace_bytes(int BHq, int BHkv, int Lq, int Lk, int d, int B) {
  const int Nq = ceil_div(Lq, B), Nk = ceil_div(Lk, B);
  // + the two counters of the list-overlap probe + the key-index tiles of the causal variant
  // + one word per 512-query workgroup (which of them the pass with running maxima has to repeat)
  return 2 * sz_kv(BHkv, Nk, B, d) + 256 + sz_kix(BHkv, Nk, B) + align_up((size_t)BHq * ceil_div(Nq * B, kWideQueries) * 4, 256);
}

basa_status launch_attn_mfma(const AttnArgs& a, hipStream_t st) {
  const int BHq = a.q.batch * a.q.heads, BHkv = a.k.batch * a.k.heads;
  const int B = a.B;
  const int Nq = ceil_div(a.q.L, B), Nk = ceil_div(a.k.L, B);
  if (BHq == 0 || Nq == 0) return BASA_OK;
  const int d = a.q.d;
  // While a workgroup builds its union list, one membership word per key block lives in the ring
  // area, whose smallest form is two stages: more key blocks than that cannot be listed.
  {
    const size_t cap = (d == 128 ? (size_t)2 * Geo<128>::kStageBytes : (size_t)2 * Geo<64>::kStageBytes) / 4;
    if ((size_t)Nk > cap) {
      set_error("attention: %d key blocks per head exceed the %zu this kernel can list (head dimension %d)", Nk, cap, d);
      return BASA_ERR_UNSUPPORTED;
    }
  }
  // the largest LDS request among the shapes that may be launched
  const size_t lds = d == 128 ? std::max(lds_bytes<128>(512, 32, Nk), lds_bytes<128>(512, 64, Nk))
                              : std::max(lds_bytes<64>(512, 32, Nk), lds_bytes<64>(512, 64, Nk));
  {
    int dev = 0, max_lds = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&max_lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
    if (e != hipSuccess) return hip_fail(e, "hipDeviceGetAttribute(shared memory per block)");
    if (lds > (size_t)max_lds) {
      set_error("attention needs %zu bytes of LDS for %d key blocks, the device offers %d", lds, Nk, max_lds);
      return BASA_ERR_UNSUPPORTED;
    }
  }
  char* ws = reinterpret_cast<char*>(a.ws);
  uint4* Kt = reinterpret_cast<uint4*>(ws);
  uint4* Vt = reinterpret_cast<uint4*>(ws + sz_kv(BHkv, Nk, B, d));
  int32_t* probe = reinterpret_cast<int32_t*>(ws + 2 * sz_kv(BHkv, Nk, B, d));
  int32_t* redo = reinterpret_cast<int32_t*>(ws + 2 * sz_kv(BHkv, Nk, B, d) + 256 + sz_kix(BHkv, Nk, B));

  {
    ProfScope prof(K_GATHER, st);
    const basa_status s = d == 128 ? launch_gathers<128>(a, Kt, Vt, BHkv, Nk, st)
                                   : launch_gathers<64>(a, Kt, Vt, BHkv, Nk, st);
    if (s != BASA_OK) return s;
  }

  MfmaArgs m;
  m.q = a.q; m.Kt = reinterpret_cast<const char*>(Kt); m.Vt = reinterpret_cast<const char*>(Vt);
  m.row_count = a.row_count; m.row_cols = a.row_cols; m.cols_stride = a.cols_stride;
  m.perm_q = a.perm_q;
  m.out = reinterpret_cast<__bf16*>(a.out); m.lse = a.lse;
  m.out_sb = a.out_sb; m.out_sh = a.out_sh; m.out_sl = a.out_sl; m.heads_q = a.q.heads;
  m.Nq = Nq; m.Nk = Nk; m.Lq = a.q.L; m.Lk = a.k.L;
  m.group = a.q.heads / a.k.heads;
  m.wgs_per_head = 0; m.total_wgs = 0;
  m.scale_log2e = 1.4426950408889634f / sqrtf((float)d);
  m.probe = nullptr; m.run_if_solo = 0; m.redo = nullptr;
  m.kix = nullptr; m.causal_off = a.causal_off;
  if (a.causal) {
    int32_t* kix = reinterpret_cast<int32_t*>(ws + 2 * sz_kv(BHkv, Nk, B, d) + 256);
    const int tiles_per_head = Nk * B / kTileKeys;
    {
      ProfScope prof(K_GATHER, st);
      hipLaunchKernelGGL(key_index_kernel, dim3(tiles_per_head, BHkv), dim3(64), 0, st, a.perm_k, a.k.L, tiles_per_head, kix);
      BASA_HIP_CHECK_LAUNCH("key_index_kernel");
    }
    m.kix = kix;
    ProfScope prof(K_ATTN, st);
    return launch_wide<true>(m, B, d, BHq, redo, a.variant != 4, st);
  }

  // Which shape of workgroup: asked for, or (B = d = 128, block lists given, enough work to pay for
  // three tiny launches) decided on the device from how much neighbouring lists overlap.
  int variant = a.variant;
  const int gsz = kWideQueries / B;
  const bool can_probe = a.row_cols != nullptr && Nq >= 2 * gsz && (int64_t)BHq * Nq * B >= 2048 * 128;
  if (variant == 0 && !can_probe) variant = a.row_cols ? BASA_ATTN_DEFAULT_LISTS : 3;   // no lists: every block shares every tile
  if (variant == 0) {
    const int groups_total = BHq * (Nq / gsz);
    hipLaunchKernelGGL(zero_probe_kernel, dim3(1), dim3(64), 0, st, probe);
    BASA_HIP_CHECK_LAUNCH("zero_probe_kernel");
    hipLaunchKernelGGL(list_overlap_kernel, dim3(ceil_div(ceil_div(groups_total, kProbeStride), 4)), dim3(256), 0, st,
                       a.row_count, a.row_cols, a.cols_stride, Nq, Nk, gsz, groups_total, probe);
    BASA_HIP_CHECK_LAUNCH("list_overlap_kernel");
    m.probe = probe;
  }
  ProfScope prof(K_ATTN, st);
  basa_status s = BASA_OK;
  if (variant == 1) return launch_shape<kSharedQueries, 32>(m, B, d, BHq, st);
  if (variant == 0 || variant == 3 || variant == 4) {
    m.run_if_solo = 0;
    if ((s = launch_wide<false>(m, B, d, BHq, redo, variant != 4, st)) != BASA_OK) return s;
  }
  if (variant == 0 || variant == 2) {
    m.run_if_solo = 1;
    s = launch_shape<kSoloQueries, 32>(m, B, d, BHq, st);
  }
  return s;
}

}  // namespace basa
