// Norm ranking (Sec. 3.3, Eq. 9-10; Alg. 1 steps 1-2): sort keys and a segmented
// merge sort of (key, index) pairs, one segment per (head, window).
//
// Key of a token = fp32 rounding of the fp64 sum of squares of its d values.  Each
// pair is packed into one 64-bit word, [segment : 6][key bits without the sign : 31][token
// index : 27]: keys are non-negative floats, whose bit patterns order like the values, so an
// unsigned compare of the packed words orders by segment, then key, and breaks ties by lower
// index, which also makes every word distinct (no stability concerns in the sort).  The
// segment field is 0 unless the caller gave a list of segments of unequal length; those are
// sorted as ONE sequence per head, and the segment field keeps every segment in its range.
#include "common.hpp"

namespace basa {
namespace {

constexpr int kSortThreads = 256;
constexpr int kTile = 4096;          // elements sorted per workgroup in LDS (32 KB)
constexpr int kMergeItems = 8;       // outputs per thread in a merge pass
constexpr int kMergeChunk = kSortThreads * kMergeItems;   // 2048 outputs per workgroup
constexpr int kIdxBits = 27;
static_assert((1 << kIdxBits) == kMaxSortLen && BASA_MAX_SEGMENTS < 64, "fields of the packed word");
__device__ __forceinline__ uint64_t pack_word(int seg, float key, int idx) {
  return ((uint64_t)(uint32_t)seg << 58) | ((uint64_t)(__float_as_uint(key) & 0x7fffffffu) << kIdxBits) | (uint32_t)idx;
}
__device__ __forceinline__ int32_t idx_of_word(uint64_t w) { return (int32_t)((uint32_t)w & ((1u << kIdxBits) - 1u)); }

// ---------------------------------------------------------------------------------
// Keys + tile sort in one kernel.  A workgroup owns one tile of up to kTile consecutive tokens
// of a segment: it streams their rows (a row of d elements is 16-byte chunks spread over LPR
// adjacent lanes; two batches of 8 rows per thread in flight), writes the packed (key, index)
// words into LDS, sorts them there with a bitonic network, and writes the sorted tile (or,
// when the tile is the whole segment, the permutation itself).  Workgroups of a compute unit
// are in different phases, so the LDS-bound sort of one hides under the HBM-bound key pass of
// the others.
// Segment s of a head covers [s*W, min((s+1)*W, L)); tiles never straddle segments.
// Up to two tensors of the same L, d and dtype are handled by one launch: rows blockIdx.y <
// BH0 belong to x0, the rest to x1; packed words and permutations of x1 follow those of x0.
// ---------------------------------------------------------------------------------
struct SegGeom {
  int L, W, segs, tiles_per_seg;
};

// ---- the tile's bitonic network, 16 words per thread in registers ------------------------
// Word i of the tile lives at LDS slot i + i/16 (one pad word per 16: a thread's 16 consecutive
// words, and the other two ownership patterns below, then hit distinct banks).
constexpr int kTileSlots = kTile + kTile / 16;
__device__ __forceinline__ int tile_slot(int i) { return i + (i >> 4); }

// Three ways of dealing the 4096 = 2^12 words to 256 threads x 16 registers; in layout G the
// register number is index bits 4G+3 .. 4G, so the compare-exchange stages whose distance 2^b
// has b in that range work on registers only.
template <int G>
__device__ __forceinline__ int word_of(int t, int r) {
  if (G == 0) return (t << 4) | r;
  if (G == 1) return ((t >> 4) << 8) | (r << 4) | (t & 15);
  return (r << 8) | t;
}
template <int G>
__device__ __forceinline__ void regs_from_lds(uint64_t (&v)[16], const uint64_t* buf, int t) {
#pragma unroll
  for (int r = 0; r < 16; ++r) v[r] = buf[tile_slot(word_of<G>(t, r))];
}
template <int G>
__device__ __forceinline__ void regs_to_lds(const uint64_t (&v)[16], uint64_t* buf, int t) {
#pragma unroll
  for (int r = 0; r < 16; ++r) buf[tile_slot(word_of<G>(t, r))] = v[r];
}
// Stages of the merge step with block size k whose compare distance 2^b has b_lo <= b <= b_hi,
// all inside layout G's register bits.  A pair is ordered ascending where index bit log2(k) is 0.
template <int G>
__device__ __forceinline__ void stages_in_regs(uint64_t (&v)[16], int t, int k, int b_hi, int b_lo) {
  asm volatile("" : "+v"(t));      // as in relayout(): recompute the word indices here
#pragma unroll
  for (int lb = 3; lb >= 0; --lb) {
    const int b = 4 * G + lb;
    if (b <= b_hi && b >= b_lo) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (r & (1 << lb)) continue;
        const int r2 = r | (1 << lb);
        const bool up = (word_of<G>(t, r) & k) == 0;
        const uint64_t a = v[r], c = v[r2];
        const bool swap = (a > c) == up;
        v[r] = swap ? c : a;
        v[r2] = swap ? a : c;
      }
    }
  }
}
// Moves the tile from layout A (registers) to layout B (registers) through LDS.
template <int A, int B>
__device__ __forceinline__ void relayout(uint64_t (&v)[16], uint64_t* buf, int t) {
  // the slot addresses are recomputed at every use (two integer ops each): left to itself the
  // compiler keeps all 48 of them in registers across the whole network and halves the occupancy
  asm volatile("" : "+v"(t));
  regs_to_lds<A>(v, buf, t);
  __syncthreads();
  regs_from_lds<B>(v, buf, t);
  __syncthreads();                 // everyone has read before anyone writes the next layout
}
// Sorts the kTile words in buf (slots tile_slot(i)) ascending; ends with the words back in buf.
__device__ __forceinline__ void sort_tile_in_lds(uint64_t* buf, int t) {
  static_assert(kTile == 4096 && kSortThreads == 256, "16 words per thread, 12 index bits in three groups of 4");
  uint64_t v[16];
  regs_from_lds<0>(v, buf, t);
  __syncthreads();
  for (int m = 1; m <= 12; ++m) {
    const int k = 1 << m;          // k = 4096: bit 12 of an index is always 0, everything ascending
    if (m > 8) {
      relayout<0, 2>(v, buf, t);
      stages_in_regs<2>(v, t, k, m - 1, 8);
      relayout<2, 1>(v, buf, t);
      stages_in_regs<1>(v, t, k, 7, 4);
      relayout<1, 0>(v, buf, t);
      stages_in_regs<0>(v, t, k, 3, 0);
    } else if (m > 4) {
      relayout<0, 1>(v, buf, t);
      stages_in_regs<1>(v, t, k, m - 1, 4);
      relayout<1, 0>(v, buf, t);
      stages_in_regs<0>(v, t, k, 3, 0);
    } else {
      stages_in_regs<0>(v, t, k, m - 1, 0);
    }
  }
  regs_to_lds<0>(v, buf, t);
  __syncthreads();
}

template <bool kBf16, int kD>
__global__ __launch_bounds__(kSortThreads) void norm_tile_sort_kernel(TensorView x0, TensorView x1, int BH0,
                                                                      uint64_t* __restrict__ out,
                                                                      int32_t* __restrict__ perm0,
                                                                      int32_t* __restrict__ perm1,
                                                                      float* __restrict__ keys_out, SegGeom g,
                                                                      SegList sl) {
  constexpr int kElem = kBf16 ? 2 : 4;
  constexpr int LPR = kD * kElem / 16;          // lanes per row: 8, 16 or 32
  constexpr int kRowsPerIter = kSortThreads / LPR;
  constexpr int kIters = 8;
  constexpr int kRowsPerPass = kRowsPerIter * kIters;
  static_assert(kTile % kRowsPerPass == 0, "a tile is a whole number of passes");
  __shared__ uint64_t buf[kTileSlots];

  const int bh = blockIdx.y;
  const int seg = blockIdx.x / g.tiles_per_seg;
  const int tile = blockIdx.x - seg * g.tiles_per_seg;
  const int seg_end = min((seg + 1) * g.W, g.L);
  const int start = seg * g.W + tile * kTile;
  if (start >= seg_end) return;
  const int n = min(kTile, seg_end - start);
  const int64_t hb = (int64_t)bh * g.L;
  const bool second = bh >= BH0;
  const TensorView& x = second ? x1 : x0;
  int32_t* perm_out = second ? (perm1 ? perm1 - (int64_t)BH0 * g.L : nullptr) : perm0;
  const char* base = reinterpret_cast<const char*>(x.ptr) + x.head_offset(second ? bh - BH0 : bh) * kElem;
  const int sub = threadIdx.x % LPR;
  const int rig = threadIdx.x / LPR;
  // segment of the tile's first token; nearly every tile lies inside one segment
  int seg_lo = 0;
  for (int j = 1; j < sl.n; ++j) seg_lo += (start >= sl.bound[j]) ? 1 : 0;
  const bool one_segment = sl.n <= 1 || start + n <= sl.bound[seg_lo + 1];

  // ---- phase 1: keys of tokens start .. start+n-1 into buf
  // Every load is unconditional, its row clamped into the tile (a row past the end reads the
  // tile's last row, whose key is never written): loads inside branches make the compiler wait
  // for ALL outstanding loads at the join, the prefetch of the next pass included, and the double
  // buffering is lost.
  const int passes = (n + kRowsPerPass - 1) / kRowsPerPass;
  auto load_pass = [&](int pass, uint4 (&raw)[kIters]) {
    // A pass past the last (the loop below asks for up to four of them) has every lane read the tile's
    // first 16 bytes, one cache line per instruction, instead of the last pass again: the loads are
    // streaming loads, which nothing caches, so a repeated pass would cost its 32 KB of HBM traffic
    // again (an eighth of the tile in all).
    const bool live = pass < passes;             // uniform over the workgroup
    const int sub_l = live ? sub : 0;
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
      const int loc = live ? min(pass * kRowsPerPass + it * kRowsPerIter + rig, n - 1) : 0;
      // (streaming loads: every row is read once here; with the hint the pass takes 0.416 instead of
      //  0.431 ms at 128K, the rows no longer push the sort words being written out of the cache)
      // (bit-cast into uint4, not held as the builtin's vector type: the compiler rotates such vectors
      //  through the three buffers as whole registers, copies that count as uses of loads still in
      //  flight, and every batch is then waited for at the top of the loop)
      typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
      raw[it] = __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + (int64_t)(start + loc) * x.stride_l * kElem) + sub_l));
    }
  };
  auto keys_of_pass = [&](int pass, const uint4 (&cur)[kIters]) {
    // per-lane partial sums of the kIters rows this lane contributes to
    double acc[kIters];
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
      acc[it] = 0.0;
      const uint32_t w[4] = {cur[it].x, cur[it].y, cur[it].z, cur[it].w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if constexpr (kBf16) {
          // |x| as a double, built from the 15 exponent+mantissa bits of the bf16 (the float to
          // double conversion instruction is many times slower than these two integer ops): the
          // high word of the double is bits << 13 plus the exponent rebias (1023-127) << 20, the
          // low word is zero.  A zero or subnormal bf16 (exponent field 0) comes out as a value
          // below 2^-126 instead; its square, below 2^-252, is lost against any sum that can
          // round to a non-zero fp32 key (>= 2^-150), exactly as the true square would be.
          const double lo = __hiloint2double((int)((__builtin_amdgcn_ubfe(w[i], 0, 15) << 13) + 0x38000000u), 0);
          const double hi = __hiloint2double((int)((__builtin_amdgcn_ubfe(w[i], 16, 15) << 13) + 0x38000000u), 0);
          acc[it] = fma(lo, lo, acc[it]);
          acc[it] = fma(hi, hi, acc[it]);
        } else {
          const double v = (double)__uint_as_float(w[i]);
          acc[it] = fma(v, v, acc[it]);
        }
      }
    }
    // Reduction over the LPR lanes of a row, all kIters rows at once: in the step with lane
    // distance 2^b a lane hands the half of its partial sums that its partner keeps to the
    // partner and halves its own set (8 -> 4 -> 2 -> 1 sums in 7 exchanges instead of 24), so
    // that after three steps lane `sub` holds one row, iteration 4*bit0 + 2*bit1 + bit2 of sub.
    static_assert(kIters == 8 && LPR >= 8, "the exchange pattern below is written for 8 rows");
#pragma unroll
    for (int b = 0; b < 3; ++b) {
      const bool upper = (sub >> b) & 1;
      const int m = kIters >> (b + 1);
#pragma unroll
      for (int i = 0; i < m; ++i) {
        const double give = upper ? acc[i] : acc[i + m];
        const double keep = upper ? acc[i + m] : acc[i];
        acc[i] = keep + __shfl_xor(give, 1 << b, LPR);
      }
    }
#pragma unroll
    for (int off = 8; off < LPR; off <<= 1) acc[0] += __shfl_xor(acc[0], off, LPR);
    const int it_mine = 4 * (sub & 1) + (sub & 2) + ((sub >> 2) & 1);
    const int loc = pass * kRowsPerPass + it_mine * kRowsPerIter + rig;
    if (sub < 8 && loc < n) {
      const float key = (float)acc[0];
      // (the segment of the tile's first token; a tile that straddles a boundary is put right below,
      //  outside this loop, whose loads the compiler can then count exactly)
      buf[tile_slot(loc)] = pack_word(seg_lo, key, start + loc);
      if (keys_out) keys_out[hb + start + loc] = key;
    }
  };
  // three batches of rows: two are in flight while the third is turned into keys (a pass past the last
  // writes nothing: its positions lie beyond n)
  uint4 b0[kIters], b1[kIters], b2[kIters];
  load_pass(0, b0);
  load_pass(1, b1);
  load_pass(2, b2);
  for (int pass = 0; pass < passes; pass += 3) {
    keys_of_pass(pass, b0);
    load_pass(pass + 3, b0);
    keys_of_pass(pass + 1, b1);
    load_pass(pass + 4, b1);
    keys_of_pass(pass + 2, b2);
    load_pass(pass + 5, b2);
  }
  if (!one_segment) {              // workgroup-uniform and rare: some tokens belong to later segments
    // (the keys stored in the loop above have to be in LDS before the barrier; the compiler's own wait
    //  was found missing on this path by lds_wait_audit, so it is spelt out)
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += kSortThreads) {
      int sg = seg_lo;
      for (int j = seg_lo + 1; j < sl.n; ++j) sg += (start + i >= sl.bound[j]) ? 1 : 0;
      if (sg != seg_lo) {
        const uint64_t w = buf[tile_slot(i)];
        buf[tile_slot(i)] = (w & ((1ull << 58) - 1ull)) | ((uint64_t)(uint32_t)sg << 58);
      }
    }
  }
  for (int i = n + threadIdx.x; i < kTile; i += kSortThreads) buf[tile_slot(i)] = ~0ull;
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __syncthreads();

  // ---- phase 2: bitonic network over the kTile words
  sort_tile_in_lds(buf, threadIdx.x);
  if (perm_out) {
    for (int i = threadIdx.x; i < n; i += kSortThreads) perm_out[hb + start + i] = idx_of_word(buf[tile_slot(i)]);
  } else {
    // (streaming stores, like the loads of the rows: another 3 % of this kernel)
    for (int i = threadIdx.x; i < n; i += kSortThreads) __builtin_nontemporal_store(buf[tile_slot(i)], &out[hb + start + i]);
  }
}

// ---------------------------------------------------------------------------------
// Merge pass: sorted runs of `run` elements are merged pairwise inside each segment.
// One workgroup produces kMergeChunk consecutive outputs of one pair, located with a
// merge-path search on the pair's two runs.
// ---------------------------------------------------------------------------------
__device__ __forceinline__ int merge_path(const uint64_t* A, int na, const uint64_t* Bv, int nb, int diag) {
  int lo = max(0, diag - nb), hi = min(diag, na);
  while (lo < hi) {
    int mid = (lo + hi) >> 1;
    if (A[mid] < Bv[diag - 1 - mid]) lo = mid + 1; else hi = mid;
  }
  return lo;
}

__global__ __launch_bounds__(kSortThreads) void merge_pass_kernel(const uint64_t* __restrict__ in,
                                                                  uint64_t* __restrict__ out,
                                                                  int32_t* __restrict__ perm0,
                                                                  int32_t* __restrict__ perm1, int BH0,
                                                                  SegGeom g, int run,
                                                                  int chunks_per_pair, int pairs_per_seg) {
  __shared__ uint64_t buf[kMergeChunk];
  __shared__ int split[2];
  const int bh = blockIdx.y;
  int id = blockIdx.x;
  const int chunk = id % chunks_per_pair; id /= chunks_per_pair;
  const int pair = id % pairs_per_seg;
  const int seg = id / pairs_per_seg;
  const int seg_end = min((seg + 1) * g.W, g.L);
  const int a0 = seg * g.W + pair * 2 * run;
  if (a0 >= seg_end) return;
  const int na = min(run, seg_end - a0);
  const int b0 = a0 + na;
  const int nb = min(run, seg_end - b0);
  const int total = na + nb;
  const int diag0 = chunk * kMergeChunk;
  if (diag0 >= total) return;
  const int diag1 = min(diag0 + kMergeChunk, total);
  const int64_t hb = (int64_t)bh * g.L;
  int32_t* perm_out = bh < BH0 ? perm0 : (perm1 ? perm1 - (int64_t)BH0 * g.L : nullptr);
  const uint64_t* A = in + hb + a0;
  const uint64_t* Bv = in + hb + b0;

  if (threadIdx.x < 2) split[threadIdx.x] = merge_path(A, na, Bv, nb, threadIdx.x == 0 ? diag0 : diag1);
  __syncthreads();
  const int as = split[0], ae = split[1];
  const int bs = diag0 - as, be = diag1 - ae;
  const int ca = ae - as, cb = be - bs;          // ca + cb == diag1 - diag0
  const int n = ca + cb;
  {
    // the chunk's share of the two runs, side by side in LDS; the kMergeItems loads of a thread
    // are unconditional (index clamped into the chunk, n >= 1) so that they are in flight together
    uint64_t w[kMergeItems];
#pragma unroll
    for (int e = 0; e < kMergeItems; ++e) {
      const int i = min(e * kSortThreads + (int)threadIdx.x, n - 1);
      w[e] = i < ca ? A[as + i] : Bv[bs + i - ca];
    }
#pragma unroll
    for (int e = 0; e < kMergeItems; ++e) {
      const int i = e * kSortThreads + threadIdx.x;
      if (i < n) buf[i] = w[e];
    }
  }
  __syncthreads();

  const int d0 = min(threadIdx.x * kMergeItems, n);
  const int d1 = min(d0 + kMergeItems, n);
  int ia = merge_path(buf, ca, buf + ca, cb, d0);
  int ib = d0 - ia;
  // merge kMergeItems outputs into registers, then hand them back through LDS so that the
  // global stores of the workgroup are consecutive
  uint64_t res[kMergeItems];
#pragma unroll
  for (int e = 0; e < kMergeItems; ++e) {
    uint64_t va = ia < ca ? buf[ia] : ~0ull;
    uint64_t vb = ib < cb ? buf[ca + ib] : ~0ull;
    if (va < vb) { res[e] = va; ++ia; } else { res[e] = vb; ++ib; }
  }
  __syncthreads();                       // everyone is done reading the two runs
#pragma unroll
  for (int e = 0; e < kMergeItems; ++e)
    if (d0 + e < d1) buf[d0 + e] = res[e];
  __syncthreads();
  const int64_t obase = hb + a0 + diag0;
  if (perm_out) {
    for (int i = threadIdx.x; i < n; i += kSortThreads) perm_out[obase + i] = idx_of_word(buf[i]);
  } else {
    for (int i = threadIdx.x; i < n; i += kSortThreads) out[obase + i] = buf[i];
  }
}

// ---------------------------------------------------------------------------------
// The first two merge passes in one: four neighbouring sorted tiles (16384 words, 128 KB) are
// brought into LDS, merged pairwise and then into one run, and written out once, so the words
// cross the memory system one time less.  1024 threads, 16 words each: a thread finds the start
// of its 16 consecutive outputs with a merge-path search in LDS, merges them into registers, and
// the workgroup puts the registers back into LDS between the two levels.  Slots past the end of
// the segment hold the all-ones word, which sorts last (no packed word has segment field 63).
// ---------------------------------------------------------------------------------
constexpr int kQuadThreads = 1024, kQuadItems = 16, kQuadWords = 4 * kTile;
static_assert(kQuadThreads * kQuadItems == kQuadWords, "one word per thread and item");

__global__ __launch_bounds__(kQuadThreads) void merge_quads_kernel(const uint64_t* __restrict__ in,
                                                                   uint64_t* __restrict__ out,
                                                                   int32_t* __restrict__ perm0,
                                                                   int32_t* __restrict__ perm1, int BH0, SegGeom g,
                                                                   int quads_per_seg, int quads_total) {
  extern __shared__ __attribute__((aligned(16))) uint64_t quad[];       // kQuadWords
  const int t = threadIdx.x;
  // A workgroup takes quads blockIdx.x, blockIdx.x + gridDim.x, ... (two of them as launched): the words
  // of the next one are requested into registers before this one is merged, so the memory system is
  // not idle while the workgroup works in LDS.
  struct Where { const uint64_t* src; int64_t obase; int n; int32_t* perm_out; };
  auto locate = [&](int id) -> Where {
    const int per_bh = g.segs * quads_per_seg;
    const int bh = id / per_bh, r = id - bh * per_bh;
    const int seg = r / quads_per_seg, q = r - seg * quads_per_seg;
    const int seg_end = min((seg + 1) * g.W, g.L);
    const int a0 = seg * g.W + q * kQuadWords;
    const int64_t hb = (int64_t)bh * g.L;
    Where w;
    w.n = max(0, min(kQuadWords, seg_end - a0));       // 0: the segment ends before this quad
    w.src = in + hb + a0;
    w.obase = hb + a0;
    w.perm_out = bh < BH0 ? perm0 : (perm1 ? perm1 - (int64_t)BH0 * g.L : nullptr);
    return w;
  };
  auto request = [&](const Where& w, uint64_t (&v)[kQuadItems]) {
    // all sixteen loads of a thread in flight together: index clamped, padding applied at the store to LDS
    if (w.n == 0) return;                        // workgroup-uniform: nothing of this quad exists
#pragma unroll
    for (int e = 0; e < kQuadItems; ++e) v[e] = w.src[min(e * kQuadThreads + t, w.n - 1)];
  };
  int id = blockIdx.x;
  if (id >= quads_total) return;
  Where cur = locate(id);
  uint64_t v[kQuadItems];
  request(cur, v);
  for (;;) {
    const int n = cur.n;
#pragma unroll
    for (int e = 0; e < kQuadItems; ++e) quad[e * kQuadThreads + t] = e * kQuadThreads + t < n ? v[e] : ~0ull;
    const int id_next = id + (int)gridDim.x;
    Where nxt = cur;
    if (id_next < quads_total) {               // workgroup-uniform
      nxt = locate(id_next);
      request(nxt, v);
    }
    __syncthreads();
    const int d0 = t * kQuadItems;               // this thread's outputs d0 .. d0 + 15 at both levels
#pragma unroll
    for (int run = kTile; run <= 2 * kTile; run *= 2) {
      const int pb = d0 & ~(2 * run - 1);        // first word of the pair of runs these outputs belong to
      const uint64_t* A = quad + pb;
      const uint64_t* Bv = quad + pb + run;
      int ia = merge_path(A, run, Bv, run, d0 - pb);
      int ib = d0 - pb - ia;
      uint64_t res[kQuadItems];
#pragma unroll
      for (int e = 0; e < kQuadItems; ++e) {
        const uint64_t va = ia < run ? A[ia] : ~0ull;
        const uint64_t vb = ib < run ? Bv[ib] : ~0ull;
        if (va <= vb) { res[e] = va; ++ia; } else { res[e] = vb; ++ib; }
      }
      __syncthreads();                           // everyone is done reading the runs
#pragma unroll
      for (int e = 0; e < kQuadItems; ++e) quad[d0 + e] = res[e];
      __syncthreads();
    }
    if (cur.perm_out) {
      for (int i = t; i < n; i += kQuadThreads) cur.perm_out[cur.obase + i] = idx_of_word(quad[i]);
    } else {
      for (int i = t; i < n; i += kQuadThreads) out[cur.obase + i] = quad[i];
    }
    if (id_next >= quads_total) break;
    __syncthreads();                             // the stores above read LDS; the next quad overwrites it
    id = id_next;
    cur = nxt;
  }
}

__global__ void iota_kernel(int32_t* perm, int L, int64_t total) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < total) perm[i] = (int32_t)(i % L);
}

}  // namespace

size_t sort_workspace_bytes(int BH, int L) {
  return 2 * align_up((size_t)BH * L * sizeof(uint64_t), 256);
}

basa_status launch_iota_perm(int32_t* perm, int BH, int L, hipStream_t st) {
  int64_t total = (int64_t)BH * L;
  if (total == 0) return BASA_OK;
  hipLaunchKernelGGL(iota_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, perm, L, total);
  BASA_HIP_CHECK_LAUNCH("iota_kernel");
  return BASA_OK;
}

// Sort one tensor (x1 == nullptr) or two tensors of identical L, d and dtype in the same launches.
static basa_status norm_sort_impl(const TensorView& x0, const TensorView* x1, int window, const SegList& segs, int32_t* perm0,
                                  int32_t* perm1, float* keys_out, void* ws, hipStream_t st) {
  const int BH0 = x0.batch * x0.heads, BH1 = x1 ? x1->batch * x1->heads : 0, L = x0.L;
  const int BH = BH0 + BH1;
  if (BH == 0 || L == 0) return BASA_OK;
  uint64_t* buf0 = reinterpret_cast<uint64_t*>(ws);
  uint64_t* buf1 = reinterpret_cast<uint64_t*>(reinterpret_cast<char*>(ws) +
                                               align_up((size_t)BH * L * sizeof(uint64_t), 256));
  const TensorView& xb = x1 ? *x1 : x0;
  const bool bf16 = x0.dtype == BASA_BF16;
  (void)buf0;

  SegGeom g;
  g.L = L;
  g.W = (window > 0 && window < L) ? window : L;      // a segment list is sorted as one run of L
  g.segs = ceil_div(L, g.W);
  g.tiles_per_seg = ceil_div(g.W, kTile);
  const bool single = g.tiles_per_seg == 1;
  {
  ProfScope prof(K_NORM_TILE_SORT, st);
  const dim3 grid(g.segs * g.tiles_per_seg, BH);
#define BASA_KEYS(BF, D)                                                                              \
  hipLaunchKernelGGL((norm_tile_sort_kernel<BF, D>), grid, dim3(kSortThreads), 0, st, x0, xb, BH0, buf1, \
                     single ? perm0 : nullptr, single ? perm1 : nullptr, keys_out, g, segs)
  if (bf16 && x0.d == 128) BASA_KEYS(true, 128);
  else if (bf16 && x0.d == 64) BASA_KEYS(true, 64);
  else if (!bf16 && x0.d == 128) BASA_KEYS(false, 128);
  else BASA_KEYS(false, 64);
#undef BASA_KEYS
  BASA_HIP_CHECK_LAUNCH("norm_tile_sort_kernel");
  }
  if (single) return BASA_OK;

  uint64_t* src = buf1;
  uint64_t* dst = buf0;
  int run0 = kTile;
  if (g.W > 2 * kTile) {
    // more than two tiles per segment: the first two passes in one launch
    const bool last = kQuadWords >= g.W;
    const int quads_per_seg = ceil_div(g.W, kQuadWords);
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&merge_quads_kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kQuadWords * 8);
    if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(dynamic LDS)");
    ProfScope prof(K_MERGE, st);
    const int quads_total = BH * g.segs * quads_per_seg;
    hipLaunchKernelGGL(merge_quads_kernel, dim3(ceil_div(quads_total, 2)), dim3(kQuadThreads), kQuadWords * 8, st,
                       src, dst, last ? perm0 : nullptr, last ? perm1 : nullptr, BH0, g, quads_per_seg, quads_total);
    BASA_HIP_CHECK_LAUNCH("merge_quads_kernel");
    uint64_t* t = src; src = dst; dst = t;
    run0 = kQuadWords;
  }
  for (int run = run0; run < g.W; run *= 2) {
    const bool last = run * 2 >= g.W;
    const int pairs_per_seg = ceil_div(ceil_div(g.W, run), 2);
    const int chunks_per_pair = ceil_div(2 * run, kMergeChunk);
    ProfScope prof(K_MERGE, st);
    hipLaunchKernelGGL(merge_pass_kernel, dim3(g.segs * pairs_per_seg * chunks_per_pair, BH),
                       dim3(kSortThreads), 0, st, src, dst, last ? perm0 : nullptr, last ? perm1 : nullptr,
                       BH0, g, run, chunks_per_pair, pairs_per_seg);
    BASA_HIP_CHECK_LAUNCH("merge_pass_kernel");
    uint64_t* t = src; src = dst; dst = t;
  }
  return BASA_OK;
}

basa_status launch_norm_sort(const TensorView& x, int window, const SegList& segs, int32_t* perm, float* keys_out,
                             void* ws, hipStream_t st) {
  return norm_sort_impl(x, nullptr, window, segs, perm, nullptr, keys_out, ws, st);
}

basa_status launch_norm_sort2(const TensorView& q, const TensorView& k, int window, const SegList& segs,
                              int32_t* perm_q, int32_t* perm_k, void* ws, hipStream_t st) {
  return norm_sort_impl(q, &k, window, segs, perm_q, perm_k, nullptr, ws, st);
}

}  // namespace basa
