// Sampling plan and stand-alone pack kernels.
//
// The keep set of a RAD store (Section 3.2: which coordinates the random
// matrix P retains) depends only on (seed, stream_id, step, element index),
// never on data.  plan_kernel therefore draws it once per row, ahead of the
// kernel that produces the data: it generates the Philox keys of the row,
// applies the selection rule (Bernoulli threshold, or the k smallest
// (key, column) pairs for the fixed-k schemes), and leaves a keep bitmap, the
// per-256-column offsets of the packed row, and the row's entry count.
// pack_kernel (and the forward GEMM epilogue) then only test bits.
#include "common.hpp"
#include "philox.hpp"
#include "kernels.hpp"

namespace rad {

namespace {

constexpr int kPlanThreads = 256;

// exclusive prefix sum over the 256 threads of a block; *total = block sum
__device__ __forceinline__ int block_excl_scan(int v, int* total, int* smem) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int t = __shfl_up(inc, o);
    if (lane >= o) inc += t;
  }
  if (lane == 63) smem[w] = inc;
  __syncthreads();
  int woff = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < kPlanThreads / 64; ++i) {
    const int s = smem[i];
    if (i < w) woff += s;
    tot += s;
  }
  __syncthreads();
  *total = tot;
  return woff + inc - v;
}

// Tail shared by both plan kernels: bitmap row in LDS -> global bitmap,
// per-bucket offsets, row count / row pointers.
__device__ __forceinline__ void finish_row(const PlanArgs& a, int prow, const uint32_t* s_bm, int* s_scan) {
  const int tid = threadIdx.x;
  uint32_t* bm_out = a.bitmap + (size_t)prow * a.bm_pitch;
  for (int w = tid; w < a.bm_pitch; w += kPlanThreads) bm_out[w] = s_bm[w];

  int cnt = 0;                          // entries of bucket `tid`
  if (tid < a.nb) {
    const int w0 = tid * (kBucket / 32);
#pragma unroll
    for (int w = 0; w < kBucket / 32; ++w)
      if (w0 + w < a.bm_pitch) cnt += __popc(s_bm[w0 + w]);
  }
  int total;
  const int off = block_excl_scan(cnt, &total, s_scan);
  // running maximum of entries per bucket over the whole store: one atomic per row at most, and only when
  // the row raises it (a plain read first keeps the common case free of atomics)
  if (a.max_seg) {
    int mx = cnt;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = max(mx, __shfl_xor(mx, o));
    if ((tid & 63) == 0) s_scan[4 + (tid >> 6)] = mx;
    __syncthreads();
    if (tid == 0) {
      mx = max(max(s_scan[4], s_scan[5]), max(s_scan[6], s_scan[7]));
      if (mx > *reinterpret_cast<volatile int*>(a.max_seg)) atomicMax(a.max_seg, mx);
    }
  }
  uint16_t* bo = a.bucket_off + (size_t)prow * (a.nb + 1);
  if (tid < a.nb) bo[tid] = (uint16_t)off;
  if (tid == 0) bo[a.nb] = (uint16_t)total;

  if (a.scheme == kBernoulli || a.scheme == kReplacePerExample) {
    if (tid == 0) a.row_cnt[prow] = (uint32_t)total;
  } else if (a.scheme == kReplaceShared) {       // every store row of this step holds the same entries
    const int r0 = prow * a.rows_per_step;
    for (int r = tid; r < a.rows_per_step; r += kPlanThreads) a.row_cnt[r0 + r] = (uint32_t)total;
  } else if (a.scheme == kFixedKPerExample) {
    if (tid == 0) {
      a.row_ptr[prow] = (uint32_t)((uint64_t)prow * a.k);
      if (prow == a.plan_rows - 1) a.row_ptr[a.plan_rows] = (uint32_t)((uint64_t)a.plan_rows * a.k);
    }
  } else {  // shared: every store row of this step holds k entries, rows k_pitch apart
    const int r0 = prow * a.rows_per_step;
    for (int r = tid; r < a.rows_per_step; r += kPlanThreads)
      a.row_ptr[r0 + r] = (uint32_t)((uint64_t)(r0 + r) * a.k_pitch);
    if (tid == 0 && prow == a.plan_rows - 1)
      a.row_ptr[a.plan_rows * a.rows_per_step] = (uint32_t)((uint64_t)a.plan_rows * a.rows_per_step * a.k_pitch);
  }
}

__device__ __forceinline__ void or_nibble(uint32_t* s_bm, uint32_t nib, int j0, int lead) {
  if (nib == 0) return;
  if (lead == 0) {
    atomicOr(&s_bm[j0 >> 5], nib << (j0 & 31));
  } else {
#pragma unroll
    for (int w = 0; w < 4; ++w)
      if ((nib >> w) & 1u) { const int j = j0 + w; atomicOr(&s_bm[j >> 5], 1u << (j & 31)); }
  }
}

// Bernoulli: keep iff key < T.  Keys are consumed as they are generated.
__global__ __launch_bounds__(kPlanThreads) void plan_bernoulli_kernel(PlanArgs a) {
  __shared__ uint32_t s_bm[2048];      // keep bitmap of the row (cols <= 65535)
  __shared__ int s_scan[8];
  const int tid = threadIdx.x;
  const int prow = blockIdx.x;
  const int t_step = prow / a.rows_per_step, b = prow % a.rows_per_step;
  const uint32_t step = a.step0 + (uint32_t)t_step;
  const uint64_t f0 = (uint64_t)b * (uint64_t)a.cols;
  const uint64_t q0 = f0 >> 2;
  const int lead = (int)(f0 & 3);
  const int nq = (int)(((f0 + (uint64_t)a.cols - 1) >> 2) - q0) + 1;
  for (int w = tid; w < a.bm_pitch; w += kPlanThreads) s_bm[w] = 0;
  __syncthreads();
  for (int qi = tid; qi < nq; qi += kPlanThreads) {
    const u32x4 k4 = element_quad_keys(q0 + (uint64_t)qi, a.stream_id, step, a.seed_lo, a.seed_hi);
    uint32_t nib = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const int j = qi * 4 + w - lead;
      if (j >= 0 && j < a.cols && (uint64_t)(k4[w] >> a.key_shift) < a.thresh) nib |= 1u << w;
    }
    or_nibble(s_bm, nib, qi * 4 - lead, lead);
  }
  __syncthreads();
  finish_row(a, prow, s_bm, s_scan);
}

// Fixed-k: the k smallest (key, column) pairs of the row.  QPT = Philox calls
// (groups of four consecutive elements) per thread; the row's keys stay in
// registers across the radix-select passes.  FULL: the row is exactly
// QPT * 4 * 256 columns and starts on a Philox call boundary, so every register
// slot holds an element and the per-element validity tests fold away.
template <int QPT, bool FULL>
__global__ __launch_bounds__(kPlanThreads) void plan_fixedk_kernel(PlanArgs a) {
  static_assert(QPT <= 16, "keep/valid masks are 64 bits");
  __shared__ uint32_t s_bm[2048];
  __shared__ int s_hist[256];
  __shared__ int s_scan[8];
  __shared__ int s_sel[3];

  const int tid = threadIdx.x;
  const int prow = blockIdx.x;         // plan row
  int t_step, b;
  if (a.scheme == kFixedKShared) { t_step = prow; b = 0; }
  else { t_step = prow / a.rows_per_step; b = prow % a.rows_per_step; }
  const uint32_t step = a.step0 + (uint32_t)t_step;

  const uint64_t f0 = (uint64_t)b * (uint64_t)a.cols;
  const uint64_t q0 = f0 >> 2;
  const int lead = (int)(f0 & 3);
  const int nq = (int)(((f0 + (uint64_t)a.cols - 1) >> 2) - q0) + 1;

  uint32_t key[QPT * 4];
  uint64_t valid = FULL ? ~0ull : 0ull;   // bit (4i+w): element exists in this row
#pragma unroll
  for (int i = 0; i < QPT; ++i) {
    const int qi = tid + i * kPlanThreads;
    u32x4 k4 = {0, 0, 0, 0};
    if (FULL || qi < nq) k4 = element_quad_keys(q0 + (uint64_t)qi, a.stream_id, step, a.seed_lo, a.seed_hi);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      key[4 * i + w] = k4[w] >> a.key_shift;
      const int j = qi * 4 + w - lead;
      if (!FULL && qi < nq && j >= 0 && j < a.cols) valid |= 1ull << (4 * i + w);
    }
  }

  // k-th smallest key: an 8-bit radix pass on the top byte, then (the usual case: a handful of keys share
  // that byte) an exact rank among those candidates; else three more radix passes
  __shared__ uint32_t s_cand[256];
  __shared__ int s_ncand;
  uint64_t keep = 0;
  uint32_t prefix = 0, pmask = 0;
  int kk = a.k;                        // rank (1-based) still to find among matching keys
  int cnt_eq = 0;
  int shift = 24;
#pragma unroll 1
  for (; shift >= 0; shift -= 8) {
    s_hist[tid] = 0;
    if (tid == 0) s_ncand = 0;
    __syncthreads();
#pragma unroll
    for (int e = 0; e < QPT * 4; ++e)
      if (((valid >> e) & 1ull) && (key[e] & pmask) == prefix)
        atomicAdd(&s_hist[(key[e] >> shift) & 255u], 1);
    __syncthreads();
    const int h = s_hist[tid];
    int tot;
    const int excl = block_excl_scan(h, &tot, s_scan);
    if (excl < kk && kk <= excl + h) { s_sel[0] = tid; s_sel[1] = kk - excl; s_sel[2] = h; }
    __syncthreads();
    prefix |= (uint32_t)s_sel[0] << shift;
    pmask |= 255u << shift;
    kk = s_sel[1];
    cnt_eq = s_sel[2];
    __syncthreads();
    if (shift > 0 && cnt_eq <= 256) {
      // candidates: keys matching the prefix so far (any order)
#pragma unroll
      for (int e = 0; e < QPT * 4; ++e)
        if (((valid >> e) & 1ull) && (key[e] & pmask) == prefix) s_cand[atomicAdd(&s_ncand, 1)] = key[e];
      __syncthreads();
      const int n = s_ncand;
      if (tid < n) {
        const uint32_t v = s_cand[tid];
        int less = 0, leq = 0;
        for (int i = 0; i < n; ++i) { const uint32_t o = s_cand[i]; less += o < v; leq += o <= v; }
        if (less < kk && kk <= leq) { s_sel[0] = (int)v; s_sel[1] = kk - less; s_sel[2] = leq - less; }
      }
      __syncthreads();
      prefix = (uint32_t)s_sel[0];
      kk = s_sel[1];
      cnt_eq = s_sel[2];
      __syncthreads();
      break;
    }
  }
  const uint32_t thr = prefix;         // the k-th smallest key; kk of its cnt_eq copies are kept
  if (cnt_eq == kk) {
#pragma unroll
    for (int e = 0; e < QPT * 4; ++e)
      if (((valid >> e) & 1ull) && key[e] <= thr) keep |= 1ull << e;
  } else {
    // equal keys straddle the cut: the lower columns win.  Column order is
    // slot-major (i), then thread, then word.
    int before = 0;
#pragma unroll
    for (int i = 0; i < QPT; ++i) {
      int mine = 0;
#pragma unroll
      for (int w = 0; w < 4; ++w)
        if (((valid >> (4 * i + w)) & 1ull) && key[4 * i + w] == thr) ++mine;
      int tot;
      int rank = before + block_excl_scan(mine, &tot, s_scan);
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const int e = 4 * i + w;
        if (!((valid >> e) & 1ull)) continue;
        if (key[e] < thr) keep |= 1ull << e;
        else if (key[e] == thr) { if (rank < kk) keep |= 1ull << e; ++rank; }
      }
      before += tot;
    }
  }

  for (int w = tid; w < a.bm_pitch; w += kPlanThreads) s_bm[w] = 0;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < QPT; ++i)
    or_nibble(s_bm, (uint32_t)(keep >> (4 * i)) & 0xFu, (tid + i * kPlanThreads) * 4 - lead, lead);
  __syncthreads();
  finish_row(a, prow, s_bm, s_scan);
}

// With replacement (Section 3.2, the matrix P as printed): draw s of the row maps its key to the column
// floor(key * cols / 2^32).  The draws are counted per column in LDS (16-bit counters: a count cannot
// exceed k <= cols <= 16384); a column with a non-zero count is kept once, and its count goes to
// mult[row][entry] in the entry order of the row, so that whoever packs the row scales entry e by
// mult[e] * cols/k.
__global__ __launch_bounds__(kPlanThreads) void plan_replace_kernel(PlanArgs a) {
  __shared__ uint32_t s_bm[512];       // cols <= 16384
  extern __shared__ uint32_t s_cnt[];  // two 16-bit counters per word: (cols + 1) / 2 words, sized at launch
  __shared__ int s_scan[8];
  const int tid = threadIdx.x;
  const int prow = blockIdx.x;
  int t_step, b;
  if (a.scheme == kReplaceShared) { t_step = prow; b = 0; }
  else { t_step = prow / a.rows_per_step; b = prow % a.rows_per_step; }
  const uint32_t step = a.step0 + (uint32_t)t_step;
  const uint64_t f0 = (uint64_t)b * (uint64_t)a.k;       // flat index of the row's first draw
  const uint64_t q0 = f0 >> 2;
  const int lead = (int)(f0 & 3);
  const int nq = (int)(((f0 + (uint64_t)a.k - 1) >> 2) - q0) + 1;

  for (int w = tid; w < (a.cols + 1) / 2; w += kPlanThreads) s_cnt[w] = 0;
  for (int w = tid; w < a.bm_pitch; w += kPlanThreads) s_bm[w] = 0;
  __syncthreads();
  for (int qi = tid; qi < nq; qi += kPlanThreads) {
    const u32x4 k4 = element_quad_keys(q0 + (uint64_t)qi, a.stream_id, step, a.seed_lo, a.seed_hi);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const int sdraw = qi * 4 + w - lead;
      if (sdraw >= 0 && sdraw < a.k) {
        const uint32_t j = (uint32_t)(((uint64_t)k4[w] * (uint64_t)(uint32_t)a.cols) >> 32);
        atomicAdd(&s_cnt[j >> 1], 1u << (16 * (j & 1u)));
        atomicOr(&s_bm[j >> 5], 1u << (j & 31u));          // keep bitmap: the column was drawn at least once
      }
    }
  }
  __syncthreads();
  auto count_of = [&](int j) { return (s_cnt[j >> 1] >> (16 * (j & 1))) & 0xFFFFu; };
  // entry index of the first kept column of words 2t, 2t+1, then the counts in entry order
  const int w0 = 2 * tid, w1 = 2 * tid + 1;
  const uint32_t b0 = w0 < a.bm_pitch ? s_bm[w0] : 0u, b1 = w1 < a.bm_pitch ? s_bm[w1] : 0u;
  int tot;
  int rel = block_excl_scan(__popc(b0) + __popc(b1), &tot, s_scan);
  uint16_t* mrow = a.mult + (size_t)prow * a.k;
  for (uint32_t bits = b0; bits; bits &= bits - 1) mrow[rel++] = (uint16_t)count_of(w0 * 32 + (__ffs(bits) - 1));
  for (uint32_t bits = b1; bits; bits &= bits - 1) mrow[rel++] = (uint16_t)count_of(w1 * 32 + (__ffs(bits) - 1));
  finish_row(a, prow, s_bm, s_scan);
}

// row_ptr = exclusive scan of row_cnt (Bernoulli).  One block; flags overflow.
__global__ __launch_bounds__(1024) void row_scan_kernel(const uint32_t* __restrict__ row_cnt,
                                                        uint32_t* __restrict__ row_ptr, int rows,
                                                        int64_t capacity, int* __restrict__ overflow) {
  __shared__ uint32_t s_w[16];
  __shared__ uint32_t s_carry;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  if (tid == 0) s_carry = 0;
  __syncthreads();
  for (int base = 0; base < rows; base += 1024) {
    const int r = base + tid;
    const uint32_t v = r < rows ? row_cnt[r] : 0u;
    uint32_t inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      uint32_t t = __shfl_up(inc, o);
      if (lane >= o) inc += t;
    }
    if (lane == 63) s_w[w] = inc;
    __syncthreads();
    uint32_t woff = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) { const uint32_t s = s_w[i]; if (i < w) woff += s; tot += s; }
    const uint32_t carry = s_carry;
    if (r < rows) row_ptr[r] = carry + woff + inc - v;
    __syncthreads();
    if (tid == 0) s_carry = carry + tot;
    __syncthreads();
  }
  if (tid == 0) {
    row_ptr[rows] = s_carry;
    if ((int64_t)s_carry > capacity) *overflow = 1;
  }
}

template <typename T> struct Vec4;
template <> struct Vec4<float> { typedef floatx4 type; };
template <> struct Vec4<uint16_t> { typedef u32x2 type; };

__device__ __forceinline__ float load_as_f32(const float* p) { return *p; }
__device__ __forceinline__ float load_as_f32(const uint16_t* p) { return bf16_bits_to_f32(*p); }
__device__ __forceinline__ void store_from_f32(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_from_f32(uint16_t* p, float v) { *p = f32_to_bf16_bits(v); }

// One workgroup packs one row.  Wave w takes the 256-column buckets w, w+4, w+8, ... four at a time, so a
// lane has four 16-byte loads in flight; lane l owns columns 4l..4l+3 of a bucket.
template <typename T>
__global__ __launch_bounds__(256) void pack_kernel(const T* __restrict__ x, StoreView s) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  T* vals = reinterpret_cast<T*>(s.values);
  const bool vec = (s.cols & 3) == 0;
  for (int row = blockIdx.x; row < s.rows; row += gridDim.x) {     // a few thousand workgroups walk all rows
  const int prow = row * s.plan_row_stride;
  const T* xr = x + (size_t)row * s.cols;
  const uint32_t* bm = s.bitmap + (size_t)prow * s.bm_pitch;
  const uint16_t* bo = s.bucket_off + (size_t)prow * (s.nb + 1);
  const int64_t base = (int64_t)s.row_ptr[row];
  for (int b0 = w; b0 < s.nb; b0 += 16) {
    float v[4][4];
    uint32_t nib[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int bucket = b0 + 4 * u;
      const int j0 = bucket * kBucket + lane * 4;
      nib[u] = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) v[u][i] = 0.f;
      if (bucket < s.nb && j0 < s.cols) {
        nib[u] = (bm[j0 >> 5] >> (j0 & 31)) & 0xFu;
        if (vec) {
          typename Vec4<T>::type raw = *reinterpret_cast<const typename Vec4<T>::type*>(xr + j0);
          const T* e = reinterpret_cast<const T*>(&raw);
#pragma unroll
          for (int i = 0; i < 4; ++i) v[u][i] = load_as_f32(e + i);
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i) if (j0 + i < s.cols) v[u][i] = load_as_f32(xr + j0 + i);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int bucket = b0 + 4 * u;
      if (bucket >= s.nb) break;
      const int j0 = bucket * kBucket + lane * 4;
      int prefix = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) prefix += lanes_below(__ballot((nib[u] >> e) & 1u));
      // entries of lower lanes come first, then this lane's own in column order
      int rel = bo[bucket] + prefix;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if ((nib[u] >> e) & 1u) {
          const int64_t pos = base + rel;
          if (pos < s.capacity) {
            // weight of the entry: the scale, times the draw count of its column for draws with replacement
            const float wgt = s.mult ? (float)s.mult[(size_t)prow * s.mult_pitch + rel] * s.scale : s.scale;
            if (s.paired) {
              reinterpret_cast<uint32_t*>(s.values)[pos] = pair_make(f32_to_bf16_bits(v[u][e] * wgt), j0 + e);
            } else {
              store_from_f32(vals + pos, v[u][e] * wgt);
              if (!s.indices) {}
              else if (!s.idx_shared) s.indices[pos] = (uint16_t)(j0 + e);
              else if (row == 0) s.indices[rel] = (uint16_t)(j0 + e);
            }
          }
          ++rel;
        }
      }
    }
  }
  }
}

// The same for rows that are whole 16-byte vectors: a wave packs 1024 consecutive columns at a time and the
// work is organised by OUTPUT entry instead of by input column, so the cost per input element is a load and
// an LDS store.  The raw span goes to LDS with contiguous 16-byte loads; lanes 0..31 fetch the span's 32
// keep words and scan their popcounts; then output slot t finds its column by rank: a binary search for the
// word that holds the t-th kept entry, then that word's (t - entries before it)-th set bit.  Consecutive
// lanes write consecutive entries.  (Walking the set bits per input lane instead measured slower.)
// MODE: what an entry is written as (kPackIdx: value + 16-bit column; kPackPaired: one 32-bit entry;
// kPackShared: value, columns once by row 0; kPackValue: value only, for index-free stores).  MULT: draw-count
// weights.  CAPCHK: positions are checked against the capacity (Bernoulli draws).  Compile-time, so the
// per-entry loop carries no branches on the store's kind.
enum { kPackIdx = 0, kPackPaired = 1, kPackShared = 2, kPackValue = 3 };
template <typename T, int MODE, bool MULT, bool CAPCHK>
__global__ __launch_bounds__(256) void pack_span_kernel(const T* __restrict__ x, StoreView s) {
  constexpr int kSpan = 1024;
  constexpr int EPL = 16 / (int)sizeof(T);       // elements per 16-byte load
  constexpr int NLD = kSpan / (64 * EPL);        // loads per lane and span
  __shared__ __align__(16) T s_x[4][kSpan];
  __shared__ uint32_t s_word[4][32];
  __shared__ uint16_t s_cum[4][32];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  T* vals = reinterpret_cast<T*>(s.values);
  const int nspan = (s.cols + kSpan - 1) / kSpan;
  if (w >= nspan) return;                        // no block barriers below: a wave without spans may leave
  // The wave's work items are (row, span) pairs: rows blockIdx.x, + gridDim.x, ..., spans w, w + 4, ...  The
  // loads of the next item are issued before the current one is ranked and written, so that a wave always has
  // a span in flight.
  int row = blockIdx.x, sp = w;
  u32x4 raw[NLD];
  uint32_t word = 0u;
  auto fetch = [&]() {
    const T* xr = x + (size_t)row * s.cols;
    const int c0 = sp * kSpan;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int lc = (i * 64 + lane) * EPL;
      raw[i] = u32x4{0u, 0u, 0u, 0u};
      if (c0 + lc < s.cols) raw[i] = *reinterpret_cast<const u32x4*>(xr + c0 + lc);
    }
    const int wg = c0 / 32 + lane;
    word = 0u;
    if (lane < 32 && wg < s.bm_pitch) word = s.bitmap[(size_t)row * s.plan_row_stride * s.bm_pitch + wg];
  };
  if (row < s.rows) fetch();
  while (row < s.rows) {
    const int cur_row = row, c0 = sp * kSpan;
    const int prow = cur_row * s.plan_row_stride;
    const uint16_t* bo = s.bucket_off + (size_t)prow * (s.nb + 1);
    const int64_t base = (int64_t)s.row_ptr[cur_row];
#pragma unroll
    for (int i = 0; i < NLD; ++i) *reinterpret_cast<u32x4*>(&s_x[w][(i * 64 + lane) * EPL]) = raw[i];
    const int cnt = __popc(word);
    int incl = cnt;
#pragma unroll
    for (int o = 1; o < 32; o <<= 1) {           // lanes 32..63 hold zero counts
      const int up = __shfl_up(incl, o);
      if (lane >= o) incl += up;
    }
    if (lane < 32) { s_word[w][lane] = word; s_cum[w][lane] = (uint16_t)(incl - cnt); }
    const int total = __shfl(incl, 31);
    const int rel0 = bo[c0 / kBucket];           // entries of the row before this span
    sp += 4;
    if (sp >= nspan) { sp = w; row += gridDim.x; }
    if (row < s.rows) fetch();                   // the next item's loads, in flight during the ranking below
    __builtin_amdgcn_wave_barrier();
    for (int t = lane; t < total; t += 64) {
      int wi = 0;
#pragma unroll
      for (int step = 16; step > 0; step >>= 1)
        if ((int)s_cum[w][wi + step] <= t) wi += step;
      uint32_t wd = s_word[w][wi];
      for (int r = t - (int)s_cum[w][wi]; r > 0; --r) wd &= wd - 1u;     // drop the lower kept entries of the word
      const int lc = wi * 32 + (__ffs(wd) - 1);
      const int col = c0 + lc;
      const int rel = rel0 + t;
      const int64_t pos = base + rel;
      if (!CAPCHK || pos < s.capacity) {
        // weight of the entry: the scale, times the draw count of its column for draws with replacement
        const float wgt = MULT ? (float)s.mult[(size_t)prow * s.mult_pitch + rel] * s.scale : s.scale;
        const float val = load_as_f32(&s_x[w][lc]) * wgt;
        if (MODE == kPackPaired) {
          reinterpret_cast<uint32_t*>(s.values)[pos] = pair_make(f32_to_bf16_bits(val), col);
        } else {
          store_from_f32(vals + pos, val);
          if (MODE == kPackIdx) s.indices[pos] = (uint16_t)col;
          else if (MODE == kPackShared && cur_row == 0) s.indices[rel] = (uint16_t)col;
        }
      }
    }
    __builtin_amdgcn_wave_barrier();             // the wave's LDS area is reused by its next item
  }
}

// Index-free stores keep only the values of the kept entries; before the backward pass the keep bitmap is
// drawn again and this kernel rebuilds what the dW kernels read: for bf16 the 32-bit (value, column) entries,
// for fp32 the 16-bit column of every entry.  Same walk as pack_span_kernel, without the input.
template <typename T>
__global__ __launch_bounds__(256) void reindex_span_kernel(StoreView s, uint32_t* __restrict__ out_pairs,
                                                           uint16_t* __restrict__ out_idx) {
  constexpr int kSpan = 1024;
  __shared__ uint32_t s_word[4][32];
  __shared__ uint16_t s_cum[4][32];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const T* vals = reinterpret_cast<const T*>(s.values);
  const int nspan = (s.cols + kSpan - 1) / kSpan;
  for (int row = blockIdx.x; row < s.rows; row += gridDim.x) {
    const int prow = row * s.plan_row_stride;
    const uint32_t* bm = s.bitmap + (size_t)prow * s.bm_pitch;
    const uint16_t* bo = s.bucket_off + (size_t)prow * (s.nb + 1);
    const int64_t base = (int64_t)s.row_ptr[row];
    for (int sp = w; sp < nspan; sp += 4) {
      const int c0 = sp * kSpan;
      uint32_t word = 0u;
      const int wg = c0 / 32 + lane;
      if (lane < 32 && wg < s.bm_pitch) word = bm[wg];
      const int cnt = __popc(word);
      int incl = cnt;
#pragma unroll
      for (int o = 1; o < 32; o <<= 1) {
        const int up = __shfl_up(incl, o);
        if (lane >= o) incl += up;
      }
      if (lane < 32) { s_word[w][lane] = word; s_cum[w][lane] = (uint16_t)(incl - cnt); }
      const int total = __shfl(incl, 31);
      const int rel0 = bo[c0 / kBucket];
      __builtin_amdgcn_wave_barrier();
      for (int t = lane; t < total; t += 64) {
        int wi = 0;
#pragma unroll
        for (int step = 16; step > 0; step >>= 1)
          if ((int)s_cum[w][wi + step] <= t) wi += step;
        uint32_t wd = s_word[w][wi];
        for (int r = t - (int)s_cum[w][wi]; r > 0; --r) wd &= wd - 1u;
        const int col = c0 + wi * 32 + (__ffs(wd) - 1);
        const int64_t pos = base + rel0 + t;
        if (pos < s.capacity) {
          if (sizeof(T) == 2) out_pairs[pos] = pair_make((uint32_t)reinterpret_cast<const uint16_t*>(vals)[pos], col);
          else out_idx[pos] = (uint16_t)col;
        }
      }
      __builtin_amdgcn_wave_barrier();
    }
  }
}

// One workgroup per store row: clear the dense row, then scatter the row's entries into it.
template <typename T>
__global__ __launch_bounds__(256) void unpack_kernel(StoreView s, T* __restrict__ dense) {
  const int row = blockIdx.x;
  T* out = dense + (size_t)row * s.cols;
  for (int j = threadIdx.x; j < s.cols; j += 256) out[j] = T(0);
  __syncthreads();
  int64_t beg = s.row_ptr[row], end = s.row_ptr[row + 1];
  if (end > s.capacity) end = s.capacity;
  if (s.paired) {
    // the bucket of an entry follows from its position: walk the row bucket by bucket (at most 256 entries each)
    const uint32_t* ent = reinterpret_cast<const uint32_t*>(s.values);
    const uint16_t* bo = s.bucket_off + (size_t)(row * s.plan_row_stride) * (s.nb + 1);
    for (int t = 0; t < s.nb; ++t) {
      const int64_t e = beg + bo[t] + threadIdx.x;
      if (e < beg + bo[t + 1] && e < end) {
        const uint32_t u = ent[e];
        reinterpret_cast<uint16_t*>(out)[pair_col(u, t)] = (uint16_t)(u >> 16);
      }
    }
    return;
  }
  const T* vals = reinterpret_cast<const T*>(s.values);
  // shared scheme: the k columns are stored once, and a row holds k entries (its pitch may be padded)
  if (s.idx_shared && end > beg + s.shared_k) end = beg + s.shared_k;
  for (int64_t e = beg + threadIdx.x; e < end; e += 256) out[s.indices[s.idx_shared ? e - beg : e]] = vals[e];
}

// The same with the row assembled in LDS (cleared and scattered there) and written out once, in 16-byte vectors:
// rows of up to 60 KB whose length is a whole number of vectors.
template <typename T>
__global__ __launch_bounds__(256) void unpack_lds_kernel(StoreView s, T* __restrict__ dense) {
  extern __shared__ __align__(16) unsigned char s_row_raw[];
  T* const srow = reinterpret_cast<T*>(s_row_raw);
  const int row = blockIdx.x;
  const int nvec = (int)((size_t)s.cols * sizeof(T) / 16);
  u32x4* const svec = reinterpret_cast<u32x4*>(s_row_raw);
  __shared__ int s_bo[260];                // bucket offsets of the row (cols <= 65535: at most 256 buckets + 1)
  if (s.paired && (int)threadIdx.x <= s.nb)
    s_bo[threadIdx.x] = s.bucket_off[(size_t)(row * s.plan_row_stride) * (s.nb + 1) + threadIdx.x];
  const u32x4 z = {0u, 0u, 0u, 0u};
  for (int v = threadIdx.x; v < nvec; v += 256) svec[v] = z;
  int64_t beg = s.row_ptr[row], end = s.row_ptr[row + 1];
  if (end > s.capacity) end = s.capacity;
  __syncthreads();
  if (s.paired) {
    const uint32_t* ent = reinterpret_cast<const uint32_t*>(s.values);
    // entry e of the row lies in the bucket t with bo[t] <= e - beg < bo[t + 1]: every thread takes entries
    // e = beg + tid, beg + tid + 256, ... (their loads go out first) and finds their buckets by walking the
    // row's offsets, which are in LDS by then
    int t = 0;
    for (int64_t e0 = beg + threadIdx.x; e0 < end; e0 += 1024) {
      uint32_t u[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) u[q] = e0 + 256 * q < end ? ent[e0 + 256 * q] : 0u;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int rel = (int)(e0 + 256 * q - beg);
        if (e0 + 256 * q >= end) break;
        while (t + 1 < s.nb && rel >= s_bo[t + 1]) ++t;
        reinterpret_cast<uint16_t*>(srow)[pair_col(u[q], t)] = (uint16_t)(u[q] >> 16);
      }
    }
  } else {
    const T* vals = reinterpret_cast<const T*>(s.values);
    if (s.idx_shared && end > beg + s.shared_k) end = beg + s.shared_k;
    for (int64_t e = beg + threadIdx.x; e < end; e += 256) srow[s.indices[s.idx_shared ? e - beg : e]] = vals[e];
  }
  __syncthreads();
  u32x4* const out = reinterpret_cast<u32x4*>(dense + (size_t)row * s.cols);
  for (int v = threadIdx.x; v < nvec; v += 256) out[v] = svec[v];
}

// The same from the keep bitmap instead of stored columns (index-free stores whose bitmap of the current draw is
// still there): entry e of a row belongs to the row's e-th kept column.
template <typename T>
__global__ __launch_bounds__(256) void unpack_bitmap_kernel(StoreView s, T* __restrict__ dense) {
  __shared__ int s_scan[8];
  const int row = blockIdx.x;
  T* out = dense + (size_t)row * s.cols;
  const uint32_t* bm = s.bitmap + (size_t)(row * s.plan_row_stride) * s.bm_pitch;
  const T* vals = reinterpret_cast<const T*>(s.values);
  int64_t pos = s.row_ptr[row];
  for (int w0 = 0; w0 < s.bm_pitch; w0 += 256) {
    const int wi = w0 + (int)threadIdx.x;
    uint32_t word = wi < s.bm_pitch ? bm[wi] : 0u;
    int total;
    int64_t e = pos + block_excl_scan(__popc(word), &total, s_scan);
    for (int b = 0; b < 32; ++b) {
      const int col = wi * 32 + b;
      if (col < s.cols) {
        T v = T(0);
        if ((word >> b) & 1u) { if (e < s.capacity) v = vals[e]; ++e; }
        out[col] = v;
      }
    }
    pos += total;
  }
}

}  // namespace

hipError_t launch_unpack_bitmap(const StoreView& s, int dtype, void* dense, hipStream_t st) {
  if (!s.bitmap || s.paired) return hipErrorInvalidValue;
  if (dtype == kF32) hipLaunchKernelGGL(unpack_bitmap_kernel<float>, dim3(s.rows), dim3(256), 0, st, s, (float*)dense);
  else hipLaunchKernelGGL(unpack_bitmap_kernel<uint16_t>, dim3(s.rows), dim3(256), 0, st, s, (uint16_t*)dense);
  return hipGetLastError();
}

hipError_t launch_unpack(const StoreView& s, int dtype, void* dense, hipStream_t st) {
  const size_t row_bytes = (size_t)s.cols * (dtype == kF32 ? 4 : 2);
  // (the row and the bucket offsets share the 64 KB of LDS a launch gets without asking for more)
  if (row_bytes % 16 == 0 && row_bytes <= 60 * 1024 && (reinterpret_cast<uintptr_t>(dense) & 15) == 0) {
    if (dtype == kF32) hipLaunchKernelGGL(unpack_lds_kernel<float>, dim3(s.rows), dim3(256), row_bytes, st, s, (float*)dense);
    else hipLaunchKernelGGL(unpack_lds_kernel<uint16_t>, dim3(s.rows), dim3(256), row_bytes, st, s, (uint16_t*)dense);
    return hipGetLastError();
  }
  if (dtype == kF32) hipLaunchKernelGGL(unpack_kernel<float>, dim3(s.rows), dim3(256), 0, st, s, (float*)dense);
  else hipLaunchKernelGGL(unpack_kernel<uint16_t>, dim3(s.rows), dim3(256), 0, st, s, (uint16_t*)dense);
  return hipGetLastError();
}

hipError_t launch_plan(const PlanArgs& a, hipStream_t st) {
  dim3 grid(a.plan_rows), block(kPlanThreads);
  if (a.cols < 1 || a.cols > 65535) return hipErrorInvalidValue;
  if (a.scheme == kBernoulli) {
    hipLaunchKernelGGL(plan_bernoulli_kernel, grid, block, 0, st, a);
    return hipGetLastError();
  }
  if (a.scheme == kReplaceShared || a.scheme == kReplacePerExample) {
    if (a.cols > 16384 || !a.mult) return hipErrorInvalidValue;
    hipLaunchKernelGGL(plan_replace_kernel, grid, block, (size_t)((a.cols + 1) / 2) * 4, st, a);
    return hipGetLastError();
  }
  // rows start on a Philox call boundary when cols is a multiple of 4
  const int nq_max = (a.cols % 4 == 0) ? a.cols / 4 : a.cols / 4 + 2;
  const int qpt = (nq_max + kPlanThreads - 1) / kPlanThreads;
  const bool full = a.cols == qpt * 4 * kPlanThreads;     // then also a multiple of 4: rows start on a call boundary
  if (qpt <= 1) {
    if (full) hipLaunchKernelGGL((plan_fixedk_kernel<1, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((plan_fixedk_kernel<1, false>), grid, block, 0, st, a);
  } else if (qpt <= 4) {
    if (full && qpt == 4) hipLaunchKernelGGL((plan_fixedk_kernel<4, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((plan_fixedk_kernel<4, false>), grid, block, 0, st, a);
  } else if (qpt <= 16) {
    if (full && qpt == 16) hipLaunchKernelGGL((plan_fixedk_kernel<16, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((plan_fixedk_kernel<16, false>), grid, block, 0, st, a);
  } else return hipErrorInvalidValue;
  return hipGetLastError();
}

// widest row the plan kernels handle for a scheme
int plan_max_cols(int scheme) { return scheme == kBernoulli ? 65535 : 16384; }

hipError_t launch_row_scan(const uint32_t* row_cnt, uint32_t* row_ptr, int rows, int64_t capacity,
                           int* overflow, hipStream_t st) {
  hipLaunchKernelGGL(row_scan_kernel, dim3(1), dim3(1024), 0, st, row_cnt, row_ptr, rows, capacity, overflow);
  return hipGetLastError();
}

hipError_t launch_pack(const void* x, int dtype, const StoreView& s, hipStream_t st) {
  dim3 grid(s.rows), block(256);
  // a workgroup per row measured best (a capped grid whose workgroups walk lists of rows, next row's loads in
  // flight, was 3 to 25 % slower on a 65536 x 4096 stream)
  const dim3 grid_span = grid;
  const size_t row_bytes = (size_t)s.cols * (dtype == kF32 ? 4 : 2);
  if (row_bytes % 16 == 0 && (reinterpret_cast<uintptr_t>(x) & 15) == 0) {     // every row is whole 16-byte vectors
    const int mode = s.paired ? kPackPaired : s.idx_shared ? kPackShared : s.indices ? kPackIdx : kPackValue;
    const bool mult = s.mult != nullptr, chk = s.may_overflow != 0;
#define RAD_PACK_CASE(T_, MODE_, MULT_, CHK_)                                                                   \
  if (mode == MODE_ && mult == MULT_ && chk == CHK_) {                                                          \
    hipLaunchKernelGGL((pack_span_kernel<T_, MODE_, MULT_, CHK_>), grid_span, block, 0, st, (const T_*)x, s);   \
    return hipGetLastError();                                                                                   \
  }
    // draw-count weights and the capacity check never occur together (Bernoulli draws have no counts)
    if (dtype == kF32) {
      RAD_PACK_CASE(float, kPackIdx, false, false) RAD_PACK_CASE(float, kPackIdx, false, true)
      RAD_PACK_CASE(float, kPackIdx, true, false) RAD_PACK_CASE(float, kPackShared, false, false)
      RAD_PACK_CASE(float, kPackValue, false, false) RAD_PACK_CASE(float, kPackValue, false, true)
      RAD_PACK_CASE(float, kPackValue, true, false)
    } else {
      RAD_PACK_CASE(uint16_t, kPackPaired, false, false) RAD_PACK_CASE(uint16_t, kPackPaired, false, true)
      RAD_PACK_CASE(uint16_t, kPackPaired, true, false) RAD_PACK_CASE(uint16_t, kPackShared, false, false)
      RAD_PACK_CASE(uint16_t, kPackValue, false, false) RAD_PACK_CASE(uint16_t, kPackValue, false, true)
      RAD_PACK_CASE(uint16_t, kPackValue, true, false)
    }
#undef RAD_PACK_CASE
    // any other combination takes the general kernel below
  }
  if (dtype == kF32)
    hipLaunchKernelGGL(pack_kernel<float>, grid, block, 0, st, (const float*)x, s);
  else
    hipLaunchKernelGGL(pack_kernel<uint16_t>, grid, block, 0, st, (const uint16_t*)x, s);
  return hipGetLastError();
}

hipError_t launch_reindex(const StoreView& s, int dtype, uint32_t* out_pairs, uint16_t* out_idx, hipStream_t st) {
  dim3 grid(s.rows), block(256);
  if (dtype == kF32) hipLaunchKernelGGL(reindex_span_kernel<float>, grid, block, 0, st, s, out_pairs, out_idx);
  else hipLaunchKernelGGL(reindex_span_kernel<uint16_t>, grid, block, 0, st, s, out_pairs, out_idx);
  return hipGetLastError();
}

}  // namespace rad
