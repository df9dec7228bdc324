// MFMA GEMM engine for gfx950: C[M,N] = A[M,K] * B[K,N], fp32 accumulate.
//
// One workgroup of 256 threads (4 waves, 2x2) owns a BM x BN output tile and
// walks K in slices of BK through a double-buffered LDS stage.  Operands reach
// LDS through loader objects (global -> registers -> LDS), which lets the same
// main loop serve every GEMM of the RAD train step:
//   forward   y  = x W          A: x  K-contiguous   B: W  N-contiguous
//   dX           = g W^T        A: g  K-contiguous   B: W  K-contiguous
//   dW (RAD)     = x~^T g       A: compressed store  B: g  N-contiguous
//   dW (dense)   = x^T g        A: x  M-contiguous   B: g  N-contiguous
// with g = dy masked by the stored ReLU bits inside the loader.
//
// fp32 operands use v_mfma_f32_32x32x2_f32 with LDS tiles laid out [k][row]
// (one float per lane per operand); bf16 operands use v_mfma_f32_32x32x16_bf16
// with LDS tiles laid out [row][k] in 16-byte units under an XOR swizzle that
// keeps both the MFMA fragment reads (32 consecutive rows, one unit column)
// and the transposing loader's writes (rows 8 apart) spread over the banks.
#pragma once
#include <type_traits>
#include <utility>
#include "kernels.hpp"

namespace rad {

constexpr int kGemmThreads = 256;

struct F32Tag {};
struct BF16Tag {};

template <class DT> struct ElemOf;
template <> struct ElemOf<F32Tag> { typedef float type; };
template <> struct ElemOf<BF16Tag> { typedef uint16_t type; };

// ------------------------------------------------------------ LDS layouts
template <int R, int BK> struct LdsF32 {
  static constexpr int P = R + 4;               // pitch in floats, keeps 16-byte alignment
  static constexpr int BYTES = BK * P * 4;
  static __device__ __forceinline__ int at(int row, int k) { return k * P + row; }
};
template <int R, int BK> struct LdsBF16 {
  static constexpr int CH = BK / 8;             // 16-byte units per row
  static constexpr int BYTES = R * BK * 2;
  static_assert(CH == 4, "the layout functions are written for 32-deep tiles");
  static __host__ __device__ __forceinline__ constexpr int unit(int row, int kc) {
    return tile_row(row) * CH + (kc ^ tile_swz(row));
  }
};
// the paired store entries carry this layout's row offset
static_assert(LdsBF16<256, 32>::unit(0xB5, 2) * 16 == (int)(pair_code(0xB5) ^ (2u << 4)), "pair_code / LDS layout");
static_assert(LdsBF16<256, 32>::unit(0x4E, 1) * 16 == (int)(pair_code(0x4E) ^ (1u << 4)), "pair_code / LDS layout");

__device__ __forceinline__ uint32_t mask_bits(const uint32_t* mask, int pitch, int outer, int inner) {
  return mask[(size_t)outer * pitch + (inner >> 5)] >> (inner & 31);
}

// Loaders move one operand tile global -> registers (fetch) -> LDS (commit).
// EDGE = false is the interior variant: the host launches it only when every
// tile is full and every row 16-byte aligned, so it carries no predicates.
// Offsets are 32-bit element offsets from the operand base (operands are
// limited to 2^31 elements by the host).

// =========================================================== fp32 loaders
// dense, K contiguous: element (row, k) at p[row*ld + k]
template <int R, int BK, bool EDGE, bool MASKED> struct F32LoadK {
  static constexpr int TOTAL = R * BK / 4;
  static constexpr int NCH = (TOTAL + kGemmThreads - 1) / kGemmThreads;
  typedef LdsF32<R, BK> L;
  floatx4 v[NCH];
  const float* p; const uint32_t* mask; uint32_t ld; int mp, r0, rmax, K;
  __device__ __forceinline__ void init(const void* ptr, int64_t ld_, const uint32_t* mask_, int mp_, int r0_,
                                       int rmax_, int K_, const StoreView&, const GemmArgs&) {
    p = static_cast<const float*>(ptr); ld = (uint32_t)ld_; mask = mask_; mp = mp_; r0 = r0_; rmax = rmax_; K = K_;
  }
  __device__ __forceinline__ void bounds(int) {}
  __device__ __forceinline__ void fetch(int k0) {
    const bool vec = (ld & 3) == 0;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = threadIdx.x + i * kGemmThreads;
      floatx4 t = {0.f, 0.f, 0.f, 0.f};
      if (TOTAL % kGemmThreads == 0 || c < TOTAL) {
        const int row = c / (BK / 4), k4 = c % (BK / 4);
        const int gr = r0 + row, gk = k0 + k4 * 4;
        const float* src = p + ((uint32_t)gr * ld + (uint32_t)gk);
        if (!EDGE) {
          t = *reinterpret_cast<const floatx4*>(src);
        } else if (gr < rmax && gk < K) {
          if (vec && gk + 3 < K) t = *reinterpret_cast<const floatx4*>(src);
          else {
#pragma unroll
            for (int e = 0; e < 4; ++e) if (gk + e < K) t[e] = src[e];
          }
        }
        if (MASKED && (!EDGE || (gr < rmax && gk < K))) {
          const uint32_t mb = mask_bits(mask, mp, gr, gk);
#pragma unroll
          for (int e = 0; e < 4; ++e) if (!((mb >> e) & 1u)) t[e] = 0.f;
        }
      }
      v[i] = t;
    }
  }
  __device__ __forceinline__ void commit(float* lds) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = threadIdx.x + i * kGemmThreads;
      if (TOTAL % kGemmThreads == 0 || c < TOTAL) {
        const int row = c / (BK / 4), k4 = c % (BK / 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) lds[L::at(row, k4 * 4 + e)] = v[i][e];
      }
    }
  }
};

// dense, M/N contiguous: element (row, k) at p[k*ld + row]
template <int R, int BK, bool EDGE, bool MASKED> struct F32LoadMN {
  static constexpr int TOTAL = R * BK / 4;
  static constexpr int NCH = (TOTAL + kGemmThreads - 1) / kGemmThreads;
  typedef LdsF32<R, BK> L;
  floatx4 v[NCH];
  const float* p; const uint32_t* mask; uint32_t ld; int mp, r0, rmax, K;
  __device__ __forceinline__ void init(const void* ptr, int64_t ld_, const uint32_t* mask_, int mp_, int r0_,
                                       int rmax_, int K_, const StoreView&, const GemmArgs&) {
    p = static_cast<const float*>(ptr); ld = (uint32_t)ld_; mask = mask_; mp = mp_; r0 = r0_; rmax = rmax_; K = K_;
  }
  __device__ __forceinline__ void bounds(int) {}
  __device__ __forceinline__ void fetch(int k0) {
    const bool vec = (ld & 3) == 0;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = threadIdx.x + i * kGemmThreads;
      floatx4 t = {0.f, 0.f, 0.f, 0.f};
      if (TOTAL % kGemmThreads == 0 || c < TOTAL) {
        const int k = c / (R / 4), m4 = c % (R / 4);
        const int gk = k0 + k, gr = r0 + m4 * 4;
        const float* src = p + ((uint32_t)gk * ld + (uint32_t)gr);
        if (!EDGE) {
          t = *reinterpret_cast<const floatx4*>(src);
        } else if (gk < K && gr < rmax) {
          if (vec && gr + 3 < rmax) t = *reinterpret_cast<const floatx4*>(src);
          else {
#pragma unroll
            for (int e = 0; e < 4; ++e) if (gr + e < rmax) t[e] = src[e];
          }
        }
        if (MASKED && (!EDGE || (gk < K && gr < rmax))) {
          const uint32_t mb = mask_bits(mask, mp, gk, gr);
#pragma unroll
          for (int e = 0; e < 4; ++e) if (!((mb >> e) & 1u)) t[e] = 0.f;
        }
      }
      v[i] = t;
    }
  }
  __device__ __forceinline__ void commit(float* lds) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = threadIdx.x + i * kGemmThreads;
      if (TOTAL % kGemmThreads == 0 || c < TOTAL) {
        const int k = c / (R / 4), m4 = c % (R / 4);
        *reinterpret_cast<floatx4*>(&lds[L::at(m4 * 4, k)]) = v[i];
      }
    }
  }
};

// Segment of a store row that falls into one 256-column bucket.
__device__ __forceinline__ void store_segment(const StoreView& s, int row, int bucket, uint32_t* beg, uint32_t* end) {
  const uint16_t* bo = s.bucket_off + (size_t)(row * s.plan_row_stride) * (s.nb + 1) + bucket;
  const uint32_t base = s.row_ptr[row];
  uint32_t b = base + bo[0], e = base + bo[1];
  const uint32_t cap = (uint32_t)s.capacity;     // an overflowed Bernoulli draw never reads past the arrays
  if (e > cap) e = cap;
  if (b > e) b = e;
  *beg = b; *end = e;
}

// compressed store as the A operand of dW: K index = store row (example b),
// M index = column j.  Wave w owns the k rows [w*BK/4, (w+1)*BK/4) of the LDS
// tile: it clears them and scatters the entries of those store rows whose
// column falls in [m0, m0+R), so no block barrier sits between clear and scatter.
template <int R, int BK, int SE> struct F32LoadSparse {
  typedef LdsF32<R, BK> L;
  static constexpr int RPW = BK / 4;            // k rows per wave
  static constexpr int LPR = 64 / RPW;          // lanes per k row
  float val[SE]; int col[SE];
  uint32_t beg, end, nbeg, nend;
  StoreView s; int m0, K;
  __device__ __forceinline__ void init(const void*, int64_t, const uint32_t*, int, int r0_, int, int K_,
                                       const StoreView& sv, const GemmArgs&) { s = sv; m0 = r0_; K = K_; }
  __device__ __forceinline__ void bounds(int k0) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int b = k0 + w * RPW + lane / LPR;
    nbeg = nend = 0;
    if (b < K) store_segment(s, b, m0 / kBucket, &nbeg, &nend);
  }
  __device__ __forceinline__ void fetch(int) {
    const int sub = (threadIdx.x & 63) % LPR;
    beg = nbeg; end = nend;
    const float* vals = reinterpret_cast<const float*>(s.values);
#pragma unroll
    for (int i = 0; i < SE; ++i) {
      const uint32_t e = beg + sub + i * LPR;
      col[i] = -1; val[i] = 0.f;
      if (e < end) { col[i] = (int)s.indices[e] - m0; val[i] = vals[e]; }
    }
  }
  __device__ __forceinline__ void commit(float* lds) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const floatx4 z = {0.f, 0.f, 0.f, 0.f};
    for (int c = lane; c < RPW * (L::P / 4); c += 64)
      *reinterpret_cast<floatx4*>(&lds[(w * RPW) * L::P + c * 4]) = z;
    const int kr = w * RPW + lane / LPR, sub = lane % LPR;
#pragma unroll
    for (int i = 0; i < SE; ++i)
      if (col[i] >= 0 && col[i] < R) lds[L::at(col[i], kr)] = val[i];
    const float* vals = reinterpret_cast<const float*>(s.values);
    for (uint32_t e = beg + sub + SE * LPR; e < end; e += LPR) {
      const int c = (int)s.indices[e] - m0;
      if (c >= 0 && c < R) lds[L::at(c, kr)] = vals[e];
    }
  }
};

// =========================================================== bf16 helper
__device__ __forceinline__ void mask_bf16x8(u32x4& t, uint32_t mb) {
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const uint32_t keep = ((mb >> (2 * e)) & 1u ? 0x0000FFFFu : 0u) | ((mb >> (2 * e + 1)) & 1u ? 0xFFFF0000u : 0u);
    t[e] &= keep;
  }
}

// ========================================================= im2col loaders
// position index gm = b*H*W + y*W + x; reduction index gk = (c*KH + u)*KW + v;
// element = src[b][c][y+u-pad][x+v-pad], zero outside the image.
__device__ __forceinline__ float im2col_at(const float* src, const GemmArgs& g, int gm, int gk) {
  const int HW = g.cv_H * g.cv_W;
  const int b = gm / HW, yx = gm - b * HW;
  const int y = yx / g.cv_W, x = yx - y * g.cv_W;
  const int c = gk / (g.cv_KH * g.cv_KW), uv = gk - c * (g.cv_KH * g.cv_KW);
  const int u = uv / g.cv_KW, v = uv - u * g.cv_KW;
  const int yy = y + u - g.cv_pad, xx = x + v - g.cv_pad;
  if (yy < 0 || yy >= g.cv_H || xx < 0 || xx >= g.cv_W) return 0.f;
  return src[((size_t)(b * g.cv_C + c) * g.cv_H + yy) * g.cv_W + xx];
}

// A of the forward / dX convolution: tile rows are positions, LDS layout [k][row]
template <int R, int BK> struct F32LoadIm2colRows {
  static constexpr int TOTAL = R * BK / 4;
  static constexpr int NCH = (TOTAL + kGemmThreads - 1) / kGemmThreads;
  typedef LdsF32<R, BK> L;
  floatx4 v[NCH];
  const float* p; int r0, rmax, K; const GemmArgs* ga;
  __device__ __forceinline__ void init(const void* ptr, int64_t, const uint32_t*, int, int r0_, int rmax_, int K_,
                                       const StoreView&, const GemmArgs& g) {
    p = static_cast<const float*>(ptr); r0 = r0_; rmax = rmax_; K = K_; ga = &g;
  }
  __device__ __forceinline__ void bounds(int) {}
  __device__ __forceinline__ void fetch(int k0) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = threadIdx.x + i * kGemmThreads;
      floatx4 t = {0.f, 0.f, 0.f, 0.f};
      if (TOTAL % kGemmThreads == 0 || c < TOTAL) {
        const int k = c / (R / 4), m4 = c % (R / 4);
        const int gk = k0 + k;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int gm = r0 + m4 * 4 + e;
          if (gk < K && gm < rmax) t[e] = im2col_at(p, *ga, gm, gk);
        }
      }
      v[i] = t;
    }
  }
  __device__ __forceinline__ void commit(float* lds) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = threadIdx.x + i * kGemmThreads;
      if (TOTAL % kGemmThreads == 0 || c < TOTAL) {
        const int k = c / (R / 4), m4 = c % (R / 4);
        *reinterpret_cast<floatx4*>(&lds[L::at(m4 * 4, k)]) = v[i];
      }
    }
  }
};

// A of the convolution dW: tile rows are (c,u,v), the K index is the position
template <int R, int BK> struct F32LoadIm2colK {
  static constexpr int TOTAL = R * BK / 4;
  static constexpr int NCH = (TOTAL + kGemmThreads - 1) / kGemmThreads;
  typedef LdsF32<R, BK> L;
  floatx4 v[NCH];
  const float* p; int r0, rmax, K; const GemmArgs* ga;
  __device__ __forceinline__ void init(const void* ptr, int64_t, const uint32_t*, int, int r0_, int rmax_, int K_,
                                       const StoreView&, const GemmArgs& g) {
    p = static_cast<const float*>(ptr); r0 = r0_; rmax = rmax_; K = K_; ga = &g;
  }
  __device__ __forceinline__ void bounds(int) {}
  __device__ __forceinline__ void fetch(int k0) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = threadIdx.x + i * kGemmThreads;
      floatx4 t = {0.f, 0.f, 0.f, 0.f};
      if (TOTAL % kGemmThreads == 0 || c < TOTAL) {
        const int row = c / (BK / 4), k4 = c % (BK / 4);
        const int gr = r0 + row;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int gk = k0 + k4 * 4 + e;
          if (gr < rmax && gk < K) t[e] = im2col_at(p, *ga, gk, gr);
        }
      }
      v[i] = t;
    }
  }
  __device__ __forceinline__ void commit(float* lds) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = threadIdx.x + i * kGemmThreads;
      if (TOTAL % kGemmThreads == 0 || c < TOTAL) {
        const int row = c / (BK / 4), k4 = c % (BK / 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) lds[L::at(row, k4 * 4 + e)] = v[i][e];
      }
    }
  }
};

// B of the convolution dW: rows are channels n of an NCHW tensor [B][cv_N][HW], the K index is (b,yx)
template <int R, int BK> struct F32LoadKBatched {
  static constexpr int TOTAL = R * BK / 4;
  static constexpr int NCH = (TOTAL + kGemmThreads - 1) / kGemmThreads;
  typedef LdsF32<R, BK> L;
  floatx4 v[NCH];
  const float* p; int r0, rmax, K, HW, CN;
  __device__ __forceinline__ void init(const void* ptr, int64_t, const uint32_t*, int, int r0_, int rmax_, int K_,
                                       const StoreView&, const GemmArgs& g) {
    p = static_cast<const float*>(ptr); r0 = r0_; rmax = rmax_; K = K_; HW = g.cv_H * g.cv_W; CN = g.cv_N;
  }
  __device__ __forceinline__ void bounds(int) {}
  __device__ __forceinline__ void fetch(int k0) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = threadIdx.x + i * kGemmThreads;
      floatx4 t = {0.f, 0.f, 0.f, 0.f};
      if (TOTAL % kGemmThreads == 0 || c < TOTAL) {
        const int row = c / (BK / 4), k4 = c % (BK / 4);
        const int gr = r0 + row;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int gk = k0 + k4 * 4 + e;
          if (gr < rmax && gk < K) {
            const int b = gk / HW, yx = gk - b * HW;
            t[e] = p[((size_t)b * CN + gr) * HW + yx];
          }
        }
      }
      v[i] = t;
    }
  }
  __device__ __forceinline__ void commit(float* lds) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = threadIdx.x + i * kGemmThreads;
      if (TOTAL % kGemmThreads == 0 || c < TOTAL) {
        const int row = c / (BK / 4), k4 = c % (BK / 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) lds[L::at(row, k4 * 4 + e)] = v[i][e];
      }
    }
  }
};

// ================================================================ operands
template <class DT, int KIND, int R, int BK, int SE, bool EDGE, bool MASKED> struct LoaderOf;
template <int R, int BK, int SE, bool EDGE, bool MASKED> struct LoaderOf<F32Tag, kOpK, R, BK, SE, EDGE, MASKED> { typedef F32LoadK<R, BK, EDGE, MASKED> type; };
template <int R, int BK, int SE, bool EDGE, bool MASKED> struct LoaderOf<F32Tag, kOpMN, R, BK, SE, EDGE, MASKED> { typedef F32LoadMN<R, BK, EDGE, MASKED> type; };
template <int R, int BK, int SE, bool EDGE, bool MASKED> struct LoaderOf<F32Tag, kOpSparse, R, BK, SE, EDGE, MASKED> { typedef F32LoadSparse<R, BK, SE> type; };

template <int R, int BK, int SE, bool EDGE, bool MASKED> struct LoaderOf<F32Tag, kOpIm2colRows, R, BK, SE, EDGE, MASKED> { typedef F32LoadIm2colRows<R, BK> type; };
template <int R, int BK, int SE, bool EDGE, bool MASKED> struct LoaderOf<F32Tag, kOpIm2colK, R, BK, SE, EDGE, MASKED> { typedef F32LoadIm2colK<R, BK> type; };
template <int R, int BK, int SE, bool EDGE, bool MASKED> struct LoaderOf<F32Tag, kOpKBatched, R, BK, SE, EDGE, MASKED> { typedef F32LoadKBatched<R, BK> type; };

template <class DT, int R, int BK> struct LdsOf;
template <int R, int BK> struct LdsOf<F32Tag, R, BK> { typedef LdsF32<R, BK> type; };
template <int R, int BK> struct LdsOf<BF16Tag, R, BK> { typedef LdsBF16<R, BK> type; };

// ============================================================== MFMA core
// Fragments of k-step s+1 are read from LDS while the MFMAs of k-step s run
// (two fragment sets), since one wave per SIMD has nobody else to hide the
// LDS latency behind.
template <class DT, int BM, int BN, int BK> struct Mma;

template <int BM, int BN, int BK> struct Mma<F32Tag, BM, BN, BK> {
  static constexpr int TM = BM / 64, TN = BN / 64, KS = BK / 2;
  typedef LdsF32<BM, BK> LA; typedef LdsF32<BN, BK> LB;
  static __device__ __forceinline__ void run(const float* As, const float* Bs, floatx16 (&acc)[TM][TN],
                                             int wm0, int wn0) {
    const int lane = threadIdx.x & 63, lr = lane & 31, lk = lane >> 5;
    float a[2][TM], b[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) a[0][i] = As[LA::at(wm0 + i * 32 + lr, lk)];
#pragma unroll
    for (int j = 0; j < TN; ++j) b[0][j] = Bs[LB::at(wn0 + j * 32 + lr, lk)];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const int c = s & 1, n = c ^ 1;
      if (s + 1 < KS) {
#pragma unroll
        for (int i = 0; i < TM; ++i) a[n][i] = As[LA::at(wm0 + i * 32 + lr, (s + 1) * 2 + lk)];
#pragma unroll
        for (int j = 0; j < TN; ++j) b[n][j] = Bs[LB::at(wn0 + j * 32 + lr, (s + 1) * 2 + lk)];
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[c][i], b[c][j], acc[i][j], 0, 0, 0);
    }
  }
};

// ============================================================== epilogues
// what the lane at quad position CTRL (a quad_perm pattern: 0xB1 = lane ^ 1, 0x4E = lane ^ 2) holds; and what
// lane + 4 of the same row of 16 holds (zero for the last four)
template <int CTRL> __device__ __forceinline__ uint32_t quad_perm(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, CTRL, 0xF, 0xF, true);
}
__device__ __forceinline__ uint32_t row_shl4(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x104, 0xF, 0xF, true);
}

__device__ __forceinline__ void put_elem(float* p, float v) { *p = v; }
__device__ __forceinline__ void put_elem(uint16_t* p, float v) { *p = f32_to_bf16_bits(v); }
// two values to the storage dtype: bf16 pairs take the hardware conversion (round to nearest even, one
// instruction for both)
__device__ __forceinline__ void put_pair(float* p, float a, float b) { p[0] = a; p[1] = b; }
__device__ __forceinline__ void put_pair(uint16_t* p, float a, float b) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  union { bf16x2 v; uint16_t h[2]; } u;
  const f32x2 f = {a, b};
  u.v = __builtin_convertvector(f, bf16x2);
  p[0] = u.h[0]; p[1] = u.h[1];
}
__device__ __forceinline__ float get_elem(const float* p) { return *p; }
__device__ __forceinline__ float get_elem(const uint16_t* p) { return bf16_bits_to_f32(*p); }

// accumulator element i of a 32x32 block sits at row (i/4)*8 + (lane/32)*4 + i%4, column lane%32
__device__ __forceinline__ int acc_row(int i, int lane) { return (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3); }

// Plain store epilogue.  Everything that varies per call is a template flag so that each copy is straight
// code over the 16*TM*TN accumulator registers (runtime branches per element made the register allocator
// spill the accumulators): EDGE guards ragged tiles, MASK zeroes outputs whose ReLU bit is 0, BETA adds to
// what is there, MAP sends tile row r to output row row_map[r].  (Split-K partial sums never meet here: every
// split stores to an array of its own and a reduction kernel adds them in a fixed order.)
template <int TM, int TN, typename OutT, bool EDGE, bool MASK, bool BETA, bool MAP>
__device__ __forceinline__ void epilogue_store(const GemmArgs& g, floatx16 (&acc)[TM][TN], int m0, int n0,
                                               int wm0, int wn0) {
  const int lane = threadIdx.x & 63;
  OutT* C = reinterpret_cast<OutT*>(g.C);
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int row = m0 + wm0 + i * 32 + acc_row(e, lane);
      int orow = row;
      if (MAP) orow = (!EDGE || row < g.M) ? (int)g.row_map[row] : 0;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn0 + j * 32 + (lane & 31);
        if (!EDGE || (row < g.M && col < g.N)) {
          OutT* dst = C + (size_t)orow * g.ldc + col;
          float v = acc[i][j][e];
          if (MASK && !((g.c_mask[(size_t)orow * g.c_mask_pitch + (col >> 5)] >> (col & 31)) & 1u)) v = 0.f;
          if (BETA) v += get_elem(dst);
          put_elem(dst, v);
        }
      }
    }
}

// picks the copy for this call; which flags can occur depends on the GEMM family
template <int AK, int TM, int TN, typename DxT, bool EDGE>
__device__ __forceinline__ void epilogue_store_dispatch(const GemmArgs& g, floatx16 (&acc)[TM][TN], int m0, int n0,
                                                        int wm0, int wn0) {
  if constexpr (AK == kOpK) {            // dX: operand dtype out, optional ReLU mask of the layer below
    if (g.c_mask) epilogue_store<TM, TN, DxT, EDGE, true, false, false>(g, acc, m0, n0, wm0, wn0);
    else epilogue_store<TM, TN, DxT, EDGE, false, false, false>(g, acc, m0, n0, wm0, wn0);
  } else if constexpr (AK == kOpSparse) { // dW from the compressed store: fp32 out, optional accumulate
    if (g.beta) epilogue_store<TM, TN, float, EDGE, false, true, false>(g, acc, m0, n0, wm0, wn0);
    else epilogue_store<TM, TN, float, EDGE, false, false, false>(g, acc, m0, n0, wm0, wn0);
  } else {                                // dW from a dense or compact store: row map for the shared scheme
    if (g.row_map) epilogue_store<TM, TN, float, EDGE, false, true, true>(g, acc, m0, n0, wm0, wn0);
    else if (g.beta) epilogue_store<TM, TN, float, EDGE, false, true, false>(g, acc, m0, n0, wm0, wn0);
    else epilogue_store<TM, TN, float, EDGE, false, false, false>(g, acc, m0, n0, wm0, wn0);
  }
}

// LDS of the forward epilogue: the output tile in the storage dtype (row pitch padded by one 16-byte vector,
// which keeps rows aligned and shifts banks).
template <typename ElemT, int BM, int BN> struct FwdEpiLds {
  static constexpr int VPL = 16 / (int)sizeof(ElemT);     // columns per 16-byte vector
  static constexpr int CP = BN + VPL;
  static constexpr int NW = BN / 32;                      // keep words per tile row
  static constexpr int BYTES = BM * CP * (int)sizeof(ElemT);
};

// Forward epilogue.  Bias, low-rank term and ReLU are applied to the accumulators, which go through LDS in the
// storage dtype; every thread then handles 16-byte vectors of the tile (8 bf16 or 4 fp32 columns of one row):
// dense y is stored as whole vectors and the (y > 0) bits of the vector are merged with those of the
// neighbouring lanes into one word of the ReLU bit array.
// If the next layer's sample is packed here, thread r then walks tile row r: it loaded the row's keep words
// and the store position of the row's first entry in this tile before the tile was staged (so those loads
// cost no waiting), and writes the kept entries, which are consecutive in the store, one after the other.
template <typename ElemT, int BM, int BN, int TM, int TN>
__device__ __forceinline__ void epilogue_fwd(const GemmArgs& g, floatx16 (&acc)[TM][TN], ElemT* ct, int m0, int n0,
                                             int wm0, int wn0) {
  typedef FwdEpiLds<ElemT, BM, BN> E;
  constexpr int CP = E::CP, NW = E::NW, VPL = E::VPL;
  constexpr int LPR = BN / VPL;                           // lanes per tile row
  constexpr int LPW = 32 / VPL;                           // lanes per 32-column word
  static_assert(BM <= kGemmThreads, "one thread per tile row packs");
  const int lane = threadIdx.x & 63;

  // everything the epilogue reads from global memory is asked for first
  float bv[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int col = n0 + wn0 + j * 32 + (lane & 31);
    bv[j] = (g.bias && col < g.N) ? g.bias[col] : 0.f;
  }
  uint32_t kw[NW];
  uint32_t pos = 0u, row_first = 0u;
  const bool packs = g.pack && (int)threadIdx.x < BM && m0 + (int)threadIdx.x < g.M;
#pragma unroll
  for (int q = 0; q < NW; ++q) kw[q] = 0u;
  if (packs) {
    const int row = m0 + (int)threadIdx.x;
    const int prow = row * g.next.plan_row_stride;
    const uint32_t* bm_row = g.next.bitmap + (size_t)prow * g.next.bm_pitch;
    const int bucket = n0 / kBucket;
    row_first = g.next.row_ptr[row];
    pos = row_first + g.next.bucket_off[(size_t)prow * (g.next.nb + 1) + bucket];
    for (int wd = bucket * (kBucket / 32); wd < n0 / 32; ++wd) pos += __popc(bm_row[wd]);
#pragma unroll
    for (int q = 0; q < NW; ++q)
      if (n0 / 32 + q < g.next.bm_pitch) kw[q] = bm_row[n0 / 32 + q];
  }

  // The staging loop is the epilogue's arithmetic: per accumulator element it is kept to a multiply-add, a
  // maximum, half a conversion and an LDS write at a constant offset from one base address per lane (the ReLU
  // choice is a compile-time copy of the loop; the low-rank term exists in the fp32 build only, where the recurrent
  // model uses it).
  ElemT* const cbase = ct + (wm0 + 4 * (lane >> 5)) * CP + wn0 + (lane & 31);
  const int row_base = m0 + wm0 + 4 * (lane >> 5);
  auto stage = [&](auto RELU_) {
    constexpr bool kRelu = decltype(RELU_)::value;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = n0 + wn0 + j * 32 + (lane & 31);
#pragma unroll
      for (int e0 = 0; e0 < 16; e0 += 2) {                // elements e0 and e0 + 1: rows r0 and r0 + 1 of this column
        const int r0 = i * 32 + (e0 >> 2) * 8 + (e0 & 3);
        float h[2];
#pragma unroll
        for (int d = 0; d < 2; ++d) {
          h[d] = (g.out_scale != 0.f ? acc[i][j][e0 + d] * g.out_scale : acc[i][j][e0 + d]) + bv[j];
          if constexpr (std::is_same<ElemT, float>::value) {
            const int row = row_base + r0 + d;
            if (g.u_n > 0 && row < g.M && col < g.N)
              for (int q = 0; q < g.u_n; ++q) h[d] += g.u[(size_t)row * g.u_ld + q] * g.V[(size_t)q * g.N + col];
          }
          if (kRelu) h[d] = h[d] > 0.f ? h[d] : 0.f;
        }
        ElemT st[2];
        put_pair(st, h[0], h[1]);
        cbase[r0 * CP + j * 32] = st[0];
        cbase[(r0 + 1) * CP + j * 32] = st[1];
      }
    }
  };
  if (g.relu) stage(std::true_type()); else stage(std::false_type());
  __syncthreads();

  // Every thread takes 16-byte vectors of the staged tile (VPL columns of one row): dense y is stored as whole
  // vectors, and the (y > 0) bits of the vector, taken from the values as stored, are merged with those of the
  // neighbouring lanes (the LPW lanes of a 32-column word are neighbours) by lane-permuting moves.
  ElemT* Y = reinterpret_cast<ElemT*>(g.y);
  const bool yvec = Y && (g.ldy % VPL) == 0 && (reinterpret_cast<uintptr_t>(Y) & 15) == 0;
  constexpr int NV = BM * LPR / kGemmThreads;
  static_assert(BM * LPR % kGemmThreads == 0, "every thread takes the same number of vectors");
#pragma unroll
  for (int it = 0; it < NV; ++it) {
    const int c = (int)threadIdx.x + it * kGemmThreads;
    const int r = c / LPR, ch = c % LPR;
    const int row = m0 + r, col = n0 + ch * VPL;
    const int valid = (row < g.M && col < g.N) ? min(VPL, g.N - col) : 0;   // columns of this vector inside the output
    const u32x4 raw = *reinterpret_cast<const u32x4*>(&ct[r * CP + ch * VPL]);
    const ElemT* re = reinterpret_cast<const ElemT*>(&raw);
    if (Y && valid > 0) {
      ElemT* dst = Y + (size_t)row * g.ldy + col;
      if (yvec && valid == VPL) {
        *reinterpret_cast<u32x4*>(dst) = raw;
      } else {                                             // (constant element numbers: the vector stays in registers)
#pragma unroll
        for (int e = 0; e < VPL; ++e) if (e < valid) dst[e] = re[e];
      }
    }
    if (g.bits) {
      uint32_t pbits = 0u;                                 // no branches: a bit per element, then the valid ones
#pragma unroll
      for (int e = 0; e < VPL; ++e) pbits |= (get_elem(re + e) > 0.f ? 1u : 0u) << e;
      pbits &= (1u << valid) - 1u;
      uint32_t word = pbits << (VPL * (ch % LPW));
      word |= quad_perm<0xB1>(word);                       // lane ^ 1
      word |= quad_perm<0x4E>(word);                       // lane ^ 2
      if (LPW == 8) word |= row_shl4(word);                // lanes 0 .. 3 of the eight: the other quad's bits
      const int wi = col >> 5;
      if ((ch % LPW) == 0 && row < g.M && wi < g.bits_pitch) g.bits[(size_t)row * g.bits_pitch + wi] = word;
    }
  }

  if (packs) {
    const int r = (int)threadIdx.x, row = m0 + r;
    // weights of draws with replacement: the draw count of an entry, in entry order
    const uint16_t* mrow = g.next.mult ? g.next.mult + (size_t)(row * g.next.plan_row_stride) * g.next.mult_pitch : nullptr;
    uint32_t p = pos;
    const ElemT* const crow = ct + r * CP;
    auto emit = [&](int lc, ElemT raw) {
      const int col = n0 + lc;
      if (col < g.N && (int64_t)p < g.next.capacity) {
        const float wgt = mrow ? (float)mrow[p - row_first] * g.next.scale : g.next.scale;
        const float yv = get_elem(&raw) * wgt;
        if (g.next.paired) {
          reinterpret_cast<uint32_t*>(g.next.values)[p] = pair_make(f32_to_bf16_bits(yv), col);
        } else {
          put_elem(reinterpret_cast<ElemT*>(g.next.values) + p, yv);
          if (!g.next.indices) {}
          else if (!g.next.idx_shared) g.next.indices[p] = (uint16_t)col;
          else if (row == 0) g.next.indices[p - g.next.row_ptr[0]] = (uint16_t)col;
        }
      }
      ++p;
    };
#pragma unroll
    for (int q = 0; q < NW; ++q) {
      uint32_t kb = kw[q];
      while (kb) {
        // four kept columns at a time, so that their LDS reads are in flight together (__ffs(0) - 1 = -1
        // marks a slot past the last kept column)
        int e[4]; ElemT v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) { e[i] = __ffs(kb) - 1; kb &= kb - 1u; }
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = crow[q * 32 + (e[i] < 0 ? 0 : e[i])];
#pragma unroll
        for (int i = 0; i < 4; ++i) if (e[i] >= 0) emit(q * 32 + e[i], v[i]);
      }
    }
  }
}

// Convolution epilogue: tile rows are positions (b,yx) of one image (H*W is a multiple of BM), tile columns
// are output channels; the output is NCHW.  The tile goes through LDS transposed, so that a wave walks one
// channel at a time with lanes on consecutive positions: stores are contiguous and a ballot of (y > 0) is
// two words of the ReLU bit array of the example (bit index = c*H*W + yx).
template <int BM, int BN, int TM, int TN>
__device__ __forceinline__ void epilogue_conv(const GemmArgs& g, floatx16 (&acc)[TM][TN], float* ct, int m0, int n0,
                                              int wm0, int wn0) {
  constexpr int CP = BM + 1;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int lc = wn0 + j * 32 + (lane & 31);
      const int col = n0 + lc;
      const float bv = (g.bias && col < g.N) ? g.bias[col] : 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int lrow = wm0 + i * 32 + acc_row(e, lane);
        float h = acc[i][j][e] + bv;
        if (g.relu) h = h > 0.f ? h : 0.f;
        ct[lc * CP + lrow] = h;
      }
    }
  __syncthreads();
  const int HW = g.cv_H * g.cv_W;
  const int b = m0 / HW, yx0 = m0 - b * HW;
  float* Y = reinterpret_cast<float*>(g.y);
  for (int c = w; c < BN; c += 4) {
    const int co = n0 + c;
    if (co >= g.N) break;
#pragma unroll
    for (int p0 = 0; p0 < BM; p0 += 64) {
      const int pos = m0 + p0 + lane;
      const float yv = ct[c * CP + p0 + lane];
      if (pos < g.M) Y[((size_t)b * g.N + co) * HW + yx0 + p0 + lane] = yv;
      if (g.bits) {
        const uint64_t bal = __ballot(pos < g.M && yv > 0.f);
        const int wi = (co * HW + yx0 + p0) / 32;
        if (lane == 0 && wi < g.bits_pitch) g.bits[(size_t)b * g.bits_pitch + wi] = (uint32_t)bal;
        if (lane == 32 && wi + 1 < g.bits_pitch) g.bits[(size_t)b * g.bits_pitch + wi + 1] = (uint32_t)(bal >> 32);
      }
    }
  }
}

// ============================================================ the kernel
template <class DT, int AK, int BKIND, int EPI, int BM, int BN, int BK, int SE>
struct GemmSmem {
  typedef typename LdsOf<DT, BM, BK>::type LA;
  typedef typename LdsOf<DT, BN, BK>::type LB;
  typedef typename ElemOf<DT>::type ElemT;
  static constexpr int STAGE = LA::BYTES + LB::BYTES;
  static constexpr int MAIN = 2 * STAGE;
  static constexpr int CT = FwdEpiLds<ElemT, BM, BN>::BYTES;
  static constexpr int CTC = BN * (BM + 1) * 4;
  static constexpr int BYTES = (EPI == kEpiFwd && CT > MAIN) ? CT : (EPI == kEpiConv && CTC > MAIN) ? CTC : MAIN;
};

// Pipeline of one K slice (registers always hold the slice after the one in
// LDS): write slice kt+1 from registers into the idle LDS stage, start the
// global loads of slice kt+2 into the same registers, run the MFMAs of slice
// kt from the other stage, barrier.  Global latency is hidden behind a whole
// slice of MFMAs, LDS writes overlap them as well.
// FLAGS: kFlagEdge = guarded loads for ragged shapes, kFlagMaskA / kFlagMaskB =
// the dense A / B operand is masked by stored ReLU bits.  Compile-time, so the
// K loop stays one basic block the scheduler can interleave.
constexpr int kFlagEdge = 1, kFlagMaskA = 2, kFlagMaskB = 4;
// bf16 ring kernels only: ragged tiles whose operand rows are still whole 16-byte vectors (row pitch, K and
// the contiguous extent multiples of 8): loads are predicated by address clamping instead of branches
constexpr int kFlagEdgeVec = 8;

template <class DT, int AK, int BKIND, int EPI, int BM, int BN, int BK, int SE, int FLAGS>
__global__ __launch_bounds__(kGemmThreads) void gemm_kernel(GemmArgs g) {
  constexpr bool EDGE = (FLAGS & kFlagEdge) != 0;
  typedef typename ElemOf<DT>::type ElemT;
  typedef GemmSmem<DT, AK, BKIND, EPI, BM, BN, BK, SE> S;
  typedef typename LoaderOf<DT, AK, BM, BK, SE, EDGE, (FLAGS & kFlagMaskA) != 0>::type LoadA;
  typedef typename LoaderOf<DT, BKIND, BN, BK, SE, EDGE, (FLAGS & kFlagMaskB) != 0>::type LoadB;
  constexpr int TM = BM / 64, TN = BN / 64;
  extern __shared__ __align__(16) unsigned char smem_raw[];

  // tile order: N fastest inside a band of rows, so concurrently resident
  // workgroups share A rows (and the compressed-store bucket) through L2
  const int tiles_n = (g.N + BN - 1) / BN;
  const int tile = blockIdx.x;
  const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;
  const int w = threadIdx.x >> 6;
  const int wm0 = (w >> 1) * (BM / 2), wn0 = (w & 1) * (BN / 2);

  // LDS is addressed as offsets from the one dynamic-LDS symbol so that every
  // access stays in the LDS address space (ds_* instructions, own wait counter)
  ElemT* const smem = reinterpret_cast<ElemT*>(smem_raw);
  constexpr int kStageElems = S::STAGE / (int)sizeof(ElemT);
  constexpr int kAElems = S::LA::BYTES / (int)sizeof(ElemT);

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  LoadA la; LoadB lb;
  // split-K: blockIdx.y owns the K range [kbeg, kend)
  const int kbeg = g.k_splits > 1 ? (int)blockIdx.y * g.k_split : 0;
  const int kend = g.k_splits > 1 ? min(g.K, kbeg + g.k_split) : g.K;
  la.init(g.A, g.lda, g.a_mask, g.a_mask_pitch, m0, g.M, kend, g.sa, g);
  lb.init(g.B, g.ldb, g.b_mask, g.b_mask_pitch, n0, g.N, kend, g.sa, g);
  const int KT = (kend - kbeg + BK - 1) / BK;

  if (KT > 0) {
    la.bounds(kbeg);
    la.fetch(kbeg);
    lb.fetch(kbeg);
    if (KT > 1) la.bounds(kbeg + BK);
    la.commit(smem);
    lb.commit(smem + kAElems);
    if (KT > 1) {
      la.fetch(kbeg + BK);
      lb.fetch(kbeg + BK);
      if (KT > 2) la.bounds(kbeg + 2 * BK);
    }
  }
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    ElemT* const cur = smem + (kt & 1) * kStageElems;
    ElemT* const nxt = smem + ((kt & 1) ^ 1) * kStageElems;
    if (kt + 1 < KT) {
      la.commit(nxt);
      lb.commit(nxt + kAElems);
    }
    if (kt + 2 < KT) {
      la.fetch(kbeg + (kt + 2) * BK);
      lb.fetch(kbeg + (kt + 2) * BK);
      if (kt + 3 < KT) la.bounds(kbeg + (kt + 3) * BK);
    }
    Mma<DT, BM, BN, BK>::run(cur, cur + kAElems, acc, wm0, wn0);
    __syncthreads();
  }

  if constexpr (EPI == kEpiStore) {
    epilogue_store_dispatch<AK, TM, TN, ElemT, EDGE>(g, acc, m0, n0, wm0, wn0);
  } else if constexpr (EPI == kEpiSplitK) {
    GemmArgs gs = g;
    gs.C = static_cast<float*>(g.C) + (size_t)blockIdx.y * g.M * g.N;
    epilogue_store<TM, TN, float, true, false, false, false>(gs, acc, m0, n0, wm0, wn0);
  } else if constexpr (EPI == kEpiConv) {
    epilogue_conv<BM, BN, TM, TN>(g, acc, reinterpret_cast<float*>(smem), m0, n0, wm0, wn0);
  } else {
    epilogue_fwd<ElemT, BM, BN, TM, TN>(g, acc, smem, m0, n0, wm0, wn0);
  }
}


}  // namespace rad
