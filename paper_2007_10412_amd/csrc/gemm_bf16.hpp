// bf16 GEMM kernels for gfx950: ring pipeline over three LDS stages of
// BK = 32 with the slice after them in flight in registers.
//
// At iteration kt the workgroup
//   - runs the 2 x TM x TN MFMAs (v_mfma_f32_32x32x16_bf16) of slice kt from
//     LDS stage kt%3,
//   - moves slice kt+2 from registers into stage (kt+2)%3, last read before
//     the previous barrier, during the first half of the MFMAs,
//   - starts the global loads of slice kt+3 into each register as soon as it
//     is free, so a load has almost a whole iteration to arrive,
//   - reads the first fragments of slice kt+1 (complete since the previous
//     barrier), so nothing waits on LDS after the one barrier per iteration.
// The loop is unrolled three times so stages and slots are compile-time, and
// the steady state is a single basic block in which sched_group_barrier
// spreads LDS, global and address instructions between the MFMAs.  LDS loads
// and stores are written in the alternating order wanted, because the
// compiler keeps the relative order of LDS accesses it cannot prove disjoint.
#pragma once
#include <type_traits>

#include "gemm.hpp"

namespace rad {

// NS = K slices in flight in registers (1 or 3).  With three, a global load has three iterations to
// arrive; the 256x256 tile has no registers left for that and keeps one.
constexpr int kBK3 = 32;

// 16 bytes of zeros in device memory: what an out-of-bounds vector load of the ragged variants reads
static __device__ __align__(16) const uint32_t kZeroChunk[4] = {0u, 0u, 0u, 0u};

// An operand stored with its M/N index contiguous (element (row, k) at p[k*ld + row]) goes to LDS as it lies
// in memory, k-row by k-row, and is transposed on the way to the registers by ds_read_b64_tr_b16: within 16
// lanes, lane j receives in element e what lane 4e + j/4 addressed as its element j%4.  With source lane s
// pointing at k-row s/4, rows 4(s%4) .. 4(s%4)+3 of a 16-row block, lane j ends up with rows j, k = 0 .. 3:
// two such reads give the 8 consecutive k of an MFMA fragment.
//   LDS tile: [k][R rows], a k-row is R*2 bytes = R/8 chunks of 16 bytes; chunk c of k-row k sits at
// position c ^ 4(k%4), so the four k-rows one read touches fall into different 64-byte bank windows.
typedef short s16x4 __attribute__((ext_vector_type(4)));
template <int R> struct LdsMN {
  static_assert(R == 256, "a k-row is 32 chunks: two k-rows per load instruction");
  static __host__ __device__ __forceinline__ constexpr int byte_of(int row, int k) {
    return k * (R * 2) + (((row >> 3) ^ (4 * (k & 3))) << 4) + (row & 7) * 2;
  }
};

// fragment of k-step ks from a [k][R rows] tile: byte offset of this lane's first read (the second is
// 4 k-rows further)
template <int R> __device__ __forceinline__ uint32_t mn_frag_byte(int row0, int lane) {
  const int s = lane & 15, grp = lane >> 4;
  return (uint32_t)LdsMN<R>::byte_of(row0 + 16 * (grp & 1) + 4 * (s & 3), 8 * (grp >> 1) + (s >> 2));
}
__device__ __forceinline__ bf16x8 mn_frag_read(const unsigned char* tile, uint32_t lane_byte, int ks, int R2) {
  typedef __attribute__((address_space(3))) s16x4* lds_ptr;
  const unsigned char* p = tile + lane_byte + ks * 16 * R2;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * R2));
  union { struct { s16x4 l, h; } s; bf16x8 v; } u;
  u.s.l = lo; u.s.h = hi;
  return u.v;
}


// ------------------------------------------------------------------ loaders
// dense, K contiguous: element (row, k) at p[row*ld + k]
// EMODE: 0 = interior (no guards), 1 = ragged but every access a whole in-bounds or out-of-bounds 16-byte
// vector (guard by clamping the address and zeroing), 2 = generic element-wise guards.
template <int R, int EMODE, bool MASKED, int NS> struct RingLoadK {
  typedef LdsBF16<R, kBK3> L;
  static constexpr bool kTr = false;
  static constexpr int TOTAL = R * L::CH;
  static constexpr int NCH = (TOTAL + kGemmThreads - 1) / kGemmThreads;
  static constexpr int kDsWrites = NCH, kVmemReads = NCH * (MASKED ? 2 : 1);
  // vector ALU work worth spreading between MFMAs
  static constexpr int kValuCommit = 0, kValuFetch = 0;
  u32x4 v[NS][NCH];
  uint32_t mb[MASKED ? NS : 1][MASKED ? NCH : 1];   // ReLU bits of each chunk, applied at commit
  const uint16_t* p; const uint32_t* mask; uint32_t ld; int mp, r0, rmax, K;
  __device__ __forceinline__ void init(const void* ptr, int64_t ld_, const uint32_t* mask_, int mp_, int r0_,
                                       int rmax_, int K_, const StoreView&) {
    p = static_cast<const uint16_t*>(ptr); ld = (uint32_t)ld_; mask = mask_; mp = mp_; r0 = r0_; rmax = rmax_; K = K_;
  }
  __device__ __forceinline__ void bounds(int) {}
  __device__ __forceinline__ void configure(int) {}
  // KTAIL = false promises that the whole slice lies below K (every slice but the last)
  template <int SLOT, bool KTAIL = true> __device__ __forceinline__ void fetch(int k0) {
    const bool vec = (ld & 7) == 0;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = threadIdx.x + i * kGemmThreads;
      u32x4 t = {0u, 0u, 0u, 0u};
      if (MASKED) mb[SLOT][i] = 0u;
      if (TOTAL % kGemmThreads == 0 || c < TOTAL) {
        const int row = c / L::CH, kc = c % L::CH;
        const int gr = r0 + row, gk = k0 + kc * 8;
        const uint16_t* src = p + ((uint32_t)gr * ld + (uint32_t)gk);
        if (EMODE == 0) {
          t = *reinterpret_cast<const u32x4*>(src);
          if (MASKED) mb[SLOT][i] = mask_bits(mask, mp, gr, gk);
        } else if (EMODE == 1) {
          // Rows past the edge read the last valid row instead: they only feed output elements that are
          // never stored.  A chunk past K must be zero and is read from a block of zeros, so nothing here
          // waits for a load.
          const int grc = min(gr, rmax - 1);
          const uint16_t* srcc = p + ((uint32_t)grc * ld + (uint32_t)gk);
          const bool ok = !KTAIL || gk < K;
          t = *reinterpret_cast<const u32x4*>(ok ? srcc : reinterpret_cast<const uint16_t*>(kZeroChunk));
          if (MASKED) mb[SLOT][i] = mask_bits(mask, mp, grc, ok ? gk : 0);
        } else if (gr < rmax && gk < K) {
          if (vec && gk + 7 < K) t = *reinterpret_cast<const u32x4*>(src);
          else {
            uint16_t* te = reinterpret_cast<uint16_t*>(&t);
#pragma unroll
            for (int e = 0; e < 8; ++e) if (gk + e < K) te[e] = src[e];
          }
          if (MASKED) mb[SLOT][i] = mask_bits(mask, mp, gr, gk);
        }
      }
      v[SLOT][i] = t;
    }
  }
  // the commit in four steps, so the caller can alternate them with its own LDS reads
  template <int SLOT, int STEP> __device__ __forceinline__ void commit_step(uint16_t* lds) {
#pragma unroll
    for (int i = STEP; i < NCH; i += 4) {
      const int c = threadIdx.x + i * kGemmThreads;
      if (TOTAL % kGemmThreads == 0 || c < TOTAL) {
        const int row = c / L::CH, kc = c % L::CH;
        if (MASKED) mask_bf16x8(v[SLOT][i], mb[SLOT][i]);
        *reinterpret_cast<u32x4*>(&lds[L::unit(row, kc) * 8]) = v[SLOT][i];
      }
    }
  }
};

// dense, M/N contiguous: element (row, k) at p[k*ld + row].  Every thread owns a KPT(k) x 8(row) block
// (KPT = 4 for 256-row tiles, 2 for 128-row tiles, so that all 256 threads have one and the code is free
// of predicates) and transposes it in registers: LDS receives, for each of the 8 rows, KPT consecutive k.
template <int R, int EMODE, bool MASKED, int NS> struct RingLoadMN {
  typedef LdsBF16<R, kBK3> L;
  static constexpr bool kTr = false;
  static constexpr int RB = R / 8;               // row blocks
  static constexpr int KPT = R / 64;             // k rows per thread
  static_assert(RB * (kBK3 / KPT) == kGemmThreads, "one block per thread");
  static constexpr int kDsWrites = 8, kVmemReads = KPT * (MASKED ? 2 : 1);
  static constexpr int kValuCommit = 40, kValuFetch = 8;
  // Which block a thread owns: the SUB threads that share one 16-byte unit (k sub-positions) are neighbours,
  // the row blocks follow, and a wave fills unit column w; one write instruction then covers rows 8 apart
  // at every k sub-position, which the tile layout spreads over all banks.
  static constexpr int SUB = 8 / KPT;
  static_assert(RB * SUB == 64, "a wave covers every row block at one unit column");
  static __device__ __forceinline__ int block_rb() { return (threadIdx.x & 63) / SUB; }
  static __device__ __forceinline__ int block_kq() { return (threadIdx.x >> 6) * SUB + (threadIdx.x & 63) % SUB; }
  u32x4 v[NS][KPT];                          // v[..][kk] = 8 consecutive rows at k = kq*KPT + kk
  uint32_t mb[MASKED ? NS : 1][MASKED ? KPT : 1];
  const uint16_t* p; const uint32_t* mask; uint32_t ld; int mp, r0, rmax, K;
  __device__ __forceinline__ void init(const void* ptr, int64_t ld_, const uint32_t* mask_, int mp_, int r0_,
                                       int rmax_, int K_, const StoreView&) {
    p = static_cast<const uint16_t*>(ptr); ld = (uint32_t)ld_; mask = mask_; mp = mp_; r0 = r0_; rmax = rmax_; K = K_;
  }
  __device__ __forceinline__ void bounds(int) {}
  __device__ __forceinline__ void configure(int) {}
  template <int SLOT, bool KTAIL = true> __device__ __forceinline__ void fetch(int k0) {
    const bool vec = (ld & 7) == 0;
    const int rb = block_rb(), kq = block_kq();
    const int gr = r0 + rb * 8;
#pragma unroll
    for (int kk = 0; kk < KPT; ++kk) {
      u32x4 t = {0u, 0u, 0u, 0u};
      const int gk = k0 + kq * KPT + kk;
      if (MASKED) mb[SLOT][kk] = 0u;
      const uint16_t* src = p + ((uint32_t)gk * ld + (uint32_t)gr);
      if (EMODE == 0) {
        t = *reinterpret_cast<const u32x4*>(src);
        if (MASKED) mb[SLOT][kk] = mask_bits(mask, mp, gk, gr);
      } else if (EMODE == 1) {
        // as in the K-contiguous loader: blocks past the edge read the last valid block, rows past K read zeros
        const int grc = min(gr, rmax - 8);
        const uint16_t* srcc = p + ((uint32_t)gk * ld + (uint32_t)grc);
        const bool ok = !KTAIL || gk < K;
        t = *reinterpret_cast<const u32x4*>(ok ? srcc : reinterpret_cast<const uint16_t*>(kZeroChunk));
        if (MASKED) mb[SLOT][kk] = mask_bits(mask, mp, ok ? gk : 0, grc);
      } else if (gk < K && gr < rmax) {
        if (vec && gr + 7 < rmax) t = *reinterpret_cast<const u32x4*>(src);
        else {
          uint16_t* te = reinterpret_cast<uint16_t*>(&t);
#pragma unroll
          for (int e = 0; e < 8; ++e) if (gr + e < rmax) te[e] = src[e];
        }
        if (MASKED) mb[SLOT][kk] = mask_bits(mask, mp, gk, gr);
      }
      v[SLOT][kk] = t;
    }
  }
  // step D transposes dword D of the block: rows 2D (low halves) and 2D+1 (high halves)
  template <int SLOT, int D> __device__ __forceinline__ void commit_step(uint16_t* lds) {
    const int rb = block_rb(), kq = block_kq();
    if (MASKED && D == 0) {
#pragma unroll
      for (int kk = 0; kk < KPT; ++kk) mask_bf16x8(v[SLOT][kk], mb[SLOT][kk]);
    }
    const int kfirst = kq * KPT;                   // first k of this thread inside the slice
    uint16_t* dlo = &lds[L::unit(rb * 8 + 2 * D, kfirst >> 3) * 8 + (kfirst & 7)];
    uint16_t* dhi = &lds[L::unit(rb * 8 + 2 * D + 1, kfirst >> 3) * 8 + (kfirst & 7)];
    if constexpr (KPT == 4) {
      u32x2 lo, hi;
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const uint32_t a = v[SLOT][2 * q][D], b = v[SLOT][2 * q + 1][D];
        lo[q] = __builtin_amdgcn_perm(b, a, 0x05040100u);   // (a.lo, b.lo)
        hi[q] = __builtin_amdgcn_perm(b, a, 0x07060302u);   // (a.hi, b.hi)
      }
      *reinterpret_cast<u32x2*>(dlo) = lo;
      *reinterpret_cast<u32x2*>(dhi) = hi;
    } else if constexpr (KPT == 2) {
      const uint32_t a = v[SLOT][0][D], b = v[SLOT][1][D];
      *reinterpret_cast<uint32_t*>(dlo) = __builtin_amdgcn_perm(b, a, 0x05040100u);
      *reinterpret_cast<uint32_t*>(dhi) = __builtin_amdgcn_perm(b, a, 0x07060302u);
    } else {
      const uint32_t a = v[SLOT][0][D];
      *dlo = (uint16_t)a;
      *dhi = (uint16_t)(a >> 16);
    }
  }
};

// dense, M/N contiguous, kept in LDS as it lies in memory (LdsMN) and transposed by the fragment reads: no
// transposition in registers, four 16-byte LDS writes per thread and slice.  256-row tiles, whole vectors only.
template <int R, int EMODE, int NS> struct RingLoadMNT {
  static_assert(R == 256 && EMODE < 2, "interior and vector-predicated variants of 256-row tiles");
  static constexpr bool kTr = true;
  static constexpr int NCH = 4;                  // 32 k-rows x 32 chunks over 256 threads
  static constexpr int kDsWrites = NCH, kVmemReads = NCH, kValuCommit = 0, kValuFetch = 0;
  u32x4 v[NS][NCH];
  const uint16_t* p; uint32_t ld; int r0, rmax, K;
  __device__ __forceinline__ void init(const void* ptr, int64_t ld_, const uint32_t*, int, int r0_, int rmax_, int K_,
                                       const StoreView&) {
    p = static_cast<const uint16_t*>(ptr); ld = (uint32_t)ld_; r0 = r0_; rmax = rmax_; K = K_;
  }
  __device__ __forceinline__ void bounds(int) {}
  __device__ __forceinline__ void configure(int) {}
  template <int SLOT, bool KTAIL = true> __device__ __forceinline__ void fetch(int k0) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int q = i * kGemmThreads + (int)threadIdx.x;
      const int gk = k0 + (q >> 5), gr = r0 + (q & 31) * 8;
      if (EMODE == 0) {
        v[SLOT][i] = *reinterpret_cast<const u32x4*>(p + ((uint32_t)gk * ld + (uint32_t)gr));
      } else {
        // as in the K-contiguous loader: chunks past the edge read the last valid chunk, k-rows past K read zeros
        const int grc = min(gr, rmax - 8);
        const bool ok = !KTAIL || gk < K;
        const uint16_t* src = p + ((uint32_t)gk * ld + (uint32_t)grc);
        v[SLOT][i] = *reinterpret_cast<const u32x4*>(ok ? src : reinterpret_cast<const uint16_t*>(kZeroChunk));
      }
    }
  }
  template <int SLOT, int STEP> __device__ __forceinline__ void commit_step(uint16_t* lds) {
    const int q = STEP * kGemmThreads + (int)threadIdx.x;
    *reinterpret_cast<u32x4*>(reinterpret_cast<unsigned char*>(lds) + LdsMN<R>::byte_of((q & 31) * 8, q >> 5)) = v[SLOT][STEP];
  }
};

// compressed store as the A operand of dW: K index = store row (example b),
// M index = column j.  The LDS tile is [row j][k b]; wave w owns the k columns
// [8w, 8w+8), one 16-byte unit of every tile row: it clears them and scatters
// into them the entries of its eight store rows (eight lanes per store row),
// so no block barrier is needed between clearing and scattering.
template <int R, int SE, int NS> struct RingLoadSparse {
  static_assert(R == kBucket && kBK3 == 32, "a tile is one bucket of the store; entries carry the 32-deep tile layout");
  typedef LdsBF16<R, kBK3> L;
  static constexpr bool kTr = false;
  static constexpr int RPW = kBK3 / 4;          // store rows per wave
  static constexpr int LPR = 64 / RPW;          // lanes per store row
  static constexpr int NZ = R / 64;             // clearing stores per lane
  static constexpr int kCap = SE * LPR;         // entries of one (store row, bucket) segment held in registers
  static constexpr int kDsWrites = NZ + SE, kVmemReads = SE + 3;
  static constexpr int kValuCommit = 4 * SE, kValuFetch = 16;
  uint32_t ent[NS][SE];                      // paired store entries: value bits << 16 | row offset in the tile
  int rem[NS];                               // entries left in the segment from this lane's first one on
  uint32_t nbeg, nend;
  uint32_t raw_base; uint16_t raw_b0, raw_b1;    // loaded by bounds(), turned into [nbeg, nend) by the next fetch
  StoreView s; int m0, K, dummy;
  __device__ __forceinline__ void init(const void*, int64_t, const uint32_t*, int, int r0_, int, int K_,
                                       const StoreView& sv) { s = sv; m0 = r0_; K = K_; dummy = 0; }
  // LDS byte offset (from the A tile) of 64 spare bytes that absorb the stores of empty register entries
  __device__ __forceinline__ void configure(int dummy_elems) { dummy = (dummy_elems + (threadIdx.x & 31)) * 2; }
  // Segment of the next slice's store row inside this tile's 256-column bucket.  Only the loads are issued
  // here; the arithmetic on them waits until the next fetch, one whole iteration later.
  __device__ __forceinline__ void bounds(int k0) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int b = k0 + w * RPW + lane / LPR;
    // no branch: rows past K read row K-1 and get an empty segment
    const int row = b < K ? b : K - 1;
    const uint16_t* bo = s.bucket_off + (size_t)(row * s.plan_row_stride) * (s.nb + 1) + m0 / kBucket;
    raw_base = s.row_ptr[row];
    raw_b0 = bo[0];
    raw_b1 = b < K ? bo[1] : (uint16_t)0;
  }
  __device__ __forceinline__ void segment() {
    const uint32_t cap = (uint32_t)s.capacity;     // an overflowed Bernoulli draw never reads past the arrays
    uint32_t b = raw_base + raw_b0, e = raw_base + raw_b1;
    e = e > cap ? cap : e;
    nbeg = b > e ? e : b; nend = e;
  }
  // A lane reads its SE entries without looking at the segment end (the store is allocated kPairPad
  // entries past its capacity); entries beyond the end are dropped at commit time.  Entries beyond kCap
  // of a segment are not handled here: the host runs the overflow kernel after this GEMM, which adds them
  // to dW (it exits at once unless the plan saw a segment that long).
  template <int SLOT, bool KTAIL = true> __device__ __forceinline__ void fetch(int) {
    segment();
    const uint32_t e0 = nbeg + (threadIdx.x & 63) % LPR;
    const uint32_t* ents = reinterpret_cast<const uint32_t*>(s.values) + e0;
    rem[SLOT] = (int)(nend - e0);
#pragma unroll
    for (int i = 0; i < SE; ++i) ent[SLOT][i] = ents[i * LPR];
  }
  // steps 0 and 1 clear the wave's unit column of the tile, steps 2 and 3 scatter the entries into it
  template <int SLOT, int STEP> __device__ __forceinline__ void commit_step(uint16_t* lds) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (STEP < 2) {
      const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int q = STEP * (NZ / 2); q < (STEP + 1) * (NZ / 2); ++q)
        *reinterpret_cast<u32x4*>(&lds[L::unit(lane + q * 64, w) * 8]) = z;
    } else {
      const int kr = w * RPW + lane / LPR;
      const uint32_t kpart = (uint32_t)(((kr >> 3) << 4) | ((kr & 7) << 1));   // byte offset of k inside a tile row
      constexpr int H = (SE + 1) / 2;
      unsigned char* const base = reinterpret_cast<unsigned char*>(lds);
#pragma unroll
      for (int i = (STEP - 2) * H; i < (STEP == 2 ? H : SE); ++i) {
        // both offsets are computed first so that the choice is a select, not a predicated region
        const uint32_t off_real = (ent[SLOT][i] & 0xFFFFu) ^ kpart;
        const uint32_t off = rem[SLOT] > i * LPR ? off_real : (uint32_t)dummy;
        *reinterpret_cast<uint16_t*>(base + off) = (uint16_t)(ent[SLOT][i] >> 16);
      }
    }
  }
};

template <int KIND, int R, int SE, int EMODE, bool MASKED, int NS> struct RingLoaderOf;
template <int R, int SE, int EMODE, bool MASKED, int NS> struct RingLoaderOf<kOpK, R, SE, EMODE, MASKED, NS> { typedef RingLoadK<R, EMODE, MASKED, NS> type; };
template <int R, int SE, int EMODE, bool MASKED, int NS> struct RingLoaderOf<kOpMN, R, SE, EMODE, MASKED, NS> {
  static constexpr bool kT = R == 256 && EMODE < 2 && !MASKED;
  // (the transposing-read loader is only named when it is the one chosen: its static_asserts)
  template <bool T, int DUMMY = 0> struct Pick { typedef RingLoadMN<R, EMODE, MASKED, NS> type; };
  template <int DUMMY> struct Pick<true, DUMMY> { typedef RingLoadMNT<R, EMODE < 2 ? EMODE : 0, NS> type; };
  typedef typename Pick<kT>::type type;
};
template <int R, int SE, int EMODE, bool MASKED, int NS> struct RingLoaderOf<kOpSparse, R, SE, EMODE, MASKED, NS> { typedef RingLoadSparse<R, SE, NS> type; };

template <class LD, int SLOT> __device__ __forceinline__ void commit_all(LD& l, uint16_t* lds) {
  l.template commit_step<SLOT, 0>(lds); l.template commit_step<SLOT, 1>(lds);
  l.template commit_step<SLOT, 2>(lds); l.template commit_step<SLOT, 3>(lds);
}

// ------------------------------------------------------------------ MFMA side
// one 32 x 16 fragment of k-step ks (0 or 1) of a 32-deep tile of R rows: a 16-byte read from the K-contiguous
// layout, or two transposing reads from the M/N-contiguous one (tr_byte: this lane's offset for the fragment)
template <bool TR, int R>
__device__ __forceinline__ bf16x8 read_frag32(const uint16_t* tile, int row0, uint32_t tr_byte, int ks, int lr, int lk) {
  if constexpr (TR) return mn_frag_read(reinterpret_cast<const unsigned char*>(tile), tr_byte, ks, R * 2);
  else return *reinterpret_cast<const bf16x8*>(&tile[LdsBF16<R, kBK3>::unit(row0 + lr, ks * 2 + lk) * 8]);
}
template <int TM, int TN, int BM, int BN, bool AT = false, bool BT = false>
__device__ __forceinline__ void load_frags32(const uint16_t* As, const uint16_t* Bs, int ks, int wm0, int wn0,
                                             bf16x8 (&a)[TM], bf16x8 (&b)[TN], const uint32_t* atr = nullptr,
                                             const uint32_t* btr = nullptr) {
  const int lane = threadIdx.x & 63, lr = lane & 31, lk = lane >> 5;
#pragma unroll
  for (int i = 0; i < TM; ++i) a[i] = read_frag32<AT, BM>(As, wm0 + i * 32, AT ? atr[i] : 0u, ks, lr, lk);
#pragma unroll
  for (int j = 0; j < TN; ++j) b[j] = read_frag32<BT, BN>(Bs, wn0 + j * 32, BT ? btr[j] : 0u, ks, lr, lk);
}

// fragments of k-step 1 of the current stage, alternated with the four commit
// steps of each loader into the stage being refilled
template <int SLOT, int TM, int TN, int BM, int BN, class LA_, class LB_>
__device__ __forceinline__ void interleave_reads_commits(const uint16_t* As, const uint16_t* Bs, uint16_t* Aw,
                                                         uint16_t* Bw, int wm0, int wn0, bf16x8 (&a)[TM],
                                                         bf16x8 (&b)[TN], LA_& la, LB_& lb) {
  typedef LdsBF16<BM, kBK3> LA; typedef LdsBF16<BN, kBK3> LB;
  const int lane = threadIdx.x & 63, lr = lane & 31, lk = lane >> 5;
  auto ra = [&](int i) { if (i < TM) a[i] = *reinterpret_cast<const bf16x8*>(&As[LA::unit(wm0 + i * 32 + lr, 2 + lk) * 8]); };
  auto rb = [&](int j) { if (j < TN) b[j] = *reinterpret_cast<const bf16x8*>(&Bs[LB::unit(wn0 + j * 32 + lr, 2 + lk) * 8]); };
  ra(0); la.template commit_step<SLOT, 0>(Aw);
  rb(0); lb.template commit_step<SLOT, 0>(Bw);
  ra(1); la.template commit_step<SLOT, 1>(Aw);
  rb(1); lb.template commit_step<SLOT, 1>(Bw);
  ra(2); la.template commit_step<SLOT, 2>(Aw);
  rb(2); lb.template commit_step<SLOT, 2>(Bw);
  ra(3); la.template commit_step<SLOT, 3>(Aw);
  rb(3); lb.template commit_step<SLOT, 3>(Bw);
}

template <int TM, int TN>
__device__ __forceinline__ void mfma_step(const bf16x8 (&a)[TM], const bf16x8 (&b)[TN], floatx16 (&acc)[TM][TN]) {
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
}

// Order of the TM x TN MFMAs of one k-step and of the TM + TN fragment reads that feed them.  Fragments are
// read a0, b0, b1, a1, b2, a2, ... and the MFMAs walk the tile in growing squares -- (0,0); (0,1), (1,0),
// (1,1); (0,2), (1,2), (2,0), (2,1), (2,2); ... -- so the q-th fragment is first needed about as many MFMAs
// into the k-step as it was read into the previous one: every LDS read has most of a k-step to arrive, where
// a row-major walk needs all of b within its first TN MFMAs.
template <int TM, int TN> struct MfmaOrder {
  static constexpr int CNT = TM * TN, NF = TM + TN;
  // m-th MFMA: returns i * TN + j
  static constexpr int at(int m) {
    if (m == 0) return 0;
    int n = 1;
    for (int s = 1; s < (TM > TN ? TM : TN); ++s) {
      if (s < TN) for (int i = 0; i < (s < TM ? s : TM); ++i) { if (n == m) return i * TN + s; ++n; }
      if (s < TM) for (int j = 0; j < (s + 1 < TN ? s + 1 : TN); ++j) { if (n == m) return s * TN + j; ++n; }
    }
    return 0;
  }
  // q-th fragment read: returns 2 * index + (1 for b, 0 for a); -1 past the last
  static constexpr int frag(int q) {
    if (q == 0) return 0;
    if (q == 1) return 1;
    int n = 2;
    for (int s = 1; s < (TM > TN ? TM : TN); ++s) {
      if (s < TN) { if (n == q) return 2 * s + 1; ++n; }
      if (s < TM) { if (n == q) return 2 * s; ++n; }
    }
    return -1;
  }
};
static_assert(MfmaOrder<4, 4>::at(4) == 0 * 4 + 2 && MfmaOrder<4, 4>::at(9) == 0 * 4 + 3 && MfmaOrder<4, 4>::at(15) == 15, "");
static_assert(MfmaOrder<4, 4>::frag(2) == 3 && MfmaOrder<4, 4>::frag(3) == 2 && MfmaOrder<4, 4>::frag(7) == 6, "");
static_assert(MfmaOrder<4, 1>::at(3) == 3 && MfmaOrder<4, 1>::frag(4) == 6 && MfmaOrder<4, 1>::frag(5) == -1, "");
static_assert(MfmaOrder<4, 2>::at(1) == 1 && MfmaOrder<4, 2>::at(2) == 2 && MfmaOrder<4, 2>::at(7) == 7, "");

// The MFMAs of one half iteration are issued in eight pieces, each followed by its share of the other work;
// piece P takes the MFMAs m with m*8/(TM*TN) == P of that order.
template <int P, int TM, int TN>
__device__ __forceinline__ void mfma_piece(const bf16x8 (&a)[TM], const bf16x8 (&b)[TN], floatx16 (&acc)[TM][TN]) {
  constexpr int CNT = TM * TN, LO = P * CNT / 8, HI = (P + 1) * CNT / 8;
  typedef MfmaOrder<TM, TN> O;
#pragma unroll
  for (int m = LO; m < HI; ++m) {
    const int i = O::at(m) / TN, j = O::at(m) % TN;
    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  }
}
// the Q-th fragment read of a k-step: ra(i) or rb(j)
template <int Q, int TM, int TN, class RA, class RB> __device__ __forceinline__ void frag_read(RA&& ra, RB&& rb) {
  constexpr int f = MfmaOrder<TM, TN>::frag(Q);
  if constexpr (f >= 0) { if constexpr (f & 1) rb(f >> 1); else ra(f >> 1); }
}

// STAGED: the store epilogue passes the bf16 output tile through LDS (dX family)
template <int EPI, int BM, int BN, bool STAGED>
struct Gemm3Smem {
  static constexpr int STAGE = (BM + BN) * kBK3 * 2 + 128;   // + spare bytes for the sparse loader
  static constexpr int MAIN = 3 * STAGE;
  static constexpr int CT = EPI == kEpiFwd ? FwdEpiLds<uint16_t, BM, BN>::BYTES : STAGED ? BM * (BN + 8) * 2 : 0;
  static constexpr int BYTES = CT > MAIN ? CT : MAIN;
};

// Store epilogue of the dX family: the tile goes through LDS as bf16 so that global memory is written in
// whole 16-byte vectors (a lane's accumulators are 4 rows of one column, which would be 2-byte stores), and
// the ReLU bits of the layer below are applied eight columns at a time from one mask word per vector.  The mask
// words of the vectors a thread will store are asked for before the staging, so they have arrived by then; the
// staging itself is a conversion per two elements and LDS writes at constant offsets from one base per lane.
template <int BM, int BN, int TM, int TN>
__device__ __forceinline__ void epilogue_dx_staged(const GemmArgs& g, floatx16 (&acc)[TM][TN], uint16_t* ct,
                                                   int m0, int n0, int wm0, int wn0) {
  constexpr int CP = BN + 8;               // row pitch in elements: rows stay 16-byte aligned, banks shift by 4
  constexpr int CPR = BN / 8;              // 16-byte vectors per tile row
  constexpr int NV = BM * CPR / kGemmThreads;
  static_assert(BM * CPR % kGemmThreads == 0, "every thread stores the same number of vectors");
  const int lane = threadIdx.x & 63;
  uint32_t mw[(NV + 3) / 4];               // eight mask bits per vector, four vectors per register
#pragma unroll
  for (int q = 0; q < (NV + 3) / 4; ++q) mw[q] = 0u;
  if (g.c_mask) {
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int c = (int)threadIdx.x + it * kGemmThreads;
      const int row = m0 + c / CPR, col = n0 + (c % CPR) * 8;
      uint32_t wd = 0u;
      if (row < g.M && col < g.N) wd = g.c_mask[(size_t)row * g.c_mask_pitch + (col >> 5)];
      mw[it / 4] |= ((wd >> (col & 31)) & 0xFFu) << (8 * (it % 4));
    }
  }
  // the main loop ended with a barrier: no wave reads the operand stages any more
  uint16_t* const cbase = ct + (wm0 + 4 * (lane >> 5)) * CP + wn0 + (lane & 31);
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        const int r0 = i * 32 + (e >> 2) * 8 + (e & 3);
        uint16_t st[2];
        put_pair(st, acc[i][j][e], acc[i][j][e + 1]);
        cbase[r0 * CP + j * 32] = st[0];
        cbase[(r0 + 1) * CP + j * 32] = st[1];
      }
  __syncthreads();
  uint16_t* C = reinterpret_cast<uint16_t*>(g.C);
  const bool vec = (g.ldc & 7) == 0 && (reinterpret_cast<uintptr_t>(g.C) & 15) == 0;
#pragma unroll
  for (int it = 0; it < NV; ++it) {
    const int c = (int)threadIdx.x + it * kGemmThreads;
    const int r = c / CPR, ch = c % CPR;
    const int row = m0 + r, col = n0 + ch * 8;
    if (row >= g.M || col >= g.N) continue;
    u32x4 v = *reinterpret_cast<const u32x4*>(&ct[r * CP + ch * 8]);
    if (g.c_mask) mask_bf16x8(v, mw[it / 4] >> (8 * (it % 4)));
    uint16_t* dst = C + (size_t)row * g.ldc + col;
    if (vec && col + 8 <= g.N) {
      *reinterpret_cast<u32x4*>(dst) = v;
    } else {
      const uint16_t* ve = reinterpret_cast<const uint16_t*>(&v);
#pragma unroll
      for (int e = 0; e < 8; ++e) if (col + e < g.N) dst[e] = ve[e];    // (constant element numbers: v stays in registers)
    }
  }
}

template <int V> using IntC = std::integral_constant<int, V>;

template <int AK, int BKIND, int EPI, int BM, int BN, int SE, int FLAGS>
__global__ __launch_bounds__(kGemmThreads) void gemm3_bf16_kernel(GemmArgs g) {
  constexpr bool EDGE = (FLAGS & (kFlagEdge | kFlagEdgeVec)) != 0;
  constexpr int EMODE = (FLAGS & kFlagEdge) ? 2 : (FLAGS & kFlagEdgeVec) ? 1 : 0;
  constexpr int BK = kBK3;
  constexpr bool kStaged = EPI == kEpiStore && AK == kOpK;
  typedef Gemm3Smem<EPI, BM, BN, kStaged> S;
  constexpr int NS = (BM * BN >= 256 * 256) ? 1 : 3;
  typedef typename RingLoaderOf<AK, BM, SE, EMODE, (FLAGS & kFlagMaskA) != 0, NS>::type LoadA;
  typedef typename RingLoaderOf<BKIND, BN, SE, EMODE, (FLAGS & kFlagMaskB) != 0, NS>::type LoadB;
  constexpr int TM = BM / 64, TN = BN / 64;
  constexpr bool kAT = LoadA::kTr, kBT = LoadB::kTr;   // fragments of that operand come from transposing reads
  extern __shared__ __align__(16) unsigned char smem_raw[];
  uint16_t* const smem = reinterpret_cast<uint16_t*>(smem_raw);
  constexpr int kStageElems = S::STAGE / 2;
  constexpr int kAElems = BM * BK;

  // Tile order.  Workgroup ids go round-robin over the 8 XCDs, each with its own L2, so ids are first
  // regrouped into 8 contiguous chunks (one per XCD); within the sequence, tiles are walked in groups of
  // GM tile rows, column by column, so that the 32 workgroups resident on one XCD cover a GM x 32/GM block of
  // tiles and share their operand slices through that L2.
  const int tiles_n = (g.N + BN - 1) / BN, tiles_m = (g.M + BM - 1) / BM;
  const int T = tiles_m * tiles_n;
  int lin = blockIdx.x;
  if ((T & 7) == 0) lin = (lin & 7) * (T >> 3) + (lin >> 3);
  // a tile of the compressed store is a fraction of a dense operand tile, so the dW-from-store kernels
  // group tall: one XCD then streams 2 tile columns of dy instead of 8
  constexpr int GM = AK == kOpSparse ? 16 : 4;
  const int grp = lin / (GM * tiles_n), within = lin - grp * (GM * tiles_n);
  const int gh = min(GM, tiles_m - grp * GM);      // rows in this (possibly last, shorter) group
  const int tm = grp * GM + within % gh, tn = within / gh;
  const int m0 = tm * BM, n0 = tn * BN;
  const int w = threadIdx.x >> 6;
  const int wm0 = (w >> 1) * (BM / 2), wn0 = (w & 1) * (BN / 2);
  uint32_t atr[TM], btr[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) { if constexpr (kAT) atr[i] = mn_frag_byte<BM>(wm0 + i * 32, (int)(threadIdx.x & 63)); else atr[i] = 0u; }
#pragma unroll
  for (int j = 0; j < TN; ++j) { if constexpr (kBT) btr[j] = mn_frag_byte<BN>(wn0 + j * 32, (int)(threadIdx.x & 63)); else btr[j] = 0u; }

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // split K: blockIdx.y takes the K range [kbeg, kend) and the epilogue adds its partial result atomically
  const int kbeg = g.k_splits > 1 ? (int)blockIdx.y * g.k_split : 0;
  const int kend = g.k_splits > 1 ? min(g.K, kbeg + g.k_split) : g.K;
  LoadA la; LoadB lb;
  la.init(g.A, g.lda, g.a_mask, g.a_mask_pitch, m0, g.m_load > g.M ? g.m_load : g.M, kend, g.sa);
  lb.init(g.B, g.ldb, g.b_mask, g.b_mask_pitch, n0, g.N, kend, g.sa);
  la.configure((BM + BN) * BK);
  const int KT = (kend - kbeg + BK - 1) / BK;

  bf16x8 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
  // one iteration; R_ = kt % 3 fixes the LDS stages at compile time
  auto body = [&](auto R_, auto STEADY_, int kt) {
    constexpr int r = decltype(R_)::value;
    constexpr bool steady = decltype(STEADY_)::value;
    constexpr int s_nxt = (r + 1) % 3, s_wr = (r + 2) % 3;
    constexpr int sl = NS == 3 ? r : 0;              // register slot that holds slice kt+2
    uint16_t* const cur = smem + r * kStageElems;
    uint16_t* const nxt = smem + s_nxt * kStageElems;
    uint16_t* const wr = smem + s_wr * kStageElems;
    if constexpr (steady && AK == kOpK && BKIND == kOpK) {
      // two K-contiguous operands: little besides loads and stores to place, and group hints measured best
      interleave_reads_commits<sl, TM, TN, BM, BN>(cur, cur + kAElems, wr, wr + kAElems, wm0, wn0, fa1, fb1, la, lb);
      // the slot is free again: the loads of slice kt+2+NS start now and have NS iterations to arrive
      la.template fetch<sl, false>(kbeg + (kt + 2 + NS) * BK); lb.template fetch<sl, false>(kbeg + (kt + 2 + NS) * BK);
      la.bounds(kbeg + (kt + 3 + NS) * BK);
      mfma_step<TM, TN>(fa0, fb0, acc);
      load_frags32<TM, TN, BM, BN, kAT, kBT>(nxt, nxt + kAElems, 0, wm0, wn0, fa0, fb0, atr, btr);
      mfma_step<TM, TN>(fa1, fb1, acc);
      constexpr int kPairs = TM * TN / 2;             // MFMA pairs per half
      constexpr int kDsw = (LoadA::kDsWrites + LoadB::kDsWrites + kPairs - 1) / kPairs;
      constexpr int kVm = (LoadA::kVmemReads + LoadB::kVmemReads + kPairs - 1) / kPairs;
      constexpr int kDsr = (TM + TN + kPairs - 1) / kPairs;
      constexpr int kVc = (LoadA::kValuCommit + LoadB::kValuCommit + LoadA::kValuFetch + LoadB::kValuFetch + kPairs - 1) / kPairs;
#pragma unroll
      for (int i = 0; i < kPairs; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);      // 2 MFMA
        if (kVc > 0) __builtin_amdgcn_sched_group_barrier(0x002, kVc, 0);   // address / unpack arithmetic
        __builtin_amdgcn_sched_group_barrier(0x100, kDsr, 0);   // LDS reads (fragments of k-step 1)
        __builtin_amdgcn_sched_group_barrier(0x200, kDsw, 0);   // LDS writes (slice kt+2)
        __builtin_amdgcn_sched_group_barrier(0x020, kVm, 0);    // global loads (slice kt+3)
      }
#pragma unroll
      for (int i = 0; i < kPairs; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);      // 2 MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, kDsr, 0);   // LDS reads (first fragments of slice kt+1)
      }
    } else if constexpr (steady) {
      // Written out piece by piece, with a scheduling fence after each, so that every pair of MFMAs is
      // followed by its share of LDS reads, LDS writes, address arithmetic and global loads whatever the
      // loaders look like (group hints alone left the commit work of the transposing and sparse loaders in
      // one burst with no MFMA in flight).
      const int lane_ = threadIdx.x & 63, lr_ = lane_ & 31, lk_ = lane_ >> 5;
      const uint16_t* const curA = cur; const uint16_t* const curB = cur + kAElems;
      const uint16_t* const nxtA = nxt; const uint16_t* const nxtB = nxt + kAElems;
      auto ra1 = [&](int i) { if (i < TM) fa1[i] = read_frag32<kAT, BM>(curA, wm0 + i * 32, atr[i < TM ? i : 0], 1, lr_, lk_); };
      auto rb1 = [&](int j) { if (j < TN) fb1[j] = read_frag32<kBT, BN>(curB, wn0 + j * 32, btr[j < TN ? j : 0], 1, lr_, lk_); };
      auto ra0 = [&](int i) { if (i < TM) fa0[i] = read_frag32<kAT, BM>(nxtA, wm0 + i * 32, atr[i < TM ? i : 0], 0, lr_, lk_); };
      auto rb0 = [&](int j) { if (j < TN) fb0[j] = read_frag32<kBT, BN>(nxtB, wn0 + j * 32, btr[j < TN ? j : 0], 0, lr_, lk_); };
      uint16_t* const wrA = wr; uint16_t* const wrB = wr + kAElems;
#define RAD_FENCE() __builtin_amdgcn_sched_barrier(0)
      // first half: MFMAs of k-step 0; fragments of k-step 1; slice kt+2 into its stage; loads of slice kt+2+NS.
      // B goes first: it is the transposing loader here, whose first step needs all of its loads, so its
      // registers are refilled at once after its last step and have the rest of the iteration to arrive.
      mfma_piece<0, TM, TN>(fa0, fb0, acc); frag_read<0, TM, TN>(ra1, rb1); lb.template commit_step<sl, 0>(wrB); RAD_FENCE();
      mfma_piece<1, TM, TN>(fa0, fb0, acc); frag_read<1, TM, TN>(ra1, rb1); lb.template commit_step<sl, 1>(wrB); RAD_FENCE();
      mfma_piece<2, TM, TN>(fa0, fb0, acc); frag_read<2, TM, TN>(ra1, rb1); lb.template commit_step<sl, 2>(wrB); RAD_FENCE();
      mfma_piece<3, TM, TN>(fa0, fb0, acc); frag_read<3, TM, TN>(ra1, rb1); lb.template commit_step<sl, 3>(wrB);
      lb.template fetch<sl, false>(kbeg + (kt + 2 + NS) * BK); RAD_FENCE();
      mfma_piece<4, TM, TN>(fa0, fb0, acc); frag_read<4, TM, TN>(ra1, rb1); la.template commit_step<sl, 0>(wrA); RAD_FENCE();
      mfma_piece<5, TM, TN>(fa0, fb0, acc); frag_read<5, TM, TN>(ra1, rb1); la.template commit_step<sl, 1>(wrA); RAD_FENCE();
      mfma_piece<6, TM, TN>(fa0, fb0, acc); frag_read<6, TM, TN>(ra1, rb1); la.template commit_step<sl, 2>(wrA); RAD_FENCE();
      mfma_piece<7, TM, TN>(fa0, fb0, acc); frag_read<7, TM, TN>(ra1, rb1); la.template commit_step<sl, 3>(wrA);
      la.template fetch<sl, false>(kbeg + (kt + 2 + NS) * BK); la.bounds(kbeg + (kt + 3 + NS) * BK); RAD_FENCE();
      // second half: MFMAs of k-step 1; first fragments of slice kt+1
      mfma_piece<0, TM, TN>(fa1, fb1, acc); frag_read<0, TM, TN>(ra0, rb0); RAD_FENCE();
      mfma_piece<1, TM, TN>(fa1, fb1, acc); frag_read<1, TM, TN>(ra0, rb0); RAD_FENCE();
      mfma_piece<2, TM, TN>(fa1, fb1, acc); frag_read<2, TM, TN>(ra0, rb0); RAD_FENCE();
      mfma_piece<3, TM, TN>(fa1, fb1, acc); frag_read<3, TM, TN>(ra0, rb0); RAD_FENCE();
      mfma_piece<4, TM, TN>(fa1, fb1, acc); frag_read<4, TM, TN>(ra0, rb0); RAD_FENCE();
      mfma_piece<5, TM, TN>(fa1, fb1, acc); frag_read<5, TM, TN>(ra0, rb0); RAD_FENCE();
      mfma_piece<6, TM, TN>(fa1, fb1, acc); frag_read<6, TM, TN>(ra0, rb0); RAD_FENCE();
      mfma_piece<7, TM, TN>(fa1, fb1, acc); frag_read<7, TM, TN>(ra0, rb0); RAD_FENCE();
#undef RAD_FENCE
    } else {
      load_frags32<TM, TN, BM, BN, kAT, kBT>(cur, cur + kAElems, 1, wm0, wn0, fa1, fb1, atr, btr);
      if (kt + 2 < KT) { commit_all<LoadA, sl>(la, wr); commit_all<LoadB, sl>(lb, wr + kAElems); }
      mfma_step<TM, TN>(fa0, fb0, acc);
      if (kt + 2 + NS < KT) {
        la.template fetch<sl>(kbeg + (kt + 2 + NS) * BK); lb.template fetch<sl>(kbeg + (kt + 2 + NS) * BK);
        la.bounds(kbeg + (kt + 3 + NS) * BK);
      }
      if (kt + 1 < KT) load_frags32<TM, TN, BM, BN, kAT, kBT>(nxt, nxt + kAElems, 0, wm0, wn0, fa0, fb0, atr, btr);
      mfma_step<TM, TN>(fa1, fb1, acc);
    }
    __syncthreads();
    // each iteration is scheduled on its own: the group pipeline above then sees exactly one iteration
    if constexpr (steady) __builtin_amdgcn_sched_barrier(0);
  };

  // prologue: slices 0 and 1 into stages 0 and 1, slices 2 .. 1+NS into the register slots (slice s lives
  // in slot (s - 2) % NS).  The long-K path is written without conditions so that the steady loop is
  // entered with a known set of loads in flight.
  // the steady loop never fetches the last slice of a ragged K: its loads carry no K predicate
  const int KTs = (EMODE == 1 && (kend - kbeg) % BK != 0) ? KT - 1 : KT;
  const bool long_k = KTs > 4 + NS;
  int kt = 0;
  if (long_k) {
    la.bounds(kbeg + 0);
    la.template fetch<0>(kbeg + 0); lb.template fetch<0>(kbeg + 0);
    la.bounds(kbeg + BK);
    commit_all<LoadA, 0>(la, smem); commit_all<LoadB, 0>(lb, smem + kAElems);
    la.template fetch<0>(kbeg + BK); lb.template fetch<0>(kbeg + BK);
    la.bounds(kbeg + 2 * BK);
    commit_all<LoadA, 0>(la, smem + kStageElems); commit_all<LoadB, 0>(lb, smem + kStageElems + kAElems);
    // The loads left in flight must be issued in the order the loop issues them (slot by slot, A before
    // B): the wait counts inside the loop are fixed at compile time from the worse of the two orders.
    __builtin_amdgcn_sched_barrier(0);
    la.template fetch<0>(kbeg + 2 * BK); lb.template fetch<0>(kbeg + 2 * BK); la.bounds(kbeg + 3 * BK);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (NS == 3) {
      la.template fetch<1>(kbeg + 3 * BK); lb.template fetch<1>(kbeg + 3 * BK); la.bounds(kbeg + 4 * BK);
      __builtin_amdgcn_sched_barrier(0);
      la.template fetch<2>(kbeg + 4 * BK); lb.template fetch<2>(kbeg + 4 * BK); la.bounds(kbeg + 5 * BK);
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
    load_frags32<TM, TN, BM, BN, kAT, kBT>(smem, smem + kAElems, 0, wm0, wn0, fa0, fb0, atr, btr);
    // steady state, inside this branch so that the loop is entered only with the loads of the
    // prologue above in flight (the wait counts in the loop are fixed from every path that reaches it)
    do {                                // all three iterations fetch a whole slice (kt+2+2+NS < KTs)
      body(IntC<0>(), std::true_type(), kt);
      body(IntC<1>(), std::true_type(), kt + 1);
      body(IntC<2>(), std::true_type(), kt + 2);
      kt += 3;
    } while (kt + 4 + NS < KTs);
  } else {
    if (KT > 0) {
      la.bounds(kbeg + 0);
      la.template fetch<0>(kbeg + 0); lb.template fetch<0>(kbeg + 0);
      la.bounds(kbeg + BK);
      commit_all<LoadA, 0>(la, smem); commit_all<LoadB, 0>(lb, smem + kAElems);
    }
    if (KT > 1) {
      la.template fetch<0>(kbeg + BK); lb.template fetch<0>(kbeg + BK);
      la.bounds(kbeg + 2 * BK);
      commit_all<LoadA, 0>(la, smem + kStageElems); commit_all<LoadB, 0>(lb, smem + kStageElems + kAElems);
    }
    if (KT > 2) { la.template fetch<0>(kbeg + 2 * BK); lb.template fetch<0>(kbeg + 2 * BK); la.bounds(kbeg + 3 * BK); }
    if constexpr (NS == 3) {
      if (KT > 3) { la.template fetch<1>(kbeg + 3 * BK); lb.template fetch<1>(kbeg + 3 * BK); la.bounds(kbeg + 4 * BK); }
      if (KT > 4) { la.template fetch<2>(kbeg + 4 * BK); lb.template fetch<2>(kbeg + 4 * BK); la.bounds(kbeg + 5 * BK); }
    }
    __syncthreads();
    if (KT > 0) load_frags32<TM, TN, BM, BN, kAT, kBT>(smem, smem + kAElems, 0, wm0, wn0, fa0, fb0, atr, btr);
  }

  for (; kt < KT; kt += 3) {          // drain; kt is a multiple of 3 here
    body(IntC<0>(), std::false_type(), kt);
    if (kt + 1 < KT) body(IntC<1>(), std::false_type(), kt + 1);
    if (kt + 2 < KT) body(IntC<2>(), std::false_type(), kt + 2);
  }

  if constexpr (EPI == kEpiStore) {
    if (g.k_splits > 1 && g.split_stride > 0) {     // this split's partial sums go, as fp32, to an array of its own
      GemmArgs gs = g;
      gs.C = static_cast<float*>(g.C) + (int64_t)blockIdx.y * g.split_stride;
      epilogue_store<TM, TN, float, EDGE, false, false, false>(gs, acc, m0, n0, wm0, wn0);
    } else if constexpr (kStaged) {
      epilogue_dx_staged<BM, BN, TM, TN>(g, acc, smem, m0, n0, wm0, wn0);
    } else {
      epilogue_store_dispatch<AK, TM, TN, uint16_t, EDGE>(g, acc, m0, n0, wm0, wn0);
    }
  } else {
    epilogue_fwd<uint16_t, BM, BN, TM, TN>(g, acc, smem, m0, n0, wm0, wn0);
  }
}

}  // namespace rad
