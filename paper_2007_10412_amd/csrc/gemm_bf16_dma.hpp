// bf16 GEMMs whose operand tiles go from global memory straight into LDS (global_load_lds_dwordx4): no
// staging registers, no LDS store instructions, no address arithmetic in the loop.  256 x 256 tiles, M a
// multiple of 256 and N too unless B is M/N-contiguous (then N may end inside the last tile column, in whole
// 16-byte vectors); everything else takes the register-staged ring kernels.
//
// A load instruction writes the 64 x 16 bytes of its wave to consecutive LDS addresses starting at M0,
// so the tile layout is produced by choosing which global chunk each lane asks for: lane l of the load
// that fills LDS units [u0, u0 + 64) fetches the chunk whose place in the layout is unit u0 + l.
// Per thread that is a constant 32-bit offset from a wave-uniform base that advances by one slice per
// iteration on the scalar unit.  The compiler does not see these loads (they are inline assembly: its own
// wait insertion would put vmcnt(0) before every LDS read that follows a load into LDS), so the waits on
// them are written out.
#pragma once
#include "gemm_bf16.hpp"

namespace rad {

// 16 bytes per lane from gbase + voff to LDS address lds + 16 * lane; gbase and lds are wave-uniform
__device__ __forceinline__ void dma16(const void* gbase, uint32_t voff, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(voff), "s"(gbase), "s"(lds) : "memory");
}
// The same in two parts, for callers that put at least one other instruction between them (an M0 write
// needs one wait state before the load that reads it; the combined form spends a nop on it).  Nothing else in
// these kernels uses M0.
__device__ __forceinline__ void dma16_aim(uint32_t lds) { asm volatile("s_mov_b32 m0, %0" :: "s"(lds) : "memory"); }
__device__ __forceinline__ void dma16_go(const void* gbase, uint32_t voff) {
  asm volatile("global_load_lds_dwordx4 %0, %1" :: "v"(voff), "s"(gbase) : "memory");
}
// the load alone with a per-lane 64-bit address (ragged last slice: lanes past K read a block of zeros)
__device__ __forceinline__ void dma16_go_at(const void* addr) {
  asm volatile("global_load_lds_dwordx4 %0, off" :: "v"(addr) : "memory");
}
template <int N> __device__ __forceinline__ void dma_wait() {   // at most N of this wave's loads still in flight
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// ------------------------------------------------------------------ 64-deep slices, two stages
// The same idea with K slices of 64 (whole 128-byte lines per row and load, half as many barriers per
// flop) in two LDS stages of 64 KB.  Iteration kt runs four k-steps of 16 on stage kt%2:
//   k-step 0: MFMAs | fragments of k-step 1 | second half of the loads of slice kt+1 into the other stage
//   k-step 1: MFMAs | fragments of k-step 2
//   k-step 2: MFMAs | fragments of k-step 3
//   wait for the loads of slice kt+1 and for the fragment reads; barrier
//   k-step 3: MFMAs | first fragments of slice kt+1 | first half of the loads of slice kt+2 into this
//             stage, which every wave has finished reading
template <int R> struct Lds64 {
  // 16-byte unit of (row, k chunk 0..7): rows are 128 bytes; the chunk is swizzled with bits 1..3 of the
  // row so that 16 consecutive rows at one chunk touch every bank once
  static __host__ __device__ __forceinline__ constexpr int unit(int row, int kc) { return row * 8 + (kc ^ ((row >> 1) & 7)); }
};

template <int R> struct DmaOperandK64 {
  static constexpr int NI = R / 32;     // loads per thread and slice: R rows x 8 units over 256 threads
  uint32_t voff[NI];
  const unsigned char* base;
  uint32_t wave_lds;
  __device__ __forceinline__ void init(const void* p, int64_t ld, int r0, int kbeg, int) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int u = i * kGemmThreads + (int)threadIdx.x;
      const int row = u >> 3, kc = (u & 7) ^ ((row >> 1) & 7);          // inverse of Lds64::unit
      voff[i] = (uint32_t)row * (uint32_t)ld * 2u + (uint32_t)kc * 16u;
    }
    base = static_cast<const unsigned char*>(p) + ((int64_t)r0 * ld + kbeg) * 2;
    wave_lds = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) * 1024u;
  }
  template <int I> __device__ __forceinline__ void issue(uint32_t lds, int k) const {
    if constexpr (I < NI) dma16(base + (int64_t)k * 2, voff[I], lds + wave_lds + (uint32_t)I * 4096u);
  }
  template <int I> __device__ __forceinline__ void aim(uint32_t lds) const {
    if constexpr (I < NI) dma16_aim(lds + wave_lds + (uint32_t)I * 4096u);
  }
  template <int I> __device__ __forceinline__ void go(int k) const {
    if constexpr (I < NI) dma16_go(base + (int64_t)k * 2, voff[I]);
  }
  // last slice of a K that is not a multiple of 64: krem valid k from the slice start on
  template <int I> __device__ __forceinline__ void go_tail(int k, int krem) const {
    if constexpr (I < NI) {
      const int u = I * kGemmThreads + (int)threadIdx.x;
      const int kc = (u & 7) ^ ((u >> 4) & 7);
      const void* src = base + (int64_t)k * 2 + voff[I];
      dma16_go_at(kc * 8 < krem ? src : static_cast<const void*>(kZeroChunk));
    }
  }
};

// M/N-contiguous operand (LdsMN layout, 64 k-rows): a load instruction fills two k-rows (1 KB); load I of
// wave w fills k-rows 2(4I + w) and 2(4I + w) + 1.
template <int R> struct DmaOperandMN64 {
  static constexpr int NI = 8;
  uint32_t voff[NI];
  const unsigned char* base;
  int64_t slice_bytes;            // 64 k-rows
  uint32_t wave_lds;
  // rmax: rows (columns of the matrix) the operand has, a multiple of 8.  A tile that reaches past them reads its
  // last whole chunk again instead: those LDS columns only feed outputs that are never stored.
  __device__ __forceinline__ void init(const void* p, int64_t ld, int r0, int kbeg, int rmax) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int cmax = (rmax - r0) / 8 - 1;                              // last whole chunk of this tile (>= 0)
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int k = 2 * (4 * i + w) + (lane >> 5);
      const int c = min((lane & 31) ^ (4 * (k & 3)), cmax);            // logical chunk at this LDS position
      voff[i] = (uint32_t)k * (uint32_t)ld * 2u + (uint32_t)c * 16u;
    }
    base = static_cast<const unsigned char*>(p) + ((int64_t)kbeg * ld + r0) * 2;
    slice_bytes = 64 * ld * 2;
    wave_lds = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) * 1024u;
  }
  template <int I> __device__ __forceinline__ void issue(uint32_t lds, int k) const {
    dma16(base + (int64_t)(k >> 6) * slice_bytes, voff[I], lds + wave_lds + (uint32_t)I * 4096u);
  }
  template <int I> __device__ __forceinline__ void aim(uint32_t lds) const { dma16_aim(lds + wave_lds + (uint32_t)I * 4096u); }
  template <int I> __device__ __forceinline__ void go(int k) const { dma16_go(base + (int64_t)(k >> 6) * slice_bytes, voff[I]); }
  template <int I> __device__ __forceinline__ void go_tail(int k, int krem) const {
    const int krow = 2 * (4 * I + (int)(threadIdx.x >> 6)) + (int)((threadIdx.x & 63) >> 5);
    const void* src = base + (int64_t)(k >> 6) * slice_bytes + voff[I];
    dma16_go_at(krow < krem ? src : static_cast<const void*>(kZeroChunk));
  }
};

template <int EPI, int BM, int BN> struct GemmDma64Smem {
  static constexpr int STAGE = (BM + BN) * 64 * 2;
  static constexpr int MAIN = 2 * STAGE;
  static constexpr int CT = EPI == kEpiFwd ? FwdEpiLds<uint16_t, BM, BN>::BYTES : BM * (BN + 8) * 2;
  static constexpr int BYTES = CT > MAIN ? CT : MAIN;
};

template <int AKIND, int BKIND, int EPI, int BM, int BN>
__global__ __launch_bounds__(kGemmThreads) void gemm_dma64_bf16_kernel(GemmArgs g) {
  constexpr int BK = 64, TM = BM / 64, TN = BN / 64;
  constexpr bool kAT = AKIND == kOpMN, kBT = BKIND == kOpMN;   // M/N contiguous: transposing fragment reads
  typedef GemmDma64Smem<EPI, BM, BN> S;
  typedef Lds64<BM> LYA; typedef Lds64<BN> LYB;
  typedef typename std::conditional<kAT, DmaOperandMN64<BM>, DmaOperandK64<BM>>::type LoadA;
  typedef typename std::conditional<kBT, DmaOperandMN64<BN>, DmaOperandK64<BN>>::type LoadB;
  static_assert(LoadA::NI == 8 && LoadB::NI == 8, "the schedule below places 8 + 8 loads");
  // every piece that aims a load also reads a fragment between aiming and issuing: the M0 wait state
  static_assert(TM + TN == 8, "one fragment read per piece");
  extern __shared__ __align__(16) unsigned char smem_raw[];
  uint16_t* const smem = reinterpret_cast<uint16_t*>(smem_raw);
  const uint32_t smem_lds = (uint32_t)reinterpret_cast<uintptr_t>(smem_raw);
  constexpr int kStageElems = S::STAGE / 2, kAElems = BM * BK;

  const int tiles_n = (g.N + BN - 1) / BN, tiles_m = g.M / BM;     // (N may be ragged for an M/N-contiguous B)
  const int T = tiles_m * tiles_n;
  int lin = blockIdx.x;
  if ((T & 7) == 0) lin = (lin & 7) * (T >> 3) + (lin >> 3);
  constexpr int GM = 4;
  const int grp = lin / (GM * tiles_n), within = lin - grp * (GM * tiles_n);
  const int gh = min(GM, tiles_m - grp * GM);
  const int tm = grp * GM + within % gh, tn = within / gh;
  const int m0 = tm * BM, n0 = tn * BN;
  const int w = threadIdx.x >> 6;
  const int wm0 = (w >> 1) * (BM / 2), wn0 = (w & 1) * (BN / 2);
  const int lane = threadIdx.x & 63, lr = lane & 31, lk = lane >> 5;

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int kbeg = g.k_splits > 1 ? (int)blockIdx.y * g.k_split : 0;
  const int kend = g.k_splits > 1 ? min(g.K, kbeg + g.k_split) : g.K;
  const int KT = (kend - kbeg + BK - 1) / BK;
  const int krem = kend - kbeg - (KT - 1) * BK;        // valid k of the last slice
  const bool ragged = krem < BK;                       // its loads read zeros past K; the steady loop never issues it
  const int KTs = ragged ? KT - 1 : KT;
  LoadA la; LoadB lb;
  la.init(g.A, g.lda, m0, kbeg, g.M);
  lb.init(g.B, g.ldb, n0, kbeg, g.N);

  // load number Q (0 .. 15) of slice s into stage st: A and B alternate
  auto issue = [&](auto Q_, int st, int s) {
    constexpr int Q = decltype(Q_)::value;
    const uint32_t a_lds = smem_lds + (uint32_t)st * S::STAGE;
    if (ragged && s == KT - 1) {
      if constexpr ((Q & 1) == 0) { la.template aim<Q / 2>(a_lds); asm volatile("s_nop 0"); la.template go_tail<Q / 2>(s * BK, krem); }
      else { lb.template aim<Q / 2>(a_lds + kAElems * 2); asm volatile("s_nop 0"); lb.template go_tail<Q / 2>(s * BK, krem); }
    } else {
      if constexpr ((Q & 1) == 0) la.template issue<Q / 2>(a_lds, s * BK);
      else lb.template issue<Q / 2>(a_lds + kAElems * 2, s * BK);
    }
  };

  // One load per piece: the first eight of a slice during k-step 3 of the iteration before, the other eight
  // during k-step 0 (two per piece, all in k-step 3, measured 6 % slower).  M0 is aimed before the piece's
  // MFMAs and the load issued after its fragment read.
#define RAD_K0_AIM(Q) if (more) aim(IntC<Q>(), r ^ 1);
#define RAD_K0_DMA(Q) if (more) go(IntC<Q>(), kt + 1, tail1);
#define RAD_K3_AIM(Q) if (more2) aim(IntC<Q>(), r);
#define RAD_K3_DMA(Q) if (more2) go(IntC<Q>(), kt + 2, tail2);
  uint32_t afrag[TM], bfrag[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) { if constexpr (kAT) afrag[i] = mn_frag_byte<BM>(wm0 + i * 32, lane); else afrag[i] = 0u; }
#pragma unroll
  for (int j = 0; j < TN; ++j) { if constexpr (kBT) bfrag[j] = mn_frag_byte<BN>(wn0 + j * 32, lane); else bfrag[j] = 0u; }
  auto aim = [&](auto Q_, int st) {
    constexpr int Q = decltype(Q_)::value;
    const uint32_t a_lds = smem_lds + (uint32_t)st * S::STAGE;
    if constexpr ((Q & 1) == 0) la.template aim<Q / 2>(a_lds); else lb.template aim<Q / 2>(a_lds + kAElems * 2);
  };
  auto go = [&](auto Q_, int s, bool tail) {
    constexpr int Q = decltype(Q_)::value;
    if (tail) {
      if constexpr ((Q & 1) == 0) la.template go_tail<Q / 2>(s * BK, krem); else lb.template go_tail<Q / 2>(s * BK, krem);
    } else {
      if constexpr ((Q & 1) == 0) la.template go<Q / 2>(s * BK); else lb.template go<Q / 2>(s * BK);
    }
  };
  bf16x8 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
#define RAD_FENCE() __builtin_amdgcn_sched_barrier(0)
  auto body = [&](auto R_, auto STEADY_, int kt) {
    constexpr int r = decltype(R_)::value;
    constexpr bool steady = decltype(STEADY_)::value;
    const uint16_t* const curA = smem + r * kStageElems; const uint16_t* const curB = curA + kAElems;
    const uint16_t* const nxtA = smem + (r ^ 1) * kStageElems; const uint16_t* const nxtB = nxtA + kAElems;
    // fragment readers: FA/FB destination set, stage, k-step
    auto rd = [&](bf16x8 (&fa)[TM], bf16x8 (&fb)[TN], const uint16_t* A_, const uint16_t* B_, int ks) {
      return std::make_pair(
          [&, A_, ks](int i) {
            if (i < TM) {
              if constexpr (kAT) fa[i] = mn_frag_read(reinterpret_cast<const unsigned char*>(A_), afrag[i], ks, BM * 2);
              else fa[i] = *reinterpret_cast<const bf16x8*>(&A_[LYA::unit(wm0 + i * 32 + lr, 2 * ks + lk) * 8]);
            }
          },
          [&, B_, ks](int j) {
            if (j < TN) {
              if constexpr (kBT) fb[j] = mn_frag_read(reinterpret_cast<const unsigned char*>(B_), bfrag[j], ks, BN * 2);
              else fb[j] = *reinterpret_cast<const bf16x8*>(&B_[LYB::unit(wn0 + j * 32 + lr, 2 * ks + lk) * 8]);
            }
          });
    };
    const bool more = steady || kt + 1 < KT;     // slice kt+1 exists
    const bool more2 = steady || kt + 2 < KT;    // slice kt+2 exists
    const bool tail1 = !steady && ragged && kt + 1 == KT - 1, tail2 = !steady && ragged && kt + 2 == KT - 1;
    {  // k-step 0
      auto f = rd(fa1, fb1, curA, curB, 1);
      RAD_K0_AIM(8) mfma_piece<0, TM, TN>(fa0, fb0, acc); frag_read<0, TM, TN>(f.first, f.second); RAD_K0_DMA(8) RAD_FENCE();
      RAD_K0_AIM(9) mfma_piece<1, TM, TN>(fa0, fb0, acc); frag_read<1, TM, TN>(f.first, f.second); RAD_K0_DMA(9) RAD_FENCE();
      RAD_K0_AIM(10) mfma_piece<2, TM, TN>(fa0, fb0, acc); frag_read<2, TM, TN>(f.first, f.second); RAD_K0_DMA(10) RAD_FENCE();
      RAD_K0_AIM(11) mfma_piece<3, TM, TN>(fa0, fb0, acc); frag_read<3, TM, TN>(f.first, f.second); RAD_K0_DMA(11) RAD_FENCE();
      RAD_K0_AIM(12) mfma_piece<4, TM, TN>(fa0, fb0, acc); frag_read<4, TM, TN>(f.first, f.second); RAD_K0_DMA(12) RAD_FENCE();
      RAD_K0_AIM(13) mfma_piece<5, TM, TN>(fa0, fb0, acc); frag_read<5, TM, TN>(f.first, f.second); RAD_K0_DMA(13) RAD_FENCE();
      RAD_K0_AIM(14) mfma_piece<6, TM, TN>(fa0, fb0, acc); frag_read<6, TM, TN>(f.first, f.second); RAD_K0_DMA(14) RAD_FENCE();
      RAD_K0_AIM(15) mfma_piece<7, TM, TN>(fa0, fb0, acc); frag_read<7, TM, TN>(f.first, f.second); RAD_K0_DMA(15) RAD_FENCE();
    }
    {  // k-step 1
      auto f = rd(fa0, fb0, curA, curB, 2);
      mfma_piece<0, TM, TN>(fa1, fb1, acc); frag_read<0, TM, TN>(f.first, f.second); RAD_FENCE();
      mfma_piece<1, TM, TN>(fa1, fb1, acc); frag_read<1, TM, TN>(f.first, f.second); RAD_FENCE();
      mfma_piece<2, TM, TN>(fa1, fb1, acc); frag_read<2, TM, TN>(f.first, f.second); RAD_FENCE();
      mfma_piece<3, TM, TN>(fa1, fb1, acc); frag_read<3, TM, TN>(f.first, f.second); RAD_FENCE();
      mfma_piece<4, TM, TN>(fa1, fb1, acc); frag_read<4, TM, TN>(f.first, f.second); RAD_FENCE();
      mfma_piece<5, TM, TN>(fa1, fb1, acc); frag_read<5, TM, TN>(f.first, f.second); RAD_FENCE();
      mfma_piece<6, TM, TN>(fa1, fb1, acc); frag_read<6, TM, TN>(f.first, f.second); RAD_FENCE();
      mfma_piece<7, TM, TN>(fa1, fb1, acc); frag_read<7, TM, TN>(f.first, f.second); RAD_FENCE();
    }
    {  // k-step 2: its fragment reads are the last of this stage and go first, two per piece
      auto f = rd(fa1, fb1, curA, curB, 3);
      mfma_piece<0, TM, TN>(fa0, fb0, acc); frag_read<0, TM, TN>(f.first, f.second); frag_read<1, TM, TN>(f.first, f.second); RAD_FENCE();
      mfma_piece<1, TM, TN>(fa0, fb0, acc); frag_read<2, TM, TN>(f.first, f.second); frag_read<3, TM, TN>(f.first, f.second); RAD_FENCE();
      mfma_piece<2, TM, TN>(fa0, fb0, acc); frag_read<4, TM, TN>(f.first, f.second); frag_read<5, TM, TN>(f.first, f.second); RAD_FENCE();
      mfma_piece<3, TM, TN>(fa0, fb0, acc); frag_read<6, TM, TN>(f.first, f.second); frag_read<7, TM, TN>(f.first, f.second); RAD_FENCE();
      mfma_piece<4, TM, TN>(fa0, fb0, acc); RAD_FENCE();
      mfma_piece<5, TM, TN>(fa0, fb0, acc); RAD_FENCE();
      mfma_piece<6, TM, TN>(fa0, fb0, acc); RAD_FENCE();
      mfma_piece<7, TM, TN>(fa0, fb0, acc); RAD_FENCE();
    }
    // slice kt+1 has landed (this thread's part) and this stage is read for the last time
    dma_wait<0>();
    __syncthreads();
    RAD_FENCE();
    {  // k-step 3
      auto f = rd(fa0, fb0, nxtA, nxtB, 0);
      RAD_K3_AIM(0) mfma_piece<0, TM, TN>(fa1, fb1, acc); if (more) frag_read<0, TM, TN>(f.first, f.second); RAD_K3_DMA(0) RAD_FENCE();
      RAD_K3_AIM(1) mfma_piece<1, TM, TN>(fa1, fb1, acc); if (more) frag_read<1, TM, TN>(f.first, f.second); RAD_K3_DMA(1) RAD_FENCE();
      RAD_K3_AIM(2) mfma_piece<2, TM, TN>(fa1, fb1, acc); if (more) frag_read<2, TM, TN>(f.first, f.second); RAD_K3_DMA(2) RAD_FENCE();
      RAD_K3_AIM(3) mfma_piece<3, TM, TN>(fa1, fb1, acc); if (more) frag_read<3, TM, TN>(f.first, f.second); RAD_K3_DMA(3) RAD_FENCE();
      RAD_K3_AIM(4) mfma_piece<4, TM, TN>(fa1, fb1, acc); if (more) frag_read<4, TM, TN>(f.first, f.second); RAD_K3_DMA(4) RAD_FENCE();
      RAD_K3_AIM(5) mfma_piece<5, TM, TN>(fa1, fb1, acc); if (more) frag_read<5, TM, TN>(f.first, f.second); RAD_K3_DMA(5) RAD_FENCE();
      RAD_K3_AIM(6) mfma_piece<6, TM, TN>(fa1, fb1, acc); if (more) frag_read<6, TM, TN>(f.first, f.second); RAD_K3_DMA(6) RAD_FENCE();
      RAD_K3_AIM(7) mfma_piece<7, TM, TN>(fa1, fb1, acc); if (more) frag_read<7, TM, TN>(f.first, f.second); RAD_K3_DMA(7) RAD_FENCE();
    }
  };

  // prologue: slice 0 into stage 0; its first fragments; the first half of the loads of slice 1
  if (KT > 0) {
    issue(IntC<0>(), 0, 0); issue(IntC<1>(), 0, 0); issue(IntC<2>(), 0, 0); issue(IntC<3>(), 0, 0);
    issue(IntC<4>(), 0, 0); issue(IntC<5>(), 0, 0); issue(IntC<6>(), 0, 0); issue(IntC<7>(), 0, 0);
    issue(IntC<8>(), 0, 0); issue(IntC<9>(), 0, 0); issue(IntC<10>(), 0, 0); issue(IntC<11>(), 0, 0);
    issue(IntC<12>(), 0, 0); issue(IntC<13>(), 0, 0); issue(IntC<14>(), 0, 0); issue(IntC<15>(), 0, 0);
  }
  dma_wait<0>();
  __syncthreads();
  RAD_FENCE();
  if (KT > 0) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      if constexpr (kAT) fa0[i] = mn_frag_read(reinterpret_cast<const unsigned char*>(smem), afrag[i], 0, BM * 2);
      else fa0[i] = *reinterpret_cast<const bf16x8*>(&smem[LYA::unit(wm0 + i * 32 + lr, lk) * 8]);
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      if constexpr (kBT) fb0[j] = mn_frag_read(reinterpret_cast<const unsigned char*>(smem + kAElems), bfrag[j], 0, BN * 2);
      else fb0[j] = *reinterpret_cast<const bf16x8*>(&smem[kAElems + LYB::unit(wn0 + j * 32 + lr, lk) * 8]);
    }
  }
  if (KT > 1) {
    issue(IntC<0>(), 1, 1); issue(IntC<1>(), 1, 1); issue(IntC<2>(), 1, 1); issue(IntC<3>(), 1, 1);
    issue(IntC<4>(), 1, 1); issue(IntC<5>(), 1, 1); issue(IntC<6>(), 1, 1); issue(IntC<7>(), 1, 1);
  }
  RAD_FENCE();

  int kt = 0;
  if (KTs > 3) {
    do {                                   // both iterations issue whole slices only: kt + 1 + 2 < KTs
      body(IntC<0>(), std::true_type(), kt);
      body(IntC<1>(), std::true_type(), kt + 1);
      kt += 2;
    } while (kt + 3 < KTs);
  }
  for (; kt < KT; kt += 2) {               // drain; kt is even here
    body(IntC<0>(), std::false_type(), kt);
    if (kt + 1 < KT) body(IntC<1>(), std::false_type(), kt + 1);
  }
#undef RAD_FENCE
#undef RAD_K0_AIM
#undef RAD_K0_DMA
#undef RAD_K3_AIM
#undef RAD_K3_DMA
  // every wave is past the last barrier only after all its reads of the stages; nothing is in flight
  __syncthreads();
  if constexpr (EPI == kEpiStore) {
    if (g.k_splits > 1 && g.split_stride > 0) {            // this split's partial sums go, as fp32, to an array of its own
      GemmArgs gs = g;
      gs.C = static_cast<float*>(g.C) + (int64_t)blockIdx.y * g.split_stride;
      if (g.N % BN) epilogue_store<TM, TN, float, true, false, false, false>(gs, acc, m0, n0, wm0, wn0);
      else epilogue_store<TM, TN, float, false, false, false, false>(gs, acc, m0, n0, wm0, wn0);
      return;
    }
  }
  if constexpr (EPI == kEpiStore && AKIND == kOpMN) {      // dW from a dense store: fp32 out
    if (g.N % BN) epilogue_store_dispatch<kOpMN, TM, TN, uint16_t, true>(g, acc, m0, n0, wm0, wn0);
    else epilogue_store_dispatch<kOpMN, TM, TN, uint16_t, false>(g, acc, m0, n0, wm0, wn0);
  } else if constexpr (EPI == kEpiStore) {
    epilogue_dx_staged<BM, BN, TM, TN>(g, acc, smem, m0, n0, wm0, wn0);
  } else {
    epilogue_fwd<uint16_t, BM, BN, TM, TN>(g, acc, smem, m0, n0, wm0, wn0);
  }
}

}  // namespace rad
