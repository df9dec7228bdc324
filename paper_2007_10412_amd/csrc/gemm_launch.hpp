// Launch helper shared by the GEMM instantiation files.
#pragma once
#include <hip/hip_ext.h>

#include "gemm_bf16.hpp"
#include "gemm_bf16_dma.hpp"

namespace rad {

// Launches a GEMM kernel; with timing events in the arguments the dispatch itself records them (start and end
// of the kernel), so timing one kernel of a step puts no extra packets, and no bubbles, on the stream.
template <class K>
hipError_t launch_gemm_kernel(K kern, dim3 grid, int smem, hipStream_t st, const GemmArgs& g) {
  if (g.ev_start && g.ev_stop)
    hipExtLaunchKernelGGL(kern, grid, dim3(kGemmThreads), smem, st, static_cast<hipEvent_t>(g.ev_start),
                          static_cast<hipEvent_t>(g.ev_stop), 0, g);
  else
    hipLaunchKernelGGL(kern, grid, dim3(kGemmThreads), smem, st, g);
  return hipGetLastError();
}

template <class DT, int AK, int BKIND, int EPI, int BM, int BN, int BK, int SE, int FLAGS>
hipError_t run_gemm_variant(const GemmArgs& g, hipStream_t st) {
  auto kern = gemm_kernel<DT, AK, BKIND, EPI, BM, BN, BK, SE, FLAGS>;
  constexpr int smem = GemmSmem<DT, AK, BKIND, EPI, BM, BN, BK, SE>::BYTES;
  static_assert(smem <= 160 * 1024, "tile does not fit the 160 KB LDS of a gfx950 CU");
  static bool prepared = false;   // one host thread drives a context
  if (!prepared) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    prepared = true;
  }
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  if (tiles_m <= 0 || tiles_n <= 0) return hipSuccess;
  return launch_gemm_kernel(kern, dim3(tiles_m * tiles_n, g.k_splits > 1 ? g.k_splits : 1), smem, st, g);
}

// true when every tile is full and every operand row is 16-byte aligned: the
// interior (unguarded) kernel variant may run
template <class DT, int AK, int BM, int BN, int BK>
bool gemm_is_full(const GemmArgs& g) {
  const int vec = sizeof(typename ElemOf<DT>::type) == 2 ? 8 : 4;
  bool full = g.M % BM == 0 && g.N % BN == 0 && g.K % BK == 0 && g.K > 0;
  if (g.k_splits > 1) full = full && g.k_split % BK == 0;       // every split's range is whole K slices
  if (AK != kOpSparse) full = full && g.lda % vec == 0 && (reinterpret_cast<uintptr_t>(g.A) & 15) == 0;
  return full && g.ldb % vec == 0 && (reinterpret_cast<uintptr_t>(g.B) & 15) == 0;
}

// MASK_A / MASK_B: whether this GEMM family can carry a ReLU-bit mask on that
// operand; BOTH_EDGE: build the interior variant too (else guarded only).
template <class DT, int AK, int BKIND, int EPI, int BM, int BN, int BK, int SE, bool MASK_A, bool MASK_B,
          bool BOTH_EDGE = true>
hipError_t run_gemm(const GemmArgs& g, hipStream_t st) {
  if (g.dry_run) return hipSuccess;   // the caller only wanted the kernel's label
  const bool full = BOTH_EDGE && gemm_is_full<DT, AK, BM, BN, BK>(g);
  const bool ma = MASK_A && g.a_mask != nullptr, mb = MASK_B && g.b_mask != nullptr;
  if ((g.a_mask && !MASK_A) || (g.b_mask && !MASK_B)) return hipErrorInvalidValue;
  constexpr int FA = MASK_A ? kFlagMaskA : 0, FB = MASK_B ? kFlagMaskB : 0;
  if (BOTH_EDGE && full) {
    if (ma || mb) return run_gemm_variant<DT, AK, BKIND, EPI, BM, BN, BK, SE, FA | FB>(g, st);
    return run_gemm_variant<DT, AK, BKIND, EPI, BM, BN, BK, SE, 0>(g, st);
  }
  if (ma || mb) return run_gemm_variant<DT, AK, BKIND, EPI, BM, BN, BK, SE, kFlagEdge | FA | FB>(g, st);
  return run_gemm_variant<DT, AK, BKIND, EPI, BM, BN, BK, SE, kFlagEdge>(g, st);
}

// ---- bf16 ring-pipeline kernels (BK = 32, three LDS stages)
template <int AK, int BKIND, int EPI, int BM, int BN, int SE, int FLAGS>
hipError_t run_gemm3_variant(const GemmArgs& g, hipStream_t st) {
  auto kern = gemm3_bf16_kernel<AK, BKIND, EPI, BM, BN, SE, FLAGS>;
  constexpr int smem = Gemm3Smem<EPI, BM, BN, EPI == kEpiStore && AK == kOpK>::BYTES;
  static_assert(smem <= 160 * 1024, "tile does not fit the 160 KB LDS of a gfx950 CU");
  static bool prepared = false;   // one host thread drives a context
  if (!prepared) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    prepared = true;
  }
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  if (tiles_m <= 0 || tiles_n <= 0) return hipSuccess;
  return launch_gemm_kernel(kern, dim3(tiles_m * tiles_n, g.k_splits > 1 ? g.k_splits : 1), smem, st, g);
}

// ---- bf16 kernels whose operands go from global memory straight into LDS: whole 256-row tiles (a ragged last
// tile column only for an M/N-contiguous B), rows that are whole 16-byte vectors, no loader masks; K need not be
// a multiple of the 64-deep slice; a split K (whole slices per split) stores fp32 partial sums per split.
template <int AKIND, int BKIND, int BM, int BN>
bool gemm_dma_ok(const GemmArgs& g) {
  if (g.a_mask || g.b_mask || g.row_map || g.m_load > g.M) return false;
  // whole tiles; an M/N-contiguous B may end inside its last tile column (whole 16-byte chunks), the loads there
  // are clamped and the epilogues guard the stores
  if (g.M <= 0 || g.N <= 0 || g.K <= 0 || g.M % BM || g.K % 8 || g.lda % 8 || g.ldb % 8) return false;
  if (BKIND == kOpMN ? g.N % 8 != 0 : g.N % BN != 0) return false;
  if ((reinterpret_cast<uintptr_t>(g.A) | reinterpret_cast<uintptr_t>(g.B)) & 15) return false;
  if (g.k_splits > 1 && g.k_split % 64 != 0) return false;
  // per-thread offsets inside a tile are 32-bit byte offsets
  const int64_t a_rows = AKIND == kOpMN ? 64 : BM, b_rows = BKIND == kOpMN ? 64 : BN;
  return a_rows * g.lda * 2 < (int64_t(1) << 32) && b_rows * g.ldb * 2 < (int64_t(1) << 32);
}
template <int AKIND, int BKIND, int EPI, int BM, int BN>
hipError_t run_gemm_dma(const GemmArgs& g, hipStream_t st) {
  if (g.dry_run) return hipSuccess;
  auto kern = gemm_dma64_bf16_kernel<AKIND, BKIND, EPI, BM, BN>;
  constexpr int smem = GemmDma64Smem<EPI, BM, BN>::BYTES;
  static_assert(smem <= 160 * 1024, "tile does not fit the 160 KB LDS of a gfx950 CU");
  static bool prepared = false;   // one host thread drives a context
  if (!prepared) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    prepared = true;
  }
  return launch_gemm_kernel(kern, dim3((g.M / BM) * ((g.N + BN - 1) / BN), g.k_splits > 1 ? g.k_splits : 1), smem, st, g);
}

// ragged shapes whose every operand access is still a whole 16-byte vector: pitches, K and the extent along
// the contiguous axis are multiples of 8 elements
template <int AK, int BKIND>
bool gemm_is_vec_edge(const GemmArgs& g) {
  bool ok = g.K > 0 && (reinterpret_cast<uintptr_t>(g.B) & 15) == 0 && g.ldb % 8 == 0;
  if (AK != kOpSparse) ok = ok && (reinterpret_cast<uintptr_t>(g.A) & 15) == 0 && g.lda % 8 == 0;
  if (AK == kOpK || BKIND == kOpK) ok = ok && g.K % 8 == 0;
  if (AK == kOpMN) ok = ok && (g.m_load > g.M ? g.m_load : g.M) % 8 == 0;
  if (BKIND == kOpMN) ok = ok && g.N % 8 == 0;
  return ok;
}

// Variants built per family: interior, vector-predicated ragged and generic ragged without a loader mask;
// generic ragged with one (loader masks serve the stand-alone entry points; the train steps mask in the
// producing epilogue instead).
template <int AK, int BKIND, int EPI, int BM, int BN, int SE, bool MASK_A, bool MASK_B, bool BOTH_EDGE = true>
hipError_t run_gemm3(const GemmArgs& g, hipStream_t st) {
  if (g.dry_run) return hipSuccess;
  const bool ma = MASK_A && g.a_mask != nullptr, mb = MASK_B && g.b_mask != nullptr;
  if ((g.a_mask && !MASK_A) || (g.b_mask && !MASK_B)) return hipErrorInvalidValue;
  constexpr int FA = MASK_A ? kFlagMaskA : 0, FB = MASK_B ? kFlagMaskB : 0;
  if (ma || mb) return run_gemm3_variant<AK, BKIND, EPI, BM, BN, SE, kFlagEdge | FA | FB>(g, st);
  if (BOTH_EDGE && gemm_is_full<BF16Tag, AK, BM, BN, 32>(g)) return run_gemm3_variant<AK, BKIND, EPI, BM, BN, SE, 0>(g, st);
  if (gemm_is_vec_edge<AK, BKIND>(g)) return run_gemm3_variant<AK, BKIND, EPI, BM, BN, SE, kFlagEdgeVec>(g, st);
  return run_gemm3_variant<AK, BKIND, EPI, BM, BN, SE, kFlagEdge>(g, st);
}

hipError_t launch_gemm_f32(int a_kind, int b_kind, int epi, const GemmArgs& g, hipStream_t st, const char** name);
hipError_t launch_gemm_bf16(int a_kind, int b_kind, int epi, const GemmArgs& g, hipStream_t st, const char** name);

inline int tiles_of(const GemmArgs& g, int bm, int bn) {
  return ((g.M + bm - 1) / bm) * ((g.N + bn - 1) / bn);
}

}  // namespace rad
