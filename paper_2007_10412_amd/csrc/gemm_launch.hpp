// Launch helper shared by the GEMM instantiation files.
#pragma once
#include "gemm.hpp"

namespace rad {

template <class DT, int AK, int BKIND, int EPI, int BM, int BN, int BK, int SE>
hipError_t run_gemm(const GemmArgs& g, hipStream_t st) {
  auto kern = gemm_kernel<DT, AK, BKIND, EPI, BM, BN, BK, SE>;
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
  hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(kGemmThreads), smem, st, g);
  return hipGetLastError();
}

hipError_t launch_gemm_f32(int a_kind, int b_kind, int epi, const GemmArgs& g, hipStream_t st, const char** name);
hipError_t launch_gemm_bf16(int a_kind, int b_kind, int epi, const GemmArgs& g, hipStream_t st, const char** name);

inline int tiles_of(const GemmArgs& g, int bm, int bn) {
  return ((g.M + bm - 1) / bm) * ((g.N + bn - 1) / bn);
}

}  // namespace rad
