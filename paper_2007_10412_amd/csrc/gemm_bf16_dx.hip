// bf16 GEMM family: dX = (dy masked by ReLU bits) W^T.
#include "gemm_launch.hpp"

namespace rad {

hipError_t launch_gemm_bf16_dx(const GemmArgs& g, hipStream_t st, const char** name) {
  // 256x256 tiles (one workgroup per CU) when they give at least half a wave of workgroups
  const bool big = tiles_of(g, 256, 256) >= 128;
  if (name) *name = big ? "gemm_bf16_dx_256" : "gemm_bf16_dx_128";
  if (big) return run_gemm3<kOpK, kOpK, kEpiStore, 256, 256, 0, true, false>(g, st);
  return run_gemm3<kOpK, kOpK, kEpiStore, 128, 128, 0, true, false>(g, st);
}

}  // namespace rad
