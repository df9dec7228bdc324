// bf16 GEMM family: forward y = act(x W + b) with the fused bits / pack epilogue.
#include "gemm_launch.hpp"

namespace rad {

hipError_t launch_gemm_bf16_fwd(const GemmArgs& g, hipStream_t st, const char** name) {
  // 256x256 tiles (one workgroup per CU) when they give at least half a wave of workgroups
  const bool big = tiles_of(g, 256, 256) >= 128;
  if (name) *name = big ? "gemm_bf16_fwd_256" : "gemm_bf16_fwd_128";
  if (big) return run_gemm3<kOpK, kOpMN, kEpiFwd, 256, 256, 0, false, false>(g, st);
  return run_gemm3<kOpK, kOpMN, kEpiFwd, 128, 128, 0, false, false>(g, st);
}

}  // namespace rad
