// bf16 GEMM family: dW from a dense or compact (shared-index) store.
#include "gemm_launch.hpp"

namespace rad {

hipError_t launch_gemm_bf16_dwd(const GemmArgs& g, hipStream_t st, const char** name) {
  // 256x256 tiles (one workgroup per CU) when they give at least half a wave of workgroups
  const bool big = tiles_of(g, 256, 256) >= 128;
  if (name) *name = big ? "gemm_bf16_dw_dense_256" : "gemm_bf16_dw_dense_128";
  if (big) return run_gemm3<kOpMN, kOpMN, kEpiStore, 256, 256, 0, false, true>(g, st);
  return run_gemm3<kOpMN, kOpMN, kEpiStore, 128, 128, 0, false, true>(g, st);
}

}  // namespace rad
