// bf16 GEMM family "dw_dense" (see gemm.hpp for the operand kinds).
#include "gemm_launch.hpp"

namespace rad {

hipError_t launch_gemm_bf16_dwd(const GemmArgs& g, hipStream_t st, const char** name) {
  // a split K needs an array per split
  if (g.k_splits > 1 && g.split_stride <= 0) { if (name) *name = ""; return hipErrorInvalidValue; }
  // 256x256 tiles (one workgroup per CU) when they give at least half a wave of workgroups; otherwise the
  // widest tile that still gives every CU a workgroup
  if (tiles_of(g, 256, 256) >= 128) {
    if (gemm_dma_ok<kOpMN, kOpMN, 256, 256>(g)) {
      if (name) *name = "gemm_bf16_dw_dense_dma_256";
      return run_gemm_dma<kOpMN, kOpMN, kEpiStore, 256, 256>(g, st);
    }
    if (name) *name = "gemm_bf16_dw_dense_256";
    return run_gemm3<kOpMN, kOpMN, kEpiStore, 256, 256, 0, false, true>(g, st);
  }
  if (tiles_of(g, 256, 64) >= 192 && tiles_of(g, 128, 128) < 2 * tiles_of(g, 256, 64)) {
    if (name) *name = "gemm_bf16_dw_dense_256x64";
    return run_gemm3<kOpMN, kOpMN, kEpiStore, 256, 64, 0, false, true, false>(g, st);
  }
  if (name) *name = "gemm_bf16_dw_dense_128";
  return run_gemm3<kOpMN, kOpMN, kEpiStore, 128, 128, 0, false, true>(g, st);
}

}  // namespace rad
