// bf16 GEMM family "fwd" (see gemm.hpp for the operand kinds).
#include "gemm_launch.hpp"

namespace rad {

hipError_t launch_gemm_bf16_fwd(const GemmArgs& g, hipStream_t st, const char** name) {
  // 256x256 tiles (one workgroup per CU) when they give at least half a wave of workgroups; otherwise the
  // widest tile that still gives every CU a workgroup
  if (tiles_of(g, 256, 256) >= 128) {
    if (gemm_dma_ok<kOpK, kOpMN, 256, 256>(g)) {
      if (name) *name = "gemm_bf16_fwd_dma_256";
      return run_gemm_dma<kOpK, kOpMN, kEpiFwd, 256, 256>(g, st);
    }
    if (name) *name = "gemm_bf16_fwd_256";
    return run_gemm3<kOpK, kOpMN, kEpiFwd, 256, 256, 0, false, false>(g, st);
  }
  if (tiles_of(g, 256, 64) >= 192 && tiles_of(g, 128, 128) < 2 * tiles_of(g, 256, 64)) {
    if (name) *name = "gemm_bf16_fwd_256x64";
    return run_gemm3<kOpK, kOpMN, kEpiFwd, 256, 64, 0, false, false, false>(g, st);
  }
  if (name) *name = "gemm_bf16_fwd_128";
  return run_gemm3<kOpK, kOpMN, kEpiFwd, 128, 128, 0, false, false>(g, st);
}

// x W for a narrow layer whose K range is split over several workgroups per 256x256 tile: fp32 partial sums,
// one array per split (bias and the cast to the layer's dtype happen in the reduction kernel)
hipError_t launch_gemm_bf16_fwd_partial(const GemmArgs& g, hipStream_t st, const char** name) {
  if (g.k_splits <= 1 || g.split_stride <= 0) { if (name) *name = ""; return hipErrorInvalidValue; }
  if (gemm_dma_ok<kOpK, kOpMN, 256, 256>(g)) {
    if (name) *name = "gemm_bf16_fwd_partial_dma_256";
    return run_gemm_dma<kOpK, kOpMN, kEpiStore, 256, 256>(g, st);
  }
  if (name) *name = "gemm_bf16_fwd_partial_256";
  return run_gemm3<kOpK, kOpMN, kEpiStore, 256, 256, 0, false, false>(g, st);
}

}  // namespace rad
