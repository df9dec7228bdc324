// bf16 dW from the compressed store, kernels that keep 7 entries per lane (56 per store row and bucket) in
// registers: A tiles are unpacked into LDS and contracted on v_mfma_f32_32x32x16_bf16.  The A tile is always
// one whole 256-column bucket of the store.
#include "gemm_launch.hpp"

namespace rad {

hipError_t launch_gemm_bf16_sparse7(const GemmArgs& g, hipStream_t st, const char** name) {
  // the host splits K (the batch) when a narrow dW gives few 256x256 tiles
  if (tiles_of(g, 256, 256) * (g.k_splits > 1 ? g.k_splits : 1) >= 128) {
    if (name) *name = g.k_splits > 1 ? "gemm_bf16_dw_sparse_splitk_256" : "gemm_bf16_dw_sparse_256x256";
    return run_gemm3<kOpSparse, kOpMN, kEpiStore, 256, 256, 7, false, true>(g, st);
  }
  if (tiles_of(g, 256, 128) * (g.k_splits > 1 ? g.k_splits : 1) >= 192) {
    if (name) *name = "gemm_bf16_dw_sparse_256x128";
    return run_gemm3<kOpSparse, kOpMN, kEpiStore, 256, 128, 7, false, true, false>(g, st);
  }
  if (name) *name = "gemm_bf16_dw_sparse_256x64";
  return run_gemm3<kOpSparse, kOpMN, kEpiStore, 256, 64, 7, false, true, false>(g, st);
}

}  // namespace rad
