// bf16 dW from the compressed store: A tiles are unpacked into LDS and
// contracted on v_mfma_f32_32x32x16_bf16.  The A tile is always one whole
// 256-column bucket of the store.
#include "gemm_launch.hpp"

namespace rad {

hipError_t launch_gemm_bf16_sparse(const GemmArgs& g, hipStream_t st, const char** name) {
  const char* nm = "";
  hipError_t e = hipErrorInvalidValue;
  const bool big = tiles_of(g, 256, 256) >= 128;
  const int se = g.sparse_prefetch;
  if (big) {
    nm = "gemm_bf16_dw_sparse_256x256";
    if (se <= 4) e = run_gemm<BF16Tag, kOpSparse, kOpMN, kEpiStore, 256, 256, 64, 4, false, true>(g, st);
    else if (se <= 12) e = run_gemm<BF16Tag, kOpSparse, kOpMN, kEpiStore, 256, 256, 64, 12, false, true>(g, st);
    else e = run_gemm<BF16Tag, kOpSparse, kOpMN, kEpiStore, 256, 256, 64, 40, false, true>(g, st);
  } else {
    nm = "gemm_bf16_dw_sparse_256x128";
    if (se <= 4) e = run_gemm<BF16Tag, kOpSparse, kOpMN, kEpiStore, 256, 128, 64, 4, false, true, false>(g, st);
    else if (se <= 12) e = run_gemm<BF16Tag, kOpSparse, kOpMN, kEpiStore, 256, 128, 64, 12, false, true, false>(g, st);
    else e = run_gemm<BF16Tag, kOpSparse, kOpMN, kEpiStore, 256, 128, 64, 40, false, true, false>(g, st);
  }
  if (name) *name = nm;
  return e;
}

}  // namespace rad
