// fp32 instantiations of the GEMM engine (v_mfma_f32_32x32x2_f32).
#include "gemm_launch.hpp"

namespace rad {

hipError_t launch_gemm_f32(int a_kind, int b_kind, int epi, const GemmArgs& g, hipStream_t st, const char** name) {
  const char* nm = "";
  hipError_t e = hipErrorInvalidValue;
  // 128x128 tiles once they alone fill the chip, 64x64 otherwise
  const bool big = tiles_of(g, 128, 128) >= 192;
  if (a_kind == kOpK && b_kind == kOpMN && epi == kEpiFwd) {
    if (big) { nm = "gemm_f32_fwd_128"; e = run_gemm<F32Tag, kOpK, kOpMN, kEpiFwd, 128, 128, 16, 0, false, false>(g, st); }
    else { nm = "gemm_f32_fwd_64"; e = run_gemm<F32Tag, kOpK, kOpMN, kEpiFwd, 64, 64, 16, 0, false, false>(g, st); }
  } else if (a_kind == kOpK && b_kind == kOpK && epi == kEpiStore) {
    if (big) { nm = "gemm_f32_dx_128"; e = run_gemm<F32Tag, kOpK, kOpK, kEpiStore, 128, 128, 16, 0, true, false>(g, st); }
    else { nm = "gemm_f32_dx_64"; e = run_gemm<F32Tag, kOpK, kOpK, kEpiStore, 64, 64, 16, 0, true, false>(g, st); }
  } else if (a_kind == kOpMN && b_kind == kOpMN && epi == kEpiStore) {
    if (big) { nm = "gemm_f32_dw_dense_128"; e = run_gemm<F32Tag, kOpMN, kOpMN, kEpiStore, 128, 128, 16, 0, false, true>(g, st); }
    else { nm = "gemm_f32_dw_dense_64"; e = run_gemm<F32Tag, kOpMN, kOpMN, kEpiStore, 64, 64, 16, 0, false, true>(g, st); }
  } else if (a_kind == kOpSparse && b_kind == kOpMN && epi == kEpiStore) {
    const bool wide = g.sparse_prefetch > 4;
    if (big) {
      if (wide) { nm = "gemm_f32_dw_sparse_128"; e = run_gemm<F32Tag, kOpSparse, kOpMN, kEpiStore, 128, 128, 16, 16, false, true, false>(g, st); }
      else { nm = "gemm_f32_dw_sparse_128"; e = run_gemm<F32Tag, kOpSparse, kOpMN, kEpiStore, 128, 128, 16, 4, false, true, false>(g, st); }
    } else {
      if (wide) { nm = "gemm_f32_dw_sparse_64"; e = run_gemm<F32Tag, kOpSparse, kOpMN, kEpiStore, 64, 64, 16, 16, false, true, false>(g, st); }
      else { nm = "gemm_f32_dw_sparse_64"; e = run_gemm<F32Tag, kOpSparse, kOpMN, kEpiStore, 64, 64, 16, 4, false, true, false>(g, st); }
    }
  }
  else if (a_kind == kOpK && b_kind == kOpMN && epi == kEpiSplitK) {
    // few output tiles and a long contraction (one step of the recurrent model): partial sums per K range
    nm = "gemm_f32_fwd_splitk_64"; e = run_gemm<F32Tag, kOpK, kOpMN, kEpiSplitK, 64, 64, 32, 0, false, false>(g, st);
  } else if (a_kind == kOpK && b_kind == kOpK && epi == kEpiSplitK) {
    nm = "gemm_f32_dx_splitk_64"; e = run_gemm<F32Tag, kOpK, kOpK, kEpiSplitK, 64, 64, 32, 0, true, false>(g, st);
  }
  else if (a_kind == kOpIm2colRows && b_kind == kOpMN && epi == kEpiConv) {
    // convolution forward / dX: positions x channels, channels fit one 64-wide tile column
    nm = "gemm_f32_conv_64"; e = run_gemm<F32Tag, kOpIm2colRows, kOpMN, kEpiConv, 64, 64, 16, 0, false, false, false>(g, st);
  } else if (a_kind == kOpIm2colK && b_kind == kOpKBatched && epi == kEpiSplitK) {
    // convolution dW: (c,u,v) x channels with the positions as a split K
    nm = "gemm_f32_conv_dw_64"; e = run_gemm<F32Tag, kOpIm2colK, kOpKBatched, kEpiSplitK, 64, 64, 16, 0, false, false, false>(g, st);
  }
  if (name) *name = nm;
  return e;
}

}  // namespace rad
