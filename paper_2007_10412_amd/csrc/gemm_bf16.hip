// bf16 instantiations of the GEMM engine (v_mfma_f32_32x32x16_bf16), dense operands.
#include "gemm_launch.hpp"

namespace rad {

hipError_t launch_gemm_bf16_sparse(const GemmArgs& g, hipStream_t st, const char** name);

hipError_t launch_gemm_bf16(int a_kind, int b_kind, int epi, const GemmArgs& g, hipStream_t st, const char** name) {
  if (a_kind == kOpSparse) return launch_gemm_bf16_sparse(g, st, name);
  const char* nm = "";
  hipError_t e = hipErrorInvalidValue;
  // 256x256 tiles (one workgroup per CU) when they give at least half a wave of workgroups
  const bool big = tiles_of(g, 256, 256) >= 128;
  if (a_kind == kOpK && b_kind == kOpMN && epi == kEpiFwd) {
    if (big) { nm = "gemm_bf16_fwd_256"; e = run_gemm<BF16Tag, kOpK, kOpMN, kEpiFwd, 256, 256, 64, 0>(g, st); }
    else { nm = "gemm_bf16_fwd_128"; e = run_gemm<BF16Tag, kOpK, kOpMN, kEpiFwd, 128, 128, 64, 0>(g, st); }
  } else if (a_kind == kOpK && b_kind == kOpK && epi == kEpiStore) {
    if (big) { nm = "gemm_bf16_dx_256"; e = run_gemm<BF16Tag, kOpK, kOpK, kEpiStore, 256, 256, 64, 0>(g, st); }
    else { nm = "gemm_bf16_dx_128"; e = run_gemm<BF16Tag, kOpK, kOpK, kEpiStore, 128, 128, 64, 0>(g, st); }
  } else if (a_kind == kOpMN && b_kind == kOpMN && epi == kEpiStore) {
    if (big) { nm = "gemm_bf16_dw_dense_256"; e = run_gemm<BF16Tag, kOpMN, kOpMN, kEpiStore, 256, 256, 64, 0>(g, st); }
    else { nm = "gemm_bf16_dw_dense_128"; e = run_gemm<BF16Tag, kOpMN, kOpMN, kEpiStore, 128, 128, 64, 0>(g, st); }
  }
  if (name) *name = nm;
  return e;
}

hipError_t launch_gemm(int dtype, int a_kind, int b_kind, int epi, const GemmArgs& g, hipStream_t st,
                       const char** name) {
  if (dtype == kBF16) return launch_gemm_bf16(a_kind, b_kind, epi, g, st, name);
  if (dtype == kF32) return launch_gemm_f32(a_kind, b_kind, epi, g, st, name);
  return hipErrorInvalidValue;
}

}  // namespace rad
