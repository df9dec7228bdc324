// bf16 GEMM dispatch (v_mfma_f32_32x32x16_bf16); the kernel families are
// instantiated in gemm_bf16_{fwd,dx,dwd,sparse}.hip.
#include "gemm_launch.hpp"

namespace rad {

hipError_t launch_gemm_bf16_fwd(const GemmArgs& g, hipStream_t st, const char** name);
hipError_t launch_gemm_bf16_fwd_partial(const GemmArgs& g, hipStream_t st, const char** name);
hipError_t launch_gemm_bf16_dx(const GemmArgs& g, hipStream_t st, const char** name);
hipError_t launch_gemm_bf16_dwd(const GemmArgs& g, hipStream_t st, const char** name);
hipError_t launch_gemm_bf16_sparse(const GemmArgs& g, hipStream_t st, const char** name);

hipError_t launch_gemm_bf16(int a_kind, int b_kind, int epi, const GemmArgs& g, hipStream_t st, const char** name) {
  if (a_kind == kOpSparse && b_kind == kOpMN && epi == kEpiStore) return launch_gemm_bf16_sparse(g, st, name);
  if (a_kind == kOpK && b_kind == kOpMN && epi == kEpiFwd) return launch_gemm_bf16_fwd(g, st, name);
  if (a_kind == kOpK && b_kind == kOpMN && epi == kEpiStore) return launch_gemm_bf16_fwd_partial(g, st, name);
  if (a_kind == kOpK && b_kind == kOpK && epi == kEpiStore) return launch_gemm_bf16_dx(g, st, name);
  if (a_kind == kOpMN && b_kind == kOpMN && epi == kEpiStore) return launch_gemm_bf16_dwd(g, st, name);
  if (name) *name = "";
  return hipErrorInvalidValue;
}

hipError_t launch_gemm(int dtype, int a_kind, int b_kind, int epi, const GemmArgs& g, hipStream_t st,
                       const char** name) {
  if (dtype == kBF16) return launch_gemm_bf16(a_kind, b_kind, epi, g, st, name);
  if (dtype == kF32) return launch_gemm_f32(a_kind, b_kind, epi, g, st, name);
  return hipErrorInvalidValue;
}

}  // namespace rad
