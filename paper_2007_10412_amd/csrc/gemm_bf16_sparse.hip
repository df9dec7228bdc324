// bf16 dW from the compressed store: picks the kernel by the number of entries a lane must hold.
#include "gemm_launch.hpp"

namespace rad {

hipError_t launch_gemm_bf16_sparse3(const GemmArgs& g, hipStream_t st, const char** name);
hipError_t launch_gemm_bf16_sparse7(const GemmArgs& g, hipStream_t st, const char** name);

// largest sparse_prefetch a fused kernel exists for; denser stores are unpacked to a dense operand first
int gemm_bf16_sparse_max_prefetch() { return 7; }

// register entries per lane of the kernel picked for `sparse_prefetch`, times the eight lanes of a store row
int gemm_bf16_sparse_cap(int sparse_prefetch) { return (sparse_prefetch <= 3 ? 3 : 7) * 8; }

hipError_t launch_gemm_bf16_sparse(const GemmArgs& g, hipStream_t st, const char** name) {
  if (g.sparse_prefetch <= 3) return launch_gemm_bf16_sparse3(g, st, name);
  return launch_gemm_bf16_sparse7(g, st, name);
}

}  // namespace rad
