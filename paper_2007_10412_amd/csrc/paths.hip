// Reverse-mode AD with path sampling on a linearised computational graph (Appendix C, Algorithm 1).
// Vertices are numbered in topological order and grouped in levels whose edges lead to later levels only, so a
// level is one launch: going up, every reached vertex draws k of its outgoing edges and marks their heads as
// reached; going down, a reached vertex's estimate is (d_v / k) times the sum over its k draws of the edge
// partial times the head's estimate.  The draws are made again on the way down (draw s of vertex v is the key
// of flat index v k + s, mapped to edge floor(key d_v / 2^32)), so nothing is stored per edge: the memory the
// method saves.  fp64; a vertex's sum runs over its draws in order, so results do not depend on the launch.
#include "kernels.hpp"
#include "philox.hpp"

namespace rad {

namespace {

struct PathArgs {
  int n, k, y; int64_t n_edges;
  const int32_t* succ_ptr; const int32_t* succ; const double* partial;
  uint32_t* reached; double* adj; int* bad;
  uint32_t seed_lo, seed_hi, stream_id;
};

__device__ __forceinline__ uint32_t draw_key(const PathArgs& a, int v, int s) {
  const uint64_t f = (uint64_t)v * (uint64_t)a.k + (uint64_t)s;
  const u32x4 k4 = element_quad_keys(f >> 2, a.stream_id, 0u, a.seed_lo, a.seed_hi);
  return k4[f & 3];
}

// edge number of draw s of vertex v, or -1 if the vertex has no edges; inconsistent arrays raise the flag
__device__ __forceinline__ int64_t draw_edge(const PathArgs& a, int v, int s, int level_end) {
  const int64_t e0 = a.succ_ptr[v], e1 = a.succ_ptr[v + 1];
  if (e1 == e0) return -1;
  if (e0 < 0 || e1 < e0 || e1 > a.n_edges) { *a.bad = 1; return -1; }
  const uint64_t d = (uint64_t)(e1 - e0);
  const int64_t e = e0 + (int64_t)(((uint64_t)draw_key(a, v, s) * d) >> 32);
  const int u = a.succ[e];
  if (u < level_end || u >= a.n) { *a.bad = 1; return -1; }   // edges lead to later levels only
  return e;
}

__global__ __launch_bounds__(256) void path_inputs_kernel(PathArgs a, const int32_t* __restrict__ inputs, int n_inputs) {
  const int q = blockIdx.x * 256 + threadIdx.x;
  if (q >= n_inputs) return;
  const int v = inputs[q];
  if (v < 0 || v >= a.n) { *a.bad = 1; return; }
  a.reached[v] = 1u;
}

// one thread per (vertex of the level, draw)
__global__ __launch_bounds__(256) void path_mark_kernel(PathArgs a, int v0, int v1) {
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t v = v0 + q / a.k;
  if (v >= v1 || !a.reached[v]) return;
  const int64_t e = draw_edge(a, (int)v, (int)(q % a.k), v1);
  if (e >= 0) a.reached[a.succ[e]] = 1u;
}

// one thread per vertex of the level
__global__ __launch_bounds__(256) void path_adjoint_kernel(PathArgs a, int v0, int v1) {
  const int v = v0 + blockIdx.x * 256 + threadIdx.x;
  if (v >= v1) return;
  if (v == a.y) { a.adj[v] = a.reached[v] ? 1.0 : 0.0; return; }
  double sum = 0.0;
  int64_t d = 0;
  if (a.reached[v]) {
    d = (int64_t)a.succ_ptr[v + 1] - (int64_t)a.succ_ptr[v];
    for (int s = 0; s < a.k; ++s) {
      const int64_t e = draw_edge(a, v, s, v1);
      if (e < 0) break;
      sum += a.partial[e] * a.adj[a.succ[e]];
    }
  }
  a.adj[v] = d > 0 ? ((double)d / (double)a.k) * sum : 0.0;
}

}  // namespace

hipError_t launch_path_sampling(int n, int n_levels, const int32_t* level_ptr_host, int64_t n_edges,
                                const int32_t* succ_ptr, const int32_t* succ, const double* partial, int y,
                                const int32_t* inputs, int n_inputs, int k, uint32_t seed_lo, uint32_t seed_hi,
                                uint32_t stream_id, double* adj, uint32_t* reached, int* bad, hipStream_t st) {
  PathArgs a;
  a.n = n; a.k = k; a.y = y; a.n_edges = n_edges; a.succ_ptr = succ_ptr; a.succ = succ; a.partial = partial;
  a.reached = reached; a.adj = adj; a.bad = bad; a.seed_lo = seed_lo; a.seed_hi = seed_hi; a.stream_id = stream_id;
  hipError_t e = launch_fill_u32(reached, 0u, n, st);
  if (e != hipSuccess) return e;
  e = launch_fill_u32(reinterpret_cast<uint32_t*>(bad), 0u, 1, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(path_inputs_kernel, dim3((unsigned)((n_inputs + 255) / 256)), dim3(256), 0, st, a, inputs, n_inputs);
  for (int l = 0; l < n_levels; ++l) {
    const int v0 = level_ptr_host[l], v1 = level_ptr_host[l + 1];
    const int64_t threads = (int64_t)(v1 - v0) * k;
    if (threads > 0)
      hipLaunchKernelGGL(path_mark_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, a, v0, v1);
  }
  for (int l = n_levels - 1; l >= 0; --l) {
    const int v0 = level_ptr_host[l], v1 = level_ptr_host[l + 1];
    if (v1 > v0)
      hipLaunchKernelGGL(path_adjoint_kernel, dim3((unsigned)((v1 - v0 + 255) / 256)), dim3(256), 0, st, a, v0, v1);
  }
  return hipGetLastError();
}

}  // namespace rad
