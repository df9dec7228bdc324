// Parameter updates (Section 4.3 and Appendix A, training details): plain SGD for the recurrent model, Adam for the
// feedforward ones, each with an l2 term added to the gradient as l2 * w.  One pass over a tensor: every operand
// is read once and every result written once, so the kernels are HBM streams (SGD 8 bytes read + 4 written per
// fp32 parameter; Adam 16 read + 12 written, 2 more written when a bf16 copy of the parameter is kept).
#include "kernels.hpp"

namespace rad {

namespace {

__device__ __forceinline__ uint16_t to_bf16(float f) {      // round to nearest even
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <bool ADAM>
__device__ __forceinline__ float update_one(float w, float g, float& m, float& v, const OptimArgs& a) {
  g += a.l2 * w;
  if constexpr (ADAM) {
    m = a.beta1 * m + a.omb1 * g;
    v = a.beta2 * v + a.omb2 * g * g;
    const float m_hat = m * a.inv_bc1, v_hat = v * a.inv_bc2;
    return w - a.lr * m_hat / (sqrtf(v_hat) + a.eps);
  } else {
    return w - a.lr * g;
  }
}

// w: the fp32 parameter (or the fp32 master copy); lo: bf16 copy to refresh, or null.  VEC = 4: whole 16-byte
// vectors of every array; VEC = 1: any alignment, and the tail of the vector form.
template <bool ADAM, int VEC>
__global__ __launch_bounds__(256) void optim_kernel(float* __restrict__ w, uint16_t* __restrict__ lo,
                                                    const float* __restrict__ g, float* __restrict__ m,
                                                    float* __restrict__ v, int64_t first, int64_t n, OptimArgs a) {
  const int64_t i = first + ((int64_t)blockIdx.x * 256 + threadIdx.x) * VEC;
  if (i >= n) return;
  if constexpr (VEC == 4) {
    auto ld = [](const float* p) { return *reinterpret_cast<const float4*>(p); };
    auto stv = [](float* p, float4 x) { *reinterpret_cast<float4*>(p) = x; };
    float4 wv = ld(w + i);
    const float4 gv = ld(g + i);
    float4 mv = make_float4(0.f, 0.f, 0.f, 0.f), vv = mv;
    if constexpr (ADAM) { mv = ld(m + i); vv = ld(v + i); }
    wv.x = update_one<ADAM>(wv.x, gv.x, mv.x, vv.x, a);
    wv.y = update_one<ADAM>(wv.y, gv.y, mv.y, vv.y, a);
    wv.z = update_one<ADAM>(wv.z, gv.z, mv.z, vv.z, a);
    wv.w = update_one<ADAM>(wv.w, gv.w, mv.w, vv.w, a);
    stv(w + i, wv);
    if constexpr (ADAM) { stv(m + i, mv); stv(v + i, vv); }
    if (lo) {
      uint2 p;
      p.x = (uint32_t)to_bf16(wv.x) | ((uint32_t)to_bf16(wv.y) << 16);
      p.y = (uint32_t)to_bf16(wv.z) | ((uint32_t)to_bf16(wv.w) << 16);
      *reinterpret_cast<uint2*>(lo + i) = p;
    }
  } else {
    float mm = 0.f, vv = 0.f;
    if constexpr (ADAM) { mm = m[i]; vv = v[i]; }
    const float wn = update_one<ADAM>(w[i], g[i], mm, vv, a);
    w[i] = wn;
    if constexpr (ADAM) { m[i] = mm; v[i] = vv; }
    if (lo) lo[i] = to_bf16(wn);
  }
}

template <bool ADAM>
hipError_t run(float* w, uint16_t* lo, const float* g, float* m, float* v, int64_t n, const OptimArgs& a,
               hipStream_t st) {
  const uintptr_t align = reinterpret_cast<uintptr_t>(w) | reinterpret_cast<uintptr_t>(g) |
                          reinterpret_cast<uintptr_t>(m) | reinterpret_cast<uintptr_t>(v) |
                          (reinterpret_cast<uintptr_t>(lo) << 1);        // 8-byte vectors of the bf16 copy
  const int64_t nv = (align & 15) ? 0 : n & ~int64_t(3);
  if (nv) {
    const int64_t threads = nv / 4;
    hipLaunchKernelGGL((optim_kernel<ADAM, 4>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, w, lo, g, m,
                       v, int64_t(0), nv, a);
  }
  if (n > nv) {
    hipLaunchKernelGGL((optim_kernel<ADAM, 1>), dim3((unsigned)((n - nv + 255) / 256)), dim3(256), 0, st, w, lo, g, m,
                       v, nv, n, a);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_optim(bool adam, float* w, uint16_t* lo, const float* g, float* m, float* v, int64_t n,
                        const OptimArgs& a, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  return adam ? run<true>(w, lo, g, m, v, n, a, st) : run<false>(w, lo, g, m, v, n, a, st);
}

}  // namespace rad
