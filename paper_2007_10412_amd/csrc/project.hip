// Projection with a Rademacher matrix per example (Appendix A, "different project": a different random matrix
// for each mini-batch element; Section 3.2, P = R R^T / k).  Nothing of R_b is ever stored: its signs are
// drawn where they are used, 128 per Philox call.  Row (b, j) of the sign tensor owns the C = ceil(k / 128)
// calls numbered (b d + j) C .. + C - 1; sign s is bit s mod 32 of word (s / 32) mod 4 of call s / 128, a
// set bit meaning -1.  There is no operand reuse between examples (each is a vector times its own matrix), so
// this is vector-ALU work, three instructions per sign, not a matrix-core contraction.
#include "kernels.hpp"
#include "philox.hpp"

namespace rad {

namespace {

__device__ __forceinline__ float ld_elem(const float* p) { return *p; }
__device__ __forceinline__ float ld_elem(const uint16_t* p) { return bf16_bits_to_f32(*p); }
__device__ __forceinline__ void st_elem(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_elem(uint16_t* p, float v) { *p = f32_to_bf16_bits(v); }

constexpr int kRedPitch = 257;      // 256 partial sums per column, padded so that rows and columns are conflict-free

// z[b, 128 c .. 128 c + 127] = scale * sum_j x[b, j] R_b[j, .]: workgroup (b, c); thread t takes j = t, t + 256, ...
// and keeps 128 partial sums, which are then added across the workgroup in a fixed order.
template <typename T>
__global__ __launch_bounds__(256) void project_rows_fwd_kernel(const T* __restrict__ x, int d, int k, int kp, float scale,
                                                               T* __restrict__ z, uint32_t seed_lo, uint32_t seed_hi,
                                                               uint32_t stream_id, uint32_t step) {
  __shared__ float red[32 * kRedPitch];
  __shared__ float red2[256];
  const int b = blockIdx.x, c = blockIdx.y, C = gridDim.y;
  float acc[128];
#pragma unroll
  for (int i = 0; i < 128; ++i) acc[i] = 0.f;
  for (int j = threadIdx.x; j < d; j += 256) {
    const uint32_t xb = __float_as_uint(ld_elem(x + (size_t)b * d + j));
    const uint32_t mag = xb & 0x7fffffffu;
    const uint32_t flip = (uint32_t)((int32_t)xb >> 31);            // all ones if x < 0
    const u32x4 w = element_quad_keys(((uint64_t)b * d + j) * C + c, stream_id, step, seed_lo, seed_hi);
#pragma unroll
    for (int wi = 0; wi < 4; ++wi) {
      const uint32_t ws = w[wi] ^ flip;                             // sign of x R[j, s] in bit s
#pragma unroll
      for (int i = 0; i < 32; ++i) acc[wi * 32 + i] += __uint_as_float(((ws << (31 - i)) & 0x80000000u) | mag);
    }
  }
  // 256 partial sums per column, added in a fixed order, 32 columns at a time (a quarter of the LDS of doing all
  // 128 at once, so that three workgroups fit a CU): thread (part, col) adds 32 of them, then 8 parts per column
  const int col = threadIdx.x & 31, part = threadIdx.x >> 5;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 32; ++i) red[i * kRedPitch + threadIdx.x] = acc[r * 32 + i];
    __syncthreads();
    float s = 0.f;
    for (int u = 0; u < 32; ++u) s += red[col * kRedPitch + part * 32 + u];
    red2[part * 32 + col] = s;
    __syncthreads();
    if (threadIdx.x < 32) {
      const int out = c * 128 + r * 32 + (int)threadIdx.x;
      if (out < kp) {
        const float t = ((red2[col] + red2[32 + col]) + (red2[64 + col] + red2[96 + col])) +
                        ((red2[128 + col] + red2[160 + col]) + (red2[192 + col] + red2[224 + col]));
        st_elem(z + (size_t)b * kp + out, out < k ? t * scale : 0.f);
      }
    }
  }
}

// xt[b, j] = scale * sum_s z[b, s] R_b[j, s]: workgroup = 256 consecutive j of example b; z[b, :] sits in LDS and is
// read as broadcasts.  With m_s = 1 for a set bit: sum_s z_s (1 - 2 m_s) = total - 2 sum_s m_s z_s.
template <typename T>
__global__ __launch_bounds__(256) void project_rows_bwd_kernel(const T* __restrict__ z, int d, int k, int kp, int C,
                                                               float scale, T* __restrict__ xt, uint32_t seed_lo,
                                                               uint32_t seed_hi, uint32_t stream_id, uint32_t step) {
  extern __shared__ __align__(16) float zs[];    // [128 C], zeros past k
  __shared__ float s_part[4];
  const int nb = (d + 255) / 256;
  const int b = (int)(blockIdx.x / (unsigned)nb), jb = (int)(blockIdx.x % (unsigned)nb);
  float part = 0.f;
  for (int i = threadIdx.x; i < 128 * C; i += 256) {
    const float v = i < k ? ld_elem(z + (size_t)b * kp + i) : 0.f;
    zs[i] = v;
    part += v;
  }
  // total of the row, the same for every thread: wave sums in lane order, then the four waves in order
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off, 64);
  if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = part;
  __syncthreads();
  const float total = (s_part[0] + s_part[1]) + (s_part[2] + s_part[3]);
  const int j = jb * 256 + (int)threadIdx.x;
  if (j >= d) return;
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  for (int c = 0; c < C; ++c) {
    const u32x4 w = element_quad_keys(((uint64_t)b * d + j) * C + c, stream_id, step, seed_lo, seed_hi);
#pragma unroll
    for (int wi = 0; wi < 4; ++wi) {
      const uint32_t ws = w[wi];
      const float4* zp = reinterpret_cast<const float4*>(zs + c * 128 + wi * 32);
#pragma unroll
      for (int i = 0; i < 32; i += 4) {
        const float4 zv = zp[i >> 2];
        // (ws << (31 - i)) >> 31 is all ones where bit i is set
        a0 += __uint_as_float((uint32_t)((int32_t)(ws << (31 - i)) >> 31) & __float_as_uint(zv.x));
        a1 += __uint_as_float((uint32_t)((int32_t)(ws << (30 - i)) >> 31) & __float_as_uint(zv.y));
        a2 += __uint_as_float((uint32_t)((int32_t)(ws << (29 - i)) >> 31) & __float_as_uint(zv.z));
        a3 += __uint_as_float((uint32_t)((int32_t)(ws << (28 - i)) >> 31) & __float_as_uint(zv.w));
      }
    }
  }
  st_elem(xt + (size_t)b * d + j, (total - 2.f * ((a0 + a1) + (a2 + a3))) * scale);
}

template <typename K>
hipError_t allow_lds(K kern, int bytes) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

}  // namespace

hipError_t launch_project_rows_fwd(const void* x, int dtype, int rows, int d, int k, int kp, float scale, void* z,
                                   uint32_t seed_lo, uint32_t seed_hi, uint32_t stream_id, uint32_t step,
                                   hipStream_t st) {
  const int C = (k + 127) / 128;
  if (C > 65535) return hipErrorInvalidValue;
  dim3 grid((unsigned)rows, (unsigned)C), block(256);
  if (dtype == kF32) {
    auto kern = project_rows_fwd_kernel<float>;
    hipLaunchKernelGGL(kern, grid, block, 0, st, (const float*)x, d, k, kp, scale, (float*)z, seed_lo, seed_hi,
                       stream_id, step);
  } else {
    auto kern = project_rows_fwd_kernel<uint16_t>;
    hipLaunchKernelGGL(kern, grid, block, 0, st, (const uint16_t*)x, d, k, kp, scale, (uint16_t*)z, seed_lo, seed_hi,
                       stream_id, step);
  }
  return hipGetLastError();
}

hipError_t launch_project_rows_bwd(const void* z, int dtype, int rows, int d, int k, int kp, float scale, void* xt,
                                   uint32_t seed_lo, uint32_t seed_hi, uint32_t stream_id, uint32_t step,
                                   hipStream_t st) {
  const int C = (k + 127) / 128;
  const int smem = 128 * C * 4;
  const int64_t blocks = (int64_t)rows * ((d + 255) / 256);
  if (smem > 150 * 1024 || blocks > 0x7fffffff) return hipErrorInvalidValue;
  dim3 grid((unsigned)blocks), block(256);
  if (dtype == kF32) {
    auto kern = project_rows_bwd_kernel<float>;
    hipError_t e = allow_lds(kern, smem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, block, smem, st, (const float*)z, d, k, kp, C, scale, (float*)xt, seed_lo, seed_hi,
                       stream_id, step);
  } else {
    auto kern = project_rows_bwd_kernel<uint16_t>;
    hipError_t e = allow_lds(kern, smem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, block, smem, st, (const uint16_t*)z, d, k, kp, C, scale, (uint16_t*)xt, seed_lo,
                       seed_hi, stream_id, step);
  }
  return hipGetLastError();
}

}  // namespace rad
