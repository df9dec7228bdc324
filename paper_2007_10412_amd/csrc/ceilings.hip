// Measured ceilings of the chip the library runs on: what a kernel with nothing else to do reaches for the
// three resources the hot path is bound by.  HBM: a streaming read (16-byte loads, four in flight per lane)
// and a copy.  MFMA: register-resident loops of the matrix instructions the GEMM kernels issue, on whatever
// operand values the caller supplies (random values draw more power than zeros and run at a lower clock).
// Integer ALU: independent 32 x 32 -> 64-bit multiply-adds, the instruction Philox spends its time in.
#include "kernels.hpp"

namespace rad {

namespace {

__global__ __launch_bounds__(256) void probe_read_kernel(const floatx4* __restrict__ a, float* sink, size_t n) {
  const size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
  floatx4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int u = 0; u < 4; ++u) if (i + u * 256 < n) s += a[i + u * 256];
  if (s[0] + s[1] + s[2] + s[3] == 12345.678f) sink[0] = s[0];      // keeps the loads alive; practically never true
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const floatx4* __restrict__ a, floatx4* __restrict__ b, size_t n) {
  const size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
  floatx4 v[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) if (i + u * 256 < n) v[u] = a[i + u * 256];
#pragma unroll
  for (int u = 0; u < 4; ++u) if (i + u * 256 < n) b[i + u * 256] = v[u];
}

// one workgroup per CU, 4 waves; per iteration a wave issues 32 MFMAs of 32768 flop (16 x 32x32x16) or 64 of 16384
template <int SHAPE>
__global__ __launch_bounds__(256) void probe_mfma_bf16_kernel(const uint16_t* __restrict__ A, float* sink, int iters) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  float s = 0.f;
  if (SHAPE == 0) {
    bf16x8 a[4], b[4];
    for (int i = 0; i < 4; ++i) {
      a[i] = *reinterpret_cast<const bf16x8*>(A + (size_t)(t * 8 + i) * 8);
      b[i] = *reinterpret_cast<const bf16x8*>(A + (size_t)(t * 8 + 4 + i) * 8);
    }
    floatx16 acc[4][4];
    for (int i = 0; i < 4; ++i) for (int j = 0; j < 4; ++j) for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    for (int i = 0; i < 4; ++i) for (int j = 0; j < 4; ++j) for (int e = 0; e < 16; ++e) s += acc[i][j][e];
  } else {
    bf16x8 a[8], b[8];
    for (int i = 0; i < 8; ++i) {
      a[i] = *reinterpret_cast<const bf16x8*>(A + (size_t)(t * 16 + i) * 8);
      b[i] = *reinterpret_cast<const bf16x8*>(A + (size_t)(t * 16 + 8 + i) * 8);
    }
    floatx4 acc[8][8];
    for (int i = 0; i < 8; ++i) for (int j = 0; j < 8; ++j) for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    for (int i = 0; i < 8; ++i) for (int j = 0; j < 8; ++j) for (int e = 0; e < 4; ++e) s += acc[i][j][e];
  }
  if (s == 12345.678f) sink[threadIdx.x] = s;
}

// fp32: v_mfma_f32_32x32x2_f32, 16 accumulator tiles per wave, 4096 flop per instruction
__global__ __launch_bounds__(256) void probe_mfma_f32_kernel(const float* __restrict__ A, float* sink, int iters) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  float a[4], b[4];
  for (int i = 0; i < 4; ++i) { a[i] = A[(size_t)t * 8 + i]; b[i] = A[(size_t)t * 8 + 4 + i]; }
  floatx16 acc[4][4];
  for (int i = 0; i < 4; ++i) for (int j = 0; j < 4; ++j) for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
  }
  float s = 0.f;
  for (int i = 0; i < 4; ++i) for (int j = 0; j < 4; ++j) for (int e = 0; e < 16; ++e) s += acc[i][j][e];
  if (s == 12345.678f) sink[threadIdx.x] = s;
}

// eight independent chains of 32 x 32 + 64 -> 64-bit multiply-adds per lane
__global__ __launch_bounds__(256) void probe_mad64_kernel(const uint32_t* __restrict__ A, float* sink, int iters) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  uint64_t c[8];
  uint32_t m[8];
  for (int i = 0; i < 8; ++i) { m[i] = A[(size_t)t * 8 + i] | 1u; c[i] = m[i]; }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) c[i] = (uint64_t)m[i] * (uint32_t)c[i] + (c[i] >> 32);
  }
  uint64_t s = 0;
  for (int i = 0; i < 8; ++i) s ^= c[i];
  if (s == 0x123456789ull) sink[threadIdx.x] = 1.f;
}

}  // namespace

// work units one launch of probe `kind` performs: bytes moved (read: bytes; copy: 2 x bytes), flop, or multiply-adds
double probe_units(int kind, uint64_t bytes, int iters) {
  switch (kind) {
    case 0: return (double)bytes;
    case 1: return 2.0 * (double)bytes;
    case 2: case 3: return 256.0 * 4 * (double)iters * 32 * 32768.0;
    case 4: return 256.0 * 4 * (double)iters * 16 * 4096.0;
    case 5: return 2048.0 * 256 * 8 * (double)iters;
    default: return 0.0;
  }
}

// smallest operand buffer the probe reads
uint64_t probe_min_bytes(int kind) {
  switch (kind) {
    case 2: return (uint64_t)65536 * 8 * 16;
    case 3: return (uint64_t)65536 * 16 * 16;
    case 4: return (uint64_t)65536 * 8 * 4;
    case 5: return (uint64_t)2048 * 256 * 8 * 4;
    default: return 64;
  }
}

hipError_t launch_probe(int kind, const void* a, void* b, uint64_t bytes, int iters, hipStream_t st) {
  const size_t n = (size_t)(bytes / 16);
  const dim3 grid_stream((unsigned)((n + 1023) / 1024)), block(256);
  switch (kind) {
    case 0: hipLaunchKernelGGL(probe_read_kernel, grid_stream, block, 0, st, (const floatx4*)a, (float*)b, n); break;
    case 1: hipLaunchKernelGGL(probe_copy_kernel, grid_stream, block, 0, st, (const floatx4*)a, (floatx4*)b, n); break;
    case 2: hipLaunchKernelGGL(probe_mfma_bf16_kernel<0>, dim3(256), block, 0, st, (const uint16_t*)a, (float*)b, iters); break;
    case 3: hipLaunchKernelGGL(probe_mfma_bf16_kernel<1>, dim3(256), block, 0, st, (const uint16_t*)a, (float*)b, iters); break;
    case 4: hipLaunchKernelGGL(probe_mfma_f32_kernel, dim3(256), block, 0, st, (const float*)a, (float*)b, iters); break;
    case 5: hipLaunchKernelGGL(probe_mad64_kernel, dim3(2048), block, 0, st, (const uint32_t*)a, (float*)b, iters); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace rad
