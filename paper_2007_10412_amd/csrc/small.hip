// Loss, bias-gradient and fill kernels of the RAD train step.
#include "philox.hpp"
#include "kernels.hpp"

namespace rad {
namespace {

__device__ __forceinline__ float ld_elem(const float* p) { return *p; }
__device__ __forceinline__ float ld_elem(const uint16_t* p) { return bf16_bits_to_f32(*p); }
__device__ __forceinline__ void st_elem(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_elem(uint16_t* p, float v) { *p = f32_to_bf16_bits(v); }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// One wave per example: loss_b = -log softmax(z_b)[label_b],
// dz_b = (softmax(z_b) - onehot(label_b)) / rows.  The logits stay dense
// (Appendix A: the softmax input is not sampled).
template <typename T>
__global__ __launch_bounds__(256) void softmax_ce_kernel(const T* __restrict__ z, const int32_t* __restrict__ labels,
                                                         int rows, int classes, T* __restrict__ dz,
                                                         float* __restrict__ row_loss) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const T* zr = z + (size_t)row * classes;
  float m = -INFINITY;
  for (int c = lane; c < classes; c += 64) m = fmaxf(m, ld_elem(zr + c));
  m = wave_max(m);
  float s = 0.f;
  for (int c = lane; c < classes; c += 64) s += expf(ld_elem(zr + c) - m);
  s = wave_sum(s);
  const int lab = labels[row];
  const bool lab_ok = lab >= 0 && lab < classes;     // a bad label poisons the loss instead of the address
  const float inv = 1.f / s, invb = 1.f / (float)rows;
  T* dr = dz + (size_t)row * classes;
  for (int c = lane; c < classes; c += 64) {
    float p = expf(ld_elem(zr + c) - m) * inv;
    if (c == lab) p -= 1.f;
    st_elem(dr + c, p * invb);
  }
  if (lane == 0) row_loss[row] = lab_ok ? -(ld_elem(zr + lab) - m - logf(s)) : NAN;
}

// The same for rows that are whole 16-byte vectors and at most NV of them per lane: a lane keeps its part of
// the row in registers, so the row is read once (16-byte loads) and every exponential is taken once.
template <typename T, int NV>
__global__ __launch_bounds__(256) void softmax_ce_vec_kernel(const T* __restrict__ z, const int32_t* __restrict__ labels,
                                                             int rows, int classes, T* __restrict__ dz, int dz_ld,
                                                             float* __restrict__ row_loss) {
  constexpr int VPL = 16 / (int)sizeof(T);            // elements per vector
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int nvec = classes / VPL;
  const T* zr = z + (size_t)row * classes;
  float v[NV][VPL];
  float m = -INFINITY;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int q = lane + i * 64;
    u32x4 raw = {0u, 0u, 0u, 0u};
    if (q < nvec) raw = *reinterpret_cast<const u32x4*>(zr + (size_t)q * VPL);
    const T* re = reinterpret_cast<const T*>(&raw);
#pragma unroll
    for (int e = 0; e < VPL; ++e) {
      v[i][e] = q < nvec ? ld_elem(re + e) : -INFINITY;
      m = fmaxf(m, v[i][e]);
    }
  }
  m = wave_max(m);
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i)
#pragma unroll
    for (int e = 0; e < VPL; ++e) { v[i][e] = expf(v[i][e] - m); s += v[i][e]; }     // exp(-inf) = 0 past the row
  s = wave_sum(s);
  const int lab = labels[row];
  const bool lab_ok = lab >= 0 && lab < classes;     // a bad label poisons the loss instead of the address
  const float inv = 1.f / s, invb = 1.f / (float)rows;
  // dz rows are dz_ld apart (a multiple of VPL, at most 64 NV vectors); columns past `classes` are written as zeros
  T* dr = dz + (size_t)row * dz_ld;
  const int nvec_out = dz_ld / VPL;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int q = lane + i * 64;
    u32x4 out;
    T* oe = reinterpret_cast<T*>(&out);
#pragma unroll
    for (int e = 0; e < VPL; ++e) {
      float p = v[i][e] * inv;
      if (q * VPL + e == lab) p -= 1.f;
      st_elem(oe + e, p * invb);
    }
    if (q < nvec) *reinterpret_cast<u32x4*>(dr + (size_t)q * VPL) = out;
    else if (q < nvec_out) *reinterpret_cast<u32x4*>(dr + (size_t)q * VPL) = u32x4{0u, 0u, 0u, 0u};
  }
  if (lane == 0) row_loss[row] = lab_ok ? -(ld_elem(zr + lab) - m - logf(s)) : NAN;
}

// deterministic mean of the per-example losses
__global__ __launch_bounds__(256) void loss_mean_kernel(const float* __restrict__ row_loss, int rows,
                                                        float* __restrict__ loss) {
  __shared__ float s_w[4];
  float acc = 0.f;
  for (int r = threadIdx.x; r < rows; r += 256) acc += row_loss[r];
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) s_w[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) *loss = (s_w[0] + s_w[1] + s_w[2] + s_w[3]) / (float)rows;
}

constexpr int kMaxU = 8;

// stage 1 of the weighted column sums of g = dy * bits
template <typename T>
__global__ __launch_bounds__(256) void colsum_partial_kernel(const T* __restrict__ dy, int rows, int N, int64_t ldy,
                                                             const uint32_t* __restrict__ bits, int bits_pitch,
                                                             const float* __restrict__ u, int64_t u_ld, int u_n,
                                                             int u_block_rows, int64_t u_block_stride,
                                                             float* __restrict__ partial, int splits,
                                                             float* __restrict__ out_bias, float* __restrict__ out_u,
                                                             int beta) {
  __shared__ float s_red[4][kMaxU + 1][64];
  const int cx = threadIdx.x & 63, ry = threadIdx.x >> 6;
  const int col = blockIdx.x * 64 + cx;
  const int split = blockIdx.y;
  const int per = (rows + splits - 1) / splits;
  const int rbeg = split * per, rend = min(rows, rbeg + per);
  float acc[kMaxU + 1];
#pragma unroll
  for (int i = 0; i <= kMaxU; ++i) acc[i] = 0.f;
  if (col < N) {
    for (int r = rbeg + ry; r < rend; r += 4) {
      float g = ld_elem(dy + (size_t)r * ldy + col);
      if (bits && !((bits[(size_t)r * bits_pitch + (col >> 5)] >> (col & 31)) & 1u)) g = 0.f;
      acc[0] += g;
      // rows come in blocks of u_block_rows (time steps): row b of block q weighs with u[b u_ld + q u_block_stride + i]
      const int q = r / u_block_rows;
      const float* ur = u + (size_t)(r - q * u_block_rows) * u_ld + (size_t)q * u_block_stride;
#pragma unroll
      for (int i = 0; i < kMaxU; ++i) if (i < u_n) acc[i + 1] += ur[i] * g;
    }
  }
#pragma unroll
  for (int i = 0; i <= kMaxU; ++i) s_red[ry][i][cx] = acc[i];
  __syncthreads();
  if (ry == 0 && col < N) {
    for (int i = 0; i <= u_n; ++i) {
      const float v = s_red[0][i][cx] + s_red[1][i][cx] + s_red[2][i][cx] + s_red[3][i][cx];
      if (splits > 1) { partial[((size_t)split * (u_n + 1) + i) * N + col] = v; continue; }
      // one split: this is the result (few rows: a second launch would cost more than it adds)
      float* dst = i == 0 ? (out_bias ? out_bias + col : nullptr) : (out_u ? out_u + (size_t)(i - 1) * N + col : nullptr);
      if (dst) *dst = beta ? *dst + v : v;
    }
  }
}

__global__ __launch_bounds__(256) void colsum_final_kernel(const float* __restrict__ partial, int splits, int N,
                                                           int u_n, float* __restrict__ out_bias,
                                                           float* __restrict__ out_u, int beta) {
  const int col = blockIdx.x * 256 + threadIdx.x;
  if (col >= N) return;
  for (int i = 0; i <= u_n; ++i) {
    float v = 0.f;
    for (int s = 0; s < splits; ++s) v += partial[((size_t)s * (u_n + 1) + i) * N + col];
    float* dst = i == 0 ? (out_bias ? out_bias + col : nullptr) : (out_u ? out_u + (size_t)(i - 1) * N + col : nullptr);
    if (dst) *dst = beta ? *dst + v : v;
  }
}

// Entries of a (store row, bucket) segment beyond the first `cap` are left out by the MFMA dW kernel,
// whose registers hold `cap` of them; this kernel adds their contribution dW[j, :] += value * g[b, :].
// One wave per segment.  *max_seg is the plan's running maximum segment length: the kernel leaves at once
// when no segment is that long, which is the normal case (cap sits six standard deviations above the mean).
template <typename T>
__global__ __launch_bounds__(256) void dw_overflow_kernel(StoreView s, int rows, const T* __restrict__ dy, int N,
                                                          int64_t ldy, const uint32_t* __restrict__ bits, int bits_pitch,
                                                          float* __restrict__ dW, int cap,
                                                          const int* __restrict__ max_seg) {
  if (*max_seg <= cap) return;
  const int lane = threadIdx.x & 63;
  for (int seg = blockIdx.x * 4 + (threadIdx.x >> 6); seg < rows * s.nb; seg += gridDim.x * 4) {
  const int b = seg / s.nb, t = seg % s.nb;
  const uint16_t* bo = s.bucket_off + (size_t)(b * s.plan_row_stride) * (s.nb + 1) + t;
  const int64_t base = s.row_ptr[b];
  int64_t beg = base + bo[0], end = base + bo[1];
  if (end > s.capacity) end = s.capacity;
  const T* vals = reinterpret_cast<const T*>(s.values);
  for (int64_t e = beg + cap; e < end; ++e) {
    int j; float v;
    if (s.paired) {
      const uint32_t u = reinterpret_cast<const uint32_t*>(s.values)[e];
      j = pair_col(u, t); v = __uint_as_float(u & 0xFFFF0000u);
    } else {
      j = s.indices[e]; v = ld_elem(vals + e);
    }
    for (int n = lane; n < N; n += 64) {
      float g = ld_elem(dy + (size_t)b * ldy + n);
      if (bits && !((bits[(size_t)b * bits_pitch + (n >> 5)] >> (n & 31)) & 1u)) g = 0.f;
      atomicAdd(&dW[(size_t)j * N + n], v * g);
    }
  }
  }
}

__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, int splits, int64_t n,
                                                            float* __restrict__ out, int beta) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  float v = 0.f;
  for (int s = 0; s < splits; ++s) v += partial[(size_t)s * n + i];
  out[i] = beta ? out[i] + v : v;
}
// the same four elements at a time (n a multiple of 4, 16-byte aligned arrays)
__global__ __launch_bounds__(256) void splitk_reduce4_kernel(const float4* __restrict__ partial, int splits, int64_t n4,
                                                             float4* __restrict__ out, int beta) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  float4 v = partial[i];
  for (int s = 1; s < splits; ++s) {
    const float4 t = partial[(size_t)s * n4 + i];
    v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
  }
  if (beta) { const float4 o = out[i]; v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w; }
  out[i] = v;
}
// Many splits, few outputs (a convolution's dW: a few thousand numbers, a partial sum per workgroup of the kernel
// before): 16 threads share an output vector, thread j adds splits j, j + 16, ... in order, and the 16 sums are
// added pairwise in a fixed tree.  The result depends on `splits` alone, never on timing.
__global__ __launch_bounds__(256) void splitk_reduce_wide_kernel(const float4* __restrict__ partial, int splits, int64_t n4,
                                                                 float4* __restrict__ out, int beta) {
  __shared__ float4 s_sum[16][17];
  const int o = threadIdx.x & 15, j = threadIdx.x >> 4;
  const int64_t i = (int64_t)blockIdx.x * 16 + o;
  float4 v = {0.f, 0.f, 0.f, 0.f};
  if (i < n4)
    for (int s = j; s < splits; s += 16) {
      const float4 t = partial[(size_t)s * n4 + i];
      v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
    }
  s_sum[j][o] = v;
  __syncthreads();
  for (int half = 8; half > 0; half >>= 1) {
    if (j < half) {
      const float4 a = s_sum[j][o], b = s_sum[j + half][o];
      s_sum[j][o] = float4{a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w};
    }
    __syncthreads();
  }
  if (j == 0 && i < n4) {
    float4 r = s_sum[0][o];
    if (beta) { const float4 p = out[i]; r.x += p.x; r.y += p.y; r.z += p.z; r.w += p.w; }
    out[i] = r;
  }
}
// Sum of the splits of a compact dW (shared index set): partial [splits][rows][N] in a fixed order, tile row r
// goes to output row row_map[r] (or r); V = float4 when N and ld are multiples of 4, else float
template <typename V>
__global__ __launch_bounds__(256) void splitk_reduce_rows_kernel(const V* __restrict__ partial, int splits, int64_t stride,
                                                                 int rows, int NV, const uint16_t* __restrict__ row_map,
                                                                 V* __restrict__ out, int64_t ldv, int beta, int64_t in_ldv) {
  const int64_t i0 = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i0 >= (int64_t)rows * NV) return;
  const int r = (int)(i0 / NV), n = (int)(i0 - (int64_t)r * NV);
  const int64_t i = (int64_t)r * in_ldv + n;             // rows of a partial array are in_ldv apart
  float acc[sizeof(V) / 4];
  const V first = partial[i];
#pragma unroll
  for (int e = 0; e < (int)(sizeof(V) / 4); ++e) acc[e] = reinterpret_cast<const float*>(&first)[e];
  for (int s = 1; s < splits; ++s) {
    const V t = partial[(size_t)s * stride + i];
#pragma unroll
    for (int e = 0; e < (int)(sizeof(V) / 4); ++e) acc[e] += reinterpret_cast<const float*>(&t)[e];
  }
  V* dst = out + (size_t)(row_map ? (int)row_map[r] : r) * ldv + n;
  if (beta) {
    const V o = *dst;
#pragma unroll
    for (int e = 0; e < (int)(sizeof(V) / 4); ++e) acc[e] += reinterpret_cast<const float*>(&o)[e];
  }
  V res;
#pragma unroll
  for (int e = 0; e < (int)(sizeof(V) / 4); ++e) reinterpret_cast<float*>(&res)[e] = acc[e];
  *dst = res;
}
// Sum of the splits of a forward GEMM, plus bias, into the layer output (no activation): partial [splits][M][N]
template <typename T>
__global__ __launch_bounds__(256) void splitk_bias_kernel(const float* __restrict__ partial, int splits, int M, int N,
                                                          int64_t pld, int64_t pstride, const float* __restrict__ bias,
                                                          T* __restrict__ out) {
  const int64_t n = (int64_t)M * N;
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= n) return;
  // N is a multiple of 4 here, so the four elements share a row; the rows of a partial array are pld apart
  const int64_t row = i / N;
  const int col = (int)(i - row * N);
  const float* src = partial + row * pld + col;
  float4 v = *reinterpret_cast<const float4*>(src);
  for (int s = 1; s < splits; ++s) {
    const float4 t = *reinterpret_cast<const float4*>(src + (size_t)s * pstride);
    v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
  }
  if (bias) { v.x += bias[col]; v.y += bias[col + 1]; v.z += bias[col + 2]; v.w += bias[col + 3]; }
  st_elem(out + i, v.x); st_elem(out + i + 1, v.y); st_elem(out + i + 2, v.z); st_elem(out + i + 3, v.w);
}

// 2x2 max pool, stride 2.  One thread produces 16 consecutive outputs of a plane row-major and the word of
// their 2-bit window positions; the first maximum in (dy, dx) row-major order wins.
__global__ __launch_bounds__(256) void maxpool_fwd_kernel(const float* __restrict__ y, int planes, int H, int W,
                                                          float* __restrict__ pooled, uint32_t* __restrict__ arg) {
  const int Ho = H / 2, Wo = W / 2;
  const int64_t total = (int64_t)planes * Ho * Wo;
  const int64_t q0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 16;
  if (q0 >= total) return;
  uint32_t word = 0;
  for (int e = 0; e < 16; ++e) {
    const int64_t q = q0 + e;
    if (q >= total) break;
    const int64_t pl = q / (Ho * Wo);
    const int r = (int)(q - pl * (Ho * Wo));
    const int oy = r / Wo, ox = r - oy * Wo;
    const float* src = y + (size_t)pl * H * W + (size_t)(2 * oy) * W + 2 * ox;
    float best = src[0]; uint32_t pos = 0;
    if (src[1] > best) { best = src[1]; pos = 1; }
    if (src[W] > best) { best = src[W]; pos = 2; }
    if (src[W + 1] > best) { best = src[W + 1]; pos = 3; }
    pooled[q] = best;
    word |= pos << (2 * e);
  }
  arg[q0 / 16] = word;
}

// The same for planes whose output rows are WO = 4, 8 or 16 wide: a thread's 16 consecutive outputs are whole
// output rows, and their 64 inputs lie in one contiguous run of the plane, read as sixteen 16-byte vectors.
template <int WO>
__global__ __launch_bounds__(256) void maxpool_rows_kernel(const float* __restrict__ y, int64_t total,
                                                           float* __restrict__ pooled, uint32_t* __restrict__ arg) {
  const int64_t q0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 16;
  if (q0 >= total) return;
  // output q = (plane, oy, ox) row-major with rows of WO; its window starts at input offset 4 q - 2 (q % WO)
  const floatx4* src = reinterpret_cast<const floatx4*>(y + 4 * q0);
  float f[64];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const floatx4 v = src[i];
#pragma unroll
    for (int e = 0; e < 4; ++e) f[4 * i + e] = v[e];
  }
  uint32_t word = 0;
  float out[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    constexpr int W = 2 * WO;
    const int i00 = (2 * (e / WO)) * W + 2 * (e % WO);
    float best = f[i00]; uint32_t pos = 0;
    if (f[i00 + 1] > best) { best = f[i00 + 1]; pos = 1; }
    if (f[i00 + W] > best) { best = f[i00 + W]; pos = 2; }
    if (f[i00 + W + 1] > best) { best = f[i00 + W + 1]; pos = 3; }
    out[e] = best;
    word |= pos << (2 * e);
  }
  floatx4* dst = reinterpret_cast<floatx4*>(pooled + q0);
#pragma unroll
  for (int i = 0; i < 4; ++i) dst[i] = floatx4{out[4 * i], out[4 * i + 1], out[4 * i + 2], out[4 * i + 3]};
  arg[q0 / 16] = word;
}

// 2x2 average pool, stride 2 (the pooling of the convolutional architecture in Appendix A): one thread per
// output; nothing is kept for the backward pass.
__global__ __launch_bounds__(256) void avgpool_fwd_kernel(const float* __restrict__ y, int planes, int H, int W,
                                                          float* __restrict__ pooled) {
  const int Ho = H / 2, Wo = W / 2;
  const int64_t total = (int64_t)planes * Ho * Wo;
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (q >= total) return;
  const int64_t pl = q / (Ho * Wo);
  const int r = (int)(q - pl * (Ho * Wo));
  const int oy = r / Wo, ox = r - oy * Wo;
  const float* src = y + (size_t)pl * H * W + (size_t)(2 * oy) * W + 2 * ox;
  const float2 top = *reinterpret_cast<const float2*>(src), bot = *reinterpret_cast<const float2*>(src + W);
  pooled[q] = 0.25f * ((top.x + top.y) + (bot.x + bot.y));
}

// g = (dy routed back through the pool, if any) masked by the ReLU bits of the layer output [B][C*H*W];
// pool: 0 none, 1 max pool (2-bit window positions in arg), 2 average pool
__global__ __launch_bounds__(256) void unpool_mask_kernel(const float* __restrict__ dy, int batch, int C, int H, int W,
                                                          int pool, const uint32_t* __restrict__ arg,
                                                          const uint32_t* __restrict__ bits, int bits_pitch,
                                                          float* __restrict__ g) {
  const int64_t per = (int64_t)C * H * W;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= batch * per) return;
  const int b = (int)(i / per);
  const int64_t f = i - (int64_t)b * per;
  float v;
  if (pool) {
    const int Ho = H / 2, Wo = W / 2;
    const int c = (int)(f / (H * W)), yx = (int)(f - (int64_t)c * H * W);
    const int y = yx / W, x = yx - y * W;
    const int64_t q = ((int64_t)(b * C + c) * Ho + y / 2) * Wo + x / 2;
    if (pool == 1) {
      const uint32_t pos = (arg[q / 16] >> (2 * (q % 16))) & 3u;
      v = (pos == (uint32_t)((y & 1) * 2 + (x & 1))) ? dy[q] : 0.f;
    } else {
      v = 0.25f * dy[q];
    }
  } else {
    v = dy[i];
  }
  if (bits && !((bits[(size_t)b * bits_pitch + (f >> 5)] >> (f & 31)) & 1u)) v = 0.f;
  g[i] = v;
}

// The same, four consecutive x per thread (W a multiple of 4): one index decomposition, one mask word, one
// 16-byte store.
__global__ __launch_bounds__(256) void unpool_mask4_kernel(const float* __restrict__ dy, int batch, int C, int H, int W,
                                                           int pool, const uint32_t* __restrict__ arg,
                                                           const uint32_t* __restrict__ bits, int bits_pitch,
                                                           float* __restrict__ g) {
  const int64_t per = (int64_t)C * H * W;
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= batch * per) return;
  const int b = (int)(i / per);
  const int64_t f = i - (int64_t)b * per;
  floatx4 v;
  if (pool) {
    const int Ho = H / 2, Wo = W / 2;
    const int c = (int)(f / (H * W)), yx = (int)(f - (int64_t)c * H * W);
    const int y = yx / W, x = yx - y * W;                  // x is a multiple of 4
    const int64_t q = ((int64_t)(b * C + c) * Ho + y / 2) * Wo + x / 2;      // even: q and q + 1 share an arg word
    const float d0 = dy[q], d1 = dy[q + 1];
    if (pool == 1) {
      const uint32_t pw = arg[q / 16] >> (2 * (q % 16));
      const uint32_t p0 = pw & 3u, p1 = (pw >> 2) & 3u, top = (uint32_t)((y & 1) * 2);
      v = floatx4{p0 == top ? d0 : 0.f, p0 == top + 1 ? d0 : 0.f, p1 == top ? d1 : 0.f, p1 == top + 1 ? d1 : 0.f};
    } else {
      v = floatx4{0.25f * d0, 0.25f * d0, 0.25f * d1, 0.25f * d1};
    }
  } else {
    v = *reinterpret_cast<const floatx4*>(dy + i);
  }
  if (bits) {
    const uint32_t m = bits[(size_t)b * bits_pitch + (f >> 5)] >> (f & 31);
#pragma unroll
    for (int e = 0; e < 4; ++e) if (!((m >> e) & 1u)) v[e] = 0.f;
  }
  *reinterpret_cast<floatx4*>(g + i) = v;
}

// db[c] = sum_{b,yx} g[b,c,yx]; one workgroup per channel, fixed summation order
__global__ __launch_bounds__(256) void channel_sum_kernel(const float* __restrict__ g, int batch, int C, int HW,
                                                          int splits, float* __restrict__ partial) {
  // workgroup (channel c, split s) adds the planes of examples s, s + splits, ...; partial[c][s]
  __shared__ float s_w[4];
  const int c = blockIdx.x, sp = blockIdx.y;
  float acc = 0.f;
  for (int b = sp; b < batch; b += splits) {
    const float* src = g + ((size_t)b * C + c) * HW;
    for (int i = threadIdx.x; i < HW; i += 256) acc += src[i];
  }
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) s_w[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) partial[(size_t)c * splits + sp] = s_w[0] + s_w[1] + s_w[2] + s_w[3];
}

__global__ __launch_bounds__(256) void channel_sum_final_kernel(const float* __restrict__ partial, int C, int splits,
                                                                float* __restrict__ db) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= C) return;
  float v = 0.f;
  for (int s = 0; s < splits; ++s) v += partial[(size_t)c * splits + s];      // fixed order
  db[c] = v;
}

__global__ __launch_bounds__(256) void flip_weights_kernel(const float* __restrict__ W, int Ci, int KH, int KW, int Co,
                                                           float* __restrict__ Wt) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= Ci * KH * KW * Co) return;
  // i indexes Wt[(o,u,v)][c]
  const int c = i % Ci, ouv = i / Ci;
  const int v = ouv % KW, ou = ouv / KW;
  const int u = ou % KH, o = ou / KH;
  Wt[i] = W[(((size_t)c * KH + (KH - 1 - u)) * KW + (KW - 1 - v)) * Co + o];
}

__global__ __launch_bounds__(256) void fill_u32_kernel(uint32_t* __restrict__ p, uint32_t v, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = v;
}

}  // namespace

hipError_t launch_softmax_ce(const void* logits, const int32_t* labels, int rows, int classes, int dtype,
                             void* dlogits, float* row_loss, float* loss, hipStream_t st, int dz_ld) {
  dim3 grid((rows + 3) / 4), block(256);
  const int vpl = dtype == kF32 ? 4 : 8;
  if (dz_ld <= 0) dz_ld = classes;
  const bool vec = classes % vpl == 0 && dz_ld % vpl == 0 && dz_ld / vpl <= 128 &&
                   (reinterpret_cast<uintptr_t>(logits) & 15) == 0 && (reinterpret_cast<uintptr_t>(dlogits) & 15) == 0;
  if (dz_ld != classes && !vec) return hipErrorInvalidValue;      // only the vector kernels write pitched rows
  if (vec && dtype == kF32)
    hipLaunchKernelGGL((softmax_ce_vec_kernel<float, 2>), grid, block, 0, st, (const float*)logits, labels, rows, classes,
                       (float*)dlogits, dz_ld, row_loss);
  else if (vec)
    hipLaunchKernelGGL((softmax_ce_vec_kernel<uint16_t, 2>), grid, block, 0, st, (const uint16_t*)logits, labels, rows,
                       classes, (uint16_t*)dlogits, dz_ld, row_loss);
  else if (dtype == kF32)
    hipLaunchKernelGGL(softmax_ce_kernel<float>, grid, block, 0, st, (const float*)logits, labels, rows, classes,
                       (float*)dlogits, row_loss);
  else
    hipLaunchKernelGGL(softmax_ce_kernel<uint16_t>, grid, block, 0, st, (const uint16_t*)logits, labels, rows,
                       classes, (uint16_t*)dlogits, row_loss);
  if (loss) hipLaunchKernelGGL(loss_mean_kernel, dim3(1), dim3(256), 0, st, row_loss, rows, loss);   // null: gradient only
  return hipGetLastError();
}

hipError_t launch_colsum(const void* dy, int dtype, int rows, int N, const uint32_t* bits, int bits_pitch,
                         const float* u, int64_t u_ld, int u_n, float* out_bias, float* out_u, int beta,
                         float* partial, int splits, hipStream_t st, int u_block_rows, int64_t u_block_stride,
                         int64_t ldy) {
  if (u_n > kMaxU) return hipErrorInvalidValue;
  if (ldy <= 0) ldy = N;
  if (u_block_rows <= 0) { u_block_rows = rows > 0 ? rows : 1; u_block_stride = 0; }
  dim3 grid((N + 63) / 64, splits), block(256);
  if (dtype == kF32)
    hipLaunchKernelGGL(colsum_partial_kernel<float>, grid, block, 0, st, (const float*)dy, rows, N, ldy, bits, bits_pitch,
                       u, u_ld, u_n, u_block_rows, u_block_stride, partial, splits, out_bias, out_u, beta);
  else
    hipLaunchKernelGGL(colsum_partial_kernel<uint16_t>, grid, block, 0, st, (const uint16_t*)dy, rows, N, ldy, bits,
                       bits_pitch, u, u_ld, u_n, u_block_rows, u_block_stride, partial, splits, out_bias, out_u, beta);
  if (splits > 1)
    hipLaunchKernelGGL(colsum_final_kernel, dim3((N + 255) / 256), dim3(256), 0, st, partial, splits, N, u_n, out_bias,
                     out_u, beta);
  return hipGetLastError();
}

hipError_t launch_dw_overflow(const StoreView& s, int rows, const void* dy, int dtype, int N, const uint32_t* bits,
                              int bits_pitch, float* dW, int cap, const int* max_seg, hipStream_t st, int64_t ldy) {
  if (ldy <= 0) ldy = N;
  // almost always the kernel only reads *max_seg and leaves: a small grid keeps that cheap, and the
  // workgroups walk the segments in strides when there is work
  const int segs = rows * s.nb;
  const int blocks = (segs + 3) / 4;
  dim3 grid(blocks < 256 ? blocks : 256), block(256);
  if (dtype == kF32)
    hipLaunchKernelGGL(dw_overflow_kernel<float>, grid, block, 0, st, s, rows, (const float*)dy, N, ldy, bits, bits_pitch,
                       dW, cap, max_seg);
  else
    hipLaunchKernelGGL(dw_overflow_kernel<uint16_t>, grid, block, 0, st, s, rows, (const uint16_t*)dy, N, ldy, bits,
                       bits_pitch, dW, cap, max_seg);
  return hipGetLastError();
}

hipError_t launch_splitk_reduce(const float* partial, int splits, int64_t n, float* out, int beta, hipStream_t st) {
  if (n % 4 == 0 && ((reinterpret_cast<uintptr_t>(partial) | reinterpret_cast<uintptr_t>(out)) & 15) == 0) {
    const int64_t n4 = n / 4;
    if (splits >= 32 && n4 < (int64_t)splits * 256) {      // too few outputs to fill the chip with a thread each
      hipLaunchKernelGGL(splitk_reduce_wide_kernel, dim3((unsigned)((n4 + 15) / 16)), dim3(256), 0, st,
                         reinterpret_cast<const float4*>(partial), splits, n4, reinterpret_cast<float4*>(out), beta);
      return hipGetLastError();
    }
    hipLaunchKernelGGL(splitk_reduce4_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st,
                       reinterpret_cast<const float4*>(partial), splits, n4, reinterpret_cast<float4*>(out), beta);
  } else {
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, partial, splits, n,
                       out, beta);
  }
  return hipGetLastError();
}

hipError_t launch_splitk_reduce_rows(const float* partial, int splits, int64_t stride, int rows, int N,
                                     const uint16_t* row_map, float* out, int64_t ld, int beta, hipStream_t st,
                                     int64_t in_ld) {
  if (in_ld <= 0) in_ld = N;
  const bool vec = N % 4 == 0 && ld % 4 == 0 && stride % 4 == 0 && in_ld % 4 == 0 &&
                   ((reinterpret_cast<uintptr_t>(partial) | reinterpret_cast<uintptr_t>(out)) & 15) == 0;
  if (vec) {
    const int64_t total = (int64_t)rows * (N / 4);
    hipLaunchKernelGGL(splitk_reduce_rows_kernel<float4>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       reinterpret_cast<const float4*>(partial), splits, stride / 4, rows, N / 4, row_map,
                       reinterpret_cast<float4*>(out), ld / 4, beta, in_ld / 4);
  } else {
    const int64_t total = (int64_t)rows * N;
    hipLaunchKernelGGL(splitk_reduce_rows_kernel<float>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, partial,
                       splits, stride, rows, N, row_map, out, ld, beta, in_ld);
  }
  return hipGetLastError();
}

// requires N % 4 == 0 and a 16-byte aligned partial array; pld (a multiple of 4; 0: N) is the row pitch of a
// partial array
hipError_t launch_splitk_bias(const float* partial, int splits, int M, int N, const float* bias, void* out, int dtype,
                              hipStream_t st, int64_t pld) {
  if (pld <= 0) pld = N;
  const int64_t n4 = (int64_t)M * N / 4, pstride = (int64_t)M * pld;
  dim3 grid((unsigned)((n4 + 255) / 256)), block(256);
  if (dtype == kF32)
    hipLaunchKernelGGL(splitk_bias_kernel<float>, grid, block, 0, st, partial, splits, M, N, pld, pstride, bias, (float*)out);
  else
    hipLaunchKernelGGL(splitk_bias_kernel<uint16_t>, grid, block, 0, st, partial, splits, M, N, pld, pstride, bias,
                       (uint16_t*)out);
  return hipGetLastError();
}

// Sum of split-K partial sums of a forward GEMM with what its fused epilogue would have done: bias, the
// low-rank input term u V, ReLU, the (h > 0) bits.  One thread per output; with bits, N is a multiple of 64 and a
// wave covers 64 consecutive columns of a row, so a ballot gives two whole words of the bit array.
__global__ __launch_bounds__(256) void splitk_fwd_f32_kernel(const float* __restrict__ partial, int splits, int M, int N,
                                                             const float* __restrict__ bias, const float* __restrict__ u,
                                                             int64_t u_ld, int u_n, const float* __restrict__ V, int relu,
                                                             float* __restrict__ y, uint32_t* __restrict__ bits,
                                                             int bits_pitch) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t total = (int64_t)M * N;
  if (i >= total) return;                        // with bits, total is a multiple of 64: whole waves leave together
  const int row = (int)(i / N), col = (int)(i - (int64_t)row * N);
  float h = 0.f;
  for (int s = 0; s < splits; ++s) h += partial[(size_t)s * total + i];
  if (bias) h += bias[col];
  for (int q = 0; q < u_n; ++q) h += u[(size_t)row * u_ld + q] * V[(size_t)q * N + col];
  if (relu) h = h > 0.f ? h : 0.f;
  y[i] = h;
  if (bits) {
    const uint64_t b = __ballot(h > 0.f);
    const int lane = threadIdx.x & 63;
    if (lane == 0) bits[(size_t)row * bits_pitch + (col >> 5)] = (uint32_t)b;
    if (lane == 32) bits[(size_t)row * bits_pitch + (col >> 5)] = (uint32_t)(b >> 32);
  }
}

// The same for any N: a wave per output row walks the row 64 columns at a time, so that its ballots are whole
// words of the row's bits wherever the row ends.
__global__ __launch_bounds__(256) void splitk_fwd_f32_rows_kernel(const float* __restrict__ partial, int splits, int M,
                                                                  int N, const float* __restrict__ bias,
                                                                  const float* __restrict__ u, int64_t u_ld, int u_n,
                                                                  const float* __restrict__ V, int relu,
                                                                  float* __restrict__ y, uint32_t* __restrict__ bits,
                                                                  int bits_pitch) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= M) return;                          // whole waves
  const int64_t total = (int64_t)M * N;
  for (int c0 = 0; c0 < N; c0 += 64) {
    const int col = c0 + lane;
    float h = 0.f;
    if (col < N) {
      const int64_t i = (int64_t)row * N + col;
      for (int s = 0; s < splits; ++s) h += partial[(size_t)s * total + i];
      if (bias) h += bias[col];
      for (int q = 0; q < u_n; ++q) h += u[(size_t)row * u_ld + q] * V[(size_t)q * N + col];
      if (relu) h = h > 0.f ? h : 0.f;
      y[i] = h;
    }
    if (bits) {
      const uint64_t b = __ballot(col < N && h > 0.f);
      if (lane == 0) bits[(size_t)row * bits_pitch + (c0 >> 5)] = (uint32_t)b;
      if (lane == 32 && c0 + 32 < N) bits[(size_t)row * bits_pitch + (c0 >> 5) + 1] = (uint32_t)(b >> 32);
    }
  }
}

// Sum of split-K partial sums, zeroed where the mask bit of the output entry is clear (mask: [M][pitch] words
// over N columns, or null)
__global__ __launch_bounds__(256) void splitk_reduce_masked_kernel(const float* __restrict__ partial, int splits, int M,
                                                                   int N, const uint32_t* __restrict__ mask, int pitch,
                                                                   float* __restrict__ out) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t total = (int64_t)M * N;
  if (i >= total) return;
  const int row = (int)(i / N), col = (int)(i - (int64_t)row * N);
  float v = 0.f;
  for (int s = 0; s < splits; ++s) v += partial[(size_t)s * total + i];
  if (mask && !((mask[(size_t)row * pitch + (col >> 5)] >> (col & 31)) & 1u)) v = 0.f;
  out[i] = v;
}

hipError_t launch_splitk_fwd_f32(const float* partial, int splits, int M, int N, const float* bias, const float* u,
                                 int64_t u_ld, int u_n, const float* V, int relu, float* y, uint32_t* bits,
                                 int bits_pitch, hipStream_t st) {
  if (bits && N % 64 != 0) {                               // rows that do not end on a wave boundary
    hipLaunchKernelGGL(splitk_fwd_f32_rows_kernel, dim3((unsigned)((M + 3) / 4)), dim3(256), 0, st, partial, splits, M, N,
                       bias, u, u_ld, u_n, V, relu, y, bits, bits_pitch);
    return hipGetLastError();
  }
  const int64_t total = (int64_t)M * N;
  hipLaunchKernelGGL(splitk_fwd_f32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, partial, splits, M, N,
                     bias, u, u_ld, u_n, V, relu, y, bits, bits_pitch);
  return hipGetLastError();
}

hipError_t launch_splitk_reduce_masked(const float* partial, int splits, int M, int N, const uint32_t* mask, int pitch,
                                       float* out, hipStream_t st) {
  const int64_t total = (int64_t)M * N;
  hipLaunchKernelGGL(splitk_reduce_masked_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, partial, splits,
                     M, N, mask, pitch, out);
  return hipGetLastError();
}

hipError_t launch_maxpool_fwd(const float* y, int planes, int H, int W, float* pooled, uint32_t* arg, hipStream_t st) {
  const int64_t total = (int64_t)planes * (H / 2) * (W / 2);
  const int64_t threads = (total + 15) / 16;
  const int Wo = W / 2;
  const bool aligned = ((reinterpret_cast<uintptr_t>(y) | reinterpret_cast<uintptr_t>(pooled)) & 15) == 0;
  if (aligned && H % 2 == 0 && W == 2 * Wo && total % 16 == 0 && (Wo == 4 || Wo == 8 || Wo == 16)) {
    const dim3 grid((unsigned)((threads + 255) / 256)), block(256);
    if (Wo == 4) hipLaunchKernelGGL(maxpool_rows_kernel<4>, grid, block, 0, st, y, total, pooled, arg);
    else if (Wo == 8) hipLaunchKernelGGL(maxpool_rows_kernel<8>, grid, block, 0, st, y, total, pooled, arg);
    else hipLaunchKernelGGL(maxpool_rows_kernel<16>, grid, block, 0, st, y, total, pooled, arg);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(maxpool_fwd_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, y, planes, H, W,
                     pooled, arg);
  return hipGetLastError();
}

hipError_t launch_avgpool_fwd(const float* y, int planes, int H, int W, float* pooled, hipStream_t st) {
  const int64_t total = (int64_t)planes * (H / 2) * (W / 2);
  hipLaunchKernelGGL(avgpool_fwd_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, y, planes, H, W, pooled);
  return hipGetLastError();
}

hipError_t launch_unpool_mask(const float* dy, int batch, int C, int H, int W, int pool, const uint32_t* arg,
                              const uint32_t* bits, int bits_pitch, float* g, hipStream_t st) {
  const int64_t n = (int64_t)batch * C * H * W;
  if (W % 4 == 0 && H % 2 == 0 && ((reinterpret_cast<uintptr_t>(g) | reinterpret_cast<uintptr_t>(dy)) & 15) == 0) {
    hipLaunchKernelGGL(unpool_mask4_kernel, dim3((unsigned)((n / 4 + 255) / 256)), dim3(256), 0, st, dy, batch, C, H, W,
                       pool, arg, bits, bits_pitch, g);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(unpool_mask_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, dy, batch, C, H, W, pool, arg,
                     bits, bits_pitch, g);
  return hipGetLastError();
}

hipError_t launch_channel_sum(const float* g, int batch, int C, int HW, float* db, float* partial, int splits,
                              hipStream_t st) {
  hipLaunchKernelGGL(channel_sum_kernel, dim3(C, splits), dim3(256), 0, st, g, batch, C, HW, splits, partial);
  hipLaunchKernelGGL(channel_sum_final_kernel, dim3((C + 255) / 256), dim3(256), 0, st, partial, C, splits, db);
  return hipGetLastError();
}

hipError_t launch_flip_weights(const float* W, int Ci, int KH, int KW, int Co, float* Wt, hipStream_t st) {
  const int n = Ci * KH * KW * Co;
  hipLaunchKernelGGL(flip_weights_kernel, dim3((n + 255) / 256), dim3(256), 0, st, W, Ci, KH, KW, Co, Wt);
  return hipGetLastError();
}

// One Philox call per thread = 128 consecutive entries of R in row-major [d][k] order.
template <typename T>
__global__ __launch_bounds__(256) void sign_matrix_kernel(T* __restrict__ R, T* __restrict__ Rt, int d, int k, int kp,
                                                          uint32_t seed_lo, uint32_t seed_hi, uint32_t stream_id,
                                                          uint32_t step) {
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t n = (int64_t)d * k;
  int64_t f = q * 128;
  if (f >= n) return;
  const u32x4 k4 = element_quad_keys((uint64_t)q, stream_id, step, seed_lo, seed_hi);
  int j = (int)(f / k), sc = (int)(f % k);
  T plus, minus;
  if (sizeof(T) == 2) { plus = (T)0x3F80u; minus = (T)0xBF80u; }              // bf16 bits of +1 and -1
  else { const float a = 1.f, b = -1.f; plus = *reinterpret_cast<const T*>(&a); minus = *reinterpret_cast<const T*>(&b); }
#pragma unroll
  for (int w = 0; w < 4; ++w)
    for (int b = 0; b < 32 && f < n; ++b, ++f) {
      const T v = ((k4[w] >> b) & 1u) ? minus : plus;
      R[(size_t)j * kp + sc] = v;
      Rt[(size_t)sc * d + j] = v;
      if (++sc == k) { sc = 0; ++j; }
    }
}

hipError_t launch_sign_matrix(void* R, void* Rt, int dtype, int d, int k, int kp, uint32_t seed_lo, uint32_t seed_hi,
                              uint32_t stream_id, uint32_t step, hipStream_t st) {
  const int64_t calls = ((int64_t)d * k + 127) / 128;
  dim3 grid((unsigned)((calls + 255) / 256)), block(256);
  if (dtype == kF32)
    hipLaunchKernelGGL(sign_matrix_kernel<uint32_t>, grid, block, 0, st, (uint32_t*)R, (uint32_t*)Rt, d, k, kp, seed_lo,
                       seed_hi, stream_id, step);
  else
    hipLaunchKernelGGL(sign_matrix_kernel<uint16_t>, grid, block, 0, st, (uint16_t*)R, (uint16_t*)Rt, d, k, kp, seed_lo,
                       seed_hi, stream_id, step);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void scale_cast_kernel(const float* __restrict__ in, void* __restrict__ out, int bf16,
                                                         int64_t n, float scale) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const float v = in[i] * scale;
  if (bf16) reinterpret_cast<uint16_t*>(out)[i] = f32_to_bf16_bits(v);
  else reinterpret_cast<float*>(out)[i] = v;
}

hipError_t launch_scale_cast(const float* in, void* out, int dtype, int64_t n, float scale, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(scale_cast_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, in, out, dtype == kBF16 ? 1 : 0,
                     n, scale);
  return hipGetLastError();
}

hipError_t launch_fill_u32(uint32_t* p, uint32_t v, int64_t n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, v, n);
  return hipGetLastError();
}

}  // namespace rad
