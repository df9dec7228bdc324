// Convolutions of the small CNNs (Section 4.2, convolutional layers; Appendix A, architectures): stride 1, zero
// padding that keeps the spatial size, fp32, at most 64 channels, v_mfma_f32_32x32x2_f32.
//
// Both kernels are implicit GEMMs whose im2col operand never exists, not even as an address computation per
// element: a workgroup stages the patch of the input it needs (its image rows plus the halo, zero outside the
// image) in LDS once, and an element of the im2col matrix is then patch[koff(c,u,v) + poff(y,x)], the sum of an
// offset that depends on the reduction index alone and one that depends on the position alone.
//   forward / dX:  y[b,o,p] = sum_(c,u,v) x[b,c,p+(u,v)] W[(c,u,v),o]       rows: positions, K: (c,u,v)
//   dW:            dW[(c,u,v),o] = sum_(b,p) x~[b,c,p+(u,v)] g[b,o,p]       rows: (c,u,v),   K: positions
#include <type_traits>

#include "gemm.hpp"

namespace rad {

namespace {

// dst[i] = load(i) for i < n with U loads of every thread in flight at once (a plain loop waits for each load
// before it issues the next: the LDS store needs the value)
template <int U, class Load>
__device__ __forceinline__ void stage_to_lds(float* dst, int n, Load load) {
  for (int base = threadIdx.x; base < n; base += 256 * U) {
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) { const int i = base + u * 256; v[u] = i < n ? load(i) : 0.f; }
#pragma unroll
    for (int u = 0; u < U; ++u) { const int i = base + u * 256; if (i < n) dst[i] = v[u]; }
  }
}

// element i of the patch [ci][nrows][PW] of image b whose first row is image row y_top (zero outside the image)
__device__ __forceinline__ float patch_elem(const float* __restrict__ src, int i, int b, int ci, int H, int W, int pad,
                                            int nrows, int PW, int y_top) {
  const int cr = i / PW, x = i - cr * PW;
  const int c = cr / nrows, r = cr - c * nrows;
  const int yy = y_top + r, xx = x - pad;
  if (yy < 0 || yy >= H || xx < 0 || xx >= W) return 0.f;
  return src[((size_t)(b * ci + c) * H + yy) * W + xx];
}

// ------------------------------------------------------------------------------------------------ forward
// NT tiles of 32 output channels side by side, 4 / NT tiles of 32 positions: a workgroup computes 32*(4/NT)
// consecutive positions of one image for all channels.  K is walked in chunks of KC weights rows staged in LDS.
constexpr int kConvKC = 64;

// KSP = 2: two waves share an output tile and take half of every chunk's K steps each (a shorter chain of dependent
// MFMAs per wave and twice the workgroups, for layers whose positions alone do not fill the chip).
template <int NT, int KSP>
__global__ __launch_bounds__(256) void conv_fwd_direct_kernel(GemmArgs g, int nrows_max) {
  constexpr int WM = 4 / (NT * KSP), BM = 32 * WM, BN = 32 * NT;
  static_assert(BM % 64 == 0, "the epilogue walks 64 positions at a time");
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int kh = w / (WM * NT), wt = w % (WM * NT);          // K half, tile of this wave
  const int wm = wt / NT, wn = wt % NT;
  const int H = g.cv_H, W = g.cv_W, ks = g.cv_KH, pad = g.cv_pad, ci = g.cv_C;
  const int HW = H * W, PW = W + 2 * pad, K = g.K, Kpad = (K + 1) & ~1;
  const int m0 = (int)blockIdx.x * BM;
  const int b = m0 / HW, p0 = m0 - b * HW;
  const int y_first = p0 / W, y_last = (p0 + BM - 1) / W;
  const int nrows = y_last - y_first + 1 + 2 * pad;          // <= nrows_max, which sized the LDS
  float* patch = reinterpret_cast<float*>(smem_raw);
  const int patch_elems = (ci * nrows_max * PW + 3) & ~3;
  int* koff = reinterpret_cast<int*>(patch + patch_elems);
  float* Bs = reinterpret_cast<float*>(koff + ((Kpad + 3) & ~3));
  const float* src = static_cast<const float*>(g.A);
  const float* Wg = static_cast<const float*>(g.B);

  // weights of K rows k0 .. k0 + KC - 1 as this thread's WU registers, then into LDS: the loads of the next chunk
  // are issued before the MFMAs of the current one
  constexpr int WU = kConvKC * BN / 256;
  float wreg[WU];
  auto load_w = [&](int k0) {
#pragma unroll
    for (int u = 0; u < WU; ++u) {
      const int i = tid + u * 256;
      const int kk = i / BN, n = i - kk * BN;
      wreg[u] = (k0 + kk < K && n < g.N) ? Wg[(size_t)(k0 + kk) * g.N + n] : 0.f;
    }
  };
  auto store_w = [&]() {
#pragma unroll
    for (int u = 0; u < WU; ++u) Bs[tid + u * 256] = wreg[u];
  };
  load_w(0);                                                  // in flight together with the patch
  stage_to_lds<16>(patch, ci * nrows * PW, [&](int i) { return patch_elem(src, i, b, ci, H, W, pad, nrows, PW, y_first - pad); });
  for (int k = tid; k < Kpad; k += 256) {
    int o = 0;
    if (k < K) {
      const int c = k / (ks * ks), uv = k - c * ks * ks;
      const int u = uv / ks, v = uv - u * ks;
      o = (c * nrows + u) * PW + v;
    }
    koff[k] = o;
  }
  store_w();
  const int p = p0 + wm * 32 + (lane & 31);
  const int py = p / W, px = p - py * W;
  const int moff = (py - y_first) * PW + px;
  const int hi = lane >> 5;

  floatx16 acc[1][1];
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[0][0][e] = 0.f;
  for (int k0 = 0; k0 < Kpad; k0 += kConvKC) {
    __syncthreads();                                        // this chunk's weights (first pass: and the tables) are in LDS
    const bool more = k0 + kConvKC < Kpad;
    if (more) load_w(k0 + kConvKC);
    const int chunk_steps = min(kConvKC, Kpad - k0) / 2;
    // this wave's share of the chunk's steps
    const int per = (chunk_steps + KSP - 1) / KSP;
    int s = kh * per;
    const int steps = min(chunk_steps, s + per);
    // eight steps at a time: their table reads, then their operand reads, then their MFMAs, so that the LDS
    // latencies of a step overlap those of its neighbours instead of standing in front of every MFMA
    for (; s + 8 <= steps; s += 8) {
      int ko[8];
      float a[8], bb[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) ko[u] = koff[k0 + 2 * (s + u) + hi];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        a[u] = patch[ko[u] + moff];
        bb[u] = Bs[(2 * (s + u) + hi) * BN + wn * 32 + (lane & 31)];     // zero for k >= K
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], bb[u], acc[0][0], 0, 0, 0);
    }
    for (; s < steps; ++s) {
      const int kk = 2 * s + hi;
      const float a = patch[koff[k0 + kk] + moff];
      const float bb = Bs[kk * BN + wn * 32 + (lane & 31)];
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bb, acc[0][0], 0, 0, 0);
    }
    if (more) {
      __syncthreads();                                      // every wave is through with this chunk's weights
      store_w();
    }
  }
  __syncthreads();                                          // the epilogue stages the tile where the patch was
  if constexpr (KSP == 2) {
    // both waves of a tile end up with the same sums (a + b and b + a are the same number), so that it does not
    // matter which of them stores an element in the epilogue
    float* xch = patch + (size_t)BN * (BM + 1);               // behind the epilogue's tile
#pragma unroll
    for (int e = 0; e < 16; ++e) xch[(w * 16 + e) * 64 + lane] = acc[0][0][e];
    __syncthreads();
    const int other = (kh ^ 1) * (WM * NT) + wt;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[0][0][e] += xch[(other * 16 + e) * 64 + lane];
  }
  epilogue_conv<BM, BN, 1, 1>(g, acc, patch, m0, 0, wm * 32, wn * 32);
}

template <int NT, int KSP> size_t conv_fwd_smem(const GemmArgs& g, int nrows_max) {
  constexpr int BM = 32 * (4 / (NT * KSP)), BN = 32 * NT;
  const int PW = g.cv_W + 2 * g.cv_pad, Kpad = (g.K + 1) & ~1;
  size_t patch = (size_t)((g.cv_C * nrows_max * PW + 3) & ~3);
  const size_t epi = (size_t)BN * (BM + 1) + (KSP == 2 ? 4 * 16 * 64 : 0);     // + the exchange of the two K halves
  if (patch < epi) patch = (epi + 3) & ~(size_t)3;          // the epilogue's tile lies where the patch was
  return (patch + (size_t)((Kpad + 3) & ~3) + (size_t)kConvKC * BN) * 4;
}

// --------------------------------------------------------------------------------------------------- dW
// A workgroup walks `tiles_per_wg` tiles of `rows_t` image rows (PT = rows_t * W positions) and keeps the whole
// [M = ci*ks*ks][N = co] partial sum in registers: 32 x 32 tiles (mt, nt), tile q of wave w is number w + 4q.
template <int TPWV>
__global__ __launch_bounds__(256) void conv_dw_direct_kernel(const float* __restrict__ xt, const float* __restrict__ gsrc,
                                                             float* __restrict__ part, int batch, int ci, int co, int H,
                                                             int W, int ks, int pad, int rows_t, int tiles_per_wg) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, hi = lane >> 5;
  const int HW = H * W, PW = W + 2 * pad, PT = rows_t * W, M = ci * ks * ks;
  const int nrows = rows_t + 2 * pad;
  const int tiles_img = H / rows_t, total_tiles = batch * tiles_img;
  const int mt_n = (M + 31) / 32, nt_n = (co + 31) / 32, n_tiles = mt_n * nt_n;
  float* patch = reinterpret_cast<float*>(smem_raw);
  float* Gs = patch + ((ci * nrows * PW + 3) & ~3);          // [co][PT + 1]
  int* poff = reinterpret_cast<int*>(Gs + ((co * (PT + 1) + 3) & ~3));

  for (int q = tid; q < PT; q += 256) { const int y = q / W; poff[q] = y * PW + (q - y * W); }
  // this lane's rows of the im2col matrix: m = mt*32 + lane%32 -> offset of (c,u,v) in the patch
  int koffA[TPWV], ntA[TPWV];
  bool validA[TPWV];
#pragma unroll
  for (int q = 0; q < TPWV; ++q) {
    const int t = w + 4 * q;
    const int mt = t / nt_n;
    ntA[q] = (t - mt * nt_n) & 1;
    const int m = mt * 32 + (lane & 31);
    validA[q] = t < n_tiles && m < M;
    int o = 0;
    if (validA[q]) {
      const int c = m / (ks * ks), uv = m - c * ks * ks;
      const int u = uv / ks, v = uv - u * ks;
      o = (c * nrows + u) * PW + v;
    }
    koffA[q] = o;
  }
  // this lane's channel of either channel tile: row offset in the g tile (row 0 if there is no such channel)
  int gofs[2];
  bool gval[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int n = j * 32 + (lane & 31);
    gval[j] = n < co;
    gofs[j] = gval[j] ? n * (PT + 1) : 0;
  }
  floatx16 acc[TPWV];
#pragma unroll
  for (int q = 0; q < TPWV; ++q)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[q][e] = 0.f;

  const int t_beg = (int)blockIdx.x * tiles_per_wg, t_end = min(total_tiles, t_beg + tiles_per_wg);
  for (int tile = t_beg; tile < t_end; ++tile) {
    const int b = tile / tiles_img, y0 = (tile - b * tiles_img) * rows_t;
    __syncthreads();                                        // the previous tile's readers are through
    stage_to_lds<16>(patch, ci * nrows * PW, [&](int i) { return patch_elem(xt, i, b, ci, H, W, pad, nrows, PW, y0 - pad); });
    // g tile [co][PT + 1] (the odd pitch spreads the channels over the banks): 16-byte loads, PT % 4 == 0
    {
      const int n4 = co * (PT / 4);
      for (int base = tid; base < n4; base += 256 * 8) {
        floatx4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int i = base + u * 256;
          v[u] = floatx4{0.f, 0.f, 0.f, 0.f};
          if (i < n4) {
            const int n = i / (PT / 4), q4 = i - n * (PT / 4);
            v[u] = *reinterpret_cast<const floatx4*>(gsrc + ((size_t)b * co + n) * HW + y0 * W + q4 * 4);
          }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int i = base + u * 256;
          if (i < n4) {
            const int n = i / (PT / 4), q4 = i - n * (PT / 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) Gs[n * (PT + 1) + q4 * 4 + e] = v[u][e];
          }
        }
      }
    }
    __syncthreads();
    // U steps at a time (reads first, then the MFMAs), U chosen so that U * tiles operands stay in registers.
    // No branches in here: every read is in bounds whatever the lane (rows of the im2col matrix past M and
    // channels past co read element 0 and are zeroed by a select), and a wave with one tile fewer than TPWV
    // multiplies zeros into an accumulator nobody stores.
    constexpr int U = TPWV >= 5 ? 2 : TPWV >= 3 ? 4 : 8;
    auto steps_of = [&](auto UC, int s0) {
      constexpr int UU = decltype(UC)::value;
      int po[UU];
      float bv[UU][2], a[UU][TPWV];
#pragma unroll
      for (int u = 0; u < UU; ++u) po[u] = poff[2 * (s0 + u) + hi];
#pragma unroll
      for (int u = 0; u < UU; ++u) {
        const int pos = 2 * (s0 + u) + hi;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const float v = Gs[gofs[j] + pos];
          bv[u][j] = gval[j] ? v : 0.f;
        }
#pragma unroll
        for (int q = 0; q < TPWV; ++q) {
          const float v = patch[koffA[q] + po[u]];
          a[u][q] = validA[q] ? v : 0.f;
        }
      }
#pragma unroll
      for (int u = 0; u < UU; ++u)
#pragma unroll
        for (int q = 0; q < TPWV; ++q)
          acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u][q], ntA[q] ? bv[u][1] : bv[u][0], acc[q], 0, 0, 0);
    };
    int s = 0;
    for (; s + U <= PT / 2; s += U) steps_of(std::integral_constant<int, U>(), s);
    for (; s < PT / 2; ++s) steps_of(std::integral_constant<int, 1>(), s);
  }
  float* out = part + (size_t)blockIdx.x * M * co;
#pragma unroll
  for (int q = 0; q < TPWV; ++q) {
    const int t = w + 4 * q;
    if (t >= n_tiles) continue;
    const int mt = t / nt_n, nt = t - mt * nt_n;
    const int n = nt * 32 + (lane & 31);
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int m = mt * 32 + acc_row(e, lane);
      if (m < M && n < co) out[(size_t)m * co + n] = acc[q][e];
    }
  }
}

constexpr size_t kConvLdsBudget = 100 * 1024;     // leaves room for a second workgroup on the CU

}  // namespace

// Forward / dX convolution with the arguments of the im2col GEMM (A = NCHW input, B = W [(c,u,v)][co], kEpiConv
// fields).  Returns hipErrorInvalidValue when the shape is not served (the caller then takes the general kernel).
hipError_t launch_conv_fwd_direct(const GemmArgs& g, hipStream_t st) {
  const int HW = g.cv_H * g.cv_W;
  if (g.cv_KH != g.cv_KW || 2 * g.cv_pad != g.cv_KH - 1 || g.N > 64 || g.N < 1 || HW % 64 != 0 || g.M % HW != 0)
    return hipErrorInvalidValue;
  const bool wide = g.N > 32;                               // two channel tiles
  // one channel tile: 128 positions per workgroup when that alone gives every CU several workgroups, else 64
  // positions with the K steps of a tile shared by two waves
  const bool ksplit = !wide && (HW % 128 != 0 || g.M / 128 < 512);
  const int BM = (wide || ksplit) ? 64 : 128;
  // image rows a tile of BM consecutive positions can touch
  const int span = g.cv_W >= BM ? (BM % g.cv_W == 0 ? 1 : 2) : (BM % g.cv_W == 0 ? BM / g.cv_W : BM / g.cv_W + 2);
  const int nrows_max = span + 2 * g.cv_pad;
  const size_t smem = wide ? conv_fwd_smem<2, 1>(g, nrows_max) : ksplit ? conv_fwd_smem<1, 2>(g, nrows_max)
                                                                        : conv_fwd_smem<1, 1>(g, nrows_max);
  if (smem > kConvLdsBudget) return hipErrorInvalidValue;
  auto kern = wide ? conv_fwd_direct_kernel<2, 1> : ksplit ? conv_fwd_direct_kernel<1, 2> : conv_fwd_direct_kernel<1, 1>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(g.M / BM), dim3(256), smem, st, g, nrows_max);
  return hipGetLastError();
}

// How the dW kernel cuts the work: image rows per tile, tiles per workgroup, workgroups (= partial sums), LDS bytes.
// ok = false: shape not served.
struct ConvDwPlan { bool ok; int rows_t, tiles_per_wg, wgs, tpwv; size_t smem; };
static ConvDwPlan conv_dw_plan(int batch, int ci, int co, int H, int W, int ks) {
  ConvDwPlan p{false, 0, 0, 0, 0, 0};
  const int pad = (ks - 1) / 2, PW = W + 2 * pad, M = ci * ks * ks;
  const int n_tiles = ((M + 31) / 32) * ((co + 31) / 32);
  if (co > 64 || co < 1 || n_tiles > 32 || (W & 1)) return p;
  // the most image rows per tile (a divisor of H, at most 512 positions) whose patch and g tile fit
  for (int r = H; r >= 1; --r) {
    if (H % r) continue;
    const int PT = r * W;
    if (PT > 256 || PT % 4) continue;
    const size_t smem = ((size_t)((ci * (r + 2 * pad) * PW + 3) & ~3) + (size_t)((co * (PT + 1) + 3) & ~3) + (size_t)PT) * 4;
    if (smem > kConvLdsBudget) continue;
    p.ok = true; p.rows_t = r; p.smem = smem;
    break;
  }
  if (!p.ok) return p;
  const int total = batch * (H / p.rows_t);
  p.tiles_per_wg = (total + 1023) / 1024;                   // a few workgroups per CU: one stages while another computes
  if (p.tiles_per_wg < 1) p.tiles_per_wg = 1;
  p.wgs = (total + p.tiles_per_wg - 1) / p.tiles_per_wg;
  const int per_wave = (n_tiles + 3) / 4;
  p.tpwv = per_wave;                                        // 1 .. 8
  return p;
}

// number of partial sums [M][co] the dW kernel writes for this shape, 0 if the shape is not served
int conv_dw_direct_splits(int batch, int ci, int co, int H, int W, int ks) {
  const ConvDwPlan p = conv_dw_plan(batch, ci, co, H, W, ks);
  return p.ok ? p.wgs : 0;
}

// part [splits][ci*ks*ks][co] <- per-workgroup partial sums of dW from the dense x~ [B][ci][H][W] and g [B][co][H][W]
hipError_t launch_conv_dw_direct(const float* xt, const float* g, float* part, int batch, int ci, int co, int H, int W,
                                 int ks, hipStream_t st) {
  const ConvDwPlan p = conv_dw_plan(batch, ci, co, H, W, ks);
  if (!p.ok) return hipErrorInvalidValue;
  const int pad = (ks - 1) / 2;
#define RAD_CONV_DW_CASE(T_)                                                                                           \
  if (p.tpwv == T_) {                                                                                                  \
    auto kern = conv_dw_direct_kernel<T_>;                                                                             \
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                       (int)p.smem);                                                                   \
    if (e != hipSuccess) return e;                                                                                     \
    hipLaunchKernelGGL(kern, dim3(p.wgs), dim3(256), p.smem, st, xt, g, part, batch, ci, co, H, W, ks, pad, p.rows_t,  \
                       p.tiles_per_wg);                                                                                \
    return hipGetLastError();                                                                                          \
  }
  RAD_CONV_DW_CASE(1) RAD_CONV_DW_CASE(2) RAD_CONV_DW_CASE(3) RAD_CONV_DW_CASE(4)
  RAD_CONV_DW_CASE(5) RAD_CONV_DW_CASE(6) RAD_CONV_DW_CASE(7) RAD_CONV_DW_CASE(8)
#undef RAD_CONV_DW_CASE
  return hipErrorInvalidValue;
}

}  // namespace rad
