// fp32 GEMM for few output tiles and a long contraction (a time step of the recurrent model, Appendix A:
// 128 x 1024 x 1024): one launch, no partial sums through memory.  A workgroup of eight waves owns a 16 x 32
// output tile (256 workgroups for the recurrent step: one per CU); every wave takes an eighth of K, brings its own
// operand slices in through a private LDS area and runs two chains of v_mfma_f32_16x16x4_f32 (the tile's two
// 16-column halves); the eight waves' accumulators meet in LDS, are added in wave order, and the tile's epilogue
// runs in the same kernel: forward (bias, low-rank input term, ReLU, bits) or dX (output mask of the layer
// below).  Splitting K over workgroups instead needs a second launch to add the splits (the time steps are a
// chain of dependent launches, so a launch is what a step costs), and adding them in the same kernel needs
// device-coherent traffic between XCDs, which measured slower than the second launch.
#include "gemm.hpp"

namespace rad {

namespace {

constexpr int kKsWaves = 8;

// A wave's operand slices reach the MFMA through its own LDS area, 64 k at a time.  K-contiguous operands (A; for
// dX also B) are loaded with whole 256-byte rows per 16 lanes and stored [rows][64 k] at a pitch of 65 floats, so
// that lane (r = lane % 16, kq = lane / 16) reads element [r][4s + kq] of step s without bank conflicts between
// rows.  An N-contiguous B (forward) is kept as it lies in memory, [64 k][32 n].  Only the wave itself touches its
// area, so there is no workgroup barrier before the final sum.
// BK_CONTIG: B is K-contiguous (B[n * ldb + k], dX) or N-contiguous (B[k * ldb + n], forward).
constexpr int kKsPitch = 65, kKsHalf = 64;
constexpr int kKsAreaA = 16 * kKsPitch, kKsAreaB = 32 * kKsPitch;       // floats (B: the larger of the two layouts)

template <bool BK_CONTIG, int FINISH>
__global__ __launch_bounds__(64 * kKsWaves) void gemm_f32_ks_kernel(GemmArgs g) {
  extern __shared__ __align__(16) float smem_ks[];
  float (*s_acc)[2][4][64] = reinterpret_cast<float (*)[2][4][64]>(smem_ks);     // [waves][half][elem][lane], at the end
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int r = lane & 15, kq = lane >> 4;
  const int tiles_n = g.N / 32;
  const int m0 = ((int)blockIdx.x / tiles_n) * 16, n0 = ((int)blockIdx.x % tiles_n) * 32;
  const int kw = g.K / kKsWaves;               // K per wave, a multiple of 8
  const int kbeg = w * kw;
  float* As = smem_ks + w * (kKsAreaA + kKsAreaB);          // (the accumulators take this space over at the end)
  float* Bs = As + kKsAreaA;
  const float* Ag = static_cast<const float*>(g.A);
  const float* Bg = static_cast<const float*>(g.B);
  floatx4 acc[2];
#pragma unroll
  for (int jn = 0; jn < 2; ++jn) acc[jn] = floatx4{0.f, 0.f, 0.f, 0.f};

  // what the epilogue adds or masks with, fetched now so that it has arrived by then: waves 0 .. 3 finish
  // accumulator element w of every lane, for both column halves
  float addend[2] = {0.f, 0.f};
  uint32_t keepw = ~0u;
  if (w < 4) {
    const int row = m0 + 4 * kq + w;
#pragma unroll
    for (int jn = 0; jn < 2; ++jn) {
      const int col = n0 + 16 * jn + r;
      if (FINISH == 1) {
        if (g.bias) addend[jn] = g.bias[col];
        for (int q = 0; q < g.u_n; ++q) addend[jn] += g.u[(size_t)row * g.u_ld + q] * g.V[(size_t)q * g.N + col];
      }
    }
    if (FINISH == 2 && g.c_mask) keepw = g.c_mask[(size_t)row * g.c_mask_pitch + (n0 >> 5)];
  }

  // One pass = 64 k.  The loads of pass p + 1 are issued before the LDS stores and MFMAs of pass p.
  // A: [16 rows][64 k], piece f = lane + 64 i (i < 4) is row f / 16, k 4 (f % 16).  K-contiguous B: [32 rows][64 k],
  // pieces f = lane + 64 i (i < 8).  N-contiguous B: [64 k][32 n], piece f is k f / 8, n 4 (f % 8).
  floatx4 av[4], bv4[8];
  auto load_pass = [&](int k0) {
    const int kn = min(kKsHalf, kw - k0);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int f = lane + 64 * i;
      const int row = f >> 4, c4 = (f & 15) * 4;
      if (i < 4) {
        av[i] = floatx4{0.f, 0.f, 0.f, 0.f};
        if (c4 < kn) av[i] = *reinterpret_cast<const floatx4*>(Ag + (size_t)(m0 + row) * g.lda + kbeg + k0 + c4);
      }
      bv4[i] = floatx4{0.f, 0.f, 0.f, 0.f};
      if constexpr (BK_CONTIG) {
        if (c4 < kn) bv4[i] = *reinterpret_cast<const floatx4*>(Bg + (size_t)(n0 + row) * g.ldb + kbeg + k0 + c4);
      } else {
        const int kk = f >> 3, n4 = (f & 7) * 4;
        if (kk < kn) bv4[i] = *reinterpret_cast<const floatx4*>(Bg + (size_t)(kbeg + k0 + kk) * g.ldb + n0 + n4);
      }
    }
  };
  load_pass(0);
  for (int k0 = 0; k0 < kw; k0 += kKsHalf) {
    const int kn = min(kKsHalf, kw - k0);      // k in this pass, a multiple of 8
    __builtin_amdgcn_wave_barrier();           // the reads of the previous pass are done (same wave, in order)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int f = lane + 64 * i, row = f >> 4, c4 = (f & 15) * 4;
      if (i < 4) {
#pragma unroll
        for (int e = 0; e < 4; ++e) As[row * kKsPitch + c4 + e] = av[i][e];
      }
      if constexpr (BK_CONTIG) {
#pragma unroll
        for (int e = 0; e < 4; ++e) Bs[row * kKsPitch + c4 + e] = bv4[i][e];
      } else {
        *reinterpret_cast<floatx4*>(Bs + (f >> 3) * 32 + (f & 7) * 4) = bv4[i];
      }
    }
    if (k0 + kKsHalf < kw) load_pass(k0 + kKsHalf);
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int s0 = 0; s0 < kKsHalf / 4; s0 += 8) {
      float a[8], b[8][2];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int kk = 4 * (s0 + u) + kq;
        a[u] = As[r * kKsPitch + kk];
#pragma unroll
        for (int jn = 0; jn < 2; ++jn) b[u][jn] = BK_CONTIG ? Bs[(16 * jn + r) * kKsPitch + kk] : Bs[kk * 32 + 16 * jn + r];
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (4 * (s0 + u) < kn) {
#pragma unroll
          for (int jn = 0; jn < 2; ++jn) acc[jn] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u], b[u][jn], acc[jn], 0, 0, 0);
        }
    }
  }
  __syncthreads();                             // every wave is through with its operand area: the accumulators go there
#pragma unroll
  for (int jn = 0; jn < 2; ++jn)
#pragma unroll
    for (int e = 0; e < 4; ++e) s_acc[w][jn][e][lane] = acc[jn][e];
  __syncthreads();
  if (w >= 4) return;
  // accumulator element e of a 16 x 16 block sits at row 4 (lane / 16) + e, column lane % 16
  const int row = m0 + 4 * kq + w;
  float v[2];
#pragma unroll
  for (int jn = 0; jn < 2; ++jn) {
    v[jn] = s_acc[0][jn][w][lane];
#pragma unroll
    for (int q = 1; q < kKsWaves; ++q) v[jn] += s_acc[q][jn][w][lane];
    const int col = n0 + 16 * jn + r;
    if (FINISH == 1) {
      v[jn] += addend[jn];
      if (g.relu) v[jn] = v[jn] > 0.f ? v[jn] : 0.f;
    } else if (!((keepw >> (col & 31)) & 1u)) {
      v[jn] = 0.f;
    }
    static_cast<float*>(g.y)[(size_t)row * g.ldy + col] = v[jn];
  }
  if (FINISH == 1 && g.bits) {
    // a ballot holds 16 columns of each of four rows: row lane / 16 in bits 16 (lane / 16) ..
    const uint64_t b0 = __ballot(v[0] > 0.f), b1 = __ballot(v[1] > 0.f);
    const uint32_t word = (uint32_t)((b0 >> (16 * kq)) & 0xFFFFu) | ((uint32_t)((b1 >> (16 * kq)) & 0xFFFFu) << 16);
    if (r == 0) g.bits[(size_t)row * g.bits_pitch + (n0 >> 5)] = word;
  }
}

}  // namespace

// Shapes this kernel takes: whole 16 x 32 tiles, K a multiple of 64 (eight waves, groups of 8), operand rows that
// are whole 16-byte vectors; no loader masks.
bool gemm_f32_ks_ok(const GemmArgs& g, bool b_k_contig) {
  if (g.M < 16 || g.N < 32 || g.K < 512 || g.M % 16 || g.N % 32 || g.K % 64) return false;
  if (g.a_mask || g.b_mask || g.lda % 4 || (reinterpret_cast<uintptr_t>(g.A) & 15)) return false;
  if (g.ldb % 4 || (reinterpret_cast<uintptr_t>(g.B) & 15)) return false;
  return true;
}

// finish 1: y = act(A B + bias + u V) with ReLU bits (forward); finish 2: y = (A B^T) under c_mask (dX)
hipError_t launch_gemm_f32_ks(const GemmArgs& g, int finish, hipStream_t st) {
  const bool b_k = finish == 2;
  if (!gemm_f32_ks_ok(g, b_k)) return hipErrorInvalidValue;
  const dim3 grid((g.M / 16) * (g.N / 32)), block(64 * kKsWaves);
  // every wave's private operand areas; the accumulators (16 KB) take the same space over at the end
  const size_t smem = (size_t)(kKsWaves * (kKsAreaA + kKsAreaB)) * 4;
  auto kern = finish == 1 ? gemm_f32_ks_kernel<false, 1> : gemm_f32_ks_kernel<true, 2>;
  static bool prepared[2] = {false, false};   // one host thread drives a context
  if (!prepared[b_k]) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    prepared[b_k] = true;
  }
  hipLaunchKernelGGL(kern, grid, block, smem, st, g);
  return hipGetLastError();
}

}  // namespace rad
