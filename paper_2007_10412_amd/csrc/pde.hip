// Reaction-diffusion PDE-constrained optimisation with a sampled adjoint (Section 5, Appendix B).
// phi lives on the nodes (i, j), 0 <= i, j <= n <= 32, of the unit square, zero on the boundary; one explicit
// step is phi += r (4-neighbour sum - 4 phi) + dt C phi with r = D dt / dx^2 and C the seven-term series in x and
// t.  The steps depend on each other, so one problem is one workgroup of 1024 threads (a node each, the state in
// LDS, one barrier per step) and the launch runs many problems (control vectors, sampling streams) side by
// side, one per CU.  All arithmetic is fp64: the work is bound by the chain of barriers, not by flops.
//
// What is kept of phi_t for the backward pass: the interior entries whose key is below p 2^32 (entry
// c = (i-1)(n-1) + (j-1) of step t takes word c mod 4 of the Philox call c / 4 with (stream, step = t)).  Every
// wave appends its kept entries to a run of its own; the backward pass draws the same keys again and walks the
// run back (ballot + popcount give a lane's place among the wave's kept entries of a step).
#include <cmath>

#include "kernels.hpp"
#include "philox.hpp"

namespace rad {

namespace {

constexpr int kPdeThreads = 1024, kPdePitch = 33, kPdeNodes = kPdePitch * kPdePitch;
constexpr int kPdeTab = 512;         // time points per refill of the per-step tables

struct PdeThread {
  int i, j, idx, cell, lane, wave;
  bool interior;
  double s2x, c2x, phi0, tgt_xy;
  __device__ __forceinline__ void init(int n) {
    i = threadIdx.x >> 5; j = threadIdx.x & 31;
    idx = i * kPdePitch + j;
    lane = threadIdx.x & 63; wave = threadIdx.x >> 6;
    interior = i >= 1 && j >= 1 && i <= n - 1 && j <= n - 1;
    cell = interior ? (i - 1) * (n - 1) + (j - 1) : 0;
    const double x = (double)i / n, y = (double)j / n;
    s2x = sinpi(2.0 * x); c2x = cospi(2.0 * x);
    phi0 = interior ? sinpi(x) * sinpi(y) : 0.0;
    tgt_xy = interior ? s2x * sinpi(y) : 0.0;
  }
  // is this thread's entry of step t kept; how many kept entries of the wave come before it; the wave's count
  __device__ __forceinline__ bool draw(const uint32_t* keys, uint32_t thr_lo, bool keep_all, uint32_t* before,
                                       uint32_t* in_wave) const {
    const bool keep = interior && (keep_all || keys[cell] < thr_lo);
    const uint64_t b = __ballot(keep);
    *before = (uint32_t)__popcll(b & ((1ull << lane) - 1ull));
    *in_wave = (uint32_t)__popcll(b);
    return keep;
  }
};

// the keys of step t for all interior entries, four per Philox call, by the first (n-1)^2 / 4 threads
__device__ __forceinline__ void pde_fill_keys(uint32_t* keys, int cells, int64_t t, uint32_t seed_lo, uint32_t seed_hi,
                                              uint32_t stream) {
  if ((int)threadIdx.x * 4 < cells) {
    const u32x4 k4 = element_quad_keys((uint64_t)threadIdx.x, stream, (uint32_t)t, seed_lo, seed_hi);
    *reinterpret_cast<u32x4*>(keys + 4 * threadIdx.x) = k4;
  }
}

// sum over the workgroup in a fixed order; every thread gets the result
__device__ __forceinline__ double block_sum(double v, double* red) {
  __syncthreads();
  red[threadIdx.x] = v;
  __syncthreads();
  for (int s = kPdeThreads / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  return red[0];
}

struct PdeArgs {
  int n; int64_t steps; double r, dt, p;
  uint32_t thr; int keep_all;                 // keep iff key < thr; p = 1 keeps everything
  uint32_t seed_lo, seed_hi, stream_id;
  const double* theta;                        // [problems][7]
  double* vals; int64_t cap;                  // [problems][16 waves][cap] kept entries, each wave its own run
  uint32_t* wave_end;                         // [problems][16] entries each wave kept in all
  int* overflow;                              // [problems]
  double* loss; double* grad; int64_t* stored;
};

// Each wave (two grid rows) appends its kept entries to a run of its own, so a thread's place is the wave's
// running count plus the kept lanes below it: no exchange between waves, and the backward pass walks the run
// back by subtracting each step's count.

__global__ __launch_bounds__(kPdeThreads) void pde_forward_kernel(PdeArgs a) {
  __shared__ double ph[2][kPdeNodes];
  __shared__ double red[kPdeThreads];
  // for each of the next kPdeTab time points: sin(pi t), and C = ca + sin(2 pi x) cb + cos(2 pi x) cc
  __shared__ double trig_s[kPdeTab], tab_a[kPdeTab], tab_b[kPdeTab], tab_c[kPdeTab];
  __shared__ __align__(16) uint32_t keys[2][kPdeThreads];        // keys of this step and of the next
  const int pb = blockIdx.x;
  PdeThread me; me.init(a.n);
  const int cells = (a.n - 1) * (a.n - 1);
  double th[7];
#pragma unroll
  for (int k = 0; k < 7; ++k) th[k] = a.theta[(size_t)pb * 7 + k];
  const uint32_t stream = a.stream_id + (uint32_t)pb;
  double* const vals = a.vals + ((size_t)pb * 16 + me.wave) * a.cap;
  for (int q = threadIdx.x; q < 2 * kPdeNodes; q += kPdeThreads) (&ph[0][0])[q] = 0.0;
  pde_fill_keys(keys[0], cells, 0, a.seed_lo, a.seed_hi, stream);
  __syncthreads();
  if (me.interior) ph[0][me.idx] = me.phi0;
  __syncthreads();
  double mine = me.phi0, loss = 0.0;
  double ca = th[0] + th[2], cb = th[4], cc = th[6];             // C at t = 0: sin = 0, cos = 1
  int64_t offset = 0;                                            // entries this wave has kept so far
  bool over = false;
  for (int64_t t = 0; t <= a.steps; ++t) {
    const int cur = (int)(t & 1);
    if ((t & (kPdeTab - 1)) == 0) {          // a thread each works out the next kPdeTab time points
      __syncthreads();
      if (threadIdx.x < kPdeTab) {
        double sn, cs;
        sincospi((double)(t + 1 + threadIdx.x) * a.dt, &sn, &cs);
        trig_s[threadIdx.x] = sn;
        tab_a[threadIdx.x] = th[0] + th[1] * sn + th[2] * cs;
        tab_b[threadIdx.x] = th[3] * sn + th[4] * cs;
        tab_c[threadIdx.x] = th[5] * sn + th[6] * cs;
      }
      __syncthreads();
    }
    uint32_t before, in_wave;
    const bool keep = me.draw(keys[cur], a.thr, a.keep_all != 0, &before, &in_wave);
    if (keep) {
      const int64_t pos = offset + before;
      if (pos < a.cap) vals[pos] = mine; else over = true;
    }
    offset += in_wave;
    if (t == a.steps) break;
    pde_fill_keys(keys[cur ^ 1], cells, t + 1, a.seed_lo, a.seed_hi, stream);
    double nw = 0.0;
    if (me.interior) {
      const double* f = ph[cur];
      const double nb = (f[me.idx + kPdePitch] + f[me.idx - kPdePitch]) + (f[me.idx + 1] + f[me.idx - 1]);
      nw = mine + a.r * (nb - 4.0 * mine) + a.dt * (ca + me.s2x * cb + me.c2x * cc) * mine;
      ph[cur ^ 1][me.idx] = nw;
    }
    const int q = (int)(t & (kPdeTab - 1));
    const double s = trig_s[q];                                  // time t + 1
    ca = tab_a[q]; cb = tab_b[q]; cc = tab_c[q];
    if (me.interior) {
      const double d = nw - (me.phi0 + 0.25 * s * me.tgt_xy);
      loss += d * d;
      mine = nw;
    }
    __syncthreads();
  }
  if (me.lane == 0) a.wave_end[(size_t)pb * 16 + me.wave] = (uint32_t)(offset < a.cap ? offset : a.cap);
  const double total_loss = block_sum(loss, red);
  const double any_over = block_sum(over ? 1.0 : 0.0, red);
  const double kept = block_sum(me.lane == 0 ? (double)offset : 0.0, red);
  if (threadIdx.x == 0) {
    a.loss[pb] = total_loss / (double)a.steps;
    a.overflow[pb] = any_over > 0.0 ? 1 : 0;
    if (a.stored) a.stored[pb] = (int64_t)kept;
  }
}

__global__ __launch_bounds__(kPdeThreads) void pde_backward_kernel(PdeArgs a) {
  __shared__ double lb[2][kPdeNodes];
  __shared__ double red[kPdeThreads];
  // for kPdeTab time points: sin and cos of pi t, and C = ca + sin(2 pi x) cb + cos(2 pi x) cc
  __shared__ double trig_s[kPdeTab], trig_c[kPdeTab], tab_a[kPdeTab], tab_b[kPdeTab], tab_c[kPdeTab];
  __shared__ __align__(16) uint32_t keys[2][kPdeThreads];        // keys of the step being drawn and of the one before
  const int pb = blockIdx.x;
  PdeThread me; me.init(a.n);
  const int cells = (a.n - 1) * (a.n - 1);
  double th[7];
#pragma unroll
  for (int k = 0; k < 7; ++k) th[k] = a.theta[(size_t)pb * 7 + k];
  // dL/dC of this node summed over time with the weights 1, sin(pi t), cos(pi t): the node's factors
  // sin(2 pi x), cos(2 pi x) of the seven basis functions are applied once at the end
  double w1 = 0.0, ws = 0.0, wc = 0.0;
  const uint32_t stream = a.stream_id + (uint32_t)pb;
  const double* const vals = a.vals + ((size_t)pb * 16 + me.wave) * a.cap;
  int64_t offset = (int64_t)a.wave_end[(size_t)pb * 16 + me.wave];       // walks back one step's count at a time
  const double inv_p = 1.0 / a.p, w_loss = 2.0 / (double)a.steps;
  for (int q = threadIdx.x; q < 2 * kPdeNodes; q += kPdeThreads) (&lb[0][0])[q] = 0.0;

  // value of this thread's entry of step t (0 if it was not kept); keys[buf] holds the keys of step t (filled
  // before the last barrier), those of step t - 1 go to the other half
  auto fetch = [&](int64_t t, int buf, bool& keep) -> double {
    uint32_t before, in_wave;
    keep = me.draw(keys[buf], a.thr, a.keep_all != 0, &before, &in_wave);
    if (t >= 1) pde_fill_keys(keys[buf ^ 1], cells, t - 1, a.seed_lo, a.seed_hi, stream);
    offset -= in_wave;
    const int64_t pos = offset + before;
    return (keep && pos >= 0 && pos < a.cap) ? vals[pos] : 0.0;
  };
  // A: step t, B: step t - 1
  pde_fill_keys(keys[0], cells, a.steps, a.seed_lo, a.seed_hi, stream);
  __syncthreads();
  bool keepA, keepB, keepC = false;
  double valA = fetch(a.steps, 0, keepA);
  __syncthreads();
  double valB = fetch(a.steps - 1, 1, keepB);
  __syncthreads();
  double lam = 0.0, s_t, c_t;
  sincospi((double)a.steps * a.dt, &s_t, &c_t);
  int cur = 0;                      // buffers alternate from the prologue on: 0, 1, then 0 again
  for (int64_t t = a.steps; t >= 1; --t, cur ^= 1) {
    const int64_t u = t - 1;        // the time point of C and of the sampled phi of this iteration
    const int q = (int)(u & (kPdeTab - 1));
    if (t == a.steps || q == kPdeTab - 1) {
      __syncthreads();
      if (threadIdx.x < kPdeTab) {
        double sn, cs;
        sincospi((double)((u & ~(int64_t)(kPdeTab - 1)) + threadIdx.x) * a.dt, &sn, &cs);
        trig_s[threadIdx.x] = sn; trig_c[threadIdx.x] = cs;
        tab_a[threadIdx.x] = th[0] + th[1] * sn + th[2] * cs;
        tab_b[threadIdx.x] = th[3] * sn + th[4] * cs;
        tab_c[threadIdx.x] = th[5] * sn + th[6] * cs;
      }
      __syncthreads();
    }
    double valC = 0.0;
    if (t >= 2) valC = fetch(t - 2, cur, keepC);                // its load is in flight during this step
    if (keepA) lam += w_loss * inv_p * (valA - (me.phi0 + 0.25 * s_t * me.tgt_xy));
    const double s = trig_s[q], c = trig_c[q];
    {
      const double w = valB * lam;                               // times dt / p at the end
      w1 += w; ws += s * w; wc += c * w;
    }
    if (me.interior) lb[cur][me.idx] = lam;
    __syncthreads();
    if (me.interior) {
      const double* f = lb[cur];
      const double nb = (f[me.idx + kPdePitch] + f[me.idx - kPdePitch]) + (f[me.idx + 1] + f[me.idx - 1]);
      lam = lam + a.r * (nb - 4.0 * lam) + a.dt * (tab_a[q] + me.s2x * tab_b[q] + me.c2x * tab_c[q]) * lam;
    }
    valA = valB; valB = valC; keepA = keepB; keepB = keepC;
    s_t = s; c_t = c;
  }
  const double sc = a.dt * inv_p;
  const double g[7] = {w1 * sc, ws * sc, wc * sc, me.s2x * ws * sc, me.s2x * wc * sc, me.c2x * ws * sc, me.c2x * wc * sc};
#pragma unroll
  for (int k = 0; k < 7; ++k) {
    const double tot = block_sum(g[k], red);
    if (threadIdx.x == 0) a.grad[(size_t)pb * 7 + k] = tot;
  }
}

}  // namespace

hipError_t launch_pde(int problems, int n, int64_t steps, double D, double dt, double p, uint32_t seed_lo,
                      uint32_t seed_hi, uint32_t stream_id, const double* theta, double* vals, int64_t cap,
                      uint32_t* wave_end, int* overflow, double* loss, double* grad, int64_t* stored, hipStream_t st) {
  PdeArgs a;
  a.n = n; a.steps = steps; a.r = D * dt * (double)n * (double)n; a.dt = dt; a.p = p;
  const double thr = std::floor(p * 4294967296.0 + 0.5);
  a.keep_all = thr >= 4294967296.0 ? 1 : 0;
  a.thr = a.keep_all ? 0xffffffffu : (uint32_t)thr;
  a.seed_lo = seed_lo; a.seed_hi = seed_hi; a.stream_id = stream_id;
  a.theta = theta; a.vals = vals; a.cap = cap; a.wave_end = wave_end; a.overflow = overflow;
  a.loss = loss; a.grad = grad; a.stored = stored;
  hipLaunchKernelGGL(pde_forward_kernel, dim3((unsigned)problems), dim3(kPdeThreads), 0, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(pde_backward_kernel, dim3((unsigned)problems), dim3(kPdeThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace rad
