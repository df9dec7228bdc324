// Host-visible launch interfaces of the RAD kernels.
#pragma once
#include "common.hpp"

namespace rad {

struct PlanArgs {
  uint32_t seed_lo, seed_hi, stream_id, step0;
  int scheme;          // kBernoulli, kFixedKShared, kFixedKPerExample
  int plan_rows;       // rows drawn: steps*rows, or steps for the shared scheme
  int rows_per_step;   // rows of one step block of the store
  int cols;
  int k;               // fixed-k schemes
  int k_pitch;         // shared scheme: entries between consecutive rows of the compact values (>= k)
  uint64_t thresh;     // Bernoulli: keep iff key < thresh
  int key_shift;       // 0; tests raise it to force equal keys
  uint32_t* bitmap;    // [plan_rows][bm_pitch]
  int bm_pitch;
  uint16_t* bucket_off;  // [plan_rows][nb+1]
  int nb;
  uint32_t* row_cnt;   // [plan_rows], Bernoulli only
  uint32_t* row_ptr;   // [steps*rows + 1], written here for the fixed-k schemes
  int* max_seg;        // running maximum of entries per (row, 256-column bucket)
  uint16_t* mult;      // with-replacement draws: draw counts of the kept columns, [plan_rows][k] in entry order
};

hipError_t launch_plan(const PlanArgs& a, hipStream_t st);
int plan_max_cols(int scheme);
hipError_t launch_row_scan(const uint32_t* row_cnt, uint32_t* row_ptr, int rows, int64_t capacity,
                           int* overflow, hipStream_t st);
hipError_t launch_pack(const void* x, int dtype, const StoreView& s, hipStream_t st);

// ---------------------------------------------------------------- GEMM family
// C[M,N] = A[M,K] * B[K,N] on MFMA with fp32 accumulation.  Operand sources:
enum OpKind : int {
  kOpK = 0,      // dense, K contiguous:  A[m*ld + k]   / B[n*ld + k]
  kOpMN = 1,     // dense, M/N contiguous: A[k*ld + m]  / B[k*ld + n]
  kOpSparse = 2, // A only: rows of a compressed store are the K index, columns the M index
  // convolution as an implicit im2col GEMM over an NCHW tensor [B][cv_C][cv_H][cv_W] (stride 1, zero pad):
  kOpIm2colRows = 3,  // A: tile rows are output positions (b,y,x), K index is (c,u,v): forward and dX
  kOpIm2colK = 4,     // A: tile rows are (c,u,v), K index is the position (b,y,x): dW
  kOpKBatched = 5     // B: rows are channels n, K index is the position (b,yx): element at B[(b*cv_N + n)*HW + yx]
};
enum EpiKind : int {
  kEpiStore = 0, // C (+= if beta) = acc, optional output row map
  kEpiFwd = 1,   // bias / rank-u addend / ReLU / bits / dense y / pack next store
  kEpiConv = 2,  // rows are positions (b,yx), columns channels: bias / ReLU / bits, NCHW output
  kEpiSplitK = 3 // plain store of the split's partial sums to C + split*M*N
};

struct GemmArgs {
  int dry_run;                  // select the kernel and report its label, launch nothing
  int M, N, K;
  float out_scale;              // forward epilogue: accumulators are multiplied by this first (0 = no scaling)
  int m_load;                   // 0, or > M: operand A is readable (as zeros) up to this many rows
  const void* A; int64_t lda;
  const void* B; int64_t ldb;
  // optional bit mask over a dense operand: element (outer, inner) is zeroed when
  // bit (inner % 32) of mask[outer * pitch + inner / 32] is 0 (inner = contiguous index)
  const uint32_t* a_mask; int a_mask_pitch;
  const uint32_t* b_mask; int b_mask_pitch;
  StoreView sa;                 // kOpSparse A
  int sparse_prefetch;          // entries per lane held in registers (host picks)
  // kEpiStore
  void* C; int64_t ldc; int beta; int c_dtype;   // c_dtype: kF32 or kBF16
  const uint16_t* row_map;      // output row of tile row r (null = r)
  const uint32_t* c_mask; int c_mask_pitch;      // kEpiStore: zero C[m,n] where bit n%32 of c_mask[m*pitch + n/32] is 0
  // kEpiFwd
  const float* bias; int relu;
  void* y; int64_t ldy;         // dense output, operand dtype
  uint32_t* bits; int bits_pitch;
  int pack; StoreView next;     // pack the output tile into `next` (rows = M, cols = N)
  const float* u; int64_t u_ld; int u_n; const float* V;   // h += sum_i u[m*u_ld+i] * V[i*N+n]
  // convolution geometry (im2col operand kinds, kEpiConv) and split-K
  int cv_C, cv_H, cv_W, cv_KH, cv_KW, cv_pad, cv_N;   // cv_N: channels of the kOpKBatched / kEpiConv tensor
  int k_split, k_splits;       // K range per blockIdx.y (multiple of the K slice), number of splits (0/1 = none)
  int64_t split_stride;        // > 0: split s stores its partial sums plainly at C + s*split_stride (else fp32 atomics into C)
  // host side only: when set, the launch itself carries these two HIP events (start and end of the kernel),
  // which costs no extra packets on the stream
  void* ev_start; void* ev_stop;
};

// dtype: operand element type; returns hipErrorInvalidValue for combinations
// without a kernel.  `name` (out, may be null) receives the kernel's label.
hipError_t launch_gemm(int dtype, int a_kind, int b_kind, int epi, const GemmArgs& g,
                       hipStream_t st, const char** name);

// ------------------------------------------------------------- small kernels
// dz_ld > classes: rows of dlogits are dz_ld apart and their columns past `classes` are written as zeros (whole
// 16-byte vectors only)
hipError_t launch_softmax_ce(const void* logits, const int32_t* labels, int rows, int classes,
                             int dtype, void* dlogits, float* row_loss, float* loss, hipStream_t st, int dz_ld = 0);
// out[i*N + n] (+)= sum_b w_i[b] * g[b,n], i = 0..n_w; w_0 = 1 (bias gradient),
// w_i = u[b*u_ld + i-1]; g = dy masked by bits.  partial: [splits][n_w+1][N] scratch.  With u_block_rows > 0 the
// rows come in blocks of that many (time steps) and row b of block q weighs with u[b*u_ld + q*u_block_stride + i-1].
hipError_t launch_colsum(const void* dy, int dtype, int rows, int N, const uint32_t* bits, int bits_pitch,
                         const float* u, int64_t u_ld, int u_n, float* out_bias, float* out_u,
                         int beta, float* partial, int splits, hipStream_t st, int u_block_rows = 0,
                         int64_t u_block_stride = 0, int64_t ldy = 0);       // ldy > 0: the rows of dy are ldy apart
hipError_t launch_fill_u32(uint32_t* p, uint32_t v, int64_t n, hipStream_t st);
// Rademacher matrix of the projection scheme: R [d][kp] and its transpose Rt [kp][d] in the given dtype, +1 / -1
// from the key stream (entry (j, s) = bit j*k + s), zero in the padding columns s >= k (both must be zeroed first)
hipError_t launch_sign_matrix(void* R, void* Rt, int dtype, int d, int k, int kp, uint32_t seed_lo, uint32_t seed_hi,
                              uint32_t stream_id, uint32_t step, hipStream_t st);
// Projection with a matrix per example: z [rows][kp] = scale * x R_b (columns k .. kp-1 are written as zeros),
// and xt [rows][d] = scale * z R_b^T, the signs of R_b drawn in the kernels (never stored).  k <= 38400.
hipError_t launch_project_rows_fwd(const void* x, int dtype, int rows, int d, int k, int kp, float scale, void* z,
                                   uint32_t seed_lo, uint32_t seed_hi, uint32_t stream_id, uint32_t step,
                                   hipStream_t st);
hipError_t launch_project_rows_bwd(const void* z, int dtype, int rows, int d, int k, int kp, float scale, void* xt,
                                   uint32_t seed_lo, uint32_t seed_hi, uint32_t stream_id, uint32_t step,
                                   hipStream_t st);
// out[i] = in[i] * scale, stored in the given dtype
hipError_t launch_scale_cast(const float* in, void* out, int dtype, int64_t n, float scale, hipStream_t st);
// out[i] (+)= sum over `splits` partial arrays of n elements
hipError_t launch_splitk_reduce(const float* partial, int splits, int64_t n, float* out, int beta, hipStream_t st);
// out[row_map[r] * ld + n] (+)= sum over `splits` arrays (stride elements apart) of partial[r * N + n], r < rows,
// added in split order; row_map may be null (row r); in_ld > 0: the rows of a partial array are in_ld apart
hipError_t launch_splitk_reduce_rows(const float* partial, int splits, int64_t stride, int rows, int N,
                                     const uint16_t* row_map, float* out, int64_t ld, int beta, hipStream_t st,
                                     int64_t in_ld = 0);
// fp32 forward GEMM finished from split-K partial sums [splits][M][N]: bias, low-rank term u V, ReLU, (h > 0) bits
// (N a multiple of 64); and a dX finished from partial sums with the output mask of the layer below
hipError_t launch_splitk_fwd_f32(const float* partial, int splits, int M, int N, const float* bias, const float* u,
                                 int64_t u_ld, int u_n, const float* V, int relu, float* y, uint32_t* bits,
                                 int bits_pitch, hipStream_t st);
hipError_t launch_splitk_reduce_masked(const float* partial, int splits, int M, int N, const uint32_t* mask, int pitch,
                                       float* out, hipStream_t st);
hipError_t launch_splitk_bias(const float* partial, int splits, int M, int N, const float* bias, void* out, int dtype,
                              hipStream_t st, int64_t pld = 0);
// 2x2/stride-2 max pool over NCHW planes; arg packs the 2-bit window position (dy*2+dx of the first maximum)
// of 16 consecutive outputs per word
hipError_t launch_maxpool_fwd(const float* y, int planes, int H, int W, float* pooled, uint32_t* arg, hipStream_t st);
// 2x2/stride-2 average pool over NCHW planes (even H and W)
hipError_t launch_avgpool_fwd(const float* y, int planes, int H, int W, float* pooled, hipStream_t st);
// g[b,c,y,x] = upstream gradient routed through the pool (pool: 0 none, 1 max pool with positions in arg,
// 2 average pool) and masked by the ReLU bits of the layer
hipError_t launch_unpool_mask(const float* dy, int batch, int C, int H, int W, int pool, const uint32_t* arg,
                              const uint32_t* bits, int bits_pitch, float* g, hipStream_t st);
// Reaction-diffusion study: `problems` independent (theta, sampling stream) pairs, one workgroup each; forward
// pass keeping the sampled entries of every state in vals [problems][16][cap] (a run per wave) and the runs' lengths
// in wave_end [problems][16], then the sampled adjoint pass.  n <= 32, steps >= 1.
hipError_t launch_pde(int problems, int n, int64_t steps, double D, double dt, double p, uint32_t seed_lo,
                      uint32_t seed_hi, uint32_t stream_id, const double* theta, double* vals, int64_t cap,
                      uint32_t* wave_end, int* overflow, double* loss, double* grad, int64_t* stored, hipStream_t st);
// Path sampling on a linearised graph (vertices in topological order, CSR of outgoing edges; level_ptr_host
// [n_levels + 1] on the HOST, edges lead to later levels only): reached [n] and adj [n] are outputs, *bad is set
// if the arrays are inconsistent (an edge or vertex number out of range, an edge inside a level).
hipError_t launch_path_sampling(int n, int n_levels, const int32_t* level_ptr_host, int64_t n_edges,
                                const int32_t* succ_ptr, const int32_t* succ, const double* partial, int y,
                                const int32_t* inputs, int n_inputs, int k, uint32_t seed_lo, uint32_t seed_hi,
                                uint32_t stream_id, double* adj, uint32_t* reached, int* bad, hipStream_t st);
// One optimiser step over n parameters: w (fp32, updated in place), g (fp32 gradient), Adam moments m, v (fp32,
// updated in place; unused for SGD), lo: bf16 copy of w to refresh, or null.  inv_bc1 / inv_bc2 are
// 1 / (1 - beta^t) of the step number and omb1 / omb2 are 1 - beta, all formed in double by the caller (in fp32
// 1 - 0.9f is off by 2e-7 of its value).
struct OptimArgs { float lr, l2, beta1, beta2, omb1, omb2, eps, inv_bc1, inv_bc2; };
hipError_t launch_optim(bool adam, float* w, uint16_t* lo, const float* g, float* m, float* v, int64_t n,
                        const OptimArgs& a, hipStream_t st);
// db[c] = sum over b, y, x of g[b,c,y,x]; partial: [C][splits] scratch (workgroup (c, s) adds examples s, s + splits, ...)
hipError_t launch_channel_sum(const float* g, int batch, int C, int HW, float* db, float* partial, int splits,
                              hipStream_t st);
// Wt[(o,u,v)][c] = W[c][KH-1-u][KW-1-v][o]: the weight operand of the transposed convolution (dX)
hipError_t launch_flip_weights(const float* W, int Ci, int KH, int KW, int Co, float* Wt, hipStream_t st);
// Adds to dW the entries of (row, bucket) segments beyond the first `cap`, which the MFMA kernel leaves out;
// exits at once when *max_seg <= cap (the plan's running maximum), which is the normal case.
// (ldy > 0: the rows of dy are ldy apart)
hipError_t launch_dw_overflow(const StoreView& s, int rows, const void* dy, int dtype, int N, const uint32_t* bits,
                              int bits_pitch, float* dW, int cap, const int* max_seg, hipStream_t st, int64_t ldy = 0);
// entries per (row, bucket) the bf16 sparse dW kernel chosen for `sparse_prefetch` handles itself
int gemm_bf16_sparse_cap(int sparse_prefetch);
int gemm_bf16_sparse_max_prefetch();
// dense[rows, cols] = the store's rows scattered back (zeros elsewhere): x~ as a dense operand
hipError_t launch_unpack(const StoreView& s, int dtype, void* dense, hipStream_t st);
// the same for a store that keeps values only, from the keep bitmap of its current draw (s.bitmap)
hipError_t launch_unpack_bitmap(const StoreView& s, int dtype, void* dense, hipStream_t st);
// index-free stores: rebuild the (value, column) entries (bf16: out_pairs) or the columns (fp32: out_idx) from
// the values in `s` and the keep bitmap / offsets of a fresh plan
hipError_t launch_reindex(const StoreView& s, int dtype, uint32_t* out_pairs, uint16_t* out_idx, hipStream_t st);

// fp32 GEMM with K split over the eight waves of a workgroup (gemm_f32_ks.hip), whole epilogue in the same launch.
// finish 1: forward (A K-contiguous, B N-contiguous; bias, u V, ReLU, bits -> y); finish 2: dX (A and B K-contiguous;
// c_mask -> y).  gemm_f32_ks_ok: whole 16 x 32 tiles, K % 64 == 0, 16-byte aligned rows, no loader masks.
bool gemm_f32_ks_ok(const GemmArgs& g, bool b_k_contig);
hipError_t launch_gemm_f32_ks(const GemmArgs& g, int finish, hipStream_t st);

// Convolutions through an LDS-staged input patch (conv.hip).  launch_conv_fwd_direct takes the arguments of the
// im2col GEMM (A = NCHW input, B = W [(c,u,v)][co], cv_* geometry, the kEpiConv fields) and serves forward and dX;
// launch_conv_dw_direct writes conv_dw_direct_splits(...) partial sums [ci*ks*ks][co] of dW from the dense x~ and
// g = dL/dh (both NCHW).  hipErrorInvalidValue / 0 splits: shape not served, take the general im2col kernels.
hipError_t launch_conv_fwd_direct(const GemmArgs& g, hipStream_t st);
int conv_dw_direct_splits(int batch, int ci, int co, int H, int W, int ks);
hipError_t launch_conv_dw_direct(const float* xt, const float* g, float* part, int batch, int ci, int co, int H, int W,
                                 int ks, hipStream_t st);

// Ceiling probes (ceilings.hip): kind 0 HBM read, 1 HBM copy, 2 / 3 bf16 MFMA 32x32x16 / 16x16x32 register loops,
// 4 fp32 MFMA 32x32x2, 5 integer 32 x 32 -> 64 multiply-adds.  a: operands (probe_min_bytes at least), b: sink
// (copy: destination of `bytes`; else 1 KiB).
double probe_units(int kind, uint64_t bytes, int iters);
uint64_t probe_min_bytes(int kind);
hipError_t launch_probe(int kind, const void* a, void* b, uint64_t bytes, int iters, hipStream_t st);

}  // namespace rad
