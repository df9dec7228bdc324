/*
 * rad.h: C ABI of the MI355X (gfx950) library for the hot path of Randomized
 * Automatic Differentiation (Oktay, McGreivy, Aduol, Beatson, Adams, 2020):
 * the training step of a linear layer that keeps, instead of its input x, a
 * random inverse-probability-scaled sample x~ = x P (Section 3.2: E[P] = I)
 * plus one ReLU bit per output (Section 4.2), and forms the unbiased weight
 * gradient dW~ = x~^T g from that compressed store while dX = g W^T stays
 * exact (Section 4.2: only dh/dW is sampled).
 *
 * Conventions for every entry point
 *   - Tensor pointers are DEVICE pointers owned by the caller, row-major and
 *     contiguous, 16-byte aligned; the library keeps none of them after the
 *     call returns.  Pointers documented "host" are host memory.
 *   - x [batch, d_in], W [d_in, d_out], bias [d_out], y and dy [batch, d_out],
 *     dW [d_in, d_out] (always fp32), dX [batch, d_in].  Element type of
 *     x, W, y, dy, dX is rad_layer.dtype; bias, dW, dbias are fp32.
 *   - Work is enqueued on the HIP stream given to rad_ctx_create and is
 *     asynchronous unless the function is documented to synchronise.
 *   - Every failure is a status code; rad_last_error(ctx) has the text.  All
 *     arguments are validated before the first launch, so a failed call has
 *     no device side effects.  Nothing aborts or throws across this ABI.
 *   - There is no CPU fallback: without a HIP device rad_ctx_create fails.
 */
#ifndef RAD_H_
#define RAD_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  RAD_OK = 0,
  RAD_ERR_NULL = 1,        /* a required pointer is null */
  RAD_ERR_SHAPE = 2,       /* negative/oversized/inconsistent dimensions */
  RAD_ERR_PARAM = 3,       /* p outside (0,1], unknown enum value */
  RAD_ERR_UNSUPPORTED = 4, /* valid request this build has no kernel for */
  RAD_ERR_CAPACITY = 5,    /* a Bernoulli draw exceeded the store's capacity */
  RAD_ERR_DEVICE = 6       /* HIP runtime error */
} rad_status;

typedef enum { RAD_F32 = 0, RAD_BF16 = 1 } rad_dtype; /* accumulation is always fp32 */

/* Which entries of the layer input are stored (Section 3.2, Section 4.3).
 * EXACT keeps everything (the baseline).  BERNOULLI keeps each entry with
 * probability p and scales by 1/p.  The two FIXEDK schemes keep
 * k = rad_fixed_k(p, d_in) coordinates drawn without replacement and scale
 * by d_in/k: SHARED uses one index set for the whole minibatch (the paper's
 * "same sample"), PER_EXAMPLE an independent one per row ("different
 * sample").  The two REPLACE schemes are the matrix P of Section 3.2 as
 * printed: k indices drawn uniformly WITH replacement (draw s of row b maps
 * the key of flat index b k + s, or s for SHARED, to floor(key d_in / 2^32));
 * a coordinate drawn m times is stored once with the weight m d_in/k, so a
 * row holds between 1 and k entries.  Their stores are always kept as
 * per-row (value, column) lists.  PROJECT_SHARED is the other P of Section 3.2
 * (Appendix, "Random projections for RAD"): P = R R^T / k with R [d_in, k] a
 * matrix of independent signs drawn once per layer and step (entry (j, s) is
 * bit (j k + s) of the key stream; clear = +1).  The store is the dense
 * z = x R / sqrt(k), k numbers per row and no indices; dW is
 * R (z^T g) / sqrt(k), with R regenerated from the sampling parameters.
 * PROJECT_PER_EXAMPLE (Appendix A, "different project") gives every row b a
 * matrix R_b of its own: row (b, j) of the sign tensor owns the
 * C = ceil(k/128) Philox calls numbered (b d_in + j) C onwards, sign s is bit
 * s mod 32 of word (s / 32) mod 4 of call s / 128 (clear = +1); the store is
 * z_b = x_b R_b / sqrt(k), and dW = x~^T g with x~_b = z_b R_b^T / sqrt(k)
 * rebuilt row by row (never more than one layer's worth); k <= 38400.
 * The projection schemes serve linear layers and MLP and RNN models only. */
typedef enum {
  RAD_EXACT = 0,
  RAD_BERNOULLI = 1,
  RAD_FIXEDK_SHARED = 2,
  RAD_FIXEDK_PER_EXAMPLE = 3,
  RAD_REPLACE_SHARED = 4,
  RAD_REPLACE_PER_EXAMPLE = 5,
  RAD_PROJECT_SHARED = 6,
  RAD_PROJECT_PER_EXAMPLE = 7
} rad_scheme;

typedef enum { RAD_LINEAR = 0, RAD_CONV2D = 1 } rad_kind;

/* One linear layer (Section 4.2).  For RAD_CONV2D (Figure 5) the layer is a
 * stride-1 convolution computed as an implicit im2col GEMM: x is NCHW
 * [batch, c_in, h, w] (d_in = c_in*h*w, the flattened tensor is what is
 * sampled), W is [c_in, kh, kw, c_out], y is NCHW [batch, c_out, h, w]
 * (d_out = c_out*h*w; pad must keep the spatial size: 2*pad = kh-1 = kw-1).
 * dW is [c_in, kh, kw, c_out] and dbias [c_out]; dX is NCHW like x.  Conv
 * layers are fp32, with at most 64 input and 64 output channels and h*w a
 * multiple of 64 (RAD_ERR_UNSUPPORTED otherwise); rad_backward_dW writes conv
 * gradients (beta = 0 only).  The projection schemes do not serve them. */
typedef struct {
  int32_t kind;     /* rad_kind */
  int32_t dtype;    /* rad_dtype */
  int64_t batch;
  int64_t d_in;
  int64_t d_out;
  int32_t relu;     /* y = max(h, 0) and one stored bit per output */
  int32_t has_bias;
  int32_t c_in, h, w, c_out, kh, kw, pad; /* RAD_CONV2D only */
} rad_layer;

/* The random draw.  Keys come from Philox4x32-10 with key = (seed low word,
 * seed high word) and counter = (floor(f/4) low, floor(f/4) high, stream_id,
 * step), output word f mod 4, where f = row*d_in + column is the flat index
 * of the element in the sampled tensor (f = column for RAD_FIXEDK_SHARED).
 * stream_id separates tensors/layers, step separates RNN time steps. */
typedef struct {
  int32_t scheme;   /* rad_scheme */
  double p;         /* fraction in (0, 1] */
  uint64_t seed;
  uint32_t stream_id;
  uint32_t step;
} rad_sampling;

typedef struct rad_ctx rad_ctx;     /* stream + workspaces; one per stream */
typedef struct rad_store rad_store; /* compressed store of one layer */
typedef struct rad_model rad_model; /* layer list + stores for rad_train_step */

/* Stored bytes of a store, split the way the accounting of Appendix A needs:
 * values (what the paper counts), indices and offset tables (which the paper
 * does not count), ReLU bits (1 per output entry, which it does). */
typedef struct {
  uint64_t value_bytes;
  uint64_t index_bytes;
  uint64_t bit_bytes;
  uint64_t nnz;          /* stored entries */
  uint64_t dense_bytes;  /* what storing x itself would take */
} rad_store_stats;

/* k = ceil(p*d) clamped to [1, d]: "rounded up" in Appendix A's memory
 * calculation (784->79, 300->30, 16384->1639 at p = 0.1).  Host function. */
int64_t rad_fixed_k(double p, int64_t d);

/* Creates a context bound to hip_stream (a hipStream_t, borrowed; null = the
 * default stream) on the current device.  Allocates workspaces lazily. */
rad_status rad_ctx_create(rad_ctx** out, void* hip_stream);
rad_status rad_ctx_destroy(rad_ctx* ctx);
/* Text of the last failure on this context (static string if ctx is null). */
const char* rad_last_error(const rad_ctx* ctx);
/* Blocks until everything enqueued on the context's stream has finished. */
rad_status rad_ctx_synchronize(rad_ctx* ctx);

/* Per-kernel timing with HIP events recorded on the context's stream around
 * every launch whose name contains `filter` (null = all, "" = off).
 * rad_ctx_timing_read synchronises, then returns launches and total
 * milliseconds since the last reset for kernels whose name contains `name`. */
rad_status rad_ctx_timing(rad_ctx* ctx, const char* filter);
rad_status rad_ctx_timing_read(rad_ctx* ctx, const char* name, int64_t* launches, double* total_ms);
rad_status rad_ctx_timing_reset(rad_ctx* ctx);
/* Floating-point operations of the timed GEMM launches whose name contains
 * `name` since the last reset: `executed` counts 2 M N K of each launch,
 * `algorithmic` what the operation needs by definition (for dW from a sampled
 * store, 2 d_out per kept entry; elsewhere the same as executed).  Kernels that
 * are not GEMMs count zero. */
rad_status rad_ctx_timing_read_flops(rad_ctx* ctx, const char* name, double* algorithmic, double* executed);

/* Synchronises.  Measurement aid, not part of the method: what a kernel with
 * nothing else to do reaches on this device for the three resources the hot
 * path is bound by, so that a benchmark can quote its kernels against measured
 * ceilings beside the published peaks.  kind: 0 streaming HBM read of `bytes`
 * from `operands` (units: bytes), 1 copy of `bytes` from `operands` to `sink`
 * (units: bytes read + written), 2 / 3 register-resident loops of the bf16
 * matrix instructions 32x32x16 / 16x16x32 and 4 of the fp32 one (32x32x2) on
 * the values found in `operands` (units: flop; random values run at a lower
 * clock than zeros), 5 independent 32 x 32 + 64 -> 64-bit integer multiply-adds
 * (units: multiply-adds).  operands / sink: DEVICE, 16-byte aligned; sink holds
 * `bytes` for the copy and 1 KiB otherwise; `bytes` a multiple of 16 and at
 * least 16 MiB.  Runs `reps` launches between two events and returns
 * units per second. */
rad_status rad_probe_ceiling(rad_ctx* ctx, int32_t kind, const void* operands, void* sink,
                             uint64_t bytes, int32_t reps, double* units_per_s);

/* Test hook, not part of the method: the keys of the NEXT draw only (the next
 * call that samples one store) are shifted right by `shift` bits (and the
 * Bernoulli threshold likewise) before selection, which makes equal keys
 * frequent and so exercises the tie rule of the fixed-k draw.  The library
 * returns to normal keys after that one draw, so the hook cannot be left on;
 * 0 cancels it.  Not for index-free stores (their backward pass draws again). */
rad_status rad_debug_key_shift(rad_ctx* ctx, int32_t shift);

/* Allocates the store for `layer` under `scheme`/`p`: value and index arrays
 * sized for batch*k entries (fixed-k), batch*d_in (EXACT), or the Bernoulli
 * mean plus eight standard deviations; row pointers, per-256-column offsets,
 * and the ReLU bit array [batch, ceil(d_out/32)] words.  `steps` > 1 makes a
 * multi-step store for BPTT: steps*batch rows, row t*batch+b drawn with
 * step = sampling.step + t.  Requires d_in <= 65535 (16-bit indices). */
rad_status rad_store_create(rad_ctx* ctx, const rad_layer* layer, int32_t scheme, double p,
                            int32_t steps, rad_store** out);
rad_status rad_store_destroy(rad_store* store);
/* Synchronises.  Byte counts of what is currently stored. */
rad_status rad_store_get_stats(rad_ctx* ctx, const rad_store* store, rad_store_stats* out);
/* Synchronises.  Canonical export to HOST arrays: row_ptr [rows+1], then for
 * each row ascending column indices and the stored (already scaled) values
 * converted to fp32.  col/val must hold `capacity` entries; fails with
 * RAD_ERR_CAPACITY if the store holds more, or if a Bernoulli draw overflowed
 * the store when it was written. */
rad_status rad_store_export_csr(rad_ctx* ctx, const rad_store* store, int64_t* row_ptr,
                                int32_t* col, float* val, int64_t capacity);
/* Synchronises.  ReLU bits to a HOST array [rows, ceil(d_out/32)] of words;
 * bit (n mod 32) of word n/32 is 1[h[b,n] > 0]. */
rad_status rad_store_export_bits(rad_ctx* ctx, const rad_store* store, uint32_t* words);
/* Overwrites the ReLU bits from a HOST array (same layout); for tests that
 * feed one side's bits to the other. */
rad_status rad_store_import_bits(rad_ctx* ctx, rad_store* store, const uint32_t* words);

/* Sampling alone (Section 3.2 applied to a stored input): draws the keep
 * set for `sampling`, then writes value = storage(x * scale) and the column
 * index of every kept entry of x [rows, cols] into `store`, ascending column
 * within a row.  rows/cols must equal the store's batch/d_in; `step_slot`
 * selects the block of rows of a multi-step store (0 otherwise). */
rad_status rad_sample_pack(rad_ctx* ctx, const rad_sampling* sampling, const void* x,
                           rad_store* store, int32_t step_slot);

/* rad_sample_pack for callers that cannot allocate device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * rad_sample_pack keeps its transient keep bitmap (1 bit per element of x) in
 * a context workspace that it allocates on first use and when a larger store
 * comes along; this variant keeps it in a static device array of
 * RAD_STATIC_SCRATCH_BYTES that the library holds on every GPU it runs on from
 * load until the process ends, and calls no hipMalloc, hipFree or other
 * allocating routine.  Same kernels, identical results.  `store` (created
 * beforehand with rad_store_create, single-step) receives the output as in
 * rad_sample_pack.  Limits: rows * ceil(cols/32) * 4 bytes of keep words must
 * fit the array (RAD_ERR_CAPACITY otherwise, nothing launched); the projection
 * schemes are RAD_ERR_UNSUPPORTED (they need further workspaces).  Every call
 * on a GPU, from any context or stream, uses that GPU's one array: calls that
 * overlap on one GPU race, so issue them on one stream or order them yourself.
 * The array keeps the last call's contents and needs no clearing (each call
 * writes every word it later reads).  Launches are not timed by
 * rad_ctx_timing. */
#define RAD_STATIC_SCRATCH_BYTES (2u << 20)   /* 2 MiB: 16.7 M elements, e.g. 4096 x 4096 */
rad_status rad_sample_pack_static(rad_ctx* ctx, const rad_sampling* sampling, const void* x,
                                  rad_store* store);

/* Forward of one layer with the exact x (Section 3: the forward pass uses the
 * original graph): y = act(x W + bias); stores the sample of x drawn by
 * `sampling` and, if layer.relu, the bits 1[h > 0] into `store`.  bias may be
 * null iff !layer.has_bias. */
rad_status rad_forward_sample(rad_ctx* ctx, const rad_layer* layer, const rad_sampling* sampling,
                              const void* x, const void* W, const void* bias, void* y,
                              rad_store* store);

/* dW = beta*dW + x~^T g with g = dy * bits (g = dy if !layer.relu), from the
 * compressed store (the sampled Jacobian dh/dW of Section 4.2); dbias (may be
 * null) = beta*dbias + sum over rows of g.  beta must be 0 or 1 (1 accumulates
 * over time steps in BPTT).  dW and dbias are fp32. */
rad_status rad_backward_dW(rad_ctx* ctx, const rad_layer* layer, const rad_store* store,
                           const void* dy, float* dW, float* dbias, float beta);

/* dX = g W^T, exact: independent of p, scheme and seed (Section 4.2).  The
 * store is read only for its ReLU bits. */
rad_status rad_backward_dX(rad_ctx* ctx, const rad_layer* layer, const rad_store* store,
                           const void* dy, const void* W, void* dX);

/* Mean softmax cross-entropy over `rows` examples and its gradient
 * dlogits = (softmax - onehot)/rows in the dtype of logits; labels are int32
 * device values in [0, classes).  loss_dev is one fp32 on the device.  The
 * softmax input is kept dense (Appendix A). */
rad_status rad_softmax_ce(rad_ctx* ctx, const void* logits, const int32_t* labels, int64_t rows,
                          int64_t classes, int32_t dtype, void* dlogits, float* loss_dev);

/* ---- whole training steps ------------------------------------------------
 * A model owns its stores and transient activation buffers; parameters and
 * gradients stay with the caller.  `params` / `grads` are HOST arrays of
 * device pointers in the order documented per model; all gradients are fp32
 * and are overwritten.  Layer l of a model samples with
 * stream_id = sampling.stream_id + l.  rad_train_step synchronises to return
 * the loss in *loss_host. */

/* MLP: n_layers linear layers dims[0] -> dims[1] -> ... -> dims[n_layers],
 * ReLU after all but the last, softmax cross-entropy on the last output.
 * params = {W_0, b_0, W_1, b_1, ...} (b_l entries present iff has_bias),
 * grads likewise. */
rad_status rad_model_create_mlp(rad_ctx* ctx, int32_t dtype, int64_t batch, int32_t n_layers,
                                const int64_t* dims, int32_t has_bias, int32_t scheme, double p,
                                rad_model** out);

/* Vanilla ReLU RNN of Appendix A: h_t = ReLU(x_t W_ih + h_{t-1} W_hh + b),
 * h_0 = 0, t = 1..T; logits = h_T W_ho + b_o; fp32.  x is [batch, T, d_input].
 * h_{t-1} is sampled afresh at each step (stream_id, step = t), the output
 * layer samples h_T with stream_id+1, step 0; x_t is kept whole.
 * params = {W_ih [d_input, hidden], W_hh [hidden, hidden], b [hidden],
 * W_ho [hidden, classes], b_o [classes]}, grads likewise. */
rad_status rad_model_create_rnn(rad_ctx* ctx, int64_t batch, int64_t T, int64_t d_input,
                                int64_t hidden, int64_t classes, int32_t scheme, double p,
                                rad_model** out);

/* Small CNN: n_conv stride-1 convolutions (each + bias + ReLU, then a 2x2 max
 * pool where pool[l] == 1, a 2x2 average pool, for which nothing is stored,
 * where pool[l] == 2 (Appendix A, architectures used), none where 0; other
 * values: RAD_ERR_PARAM), then one linear layer to `classes`; fp32, NCHW.
 * channels[0..n_conv] are c_in, c_out_0, ..., ksize is the square kernel size
 * with pad (ksize-1)/2.  Every conv input and the linear input are sampled.
 * params = {W_0 [c_in,k,k,c_out], b_0, ..., W_fc [d, classes], b_fc}. */
rad_status rad_model_create_cnn(rad_ctx* ctx, int64_t batch, int32_t n_conv, const int32_t* channels,
                                const int32_t* pool, int32_t ksize, int32_t height, int32_t width,
                                int32_t classes, int32_t scheme, double p, rad_model** out);

rad_status rad_model_destroy(rad_model* model);
/* Index-free storage (MLP models; stores of the Bernoulli, per-example fixed-k and with-replacement
 * schemes): only the values of the kept entries stay in the store, which is then the size the paper's
 * accounting gives (Appendix A: k values per sampled row plus the ReLU bits).  The columns are a pure
 * function of the sampling parameters, so the backward pass draws the keep sets again and rebuilds the
 * (value, column) entries of one layer at a time in a context workspace.  Costs one more plan and one
 * small kernel per layer and step.  Synchronises and reallocates; contents of the store are lost. */
rad_status rad_store_set_index_free(rad_ctx* ctx, rad_store* store, int32_t on);
rad_status rad_model_set_index_free(rad_ctx* ctx, rad_model* model, int32_t on);
/* Number of stores and borrowed access to store l (for export and stats). */
int32_t rad_model_num_stores(const rad_model* model);
rad_store* rad_model_store(rad_model* model, int32_t l);
/* Synchronises.  CNN models: the 2-bit max-pool window positions (dy*2+dx of the first maximum) kept for
 * conv layer l, one byte per pooled output, to a HOST array [batch*c_out*(h/2)*(w/2)]; RAD_ERR_PARAM if the
 * layer has no max pool. */
rad_status rad_model_export_pool_arg(rad_ctx* ctx, const rad_model* model, int32_t l, uint8_t* out);
/* Device pointer to the logits of the last step ([batch, classes], model dtype). */
const void* rad_model_logits(const rad_model* model);

/* One training step: forward with exact activations (storing only samples and
 * bits), loss, backward from the stores.  x is the model input, labels int32
 * device [batch].  With loss_host the call synchronises, *loss_host (HOST)
 * receives the mean loss, and RAD_ERR_CAPACITY is returned if a Bernoulli draw
 * overflowed a store in this step or in an earlier one that was only enqueued.
 * With loss_host null the step is only enqueued on the context's stream:
 * nothing is read back, the mean loss is not formed and the call does not
 * wait; gradients are complete once the stream has been synchronised. */
rad_status rad_train_step(rad_ctx* ctx, rad_model* model, const rad_sampling* sampling,
                          const void* x, const int32_t* labels, void* const* params,
                          void* const* grads, float* loss_host);

/* ---- parameter updates ---------------------------------------------------
 * Section 4.3 and Appendix A (training details): the feedforward networks are
 * trained with Adam with a tuned learning rate and l2 regularisation, the
 * recurrent one with SGD without momentum.  The l2 term enters the gradient
 * as l2 * w.  Learning-rate schedules are the caller's: lr is per call. */
typedef enum { RAD_SGD = 0, RAD_ADAM = 1 } rad_optimizer_kind;
typedef struct {
  int32_t kind;             /* rad_optimizer_kind */
  double lr, l2;            /* lr > 0; l2 >= 0 */
  double beta1, beta2, eps; /* RAD_ADAM only: 0 <= beta < 1, eps > 0 */
} rad_optimizer;

/* One optimiser step, number t = 1, 2, ... (Adam's bias correction uses it),
 * over n_tensors tensors of counts[i] elements; all arithmetic in fp32:
 *   g' = g + l2 w
 *   SGD:  w -= lr g'
 *   Adam: m = beta1 m + (1-beta1) g';  v = beta2 v + (1-beta2) g'^2;
 *         w -= lr (m / (1-beta1^t)) / (sqrt(v / (1-beta2^t)) + eps)
 * counts and the pointer arrays are HOST arrays; their entries are DEVICE
 * pointers owned by the caller: grads[i] fp32 (read), m[i] and v[i] fp32
 * moments (RAD_ADAM; updated in place, zero before step 1; the arrays may be
 * null for RAD_SGD).  dtype RAD_F32: params[i] fp32, updated in place, master
 * is ignored (may be null).  dtype RAD_BF16: master[i] holds the fp32 master
 * copy that is updated in place, and params[i] (bf16) receives its rounding
 * to nearest even.  Enqueued on the context's stream; does not wait.
 * Errors (nothing is launched): RAD_ERR_NULL for a missing array or entry,
 * RAD_ERR_SHAPE for a negative count or n_tensors, RAD_ERR_PARAM for an
 * unknown kind or dtype, t < 1, or coefficients outside the ranges above. */
rad_status rad_optimizer_step(rad_ctx* ctx, const rad_optimizer* opt, int64_t t, int32_t dtype,
                              int32_t n_tensors, const int64_t* counts, void* const* params,
                              const void* const* grads, void* const* m, void* const* v,
                              void* const* master);

/* ---- reaction-diffusion PDE-constrained optimisation -----------------------
 * Section 5 and Appendix B: phi on the nodes (i, j), 0 <= i, j <= n, of the
 * unit square (x = i/n, y = j/n), zero on the boundary, stepped explicitly,
 *   phi_{t+1} = phi_t + (D dt n^2)(4-neighbour sum - 4 phi_t) + dt C_t phi_t,
 *   C = th0 + th1 sin(pi t) + th2 cos(pi t) + sin(2 pi x)(th3 sin(pi t) + th4 cos(pi t))
 *       + cos(2 pi x)(th5 sin(pi t) + th6 cos(pi t)),
 * from phi_0 = sin(pi x) sin(pi y); L = (1/steps) sum_{t=1..steps} |phi_t - target_t|^2,
 * target_t = phi_0 + (1/4) sin(pi t) sin(2 pi x) sin(pi y), time t = step * dt.
 * The gradient with respect to the seven controls is the estimator of
 * Section 5: dL/dphi_t and dphi_{t+1}/dC_t = dt diag(phi_t) are sampled with
 * the matrix P of phi_t, so only sampled entries of phi_t are kept: interior
 * entry c = (i-1)(n-1) + (j-1) of step t is kept iff the key of flat index c
 * with (stream_id, step = t) is below round(p 2^32), and weighs 1/p.  p = 1
 * keeps every state and gives the exact gradient.  The paper's grid is n = 32,
 * dt = 1/4096, D = 1/4, steps = 40960.  All arithmetic is fp64. */
typedef struct {
  int32_t n;     /* intervals per side, 2 <= n <= 32 */
  int64_t steps; /* >= 1; steps * (n-1)^2 < 2^32 */
  double D, dt;  /* D dt n^2 <= 1/4 (the stability bound of Appendix B), else RAD_ERR_PARAM */
} rad_pde_grid;

/* Bytes of device workspace rad_pde_gradient needs for `problems` problems at fraction p. */
rad_status rad_pde_workspace_bytes(rad_ctx* ctx, const rad_pde_grid* grid, double p, int32_t problems,
                                   uint64_t* bytes);

/* `problems` independent problems side by side: problem q has the controls
 * theta[q][0..6] (DEVICE, fp64) and draws with stream_id + q.  Outputs
 * (DEVICE): loss [problems], grad [problems][7], stored [problems] (number of
 * kept entries; nullable).  workspace: DEVICE memory of at least
 * rad_pde_workspace_bytes, owned by the caller, contents undefined afterwards.
 * Synchronises; RAD_ERR_CAPACITY if a draw kept more entries than the
 * workspace provides for (8 standard deviations above the mean). */
rad_status rad_pde_gradient(rad_ctx* ctx, const rad_pde_grid* grid, int32_t problems, const double* theta,
                            double p, uint64_t seed, uint32_t stream_id, void* workspace,
                            uint64_t workspace_bytes, double* loss, double* grad, int64_t* stored);

/* ---- path sampling on a general computational graph -------------------------
 * Appendix C, Algorithm 1.  The graph is linearised: vertices numbered in
 * topological order, vertex v with outgoing edges succ_ptr[v] .. succ_ptr[v+1]-1,
 * succ[e] the head of edge e and partial[e] = d succ[e] / d v.  Vertices are
 * grouped in levels (level l = vertices level_ptr[l] .. level_ptr[l+1]-1) and
 * every edge leads to a later level.  In topological order each vertex reached
 * from the inputs through drawn edges draws k of its d_v outgoing edges
 * uniformly with replacement (draw s of vertex v: the key of flat index
 * v k + s, edge floor(key d_v / 2^32)) and each draw counts (d_v / k) partial;
 * vertices no drawn edge leads to are skipped.  Back-propagation from y over
 * the drawn edges gives adjoint[v], an unbiased estimate of dy/dv (0 for
 * skipped vertices; 1 at y if y was reached); the gradient is adjoint[] at the
 * input vertices.  Nothing is stored per edge: the draws are made again on
 * the way back.  fp64. */
typedef struct {
  int32_t n_vertices, n_levels;
  int64_t n_edges;
  const int32_t* level_ptr; /* HOST [n_levels + 1], level_ptr[0] = 0, non-decreasing, last = n_vertices */
  const int32_t* succ_ptr;  /* DEVICE [n_vertices + 1] */
  const int32_t* succ;      /* DEVICE [n_edges] */
  const double* partial;    /* DEVICE [n_edges] */
} rad_graph;

/* inputs: DEVICE [n_inputs] vertex numbers; adjoint: DEVICE [n_vertices] out;
 * reached: DEVICE [n_vertices] out (1 where the vertex was visited).
 * 1 <= k <= 65536.  Synchronises; RAD_ERR_PARAM if the device arrays are
 * inconsistent (numbers out of range, an edge that does not lead to a later
 * level): outputs are then undefined, but no access leaves the arrays. */
rad_status rad_path_sample_gradient(rad_ctx* ctx, const rad_graph* graph, int32_t y, const int32_t* inputs,
                                    int32_t n_inputs, int32_t k, uint64_t seed, uint32_t stream_id,
                                    double* adjoint, uint32_t* reached);

#ifdef __cplusplus
}
#endif
#endif /* RAD_H_ */
