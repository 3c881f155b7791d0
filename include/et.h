/* et.h - C ABI of the elastic selective training step for one MI355X (gfx950).
 *
 * The library implements the hot path of ElasticTrainer: a training step in
 * which a runtime mask picks the trainable tensors (Section 2.2, Eq. 1/Eq. 3),
 * a per-tensor importance reduction (Eq. 2), a tensor timing profiler
 * (Section 5) and the tensor selector (Section 6).
 *
 * Conventions
 *   - Tensor index i = 0 .. N-1 runs in forward execution order (Section 5);
 *     i = 0 is the input-most tensor, i = N-1 the output-most one.
 *   - Every function returns an int status: 0 = ET_OK, negative = error,
 *     positive = informational.  Nothing throws; there is no global state.
 *   - "dev" pointers are device (HBM) addresses, "host" pointers ordinary host
 *     memory.  The library never allocates or frees device memory: weights,
 *     optimizer state, gradients and the workspace belong to the caller and are
 *     borrowed from et_bind() until et_destroy() or the next et_bind().
 *   - All device work is enqueued on the HIP stream given to et_create();
 *     only functions that return values to host memory wait for it.
 *   - Calls on one context must not overlap.
 */
#ifndef ET_H_
#define ET_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status codes */
#define ET_OK 0
#define ET_INFEASIBLE 1 /* the budget is below the forward time: empty mask returned */
#define ET_EINVAL (-1)  /* bad argument (null pointer, size, alignment, range)      */
#define ET_ENOMEM (-2)  /* host allocation failed or workspace too small            */
#define ET_EHIP (-3)    /* a HIP runtime call failed                                */
#define ET_ENAN (-4)    /* an importance value is NaN or infinite                   */
#define ET_ESTATE (-5)  /* call order: et_bind() has not been called                */

/* model kinds */
#define ET_MLP 0 /* ReLU multi-layer perceptron without biases                      */
#define ET_VIT 1 /* pre-LN vision transformer encoder on flattened patches          */
#define ET_RESNET 2 /* bottleneck residual CNN, BatchNorm folded into per-channel affines */
#define ET_VGG 3 /* plain 3x3 convolution stack with biases, 2x2 max pooling, linear layers   */
#define ET_MOBILENET 4 /* inverted residual blocks: 1x1 expansion, 3x3 depthwise, 1x1 projection   */

/* storage types of weights and activations */
#define ET_F32 0  /* float32 everywhere                                             */
#define ET_BF16 1 /* bf16 weights/activations, float32 accumulation and statistics  */

/* optimizers (Section 8: Adam for ViT, SGD with momentum and decoupled decay otherwise) */
#define ET_ADAM 0
#define ET_SGDW 1

#define ET_MAX_MLP_LAYERS 16
#define ET_MAX_STAGES 8

typedef struct et_ctx et_ctx;

/* Shape of the network.  Matrix weights are stored [out, in] row-major.
 * ET_MLP: dims[0..n_layers], x is [batch, dims[0]] float32; tensors fc0.W .. fc{n-1}.W.
 * ET_VIT: x is [batch, tokens-1, patch_dim]; the tensors are, in order,
 *   patch.W [width, patch_dim], patch.b, cls [width], pos [tokens, width], then per block
 *   ln1.g, ln1.b, qkv.W [3 width, width], qkv.b, proj.W, proj.b, ln2.g, ln2.b,
 *   fc1.W [mlp, width], fc1.b, fc2.W [width, mlp], fc2.b, then lnf.g, lnf.b,
 *   head.W [classes, width], head.b.  width, patch_dim, mlp, classes and the head size
 *   width/heads must be multiples of 8 (16-byte rows); tokens is arbitrary.
 * ET_RESNET: x is [batch, image, image, in_ch] (NHWC), convolution weights are [out, kh, kw, in],
 *   zero padding (k-1)/2.  Stem: 7x7/2 convolution to `stem` channels, affine, ReLU, 3x3/2 max
 *   pooling.  Stage i has stage_blocks[i] bottleneck blocks (1x1 to planes[i], 3x3 to planes[i],
 *   1x1 to 4 planes[i], an affine after each, ReLU after the first two and after the residual
 *   sum); the 3x3 of the first block of stages 1.. has stride 2; the first block of every stage
 *   has a 1x1 projection shortcut with the same stride.  Then global average pooling and a
 *   linear head.  Tensors in chain order (a branched network is unrolled by execution order,
 *   Section 5): stem.W, stem.g, stem.b; per block c1.W, c1.g, c1.b, c2.*, c3.*, then sc.W,
 *   sc.g, sc.b for a projection block; head.W [classes, 4 planes[last]], head.b.  stem, planes
 *   and classes must be multiples of 8.
 * ET_VGG: x and the convolution weights are laid out as for ET_RESNET.  Stage i is stage_blocks[i]
 *   3x3 / stride 1 / zero padding 1 convolutions to planes[i] channels, each followed by a bias and
 *   a ReLU, then a 2x2 / stride 2 max pooling (image must be divisible by 2^n_stages).  The pooled
 *   features, flattened in (h, w, c) order, pass through n_layers hidden linear layers of
 *   dims[0..n_layers-1] units (bias, ReLU) and a linear layer to `classes` logits.  Every layer is
 *   two tensors, Kernel and Bias (Section 5.1): conv{i}.W [out, 3, 3, in], conv{i}.b, ...,
 *   fc{j}.W [out, in], fc{j}.b.  planes, dims and classes must be multiples of 8.
 * ET_MOBILENET: x and the dense convolution weights as for ET_RESNET; depthwise weights [channels, 3, 3, 1];
 *   every convolution is followed by a per-channel affine (folded BatchNorm) and contributes three
 *   tensors W, g, b.  Stem: 3x3 / stride 2 convolution to `stem` channels, ReLU6.  Entry i of the
 *   settings is stage_blocks[i] blocks to planes[i] channels with expansion factor expand[i], the
 *   first of stride strides[i] (1 or 2): 1x1 expansion to expand[i] * c_in channels with ReLU6
 *   (absent when expand[i] = 1), 3x3 depthwise convolution with ReLU6, 1x1 projection without
 *   activation; a stride-1 block whose input has planes[i] channels adds its input to its output.
 *   Then a 1x1 convolution to `last` channels with ReLU6, global average pooling and a linear
 *   head.  Tensors in chain order: stem.W, stem.g, stem.b; per block [exp.W, exp.g, exp.b,] dw.W,
 *   dw.g, dw.b, proj.W, proj.g, proj.b; last.W, last.g, last.b; head.W [classes, last], head.b.
 *   All channel counts and classes must be multiples of 8.
 * Labels are int32 in [0, classes). The loss is the mean softmax cross-entropy.
 *
 * Storage contract of the ET_BF16 convolutional models (a property of the memory layout, whichever kernel
 * computes a layer): every tensor that one operation of the chain hands to the next is rounded once to bf16
 * (nearest, ties to even) -- each convolution output, each affine / activation output, pooled features, the
 * copy of the logit gradient that feeds the matrix products, and each error gradient between two backward
 * operations; sums are accumulated in float32 and rounded when the result is stored.  Two exceptions:
 * the ET_RESNET stem keeps its convolution output in float32 (the max-pooling argmax is decided on unrounded
 * values), and the column gradient d * W of a convolution with a kernel larger than 1x1 is never a stored
 * tensor: the input gradient, the sum of its shifted copies, is rounded once after the sum.  For a 1x1
 * convolution that product is the input gradient itself and is rounded like any other result.
 * Weight gradients are float32. */
typedef struct {
  int32_t kind;  /* ET_MLP | ET_VIT | ET_RESNET | ET_VGG | ET_MOBILENET */
  int32_t dtype; /* ET_F32 (MLP) | ET_BF16 (all others) */
  int32_t batch;
  int32_t n_layers;                    /* ET_MLP, ET_VGG */
  int32_t dims[ET_MAX_MLP_LAYERS + 1]; /* ET_MLP, ET_VGG */
  int32_t tokens, patch_dim, width, heads, mlp, blocks, classes; /* ET_VIT */
  float ln_eps;                        /* ET_VIT */
  int32_t image, in_ch, stem, n_stages;               /* ET_RESNET, ET_VGG, ET_MOBILENET (classes as above; stem: not ET_VGG) */
  int32_t stage_blocks[ET_MAX_STAGES], planes[ET_MAX_STAGES]; /* ET_RESNET, ET_VGG, ET_MOBILENET */
  int32_t expand[ET_MAX_STAGES], strides[ET_MAX_STAGES], last;  /* ET_MOBILENET */
} et_model_desc;

/* Optimizer hyper-parameters of one step; every constant is explicit.
 *   ET_ADAM: m = b1 m + (1-b1) g; v = b2 v + (1-b2) g^2;
 *            w -= lr (m / (1-b1^step)) / (sqrt(v / (1-b2^step)) + eps); step >= 1 is the global step.
 *   ET_SGDW: m = momentum m + g; w -= lr m + lr wd w.
 * State of a tensor that is not selected is left untouched (frozen). */
typedef struct {
  int32_t kind; /* ET_ADAM | ET_SGDW */
  float lr, beta1, beta2, eps, momentum, wd;
  uint64_t step;
} et_opt;

/* Build the static operation chain of the model.  `hip_stream` is a hipStream_t (NULL = the
 * default stream).  Allocates host memory only. */
int et_create(const et_model_desc* desc, void* hip_stream, et_ctx** out);
int et_destroy(et_ctx* ctx);

/* Number of trainable tensors N, and per tensor its element count, storage type and name
 * (the string lives as long as the context). */
int et_num_tensors(const et_ctx* ctx, int32_t* n);
int et_tensor_info(const et_ctx* ctx, int32_t i, size_t* numel, int32_t* dtype, const char** name);

/* Bytes of device workspace the context needs (activations kept for the backward pass,
 * gradient streams, reduction partials). */
size_t et_workspace_bytes(const et_ctx* ctx);

/* Number of optimizer-state buffers per tensor expected by et_bind():
 *   ET_BF16 models: 3 = { float32 master weights, m, v }  (ET_SGDW uses the first two)
 *   ET_F32  models: 2 = { m, v }                          (ET_SGDW uses the first)     */
int et_state_slots(const et_ctx* ctx, int32_t* k);

/* Lend the device buffers.  w_dev[i]: weights of tensor i in the model's storage type;
 * grad_dev[i]: float32 [numel_i]; opt_state_dev[i*k + s]: float32 [numel_i] (k from
 * et_state_slots; may be NULL as a whole if et_train_step is only called with opt == NULL);
 * workspace_dev: at least et_workspace_bytes() bytes, 256-byte aligned.  The arrays of
 * pointers are host arrays and are copied.  The workspace is cleared on the stream. */
int et_bind(et_ctx* ctx, void* const* w_dev, void* const* opt_state_dev, void* const* grad_dev,
            void* workspace_dev, size_t workspace_bytes);

/* Tensor Timing Profiler (Section 5).  Runs `warmup` untimed and `reps` timed full training
 * iterations (all tensors selected, no optimizer update of the weights), timing every kernel
 * in place with HIP events, takes the median per kernel and attributes the times to tensors:
 *   t_dw_ns[i]: computing tensor i's gradient plus its optimizer update (Section 5.1: T3, T2);
 *   t_dy_ns[i]: passing the error gradient through tensor i towards tensor i-1 (T1); biases
 *               and LayerNorm shifts have 0 (Section 5.1 footnote); backward kernels of
 *               operations without weights (ReLU/GELU, attention core, residual additions)
 *               are charged to the tensor that must be passed for them to run (Section 5.3);
 *               a LayerNorm's input-gradient kernel is charged to its gain (Section 5.2);
 *   t_fwd_ns:   the whole forward pass including the loss and its gradient.
 * Every timed iteration is followed by the same iteration without events, timed as a whole; the
 * excess of the instrumented one is the measurement's own overhead and is taken off the regions
 * in equal parts (at most half of a region's own time).
 * Host outputs; waits for the stream. */
int et_profile(et_ctx* ctx, const void* x_dev, const int32_t* y_dev, int32_t warmup, int32_t reps,
               uint64_t* t_fwd_ns, uint64_t* t_dw_ns /*[N]*/, uint64_t* t_dy_ns /*[N]*/);

/* Tensor Importance Evaluator (Eq. 2, with the gradient at the current weights, Eq. 5 at c=0):
 * one full backward pass on (x, y) without update, then
 *   importance[i] = sum_e grad_i[e] * (w_snapshot_i[e] - w_i[e])
 * for every tensor in one segmented reduction (a launch over all chunks of all tensors, then a tiny launch
 * that adds each tensor's chunk sums in a fixed order).  w_snapshot_dev[i] has the model's storage type
 * and tensor i's size: the weights that undoing the recent update would restore.  Leaves
 * the gradients of all tensors in grad_dev.  Host output; waits for the stream. */
int et_importance(et_ctx* ctx, const void* x_dev, const int32_t* y_dev, void* const* w_snapshot_dev /*[N]*/,
                  double* importance_host /*[N]*/);

/* The same evaluation with full-precision weight updates, for ET_BF16 models: delta w is taken
 * between float32 snapshots and the float32 master weights (optimizer state slot 0) instead of
 * the bf16 copies, whose rounding step is of the size of a few low-learning-rate updates
 * (Section 4 assumes updates proportional to a learning rate of 1e-4..1e-5).
 * w_snapshot_f32_dev[i]: float32 [numel_i], a copy of the master weights taken earlier.
 * Needs optimizer state bound; ET_ESTATE otherwise, ET_EINVAL for ET_F32 models (use
 * et_importance there). */
int et_importance_master(et_ctx* ctx, const void* x_dev, const int32_t* y_dev, void* const* w_snapshot_f32_dev /*[N]*/,
                         double* importance_host /*[N]*/);

/* The two importance metrics the ablation of Section 8 compares Eq. 2 with, evaluated per tensor by the
 * same single segmented reduction (the paper names them only; the reading here is the L1 norm):
 *   ET_METRIC_WEIGHT_L1: sum |w_i| over the tensor's current weights (x_dev, y_dev may be NULL);
 *   ET_METRIC_GRAD_L1:   sum |dL/dw_i| after one full backward pass on the given batch.
 * Neither is additive in the sense of Section 4; their values feed et_select like importances.
 * metric_host: N doubles.  Synchronises the stream. */
#define ET_METRIC_WEIGHT_L1 1
#define ET_METRIC_GRAD_L1 2
int et_tensor_metric(et_ctx* ctx, const void* x_dev, const int32_t* y_dev, int32_t metric, double* metric_host /*[N]*/);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the reduction of et_importance on its own,
 *   importance_dev[i] = sum_e grad_dev[i][e] * (w_snapshot_dev[i][e] - w_dev[i][e]),   i = 0 .. n-1,
 * with the same kernels, chunking and summation order (bit-identical to et_importance on the same gradients),
 * but with the chunk table and the partial sums in a fixed device array inside the library instead of a
 * caller's workspace.  It allocates nothing, on the device or through the HIP runtime, copies nothing from host
 * memory and does not wait: a few kernel launches on `hip_stream` (NULL = the default stream).
 *   grad_dev[i]: float32 [numel[i]]; w_dev[i], w_snapshot_dev[i]: `dtype` (ET_F32 | ET_BF16) [numel[i]]; the three
 *   arrays of pointers and numel are host arrays, read before the call returns; importance_dev: n doubles in
 *   device memory, written on the stream.  16-byte aligned tensors take the vector path.
 * Limits: n <= ET_STATIC_MAX_TENSORS and sum_i ceil(numel[i] / 16384) <= ET_STATIC_MAX_CHUNKS (about 1e9
 * elements), else ET_ENOMEM and nothing is launched; the array takes 2.6 MB on every GPU the library runs on,
 * until the process ends.  All calls on one GPU share that GPU's array, which keeps the last call's contents
 * (no entry has to start at zero): calls that overlap on one GPU race. */
#define ET_STATIC_MAX_TENSORS 1024
#define ET_STATIC_MAX_CHUNKS 65536
int et_importance_reduce_static(int32_t n, void* const* grad_dev, void* const* w_dev, void* const* w_snapshot_dev,
                                const uint64_t* numel, int32_t dtype, void* hip_stream, double* importance_dev);

/* Tensor Selector (Eq. 3 solved exactly on integers; Sections 3.3 and 6).  Pure host code,
 * no context, no device.  Maximises the summed importance of the selected tensors subject to
 *   t_fwd + sum_{i selected} t_dw[i] + sum_{i > i*} t_dy[i] <= rho * T_full,
 * i* being the smallest selected index and T_full the same expression for all tensors
 * selected (Section 2.2: the worked example and Eq. 7 leave out t_dy of i* itself).
 *   rho_ppm: the speed-up objective rho in parts per million (500000 = 50 %);
 *   tq:      time resolution T_q of Eq. 8: if 0 < tq < T_b (T_b = full backward time) every
 *            time becomes floor(t * tq / T_b); tq = 0 keeps nanoseconds;
 *   budget:  floor(rho_ppm * T_full / 1e6) - t_fwd; negative: ET_INFEASIBLE and an empty mask;
 *   importance is quantised to integers rint(I * 2^(40-e)), 2^(e-1) <= max|I| < 2^e;
 *   ties:    larger summed importance first; among equals the mask that is smallest when
 *            read as a binary number with tensor 0 as the most significant bit.
 * mask_out[i] = 1 if tensor i is selected.  predicted_ns (nullable) = the unquantised
 * time-model value of the returned mask. */
int et_select(int32_t n, const double* importance, const uint64_t* t_dw_ns, const uint64_t* t_dy_ns,
              uint64_t t_fwd_ns, uint32_t rho_ppm, uint32_t tq, uint8_t* mask_out /*[N]*/,
              uint64_t* predicted_ns);

/* The same selection, plus the sizes of the dynamic-programming tables on the quantised times
 * (Section 6.3, Figure 10: how much of the table the pruning of invalid and redundant cells
 * leaves).  With depth d = 1..N counted from the output and T the quantised time axis:
 *   backward_q:     quantised full backward time, budget_q: quantised budget;
 *   cells_table:    N * (max(backward_q, budget_q) + 1), the paper's table without pruning;
 *   cells_pruned:   sum over depths that fit the budget of (budget_q - reach_d + 1): cells that are
 *                   neither invalid (t above the budget) nor redundant (t below the time reach_d of
 *                   merely passing the gradient down to depth d);
 *   cells_knapsack: N * (budget_q + 1), the table this library fills (one 0/1-knapsack row per
 *                   depth serves every choice of the input-most selected tensor).
 * counts must not be NULL; it is zeroed when the call returns ET_INFEASIBLE or an error. */
typedef struct {
  uint64_t backward_q, budget_q, cells_table, cells_pruned, cells_knapsack;
} et_select_counts;
int et_select_stats(int32_t n, const double* importance, const uint64_t* t_dw_ns, const uint64_t* t_dy_ns,
                    uint64_t t_fwd_ns, uint32_t rho_ppm, uint32_t tq, uint8_t* mask_out /*[n]*/,
                    uint64_t* predicted_ns, et_select_counts* counts);

/* One elastic selective training iteration (Section 2.2): forward pass and loss; then, from
 * the output backwards, the weight gradient of every selected tensor and the error-gradient
 * passing down to (not through) the input-most selected tensor; then the optimizer update of
 * the selected tensors only.  mask_host[i] != 0 selects tensor i; it steers which kernels are
 * launched.  An empty mask launches no backward kernel.  grad_dev[i] of an unselected tensor
 * is not written; its weights and optimizer state keep their bytes.  opt == NULL skips the
 * update (gradients only).  loss_host == NULL makes the call fully asynchronous; otherwise it
 * waits for the stream and stores the loss. */
int et_train_step(et_ctx* ctx, const void* x_dev, const int32_t* y_dev, const uint8_t* mask_host /*[N]*/,
                  const et_opt* opt, float* loss_host);

/* Counters of the last et_train_step/et_importance call on this context: kernels launched in
 * the forward pass, in the backward pass and in the optimizer update. */
int et_last_launch_counts(const et_ctx* ctx, int32_t* forward, int32_t* backward, int32_t* update);

/* Measurement support.  While enabled, every launch of a kernel class below is bracketed by a
 * pair of HIP events on the context's stream, so that a benchmark can report the average
 * duration of a kernel inside real training steps.  Classes:
 *   0 forward GEMM (X W^T), 1 gradient-passing GEMM (dY W), 2 weight-gradient GEMM (dY^T X,
 *   including its split-K reduction), 3 importance reduction, 4 masked optimizer update,
 *   5 fused attention forward, 6 fused attention backward, 7 the data-movement kernels of the
 *   convolutional workload (im2col and its adjoint, affine, pooling, per-channel reductions).
 * et_kernel_timing_read waits for the stream and returns, for one class, the number of timed
 * launches since timing was enabled, their summed duration, and their summed algorithmic work
 * (floating-point operations for classes 0-2 and 5-6, bytes read plus written for classes 3-4, 7).
 * Enabling clears the records.  Outputs are host pointers and may be NULL.
 * An event pair measures more than the kernel between its events: the hand-over from one command to the next
 * is inside it too.  Enabling therefore also records 33 pairs with nothing between them on the same stream;
 * et_kernel_timing_overhead returns their median elapsed time (about 5 us on this hardware), which a caller may
 * take off every timed launch (summed durations are returned as measured). */
#define ET_NUM_KERNEL_CLASSES 8
int et_kernel_timing(et_ctx* ctx, int32_t enable);
int et_kernel_timing_read(et_ctx* ctx, int32_t kernel_class, uint64_t* launches, double* total_ns, double* work);
int et_kernel_timing_overhead(et_ctx* ctx, double* ns_per_pair);

/* Text of the HIP error behind the last ET_EHIP returned on this context ("no error" if none). */
const char* et_last_hip_error(const et_ctx* ctx);

/* Human-readable text for a status code. */
const char* et_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* ET_H_ */
