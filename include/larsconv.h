/*
 * larsconv -- one worker's share of large-batch LARS training on one MI355X (gfx950):
 * convolution forward, backward-data, backward-weight, and the layer-wise LARS update.
 *
 * The operations are those of the synchronous data-parallel iteration described in
 * "Data-Parallelism SGD" (every worker computes its local gradient independently) with the
 * optimizer named in "Scaling up Batch Size" (LARS, momentum, weight decay, poly schedule of
 * power 2 -- hyper-parameters in the caption of the AlexNet accuracy table).  The gradient
 * sum across workers that sits between the two is not part of this library.
 *
 * Conventions for every entry point
 *  - Tensor pointers are DEVICE pointers owned by the caller unless a parameter says HOST.
 *    The library never allocates, frees or keeps them.  Outputs are overwritten, inputs are
 *    not modified (lars_step updates w and v in place).
 *  - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = the default
 *    stream) and the call returns without waiting for it.  Calls on one stream are ordered.
 *  - `workspace` is caller-owned device scratch of at least the size the matching *_workspace_bytes
 *    query returns (256-byte aligned); its contents are undefined between calls.
 *  - Arguments are validated before anything is launched; errors come back as lc_status, never
 *    as exceptions or aborts, and a failing call launches nothing.
 *  - Kernels exist for gfx950 only.
 */
#ifndef LARSCONV_H
#define LARSCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LC_OK = 0,
    LC_ERR_NULL = 1,        /* a required pointer is NULL                                  */
    LC_ERR_SHAPE = 2,       /* non-positive size, empty output, negative pad, bad count     */
    LC_ERR_UNSUPPORTED = 3, /* unknown enum value or a combination that is not built        */
    LC_ERR_WORKSPACE = 4,   /* workspace NULL, misaligned or smaller than the query         */
    LC_ERR_LAUNCH = 5,      /* the HIP runtime reported an error while enqueueing           */
    LC_ERR_ALIGN = 6        /* a tensor pointer is not aligned: 4 bytes for fp32 tensors,
                               16 bytes for bf16 tensors (they are read in 16-byte vectors) */
} lc_status;

typedef enum { LC_F32 = 0, LC_BF16 = 1 } lc_dtype;   /* operand type; sums are always fp32 */
typedef enum { LC_NCHW = 0, LC_NHWC = 1 } lc_layout; /* filter is KCRS for NCHW, KRSC for NHWC */
typedef enum { LC_PASS_FWD = 0, LC_PASS_BWD_DATA = 1, LC_PASS_BWD_WEIGHT = 2 } lc_pass;

/* One convolution layer: input X[n,c,h,w], filter W[k,c,r,s], output Y[n,k,p,q] with
 * p = floor((h + 2*pad_h - r)/stride_h) + 1 (q likewise).  Cross-correlation (no filter flip),
 * zero padding, dilation 1, no bias -- the convolution of the Caffe-style layers the
 * paper's networks are made of ("Experimental Settings").  NHWC is the layout the matrix cores
 * are fed from; NCHW tensors are accepted and transposed through the workspace.
 * groups > 1: the c input channels and the k filters are cut into `groups` equal slices and filter j sees only the
 * input channels of slice j / (k/groups), so the filter (and dw) is W[k, c/groups, r, s] -- the form of the original
 * AlexNet whose 61 million parameters and 1.5 billion operations the paper's Table "Scaling Ratio for AlexNet and
 * ResNet50" lists.  c and k stay the TOTAL channel counts and must be multiples of groups; 0 means 1.  Each group
 * runs as a convolution of its own on channel slices copied through the workspace. */
typedef struct {
    int n, c, h, w;
    int k, r, s;
    int stride_h, stride_w, pad_h, pad_w;
    lc_dtype dtype;   /* type of x, w, y, dy, dx.  dw is always fp32. */
    lc_layout layout;
    int groups;       /* 0 or 1: every filter sees every input channel */
} lc_conv_desc;

/* Output height p and width q.  HOST pointers.  LC_ERR_SHAPE if the window does not fit. */
lc_status conv2d_out_shape(const lc_conv_desc* desc, int* p, int* q);

/* Scratch bytes conv2d_{fwd,bwd_data,bwd_weight} needs for `desc` (0 is possible).  Returns 0 for an
 * invalid descriptor; the call itself then reports the error.  Usually a few MB (partial tiles, split sums);
 * it holds whole tensors where the library re-lays its operands: NCHW calls (NHWC copies of all three tensors),
 * channel counts that are not a multiple of 4 (8 for bf16; a padded copy of x), and the bf16 forward and
 * backward-weight passes of a stride-2 layer with at most 4 channels (x unfolded over 2x2 pixel blocks, about
 * 5.5 times its size: 0.84 GB for 512 x 224 x 224 x 3), and grouped layers (one group's slices of x and y). */
size_t conv2d_workspace_bytes(const lc_conv_desc* desc, lc_pass pass);

/* Forward pass: the per-image work the paper counts in flops ("Benefits of Large-Batch Training",
 * "Model Selection").   y[n,k,p,q] = sum_{c,r,s} x[n,c,p*stride_h-pad_h+r, q*stride_w-pad_w+s] * w[k,c,r,s],
 * reads outside the image being zero.  x: n*c*h*w, w: k*(c/groups)*r*s, y: n*k*p*q elements of desc->dtype. */
lc_status conv2d_fwd(const lc_conv_desc* desc, const void* x, const void* w, void* y,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

/* Gradient with respect to the input (back-propagation through the layer; part of the local
 * gradient computation of "Data-Parallelism SGD").  dx[n,c,h,w] = sum over all (k,p,q,r,s) whose
 * forward read touched (h,w) of dy[n,k,p,q] * w[k,c,r,s].  dx is written in full, zeros included. */
lc_status conv2d_bwd_data(const lc_conv_desc* desc, const void* dy, const void* w, void* dx,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* Gradient with respect to the filter: the worker's local gradient that the data-parallel scheme sums
 * over workers.  dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * x[n,c,p*stride_h-pad_h+r, q*stride_w-pad_w+s].
 * dw is fp32 for every operand dtype and is overwritten.  The reduction is split over the batch and
 * summed in a fixed order: results are bit-identical from run to run. */
lc_status conv2d_bwd_weight(const lc_conv_desc* desc, const void* x, const void* dy, float* dw,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/* conv2d_bwd_weight that also hands over the squared Euclidean norm of the gradient it wrote, the quantity the
 * layer-wise rule of "Scaling up Batch Size" needs of every gradient tensor: dw_sq_pieces (DEVICE, 8-byte aligned)
 * receives conv2d_bwd_weight_sq_count(desc) doubles whose sum, taken in index order, is sum dw^2.  Where the pass ends
 * in the fixed-order sum of its batch splits (every larger layer) the pieces come out of that kernel at no extra
 * memory traffic; otherwise one more small kernel reads dw.  Everything else as conv2d_bwd_weight; the pieces are
 * bit-identical from run to run.  conv2d_bwd_weight_sq_count returns 0 for an invalid descriptor. */
size_t conv2d_bwd_weight_sq_count(const lc_conv_desc* desc);
lc_status conv2d_bwd_weight_sq(const lc_conv_desc* desc, const void* x, const void* dy, float* dw, double* dw_sq_pieces,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/* Scratch bytes lars_step needs for this list of tensor sizes (HOST array).  0 on invalid input. */
size_t lars_workspace_bytes(int n_tensors, const int64_t* numel);

/* One LARS step over a list of parameter tensors, each its own "layer" ("Scaling up Batch Size":
 * LARS with warmup; momentum and weight decay as in the AlexNet accuracy table).  For tensor l:
 *     trust_l = eta * ||w_l|| / (||g_l|| + weight_decay * ||w_l||)     (Euclidean norms; 1 if undefined)
 *     v_l <- momentum * v_l + lr * trust_l * (g_l + weight_decay * w_l)
 *     w_l <- w_l - v_l
 * w, g, v: HOST arrays of n_tensors DEVICE pointers to fp32 data (4-byte aligned; 16-byte alignment
 * takes the vector path); numel: HOST array of element counts (0 allowed).  w and v are updated in
 * place, g is read only; the three must not overlap.  trust_out: DEVICE, n_tensors floats, or NULL.
 * w_lowp_out: HOST array of DEVICE pointers receiving the new weights rounded to bf16 (nearest even),
 * or NULL; single entries may be NULL.  n_tensors = 0 is a no-op.  Norms are reduced in a fixed
 * order: results are bit-identical from run to run and independent of the other tensors in the list.
 * The pointer and size arrays are read during the call and travel to the kernels as launch arguments: a HIP graph
 * that captured the call replays with the pointers of the capture, so a changed list means capturing again. */
lc_status lars_step(int n_tensors, float* const* w, const float* const* g, float* const* v,
                    const int64_t* numel, float eta, float momentum, float weight_decay, float lr,
                    float* trust_out, void* const* w_lowp_out,
                    void* workspace, size_t workspace_bytes, void* hip_stream);

/* lars_step with per-tensor coefficients.  The paper applies the rule layer by layer ("Scaling up Batch
 * Size") and leaves open which tensors take part and with which coefficients; biases and batch-norm
 * parameters are commonly given no layer-wise scaling.  eta_per_tensor, weight_decay_per_tensor: HOST arrays
 * of n_tensors floats replacing the scalars, or NULL (the scalar for every tensor).  skip: HOST array of
 * n_tensors bytes or NULL; a tensor with a non-zero entry takes trust ratio 1, i.e. the plain momentum step
 * v <- momentum*v + lr*(g + weight_decay*w) with its weight decay, and trust_out reports 1 for it.
 * Everything else as lars_step, which is this call with the three arrays NULL. */
lc_status lars_step_ex(int n_tensors, float* const* w, const float* const* g, float* const* v,
                       const int64_t* numel, float eta, float momentum, float weight_decay, float lr,
                       const float* eta_per_tensor, const float* weight_decay_per_tensor, const uint8_t* skip,
                       float* trust_out, void* const* w_lowp_out,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* lars_step_ex that takes sum g^2 of some tensors from where their gradients were written (conv2d_bwd_weight_sq), so
 * that the norm pass does not read those gradients again: 24 instead of 28 bytes per parameter of such tensors.
 * g_sq_pieces: HOST array of n_tensors DEVICE pointers (8-byte aligned), g_sq_counts: HOST array of n_tensors counts;
 * for tensor l with a non-null pointer and a positive count, ||g_l||^2 is the sum of those doubles in index order and
 * g_l is only read by the update pass; for the others (null / 0) the norm is computed here as in lars_step_ex.  Both
 * arrays NULL: lars_step_ex.  The pieces must describe the g_l passed in the same call.  Trust ratios agree with
 * lars_step_ex to rounding (the sums are taken in a different order, both in double). */
lc_status lars_step_pre(int n_tensors, float* const* w, const float* const* g, float* const* v,
                        const int64_t* numel, float eta, float momentum, float weight_decay, float lr,
                        const float* eta_per_tensor, const float* weight_decay_per_tensor, const uint8_t* skip,
                        const double* const* g_sq_pieces, const int64_t* g_sq_counts,
                        float* trust_out, void* const* w_lowp_out,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/* lars_step_ex for callers that cannot allocate device memory or have none to pass: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and errors as lars_step_ex without
 * the workspace: the scratch memory is a fixed array of LARS_STATIC_SCRATCH_BYTES inside the library's device image
 * (each GPU the library runs on holds one copy until the process ends), and the call allocates and frees nothing.
 * A list whose lars_workspace_bytes() exceeds LARS_STATIC_SCRATCH_BYTES is refused with LC_ERR_WORKSPACE before
 * anything is launched (2 MiB holds about 420 M parameters; ResNet-50's list needs 0.14 MB, AlexNet-BN's 0.31 MB).
 * Every call on a GPU uses that GPU's one array: calls on the same GPU must be ordered (one stream, or events
 * between streams); calls that overlap on one GPU race on the scratch memory and give undefined results.  The
 * array keeps the last call's contents; nothing in it needs clearing, every value read is written first by the
 * same call.  The device is the calling thread's current device. */
#define LARS_STATIC_SCRATCH_BYTES ((size_t)2 << 20)
lc_status lars_step_ex_static(int n_tensors, float* const* w, const float* const* g, float* const* v,
                              const int64_t* numel, float eta, float momentum, float weight_decay, float lr,
                              const float* eta_per_tensor, const float* weight_decay_per_tensor, const uint8_t* skip,
                              float* trust_out, void* const* w_lowp_out, void* hip_stream);

/* Warm-up followed by the poly policy (HOST arithmetic).  The paper's warm-up scheme starts from a small rate
 * and raises it to the large one over the first few epochs ("Difficulty of Large-Batch Training"; 5 epochs
 * for ResNet-50); the ramp is taken to be linear: start_lr + (base_lr - start_lr) * iter / warmup_iters for
 * iter < warmup_iters, then base_lr * (1 - (iter - warmup_iters)/(max_iter - warmup_iters))^power.
 * warmup_iters <= 0 gives lars_poly_lr. */
float lars_warmup_poly_lr(float base_lr, float start_lr, int64_t iter, int64_t warmup_iters, int64_t max_iter, float power);

/* Poly learning-rate policy (HOST arithmetic): base_lr * (1 - iter/max_iter)^power, 0 past max_iter.
 * The paper trains with power 2; max_iter = epochs * images / batch ("Scaling Efficiency of Large
 * Batches").  The result is the `lr` argument of lars_step. */
float lars_poly_lr(float base_lr, int64_t iter, int64_t max_iter, float power);

/* ---- Glue layers of the networks the paper trains (fp32) ----
 * ReLU, max pooling, global average pooling, bias, softmax cross-entropy and the gradient at a residual
 * block's output: the paper does not discuss them (they are implied by the networks it trains, "Experimental
 * Settings"; ResNet-50 in "ImageNet training with ResNet-50"); these are the textbook definitions, memory-bound
 * streaming kernels.  All pointers DEVICE, fp32, 4-byte aligned; reductions run in a fixed order. */

/* y = max(x, 0);  dx = x > 0 ? dy : 0 (x is the forward INPUT).  count elements; the buffers must not overlap. */
lc_status relu_fwd(const float* x, float* y, size_t count, void* hip_stream);
lc_status relu_bwd(const float* x, const float* dy, float* dx, size_t count, void* hip_stream);

/* 2x2 window, stride 2, h and w even.  x: [n,c,h,w] in `layout`, y: [n,c,h/2,w/2]; idx (one byte per
 * output element, same order as y) receives the position 0..3, row-major in the window, of the first
 * maximum; the backward pass sends dy there and zeros to the rest of the window (dx written in full). */
lc_status maxpool2x2_fwd(const float* x, float* y, uint8_t* idx, int n, int c, int h, int w, lc_layout layout, void* hip_stream);
lc_status maxpool2x2_bwd(const float* dy, const uint8_t* idx, float* dx, int n, int c, int h, int w, lc_layout layout,
                         void* hip_stream);

/* Max pool with a window x window window (1..15), any stride >= 1 and 0 <= pad < window (the overlapping 3x3
 * stride-2 pools of ResNet-50 and AlexNet); output size floor((h + 2*pad - window)/stride) + 1.  Padding taps
 * never win.  idx (one byte per output element, same order as y) receives the tap, row * window + column, of
 * the first maximum in row-major window order; the backward pass gives every input element the sum of dy over
 * the outputs whose maximum it was (fixed order, no atomics; dx written in full, h and w are the INPUT's). */
lc_status maxpool_fwd(const float* x, float* y, uint8_t* idx, int n, int c, int h, int w, int window, int stride, int pad,
                      lc_layout layout, void* hip_stream);
lc_status maxpool_bwd(const float* dy, const uint8_t* idx, float* dx, int n, int c, int h, int w, int window, int stride, int pad,
                      lc_layout layout, void* hip_stream);

/* dx = y > 0 ? da + db : 0 over count elements: the gradients that meet at a residual block's output y =
 * max(branch + shortcut, 0) -- one from the next block's first convolution, one from its shortcut -- taken
 * through the block's ReLU in one pass.  db may be NULL (dx = y > 0 ? da : 0); y may be NULL when db is not
 * (dx = da + db, no ReLU at that point).  Buffers must not overlap. */
lc_status relu_add_bwd(const float* y, const float* da, const float* db, float* dx, size_t count, void* hip_stream);

/* y[n,c] = mean over h, w of x[n,c,h,w];  dx[n,c,h,w] = dy[n,c] / (h*w). */
lc_status global_avgpool_fwd(const float* x, float* y, int n, int c, int h, int w, lc_layout layout, void* hip_stream);
lc_status global_avgpool_bwd(const float* dy, float* dx, int n, int c, int h, int w, lc_layout layout, void* hip_stream);

/* y[r][j] += b[j] for rows x k values in place;  db[j] = sum over rows of dy[r][j]. */
lc_status bias_add(float* y, const float* b, size_t rows, int k, void* hip_stream);
lc_status bias_grad(const float* dy, float* db, size_t rows, int k, void* hip_stream);

/* Mean softmax cross-entropy of logits [n][k] against labels (n int32 values in [0, k)) -> loss (one float),
 * and its gradient (softmax - onehot) / n -> dlogits [n][k].  row_scratch: n floats of device scratch. */
lc_status softmax_xent(const float* logits, const int32_t* labels, float* loss, float* dlogits, float* row_scratch, int n, int k,
                       void* hip_stream);

/* ---- Batch normalisation, training mode (fp32) ----
 * The paper adds batch normalisation after each convolution of AlexNet ("Scaling up Batch Size") and trains
 * ResNet-50, which has it throughout; this is the textbook layer with batch statistics: per channel c over the
 * m = n*h*w values of the batch, mean and biased variance, xhat = (x - mean)/sqrt(var + eps),
 * y = gamma[c]*xhat + beta[c].  save_mean, save_invstd (c floats each) receive mean and 1/sqrt(var + eps) for
 * the backward pass.  Backward: dbeta[c] = sum dy, dgamma[c] = sum dy*xhat,
 * dx = gamma[c]*invstd*(dy - dbeta[c]/m - xhat*dgamma[c]/m).  No running averages.
 * x, y, dy, dx: [n,c,h,w] in `layout`, fp32, 4-byte aligned (16-byte alignment with c a multiple of 4 takes the
 * vector path); per-channel arrays fp32 DEVICE.  Sums run in a fixed order (bit-identical reruns). */
size_t batchnorm_workspace_bytes(int n, int c, int h, int w, lc_layout layout);
lc_status batchnorm_fwd(const float* x, const float* gamma, const float* beta, float* y, float* save_mean, float* save_invstd,
                        int n, int c, int h, int w, float eps, lc_layout layout, void* workspace, size_t workspace_bytes,
                        void* hip_stream);
lc_status batchnorm_bwd(const float* x, const float* dy, const float* gamma, const float* save_mean, const float* save_invstd,
                        float* dx, float* dgamma, float* dbeta, int n, int c, int h, int w, lc_layout layout, void* workspace,
                        size_t workspace_bytes, void* hip_stream);

/* Fused forms for a network step (same statistics and sums as above).
 * Forward: y = act(gamma*xhat + beta + residual); residual ([n,c,h,w] like x) may be NULL; relu != 0 clamps at
 * zero.  Backward with relu != 0: dy is the gradient with respect to max(gamma*xhat + beta, 0) and is taken as
 * zero where gamma*xhat + beta <= 0; the layer rebuilds that value from x (beta is then required, and the
 * forward pass must have had no residual) with the arithmetic of the forward pass, so the mask is the one of
 * the stored output.  relu == 0: beta may be NULL and the call is batchnorm_bwd.  Buffers must not overlap. */
lc_status batchnorm_fwd_ex(const float* x, const float* gamma, const float* beta, const float* residual, float* y,
                           float* save_mean, float* save_invstd, int n, int c, int h, int w, float eps, int relu, lc_layout layout,
                           void* workspace, size_t workspace_bytes, void* hip_stream);
lc_status batchnorm_bwd_ex(const float* x, const float* dy, const float* gamma, const float* beta, const float* save_mean,
                           const float* save_invstd, float* dx, float* dgamma, float* dbeta, int n, int c, int h, int w, int relu,
                           lc_layout layout, void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---- The same layers on bf16 activations: the rest of a mixed-precision step ----
 * The paper's fastest ResNet-50 runs train in reduced precision with fp32 master weights ("State-of-the-art
 * results"); with LC_BF16 convolutions the activations between them are bf16, and these calls take them as they
 * are.  `dtype` is the storage type of every `void*` tensor argument: LC_F32 is exactly the call of the same name
 * without `_t`; LC_BF16 means bf16 bit patterns in NHWC with c (count for relu_add_bwd_t) a multiple of 8 and
 * 16-byte aligned tensors (idx 8-byte aligned) -- anything else is LC_ERR_UNSUPPORTED / LC_ERR_ALIGN.
 * All arithmetic is fp32 on the widened values, with the operation order of the fp32 kernels; a result stored as
 * bf16 is rounded once, to nearest even.  gamma, beta, statistics, dgamma, dbeta stay fp32; the statistics are
 * those of the bf16 values of x.  global_avgpool_fwd_t gives fp32 means and global_avgpool_bwd_t takes an fp32
 * dy (the classifier behind it runs in fp32).  Workspace: batchnorm_workspace_bytes, for either type. */
lc_status batchnorm_fwd_t(lc_dtype dtype, const void* x, const float* gamma, const float* beta, const void* residual, void* y,
                          float* save_mean, float* save_invstd, int n, int c, int h, int w, float eps, int relu, lc_layout layout,
                          void* workspace, size_t workspace_bytes, void* hip_stream);
lc_status batchnorm_bwd_t(lc_dtype dtype, const void* x, const void* dy, const float* gamma, const float* beta, const float* save_mean,
                          const float* save_invstd, void* dx, float* dgamma, float* dbeta, int n, int c, int h, int w, int relu,
                          lc_layout layout, void* workspace, size_t workspace_bytes, void* hip_stream);
lc_status maxpool_fwd_t(lc_dtype dtype, const void* x, void* y, uint8_t* idx, int n, int c, int h, int w, int window, int stride,
                        int pad, lc_layout layout, void* hip_stream);
lc_status maxpool_bwd_t(lc_dtype dtype, const void* dy, const uint8_t* idx, void* dx, int n, int c, int h, int w, int window,
                        int stride, int pad, lc_layout layout, void* hip_stream);
lc_status relu_add_bwd_t(lc_dtype dtype, const void* y, const void* da, const void* db, void* dx, size_t count, void* hip_stream);
lc_status global_avgpool_fwd_t(lc_dtype dtype, const void* x, float* y, int n, int c, int h, int w, lc_layout layout, void* hip_stream);
lc_status global_avgpool_bwd_t(lc_dtype dtype, const float* dy, void* dx, int n, int c, int h, int w, lc_layout layout, void* hip_stream);

/* The gradient at a residual block's output and the sums of the batch-norm backward pass behind it, in one pass.
 * In the residual networks the paper trains ("ImageNet training with ResNet-50") the gradient that relu_add_bwd makes is
 * at once the dy of the block's last batch norm.  relu_add_bwd_bnsums_t is relu_add_bwd_t (y required, db may be NULL)
 * on [n,c,h,w] tensors that, while it writes dx, also sums dx and dx * xhat per channel against x_bn, the INPUT of that
 * batch norm (xhat from save_mean / save_invstd of its forward pass), and leaves the sums in `workspace`;
 * batchnorm_bwd_presummed_t is batchnorm_bwd_t (no ReLU) that takes them from there instead of reading x and dy once
 * more.  The pair gives bit for bit what relu_add_bwd_t followed by batchnorm_bwd_t gives, with one pass over x less.
 * Between the two calls nothing else may use the workspace (the one exception to "contents undefined between calls");
 * both need NHWC, 16-byte aligned tensors and c a multiple of 4 (fp32) or 8 (bf16): LC_ERR_UNSUPPORTED / LC_ERR_ALIGN
 * otherwise, and callers then use the two plain calls.  Workspace: batchnorm_workspace_bytes. */
lc_status relu_add_bwd_bnsums_t(lc_dtype dtype, const void* y, const void* da, const void* db, void* dx, const void* x_bn,
                                const float* save_mean, const float* save_invstd, int n, int c, int h, int w, lc_layout layout,
                                void* workspace, size_t workspace_bytes, void* hip_stream);
lc_status batchnorm_bwd_presummed_t(lc_dtype dtype, const void* x, const void* dy, const float* gamma, const float* save_mean,
                                    const float* save_invstd, void* dx, float* dgamma, float* dbeta, int n, int c, int h, int w,
                                    lc_layout layout, void* workspace, size_t workspace_bytes, void* hip_stream);
/* The same pass where the arriving gradients come out of strided 1x1 convolutions.  The first block of a stage of the
 * paper's ResNet-50 ("ImageNet training with ResNet-50") reads the previous block's output through two 1x1 convolutions of
 * stride 2 (its first convolution and its projection); their input gradients are zero except at the pixels
 * (i * grad_stride, j * grad_stride).  relu_add_bwd_bnsums_grid_t is relu_add_bwd_bnsums_t whose da and db (db may be
 * NULL) are [n, c, ceil(h / grad_stride), ceil(w / grad_stride)] tensors holding only those pixels -- what conv2d_bwd_data
 * of the same filters gives when the descriptor describes the output grid with stride 1 -- so neither the zeros nor the
 * scatter are ever written or read.  Results are bit for bit those of relu_add_bwd_bnsums_t on the scattered tensors.
 * grad_stride = 1 is relu_add_bwd_bnsums_t itself; grad_stride < 1, or more than 2^31 - 1 pixels with grad_stride > 1:
 * LC_ERR_SHAPE.  Everything else (layout, alignment, channel multiples, workspace, errors) as relu_add_bwd_bnsums_t. */
lc_status relu_add_bwd_bnsums_grid_t(lc_dtype dtype, const void* y, const void* da, const void* db, void* dx, const void* x_bn,
                                     const float* save_mean, const float* save_invstd, int n, int c, int h, int w, int grad_stride,
                                     lc_layout layout, void* workspace, size_t workspace_bytes, void* hip_stream);
/* ---- Batch-norm statistics out of the convolution ----
 * Every convolution of the paper's networks is followed by batch normalisation ("Scaling up Batch Size",
 * "ImageNet training with ResNet-50"), whose first step reads the convolution's whole output again to sum it.
 * conv2d_fwd_stats is conv2d_fwd that also hands those sums over: stats receives
 * conv2d_fwd_stats_count(desc) * k * 2 floats, [piece][channel][2] = the sum and the sum of squares, over one
 * piece of the output's pixels, of the values written to y (as written: after rounding where y is bf16).  Every pixel
 * (n, p, q) lies in exactly one piece: 64 or 128 consecutive pixels in (n, p, q) order, or -- ResNet's first layer in
 * fp32, which has a kernel of its own -- a block of 4 x 16 pixels of one image.  They come out of the output tile's registers: 1/16 (fp32) or 1/8 (bf16) of y's bytes instead of a pass over y.
 * The count is 0 -- and conv2d_fwd_stats returns LC_ERR_UNSUPPORTED -- for layers whose plan has no such epilogue: NCHW,
 * groups > 1, and operands the MFMA kernels do not take (fp32 tensors off a 16-byte boundary, channel counts not a
 * multiple of 4 resp. 8); callers then use conv2d_fwd and batchnorm_fwd_t.  stats: DEVICE, 8-byte aligned, written in full.
 * batchnorm_fwd_pre is batchnorm_fwd_t (NHWC) on x = that y with the statistics taken from `stats`
 * (stats_tiles = the count) instead of a pass over x: the pieces are added in a fixed order in double, then
 * mean = sum / m, variance = sum of squares / m - mean^2.  Without a pivot this loses accuracy where a channel's mean is
 * large against its deviation (relative error of the variance about 1e-7 * (1 + mean^2 / variance)): meant for
 * convolution outputs, whose means are of the order of their deviations. */
size_t conv2d_fwd_stats_count(const lc_conv_desc* desc);
lc_status conv2d_fwd_stats(const lc_conv_desc* desc, const void* x, const void* w, void* y, float* stats, void* workspace,
                           size_t workspace_bytes, void* hip_stream);
lc_status batchnorm_fwd_pre(lc_dtype dtype, const void* x, const float* gamma, const float* beta, const void* residual, void* y,
                            float* save_mean, float* save_invstd, int n, int c, int h, int w, float eps, int relu, lc_layout layout,
                            const float* stats, size_t stats_tiles, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Two batch norms that meet in one sum: y = relu?(bn(x) + bn2(x2)), the output of a residual block whose shortcut has a
 * projection (convolution + batch norm) in the residual networks the paper trains ("ImageNet training with ResNet-50").
 * As batchnorm_fwd_t on (x2, gamma2, beta2) without ReLU followed by batchnorm_fwd_t on (x, gamma, beta) with that result
 * as residual, except that the second batch norm's output is never stored: its statistics are made first (save_mean2,
 * save_invstd2), its scale and shift go into the coefficients of the one stream pass that reads x and x2 and writes y.
 * One tensor less written and read; in bf16 also one rounding less (the shortcut's value is not rounded to bf16 before
 * the sum).  stats / stats2: the pieces conv2d_fwd_stats handed over for x / x2 (with their counts), or NULL: then a pass
 * over that tensor makes its statistics (NULL is the only choice for NCHW).  Everything else -- layouts, types,
 * alignment, workspace (batchnorm_workspace_bytes), errors -- as batchnorm_fwd_t; x2 and y must not be NULL.  The
 * backward pass is two batchnorm_bwd_t calls on (x, dy) and (x2, dy) with the same dy, as without the fusion. */
lc_status batchnorm_fwd_pair_t(lc_dtype dtype, const void* x, const float* gamma, const float* beta, const float* stats,
                               size_t stats_tiles, const void* x2, const float* gamma2, const float* beta2, const float* stats2,
                               size_t stats_tiles2, void* y, float* save_mean, float* save_invstd, float* save_mean2,
                               float* save_invstd2, int n, int c, int h, int w, float eps, int relu, lc_layout layout, void* workspace,
                               size_t workspace_bytes, void* hip_stream);

/* Static, human-readable name of a status code. */
const char* lc_status_string(lc_status status);

/* Text of the HIP runtime error behind the most recent LC_ERR_LAUNCH returned on the calling thread
 * ("" if there was none).  The pointer stays valid until the thread's next failing call. */
const char* lc_last_error_detail(void);

#ifdef __cplusplus
}
#endif
#endif /* LARSCONV_H */
