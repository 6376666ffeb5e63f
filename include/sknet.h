/*
 * libsknet — dense pixelwise classification with strided-kernel (SK) networks and a U-Net
 * forward pass on one AMD MI355X (gfx950).  C ABI; no C++ or framework types cross it.
 *
 * Method: F. Tschopp, "Efficient Convolutional Neural Networks for Pixelwise Classification on
 * Heterogeneous Hardware Systems" (arXiv 1509.03371).  Symbols follow its Section 1.6:
 * f_in/f_out feature maps, w map size, v total context of the net, k kernel size, s layer
 * stride, d kernel stride (dilation), n minibatch.
 *
 * Pointer conventions: every pointer argument is marked HOST or DEVICE.  DEVICE buffers are
 * owned by the caller (e.g. a PyTorch tensor's data_ptr()); the library never frees or keeps
 * them beyond the call.  HOST buffers are plain caller memory.  Weights, packed weights,
 * activations, pool masks and gradients are owned by the handle.
 *
 * Errors: every function returns an sk_status (0 = success) and never throws or aborts; all
 * argument and shape checks happen on the host before anything is launched.  The message for
 * the last failure on the calling thread is available from sknet_last_error().
 *
 * Asynchrony: forward / backward / sgd_step only enqueue work on the given HIP stream
 * (a hipStream_t passed as void*, NULL = the default stream) and return; the get_* accessors
 * and sknet_time_step synchronise that stream themselves.  One handle must not be used from
 * two host threads, or on two streams, at the same time.
 */
#ifndef SKNET_H
#define SKNET_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sknet sknet_t; /* opaque */
typedef struct unet unet_t;   /* opaque */
typedef struct sknet3d sknet3d_t; /* opaque */

typedef enum {
    SK_OK = 0,
    SK_EINVAL = 1,       /* null pointer, bad enum, bad index */
    SK_ESHAPE = 2,       /* sizes that the layer rules reject */
    SK_ESTATE = 3,       /* call order: forward before plan, backward before a training forward ... */
    SK_ENOMEM = 4,       /* device or host allocation failed */
    SK_EDEVICE = 5,      /* a HIP call failed, or no usable GPU */
    SK_EUNSUPPORTED = 6  /* valid request that this build does not implement */
} sk_status;

/* Arithmetic/storage type of activations and packed weights.  Accumulation is always fp32;
 * images, probabilities, labels, weights and gradients cross the ABI as fp32 / int32. */
typedef enum { SK_F32 = 0, SK_BF16 = 1, SK_F16 = 2 } sk_dtype;

typedef enum { SK_CONV = 0, SK_MAXPOOL = 1 } sk_kind;

/* One layer of an SK net, in the terms of the paper's configuration tables (Section 3.3.2):
 *   SK_CONV    : f_out = c_out maps, kernel k x k, kernel stride d, s must be 1; relu != 0 applies
 *                max(0, .) to the output.  Y[o,y,x] = b[o] + sum_{c,i,j} W[o,c,i,j] X[c,y+i*d,x+j*d]
 *                (Section 5.2.1; cross-correlation, no padding).
 *   SK_MAXPOOL : kernel k x k, kernel stride d, layer stride s (1 for SK pooling; s = k with d = 1
 *                for an ordinary down-sampling pool).  c_out and relu are ignored.
 * Every layer with a kernel shrinks the map by (k-1)*d (Algorithm 1). */
typedef struct {
    int32_t kind;  /* sk_kind */
    int32_t c_out;
    int32_t k;
    int32_t d;
    int32_t s;
    int32_t relu;
} sk_layer;

/* A layer of a sliding-window net, input of Algorithm 1.  kind: 0 convolution (k, c_out, relu),
 * 1 pooling (k, s), 2 inner product (c_out, relu; its kernel is the whole remaining map),
 * 3 any other layer (must have k = 1, i.e. be element-wise; it is dropped from the output). */
typedef struct {
    int32_t kind;
    int32_t c_out;
    int32_t k;
    int32_t s;
    int32_t relu;
} sw_layer;

/* ---------------------------------------------------------------- host-only helpers (no GPU) */

/* Algorithm 1 (Section 3.3.1): convert a sliding-window net with patch size w0_sw into SK layers.
 * sw, sk_out: HOST arrays; sk_out must have room for n entries; *n_out receives the count
 * written.  Returns SK_ESHAPE when the algorithm's checks fail: a pool with w mod k != 0 or
 * k != s, another layer type with k > 1, a map that shrinks below 1, or a final kernel
 * stride != 1. */
sk_status sknet_convert_sw(const sw_layer *sw, int32_t n, int32_t w0_sw, sk_layer *sk_out,
                           int32_t *n_out);

/* Convolution cost model of Section 5.5: f_out * w_out^2 * (2 * f_in * k^2 - 1). */
int64_t sknet_conv_flops(int64_t f_in, int64_t f_out, int64_t k, int64_t w_out);

/* Message of the last error on this thread (never NULL; valid until the next failing call). */
const char *sknet_last_error(void);

/* ---------------------------------------------------------------- SK-Net */

/* Build a net description (host only; no GPU needed).  layers: HOST array, copied.
 * The net is: mirror padding by the context v, the layers in order, then a per-pixel softmax
 * over the maps of the last layer (Section 3.3.2's table ends in such a "prob" layer).
 * n_classes must equal the map count of the last layer.  pad_mode: 0 = reflect (edge sample not
 * repeated), 1 = symmetric (edge sample repeated).  Conv weights start as zeros.
 * SK_EINVAL for bad arguments, SK_ESHAPE for k < 1, d < 1, a pool whose s is neither 1 nor k
 * (or s = k with d != 1), SK_EUNSUPPORTED for k > 15, and for SK_BF16 / SK_F16 nets a conv whose
 * kernel the 16-bit path has no variant for: k <= 4 needs (k-1)*d <= 64; k = 5, 6, 7, 8 and 10 (the
 * sizes of the paper's SK and USK configuration tables) need a staged row 128 + (4*ceil(k/4) - 1)*d
 * of at most 256 pixels; k = 9 and k > 10 are fp32 only.  (Training plans in 16-bit storage: k <= 4.) */
sk_status sknet_create(const sk_layer *layers, int32_t n_layers, int32_t c_in, int32_t n_classes,
                       sk_dtype dtype, int32_t pad_mode, sknet_t **out);
void sknet_destroy(sknet_t *net);

/* *v = total context, the sum of (k-1)*d over all layers (only defined for nets whose pools
 * all have s = 1; SK_ESHAPE otherwise).  The image is padded by ceil(v/2) rows/columns at the
 * top/left and floor(v/2) at the bottom/right (Section 3.3.2's handling of an odd v). */
sk_status sknet_context(const sknet_t *net, int32_t *v);

/* Map sizes for an h x w image: dims (HOST) receives (n_layers + 1) triples {maps, height,
 * width}: entry 0 is the padded image, entry i the output of layer i-1.  pad != 0 applies the
 * context padding first.  SK_ESHAPE if a map would shrink below one pixel, a down-sampling pool
 * meets an odd size, or the mirror border does not fit the image. */
sk_status sknet_infer_shapes(const sknet_t *net, int32_t h, int32_t w, int32_t pad, int32_t *dims);

/* Number of convolution layers, and for conv number conv_idx (0-based, in layer order) its
 * weight shape {f_out, f_in, k, k} written to shape4 (HOST). */
sk_status sknet_num_convs(const sknet_t *net, int32_t *count);
sk_status sknet_conv_shape(const sknet_t *net, int32_t conv_idx, int32_t *shape4);

/* Set / read the fp32 master weights [f_out][f_in][k][k] and biases [f_out] of one conv (HOST
 * buffers; b may be NULL in set = keep).  May be called before or after sknet_plan; after a plan
 * the device copies are refreshed at once (synchronously). */
sk_status sknet_set_weights(sknet_t *net, int32_t conv_idx, const float *w_host, const float *b_host);
sk_status sknet_get_weights(sknet_t *net, int32_t conv_idx, float *w_host, float *b_host);

/* Fix the problem size: n images of h x w pixels, and allocate every workspace on the current
 * HIP device (hipMalloc).  pad != 0: the library mirror-pads the image by v so that the output
 * is h x w; pad = 0: the caller's image already contains its context and the output is
 * (h - v) x (w - v).
 * mode 0 = inference: layers may be fused (at present: a trailing "1x1 conv + ReLU, 1x1 conv,
 *          softmax" runs as one kernel whose hidden maps and logits never reach memory; then
 *          sknet_get_activation reports SK_ESTATE for those two layers);
 * mode 1 = training: every activation and the pool winners are kept, gradient buffers allocated;
 * mode 2 = inference with every layer's output kept in memory (for parity checks);
 * mode 3 = training as mode 1, but a trailing "1x1 conv + ReLU, 1x1 conv" and the softmax loss (Sections 4.2, 4.3)
 *          run as one kernel in each direction: the hidden maps, the logits and their gradients never reach memory
 *          (the backward kernel recomputes the hidden maps from the head's input).  16-bit storage, at most 48
 *          input maps, 208 hidden maps and 4 classes, a pool in front of the head; SK_EUNSUPPORTED otherwise.
 *          sknet_get_activation and sknet_get_activation_grad report SK_ESTATE / SK_EUNSUPPORTED for those two layers.
 * May be called again to change the size or mode.  SK_ESHAPE as in sknet_infer_shapes. */
sk_status sknet_plan(sknet_t *net, int32_t n, int32_t h, int32_t w, int32_t pad, int32_t mode);

/* Whole forward pass (Section 1.3: image in, per-pixel class probabilities out).
 * image_dev: DEVICE fp32 [n][c_in][h][w];  prob_dev: DEVICE fp32 [n][n_classes][h_out][w_out].
 * Needs a plan (SK_ESTATE otherwise). */
sk_status sknet_forward(sknet_t *net, const float *image_dev, float *prob_dev, void *hip_stream);

/* Softmax loss and exact gradients of every conv weight and bias, after a forward on a
 * training plan (SK_ESTATE otherwise).  labels_dev: DEVICE int32 [n][h_out][w_out], values in
 * [0, n_classes), or any other value (-1 by convention) for a pixel that is masked out of the error
 * map (Section 4.2's label masking: no loss, zero gradient).  loss_dev: DEVICE fp32 scalar =
 * -(1/P) * sum over the P labelled pixels of log p_label (Section 4.3: accumulated over all error
 * pixels, then normalised; P = n*h_out*w_out without masking; everything masked: loss 0, gradients 0).
 * Pool gradients go to the recorded maximum; ReLU passes gradient where its output is > 0. */
sk_status sknet_backward(sknet_t *net, const int32_t *labels_dev, float *loss_dev, void *hip_stream);

/* sknet_backward for callers that cannot allocate device memory or tolerate a call that does (code under HIP
 * graph capture, tight serving / training loops, harnesses that forbid hipMalloc): the same pass with the same
 * arguments, results and state rules, but its partial results -- the loss kernel's partial sums and counts, the
 * private copies of each weight gradient and the bias partials -- live in a buffer that is part of the library's
 * device code (32 MiB per GPU, there from the time the library is loaded on that GPU until the process ends)
 * instead of the plan's own scratch.  The call itself allocates and frees nothing.  The activation-gradient
 * buffers are the plan's, as in sknet_backward.  Limits: SK_EUNSUPPORTED if one padded copy of the net's largest
 * weight gradient, roundup(f_out,16) x roundup(f_in*k*k,16) floats plus 512 x roundup(f_out,16) floats of bias partials,
 * exceeds 8 Mi - 4096 floats, or if the loss needs more than 4096 floats (it never does: at most 4096).  A weight
 * gradient takes as many private copies as fit, so the summation order -- not the value beyond fp32 rounding --
 * can differ from sknet_backward's.  Every call on one GPU shares that GPU's buffer, whose contents are whatever
 * the last call left (nothing in it needs clearing: each kernel writes every partial that is read afterwards);
 * two such calls that overlap in time on one GPU (two streams, two handles, two threads) race and give wrong
 * gradients -- serialise them. */
sk_status sknet_backward_noalloc(sknet_t *net, const int32_t *labels_dev, float *loss_dev, void *hip_stream);

/* SGD on the fp32 master weights with the gradients of the last backward:
 * g = dW + weight_decay*W;  V = momentum*V + lr*g;  W = W - V; then the packed device weights
 * are rebuilt (rounded to the compute dtype). */
sk_status sknet_sgd_step(sknet_t *net, float lr, float momentum, float weight_decay, void *hip_stream);

/* Debug / parity accessors; each synchronises the stream of the last call first.
 * get_grad: gradients of conv conv_idx as fp32 [f_out][f_in][k][k] and [f_out] (HOST).
 * get_activation: output of layer layer_idx (-1 = the padded image) as fp32 NCHW (HOST), sized
 *   as sknet_infer_shapes reports.
 * get_pool_argmax: for max-pool number pool_idx (0-based among pools), per output element the
 *   flat offset (y*W_in + x) of the winning input sample inside its input plane, int32 NCHW
 *   (HOST).  Taps are scanned row-major and only a strictly greater value replaces the
 *   incumbent, so the first maximum wins.  Needs a training plan.
 * get_activation_grad: the error map of layer layer_idx (0-based), i.e. the gradient of the loss with respect
 *   to that layer's output with the layer's own ReLU derivative applied (what its weight gradient and the
 *   data gradient of the layer read; Section 1.6 calls it the blob's "diff"), fp32 NCHW (HOST), sized like the
 *   layer's output.  Re-runs the backward pass of the last forward with labels_dev (DEVICE, as in
 *   sknet_backward) from the loss down to that layer; this overwrites the weight gradients of the layers it
 *   passes, so sknet_get_grad reports SK_ESTATE until the next sknet_backward.  Needs a forward pass on a
 *   training plan.  Allocates and frees small temporaries. */
sk_status sknet_get_grad(sknet_t *net, int32_t conv_idx, float *dw_host, float *db_host);
sk_status sknet_get_activation(sknet_t *net, int32_t layer_idx, float *nchw_host);
sk_status sknet_get_activation_grad(sknet_t *net, int32_t layer_idx, const int32_t *labels_dev, float *nchw_host);
sk_status sknet_get_pool_argmax(sknet_t *net, int32_t pool_idx, int32_t *idx_host);

/* Number of device steps of the planned forward pass (pad, one per layer or fused group, softmax), a short
 * name for step i copied into name (HOST, at most cap bytes), and the average duration in
 * milliseconds of step i re-run iters times on hip_stream between two HIP events (the step
 * reads the activations the last forward left behind).  For benchmarking. */
sk_status sknet_num_steps(const sknet_t *net, int32_t *count);
sk_status sknet_step_name(const sknet_t *net, int32_t step, char *name, int32_t cap);
sk_status sknet_time_step(sknet_t *net, int32_t step, int32_t iters, void *hip_stream, float *avg_ms);
/* The same for one piece of the backward pass of the last forward on a training plan (for benchmarking; Section 6
 * times layers one by one): part 0 = the weight and bias gradient of convolution layer layer_idx (all its launches:
 * the gradient kernel and the reduction of its private copies), part 1 = the gradient of layer layer_idx's input (data
 * gradient of a convolution, scatter of a pool; layer_idx >= 1), part 2 = the softmax loss and its gradient (layer_idx
 * ignored).  The call first walks the backward pass from the loss down to that layer with labels_dev (DEVICE, as in
 * sknet_backward) to rebuild the layer's error map, then repeats the piece iters times between two HIP events on
 * hip_stream.  Weight gradients are overwritten on the way: sknet_get_grad reports SK_ESTATE until the next
 * sknet_backward. */
sk_status sknet_time_backward_step(sknet_t *net, const int32_t *labels_dev, int32_t layer_idx, int32_t part, int32_t iters, void *hip_stream,
                                   float *avg_ms);

/* ---------------------------------------------------------------- U-Net forward */

/* U-Net of Section 3.4's configuration table: `depth` contracting steps (two 3x3 convs + ReLU,
 * then a 2x2 stride-2 max pool), two 3x3 convs at the bottom, `depth` expanding steps (2x2
 * stride-2 up-convolution f -> f/2 without ReLU, MergeCrop with the skip connection, two 3x3
 * convs + ReLU), a 1x1 conv to n_classes and a per-pixel softmax.  Maps: base_ch * 2^level.
 * dtype: SK_F32, or SK_BF16 / SK_F16 (activations and packed weights in the 16-bit type, fp32
 * accumulation, fp32 logits and probabilities; base_ch must then be a multiple of 8, else
 * SK_EUNSUPPORTED).  Host only. */
sk_status unet_create(int32_t c_in, int32_t n_classes, int32_t depth, int32_t base_ch,
                      sk_dtype dtype, unet_t **out);
void unet_destroy(unet_t *net);

/* USK-Net of Section 3.5's configuration table, as a unet_t handle that every unet_* call below
 * accepts: two 3x3 convs + ReLU and a 2x2 stride-2 max pool (U part); on the half-resolution maps
 * the SK sequence conv k6 d1, pool k2 d1, conv k4 d2, pool k2 d2, conv k4 d4, pool k2 d4, conv k8
 * d8 ("ip1"), conv 1x1 ("ip2"), all convs + ReLU, all pools stride 1 (context 86); a 2x2 stride-2
 * up-convolution without ReLU, MergeCrop with the maps of the second 3x3 conv, two 3x3 convs + ReLU,
 * a 1x1 conv to n_classes and a per-pixel softmax.  Maps: base_ch (64 in the table), 2, 8, 4, 2, 3,
 * 2, 1 times base_ch along the path.  692 x 692 in -> 512 x 512 out.  Parameter order: "conv1",
 * "conv2", "conv3", "conv4", "conv5", "ip1", "ip2", "up1" ([4b][2b][2][2]), "conv7", "conv8",
 * "ip3".  Stages for unet_get_activation: "conv2", "pool1", "conv3", "pool2", "conv4", "pool3",
 * "conv5", "pool4", "ip1", "ip2", "up1", "conv8", "logits".  dtype: SK_F32, or SK_BF16 / SK_F16 for the
 * forward pass (base_ch a multiple of 8; training plans are fp32).  Host only. */
sk_status usknet_create(int32_t c_in, int32_t n_classes, int32_t base_ch, sk_dtype dtype, unet_t **out);

/* Parameter tensors, in forward order: per level i = 0..depth "down{i}a", "down{i}b"; then per
 * level i = depth-1..0 "up{i}", "dec{i}a", "dec{i}b"; then "head".  Convs are [f_out][f_in][k][k];
 * up-convolutions are [f_in][f_out][2][2] with Y[o,2y+a,2x+b] = bias[o] + sum_c W[c,o,a,b] X[c,y,x]
 * (the paper's fixed nearest-neighbour up-sampling followed by a 1x1 conv is the case
 * W[c,o,a,b] = W1x1[o,c]).  shape4 (HOST) receives the four extents. */
sk_status unet_num_params(const unet_t *net, int32_t *count);
sk_status unet_param_shape(const unet_t *net, int32_t idx, int32_t *shape4);
/* *kind (HOST) = 0 for a convolution ([f_out][f_in][k][k], f_out biases), 1 for an up-convolution ([f_in][f_out][2][2], f_out biases). */
sk_status unet_param_kind(const unet_t *net, int32_t idx, int32_t *kind);
sk_status unet_set_weights(unet_t *net, int32_t idx, const float *w_host, const float *b_host);

/* Output size for an input of h_in x w_in (which already contains the context; 572 -> 388 in the
 * paper's table).  SK_ESHAPE when a pool meets an odd size or a map vanishes. */
sk_status unet_output_size(const unet_t *net, int32_t h_in, int32_t w_in, int32_t *h_out, int32_t *w_out);

/* Allocate workspaces for n images of h_in x w_in on the current HIP device. */
sk_status unet_plan(unet_t *net, int32_t n, int32_t h_in, int32_t w_in);

/* image_dev: DEVICE fp32 [n][c_in][h_in][w_in];  prob_dev: DEVICE fp32 [n][n_classes][h_out][w_out].
 * MergeCrop puts the up path's maps first, then the skip maps centre-cropped with offset
 * floor((w_skip - w_up)/2) (Section 5.3.1). */
sk_status unet_forward(unet_t *net, const float *image_dev, float *prob_dev, void *hip_stream);

/* Training pass (U-Net and USK-Net handles alike; every storage type: with bf16 / fp16 the error maps are stored
 * in that type too, sums and weight gradients are fp32 and the fp32 master weights take the update.  fp16 error
 * maps carry the loss's factor 1 / (labelled pixels) unscaled and underflow on large images; bf16 does not).
 * unet_plan_training: as unet_plan, and also allocates a gradient buffer per activation, the pools'
 *   winner codes and the gradient scratch; unet_forward then records what the backward pass needs.
 * unet_backward: after a forward on a training plan (SK_ESTATE otherwise).  labels_dev: DEVICE int32
 *   [n][h_out][w_out], values in [0, n_classes) or -1 for a masked pixel; loss_dev: DEVICE fp32 scalar,
 *   both as in sknet_backward (on a training plan unet_forward keeps a copy of its image for this).
 *   Computes the gradient of the loss for every parameter by the layers' backward rules in reverse order.
 *   MergeCrop (Section 5.3.1) copies the error maps back in the inverse direction; for these nets the
 *   section enables that for input A (the up path) only, because B (the skip map) gets its differential
 *   on another path, from the down-sampling pool.  That is the default.  unet_set_merge_backward(net, 1)
 *   selects the exact derivative of the composite instead: the skip maps' part of MergeCrop's gradient
 *   also goes to the centre window of the skip map (nothing to the cropped border) and is summed with
 *   the pool's gradient; mode 0 restores the section's rule.  May be called at any time before
 *   unet_backward; SK_EINVAL for another mode.  The up-convolution's gradient is that of a 1x1
 *   convolution to the four interleaved sub-images.  Deterministic.
 * unet_get_grad: gradient of parameter idx in the layout of unet_set_weights (HOST; either may be null);
 *   synchronises. */
sk_status unet_plan_training(unet_t *net, int32_t n, int32_t h_in, int32_t w_in);
sk_status unet_set_merge_backward(unet_t *net, int32_t mode);
sk_status unet_backward(unet_t *net, const int32_t *labels_dev, float *loss_dev, void *hip_stream);
sk_status unet_get_grad(unet_t *net, int32_t idx, float *dw_host, float *db_host);
/* SGD on the fp32 weights with the gradients of the last unet_backward, as sknet_sgd_step
 * (g = dW + weight_decay*W; V = momentum*V + lr*g; W = W - V); the four taps of an up-convolution share
 * one bias, whose gradient is the sum over the taps.  unet_get_weights: the current values in the
 * layout of unet_set_weights (HOST; either may be null); synchronises.  A later unet_plan keeps them. */
sk_status unet_sgd_step(unet_t *net, float lr, float momentum, float weight_decay, void *hip_stream);
sk_status unet_get_weights(unet_t *net, int32_t idx, float *w_host, float *b_host);

/* Output of named stage (HOST fp32 NCHW): "down{i}", "up{i}", "dec{i}", "logits". *dims3 = maps,h,w. */
sk_status unet_get_activation(unet_t *net, const char *stage, float *nchw_host, int32_t *dims3);

/* ---------------------------------------------------------------- 3-D SK net forward */

/* SK net on volumes (Section 5.2.2: the convolution and max-pool layers with one more spatial axis; the
 * paper's N-dimensional layers, three dimensions here).  The layers are sk_layer entries whose k, d and s
 * act on depth, height and width alike:
 *   SK_CONV    : Y[o,z,y,x] = b[o] + sum_{c,a,i,j} W[o,c,a,i,j] X[c, z+a*d, y+i*d, x+j*d], optional ReLU;
 *   SK_MAXPOOL : Y[c,z,y,x] = max_{a,i,j<k} X[c, s*z+a*d, s*y+i*d, s*x+j*d]  (s = 1, or s = k with d = 1);
 * every layer shrinks each axis by (k-1)*d (Algorithm 1 holds per axis); a per-voxel softmax over the maps
 * of the last layer follows (forward; sknet3d_backward adds the training pass).  One volume per call, no padding: the caller's volume contains the
 * context v, the output is (dz - v) x (h - v) x (w - v).  Create is host only; errors as sknet_create.
 *
 * Layout of every volume that crosses this interface (input, probabilities, activations): SLICE-MAJOR,
 * [depth][maps][height][width] fp32 -- a stack of multi-map 2-D sections; for one input map that is the
 * plain [depth][height][width] image stack.  Weights are [f_out][f_in][k][k][k] (depth, height, width taps). */
sk_status sknet3d_create(const sk_layer *layers, int32_t n_layers, int32_t c_in, int32_t n_classes, sknet3d_t **out);
/* The same with the storage type of the activations: SK_F32 (what sknet3d_create builds), or SK_BF16 / SK_F16:
 * activations (and, on a training plan, error maps) in the 16-bit slice-major octet layout inside the library, fp32
 * accumulation, fp32 weight gradients and master weights, fp32 volumes and probabilities at this interface as before;
 * the net must end in a convolution.  SK_EUNSUPPORTED for a convolution the 16-bit kernels have no variant for (see
 * sknet_create).  As in the 2-D nets, fp16 error maps carry the loss's 1 / (labelled voxels) unscaled. */
sk_status sknet3d_create_dtype(const sk_layer *layers, int32_t n_layers, int32_t c_in, int32_t n_classes, sk_dtype dtype, sknet3d_t **out);
void sknet3d_destroy(sknet3d_t *net);
/* *v = sum of (k-1)*d over the layers (SK_ESHAPE if a pool has s != 1). */
sk_status sknet3d_context(const sknet3d_t *net, int32_t *v);
/* dims4 (HOST) receives (n_layers + 1) quadruples {maps, depth, height, width}: entry 0 the input volume,
 * entry i the output of layer i-1.  SK_ESHAPE if a map would vanish or a down-sampling pool meets a size
 * that k does not divide. */
sk_status sknet3d_infer_shapes(const sknet3d_t *net, int32_t dz, int32_t h, int32_t w, int32_t *dims4);
sk_status sknet3d_num_convs(const sknet3d_t *net, int32_t *count);
/* shape5 (HOST) = {f_out, f_in, k, k, k} */
sk_status sknet3d_conv_shape(const sknet3d_t *net, int32_t conv_idx, int32_t *shape5);
/* w_host: HOST fp32 [f_out][f_in][k][k][k]; b_host: HOST fp32 [f_out] or NULL = keep.  Before or after a
 * plan (after: the device copies are refreshed synchronously). */
sk_status sknet3d_set_weights(sknet3d_t *net, int32_t conv_idx, const float *w_host, const float *b_host);
/* Fix the volume size and allocate the workspaces on the current HIP device (hipMalloc).  mode 0: inference,
 * a trailing "1x1x1 conv + ReLU, 1x1x1 conv, softmax" may run as one kernel (then sknet3d_get_activation
 * reports SK_ESTATE for those two layers); mode 2: every layer's output is kept; mode 1: training -- every
 * activation and the pools' winners are kept, gradient buffers allocated (pools must have s = 1 and k <= 6,
 * else SK_EUNSUPPORTED).  May be called again; the current weights are kept. */
sk_status sknet3d_plan(sknet3d_t *net, int32_t dz, int32_t h, int32_t w, int32_t mode);
/* volume_dev: DEVICE fp32 [dz][c_in][h][w]; prob_dev: DEVICE fp32 [dz-v][n_classes][h-v][w-v] (for nets with
 * down-sampling pools: the sizes sknet3d_infer_shapes reports).  On an inference plan the volume must stay
 * valid until the enqueued work has run; a training plan copies it.  SK_ESTATE without a plan. */
sk_status sknet3d_forward(sknet3d_t *net, const float *volume_dev, float *prob_dev, void *hip_stream);
/* Softmax loss and the exact gradient of every weight and bias, after a forward on a training plan (SK_ESTATE
 * otherwise).  labels_dev: DEVICE int32 [dz-v][h-v][w-v], values in [0, n_classes) or -1 for a masked voxel;
 * loss_dev: DEVICE fp32 scalar; both as in sknet_backward with voxels for pixels (Sections 4.2, 4.3).  The
 * gradient of a pool goes to the recorded winner (first maximum in the order depth, row, column tap), ReLU
 * passes gradient where its output is > 0.  Deterministic. */
sk_status sknet3d_backward(sknet3d_t *net, const int32_t *labels_dev, float *loss_dev, void *hip_stream);
/* SGD on the fp32 weights with the gradients of the last backward, as sknet_sgd_step. */
sk_status sknet3d_sgd_step(sknet3d_t *net, float lr, float momentum, float weight_decay, void *hip_stream);
/* Parity accessors; each synchronises the stream of the last call first.  get_grad / get_weights: HOST fp32
 * [f_out][f_in][k][k][k] and [f_out] (either may be NULL).  get_activation: output of layer layer_idx, HOST fp32
 * [depth][maps][height][width].  get_pool_argmax: for max pool number pool_idx (0-based among pools) of a
 * training plan, per output element ([depth][maps][height][width], int32) the flat offset
 * (z_in*H_in + y_in)*W_in + x_in of the winning sample inside its map's input volume. */
sk_status sknet3d_get_grad(sknet3d_t *net, int32_t conv_idx, float *dw_host, float *db_host);
sk_status sknet3d_get_weights(sknet3d_t *net, int32_t conv_idx, float *w_host, float *b_host);
sk_status sknet3d_get_activation(sknet3d_t *net, int32_t layer_idx, float *dchw_host);
sk_status sknet3d_get_pool_argmax(sknet3d_t *net, int32_t pool_idx, int32_t *idx_host);

/* Machine probes for the benchmark (Section 6 of the paper times kernels against each device's
 * peak; these two calls measure the peaks of the device at hand).  Neither runs any step of the method.
 *
 * sk_probe_mfma: every wave of a grid of 4 x (number of CUs) workgroups of 256 threads issues
 *   iters x 8 independent MFMA instructions of the shape the convolutions use for dtype
 *   (sk_dtype: fp32 16x16x4, bf16 / fp16 16x16x32) with no memory traffic; *tflops (HOST) receives
 *   the sustained rate.  operands = 0: all MFMAs multiply the same two registers (a smooth value per
 *   lane, and ones); operands = 1: each of the 8 has operands of its own with hashed bit patterns in
 *   [-1, 1), the switching activity of real data -- the rate then shows what the chip sustains
 *   under its power limit.  1 <= iters <= 2^22.  Allocates and frees a small device buffer.
 * sk_probe_copy: copies bytes (a positive multiple of 16) from src_dev to dst_dev (DEVICE, 16-byte
 *   aligned, caller-owned, non-overlapping) reps times with a 16-bytes-per-lane grid-stride
 *   kernel; *gb_per_s (HOST) receives (bytes read + bytes written) / time.
 * Both enqueue on hip_stream, time with HIP events on that stream and synchronise it. */
sk_status sk_probe_mfma(int32_t dtype, int32_t operands, int32_t iters, void *hip_stream, double *tflops);
sk_status sk_probe_copy(const void *src_dev, void *dst_dev, uint64_t bytes, int32_t reps, void *hip_stream,
                        double *gb_per_s);

#ifdef __cplusplus
}
#endif
#endif /* SKNET_H */
