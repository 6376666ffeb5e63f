// Launchers of the gfx950 kernels.  Internal to libsknet; everything here works on raw device
// pointers and sizes.  All launchers enqueue on `stream` and return the hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sk {

// ---- implicit-GEMM SK convolution, fp32 activations, fp32 MFMA --------------------------------
// Computes, for every image b, output map o and output position (y, x) in [0,Ho) x [0,Wo):
//   acc = bias[o] + sum_{c,i,j} Wp[(c*k+i)*k+j][o] * X[b, c, y + i*d - in_off, x + j*d - in_off]
// with X read as zero outside [0,H) x [0,W)  (in_off = 0: the forward "valid" SK convolution;
// in_off = (k-1)*d with flipped, transposed weights: its data gradient),
// then optional ReLU, then optional masking (acc = mask[...] > 0 ? acc : 0, same index as the
// output), and stores it at
//   Y[((b*out_maps + o + o_off)*OH + y*oy_mul + oy_off)*OW + x*ox_mul + ox_off].
struct ConvF32Args {
    const float *x;      // [n][c_in][H][W]
    const float *wp;     // packed weights [c_pad*k*k][n_pad], c_pad = roundup(c_in, 16), n_pad = roundup(c_out, 16)
    const float *bias;   // [n_pad] or nullptr
    const float *mask;   // optional, indexed like y
    float *y;
    int n, c_in, H, W;
    int c_out, n_pad;
    int k, d, in_off;
    int Ho, Wo;
    int relu;
    int out_maps, o_off, OH, OW, oy_mul, oy_off, ox_mul, ox_off;
    // tap_maps > 0 (a multiple of 16): GEMM map o is tap t = o / tap_maps of real map o % tap_maps and is stored at
    // (y*oy_mul + t/2, x*ox_mul + t%2) -- the four taps of a 2x2 stride-2 up-convolution as one 1x1 convolution
    int tap_maps;
    // accumulate != 0: the value that y holds is added to the sum before bias and ReLU (a convolution split into
    // several launches over parts of its input maps); not with mask or tap_maps
    int accumulate;
    // distance in floats between the inputs of consecutive images; 0 = c_in*H*W (images may overlap: a 3-D
    // convolution reads a window of consecutive slices as the maps of one image)
    long x_bstride;
    // grp_maps > 0: the input maps of an image come in groups of grp_maps consecutive planes with grp_skip more
    // floats between one group and the next (the depth taps of a 3-D convolution with kernel stride > 1: a tap's
    // maps are one slice, the next tap's slice lies d slices on); see conv_f32_groups_supported
    int grp_maps;
    long grp_skip;
};
bool conv_f32_groups_supported(int k, int d, int grp_maps);
hipError_t launch_conv_f32(const ConvF32Args &a, hipStream_t stream);

// Pack OIHW fp32 master weights [c_out][c_in][k][k] into the K-major layout launch_conv_f32 reads.
// flip_transpose = 0: Wp[(c*k+i)*k+j][o] = W[o][c][i][j]                       (forward)
// flip_transpose = 1: Wp[(o*k+i)*k+j][c] = W[o][c][k-1-i][k-1-j]               (data gradient)
// Rows/columns beyond the real extents are zero.  rows = roundup(in_maps,16)*k*k, cols = n_pad.
hipError_t launch_pack_weights_f32(const float *w_oihw, float *wp, int c_out, int c_in, int k,
                                   int flip_transpose, int rows, int n_pad, hipStream_t stream);
// several packings in one launch (n <= 32 jobs)
struct PackF32Job { const float *w; float *wp; int c_out, c_in, k, flip_transpose, rows, n_pad; };
hipError_t launch_pack_weights_f32_batch(const PackF32Job *jobs, int n, hipStream_t stream);

// ---- implicit-GEMM SK convolution, 16-bit activations (dtype 1 = bf16, 2 = fp16), MFMA 16x16x32 -------
// Same contract as launch_conv_f32, on the octet layout: a tensor with C maps is stored as
// [n][ceil(C/8)][H][W][8] 16-bit elements (maps beyond C are zero).  k in 1..4, (k-1)*d <= 64.
struct ConvHArgs {
    const void *x;        // input, octet layout, c8_in octets
    const void *wp;       // packed weights (launch_pack_weights_h)
    const float *bias;    // fp32 [roundup(c_out,16)] or nullptr
    const void *mask;     // optional, octet layout, indexed like y: output zeroed where mask <= 0
    void *y;              // octet layout (out_f32 = 0) or fp32 NCHW planar [n][c_out][OH][OW] (out_f32 = 1)
    int dtype;
    int n, c8_in, H, W;
    int c_out, c8_out;    // real output maps and ceil(c_out/8)
    int k, d, in_off;
    int Ho, Wo;
    int relu, out_f32;
    int c8_out_total, o8_off, OH, OW, oy_mul, oy_off, ox_mul, ox_off;
    int mt;               // map tiles per workgroup the weights were packed for; 0 = default for (c_out, k)
    int tap_maps;         // > 0 (multiple of 16): GEMM map o = tap o / tap_maps of real map o % tap_maps, stored at (y*oy_mul + tap/2, x*ox_mul + tap%2)
    // SK pool k = 2, s = 1 fused across two launches (inference): vpool != 0: this layer's output (ReLU required) is
    // stored as max(Y[y], Y[y + d]), Ho - d rows of Wo columns (OH = Ho - d, OW = Wo); hd > 0: the input was stored that way
    // by a layer with kernel stride hd and has W + hd columns per row in memory, of which this launch reads
    // max(X[x], X[x + hd]) for x < W.  Both only where conv_h_pool_fusable() says so.
    int vpool, hd;
    int single_map;       // != 0: the layer has ONE input map (map 0 of the single input octet; the rest of the octet is padding)
    // img != nullptr (only where conv_h_reads_image() says so): the layer reads the caller's fp32 image [n][1][img_h][img_w]
    // itself instead of x -- mirror padding by pad_top / pad_left (pad_mode as in launch_pad_pack_h) to the H x W map this
    // launch convolves, each sample rounded to the storage type as launch_pad_pack_h rounds it
    const float *img;
    int img_h, img_w, pad_top, pad_left, pad_mode;
    const void *zeros;    // CONV_H_ZERO_BYTES of zeros in device memory, read in place of samples outside the image (the launcher
                          // allocates nothing: the owner of the plan provides the page)
    // Slices of a volume as images (3-D layers on the slice-major layout): xb8 > 0: image b starts xb8 octet planes after
    // image b - 1 (0: c8_in, images do not overlap); grp8 > 0: the c8_in input octets come in groups of grp8 with skip8 more
    // octet planes between two groups (the d - 1 slices between two depth taps)
    int xb8, grp8, skip8;
    // filled in by the launcher
    int m_tiles, mgroups, nchunks, xtiles, tiles_hi, tiles_lo, rem, ytiles_total, total_tiles, ypitch;
};
constexpr int CONV_H_ZERO_BYTES = 4096;
bool conv_h_supported(int k, int d);
bool conv_h_pool_fusable(int k, int d, int c_out, int c8_in, int Ho, int hd);
// ... and for a GEMM with gemm_m output maps (c_out forward, c_in for the data gradient) the tile fits the LDS
bool conv_h_supported(int k, int d, int gemm_m);
// does this launch (single_map set, img left null) run on the kernel that can read the fp32 image itself?
bool conv_h_reads_image(const ConvHArgs &a);
hipError_t launch_conv_h(const ConvHArgs &a, hipStream_t stream);
// 16-bit elements of the packed weights of a GEMM with gemm_m output maps and gemm_c8 input octets
long packed_h_elems(int gemm_m, int gemm_c8, int k, int mt = 0);
// map tiles per workgroup (mt) that suit a forward layer of this output size; pass it to the packing too
int conv_h_pick_mt(int c_out, int k, int n, int Ho, int Wo);
// ... or that value with CONV_H_TAPCOLS set: a 3x3 layer whose weights are packed (and whose launch runs) with the kernel
// columns on the lane groups; pass the value to the packing and in ConvHArgs.mt as it is
constexpr int CONV_H_TAPCOLS = 16;
int conv_h_pick_mode(int c_out, int c_in, int k, int d, int n, int Ho, int Wo);
// forward packing (flip_transpose = 0: gemm_m = c_out, input octets of c_in) or data-gradient
// packing (flip_transpose = 1: gemm_m = c_in, input octets of c_out) from OIHW fp32 master weights
hipError_t launch_pack_weights_h(const float *w_oihw, void *wp, int dtype, int c_out, int c_in, int k,
                                 int flip_transpose, int mt, hipStream_t stream);
// several packings in one launch (n <= 32 jobs, one dtype)
struct PackHJob { const float *w; void *wp; int c_out, c_in, k, flip_transpose, mt; };
hipError_t launch_pack_weights_h_batch(const PackHJob *jobs, int n, int dtype, hipStream_t stream);

// ---- HBM-bound layers on the octet layout (dtype 1 = bf16, 2 = fp16) ------------------------------------
// fp32 NCHW -> octets with optional mirror padding (top = left = 0 and ho = h, wo = w: plain conversion)
hipError_t launch_pad_pack_h(const float *in, void *out, int dtype, int n, int c, int h, int w, int top, int left,
                             int ho, int wo, int mode, hipStream_t stream);
hipError_t launch_unpack_h(const void *in, float *out, int dtype, int n, int c, int h, int w, hipStream_t stream);
// planes8 = n * ceil(C/8); tap (optional) holds one byte per element, laid out like y
hipError_t launch_maxpool_h(const void *x, void *y, void *tap, int dtype, long planes8, int H, int W, int Ho, int Wo,
                            int k, int d, int s, hipStream_t stream);
hipError_t launch_crop_copy_h(const void *src, void *dst, int n, int c8, int Hs, int Ws, int c8_total, int o8_off,
                              int H, int W, int cy, int cx, hipStream_t stream);
hipError_t launch_maxpool_bwd_h(const void *dy, const void *tap, const void *relu_src, void *dx, int dtype,
                                long planes8, int H, int W, int Ho, int Wo, int k, int d, hipStream_t stream);
// pool with layer stride s = k at d = 1: dx (H x W) from dy and the winner codes (Ho x Wo); acc != 0 adds to dx
hipError_t launch_maxpool_stride_bwd_h(const void *dy, const void *tap, const void *relu_src, void *dx, int dtype, long planes8, int H, int W,
                                       int Ho, int Wo, int k, int acc, hipStream_t stream);
// out[b][t*c8 + o][y][x] = in[b][o][2y + t/2][2x + t%2] for the first c8 of in's c8_total octets (in: 2h x 2w, out: h x w)
hipError_t launch_space_to_depth2_h(const void *in, void *out, int n, int c8_total, int c8, int h, int w, hipStream_t stream);
// dst [n][c8][Hd][Wd] = octets o8_off.. of src [n][c8_total][Hs][Ws] in the window at (cy, cx), zero elsewhere
hipError_t launch_place_h(const void *src, void *dst, int n, int c8, int Hd, int Wd, int c8_total, int o8_off, int Hs, int Ws, int cy,
                          int cx, hipStream_t stream);
hipError_t launch_tap_to_index_h(const void *tap, int32_t *idx, int n, int c, int Ho, int Wo, int W, int k, int d, int s,
                                 hipStream_t stream);
// stage 1 of the bias gradient: part[(map) * slices + slice] (8 * ceil(c/8) maps); see kernels_wgrad_f32.hip
hipError_t launch_bias_grad_h(const void *dy, float *part, int dtype, int n, int c, long plane, int slices, hipStream_t stream);

// ---- fused inference head: 1x1 conv + ReLU, 1x1 conv, per-pixel softmax (see kernels_head.hip) -------------
struct HeadArgs {
    const void *x;        // input maps: fp32 NCHW (dtype 0) or 16-bit octet layout (dtype 1 bf16, 2 fp16)
    const void *w1p;      // first conv's weights packed by launch_pack_head_w1
    const float *b1;      // [hidden]
    const float *w2;      // second conv's weights, fp32 [classes][hidden]
    const float *b2;      // [classes]
    float *prob;          // fp32 NCHW [n][classes][H][W]
    int dtype, n, c_in, H, W, hidden, classes;
    int hd;               // > 0: the input lacks the horizontal half of an SK pool at kernel stride hd (rows of W + hd samples)
    int ksteps;           // filled in by the launcher
};
bool head_supported(int dtype, int c_in, int hidden, int classes);
bool head_takes_pending_pool(int dtype, int c_in, int classes, int hd);
long head_w1_packed_bytes(int dtype, int c_in, int hidden);
hipError_t launch_pack_head_w1(const float *w1, void *out, int dtype, int hidden, int c_in, hipStream_t stream);
hipError_t launch_head_fused(HeadArgs a, hipStream_t stream);

// Backward pass of the same head with the softmax loss in one kernel (16-bit storage): nothing but x is read and
// nothing but dx, the two layers' weight / bias gradients and the loss is written.
struct HeadTrainArgs {
    const void *x;            // input maps, 16-bit octet layout [n][ceil(c_in/8)][plane][8]
    const void *w1p;          // first conv's weights packed by launch_pack_head_w1
    const float *w1;          // the same weights, fp32 [hidden][c_in]
    const float *b1, *w2, *b2;
    const int32_t *labels;    // [n][plane]; outside 0..classes-1: masked
    const int *counts;        // partial counts of the labelled pixels (launch_label_count)
    int ncounts;
    void *dx;                 // gradient of the loss with respect to x, layout of x (nullptr: not wanted)
    float *scratch;           // head_train_scratch_floats(...) floats, or fewer (fewer workgroups)
    float *dw1, *db1, *dw2, *db2, *loss;
    int dtype, n, c_in, plane, hidden, classes;
};
bool head_train_supported(int dtype, int c_in, int hidden, int classes);
size_t head_train_scratch_floats(int c_in, int hidden);
hipError_t launch_head_train_bwd(HeadTrainArgs a, size_t scratch_floats, hipStream_t stream);

// ---- weight / bias gradient of the SK convolution (fp32) ---------------------------------------
// dW[o][c][i][j] = sum_{b,y,x} dY[b,o,y,x] * X[b,c,y+i*d,x+j*d];  db[o] = sum dY[b,o,:,:].
// scratch must hold wgrad_f32_scratch_floats(...) floats (scratch_cap = 0), or scratch_cap floats with
// scratch_cap >= wgrad_min_scratch_floats(...): the kernel then takes as many private copies of the gradient
// as that holds.  The result is deterministic for a given scratch size.
size_t wgrad_f32_scratch_floats(int c_out, int c_in, int k);
size_t wgrad_min_scratch_floats(int c_out, int c_in, int k);
hipError_t launch_wgrad_f32(const float *x, const float *dy, float *dw, float *db, float *scratch,
                            int n, int c_in, int H, int W, int c_out, int k, int d,
                            hipStream_t stream, size_t scratch_cap = 0);

// the same with the input addressed as launch_conv_f32 addresses it: images x_bstride floats apart (0 = c_in*H*W),
// the c_in maps in groups of grp_maps (a power of two, or 0 = none) with grp_skip more floats between groups
hipError_t launch_wgrad_f32_grouped(const float *x, const float *dy, float *dw, float *db, float *scratch, int n, int c_in, int H,
                                    int W, int c_out, int k, int d, long x_bstride, int grp_maps, long grp_skip, hipStream_t stream);

// 16-bit storage with the input maps in groups: consecutive images start xb8 octet planes apart (0 = the octets of c_in),
// groups of grp_maps maps (a multiple of 8, 0 = none) lie skip8 more planes apart -- the depth taps of a 3-D convolution
// on slice-major volumes as input maps.  c_in is a multiple of 8; ask wgrad_h_grouped_supported first.
bool wgrad_h_grouped_supported(int c_in, int c_out, int k, int d);
hipError_t launch_wgrad_h_grouped(const void *x, const void *dy, float *dw, float *db, float *scratch, int dtype, int n, int c_in, int H, int W,
                                  int c_out, int k, int d, int xb8, int grp_maps, int skip8, hipStream_t stream, size_t scratch_cap = 0);

// zeros: at least 1 KB of zeros in device memory (the row-streaming form of the 4x4 gradient reads the gradient rows
// beyond the image from there); nullptr keeps every shape on the segment kernel
hipError_t launch_wgrad_h(const void *x, const void *dy, float *dw, float *db, float *scratch, int dtype,
                          int n, int c_in, int H, int W, int c_out, int k, int d, hipStream_t stream, size_t scratch_cap = 0,
                          const void *zeros = nullptr);
// 16-bit storage, 4x4 kernels up to 48 -> 48 maps: rows streamed through an LDS ring, operands transposed by the LDS read
bool wgrad_rows_h_supported(int c_in, int c_out, int k, int d);
size_t wgrad_rows_h_scratch_floats(int c_in, int c_out);
hipError_t launch_wgrad_rows_h(const void *x, const void *dy, const void *zeros, float *dw, float *db, float *scratch, size_t scratch_floats,
                               int dtype, int n, int c_in, int H, int W, int c_out, int d, hipStream_t stream);

// ---- HBM-bound layers ---------------------------------------------------------------------------
hipError_t launch_mirror_pad_f32(const float *in, float *out, int planes, int h, int w, int top,
                                 int left, int ho, int wo, int mode, hipStream_t stream);
// Y[p,y,x] = max_{i,j<k} X[p, s*y+i*d, s*x+j*d]; first maximum wins; tap (optional) = i*k+j.
hipError_t launch_maxpool_f32(const float *x, float *y, uint8_t *tap, int planes, int H, int W,
                              int Ho, int Wo, int k, int d, int s, hipStream_t stream);
// dX[p,u,v] = sum over outputs whose recorded winner is (u,v) of dY; if relu_src != nullptr the
// result is zeroed where relu_src[p,u,v] <= 0 (ReLU backward of the layer below, fused).  s = 1 only.
hipError_t launch_maxpool_bwd_f32(const float *dy, const uint8_t *tap, const float *relu_src,
                                  float *dx, int planes, int H, int W, int Ho, int Wo, int k, int d,
                                  hipStream_t stream);
// 3-D pool on the slice-major layout X[D][C][H][W] -> Y[Do][C][Ho][Wo]; k, d, s act on the three axes alike;
// tap (optional, k <= 6) receives the winner's code (a*k + i)*k + j, first maximum in (a, i, j) order
// the same on the 16-bit slice-major octet layout [D][ceil(C/8)][H][W][8], forward only
// tap (optional): one byte per element laid out like y, the winner's code (a k + i) k + j
hipError_t launch_maxpool3d_h(const void *x, void *y, void *tap, int dtype, int C, int D, int H, int W, int Do, int Ho, int Wo, int k, int d,
                              int s, hipStream_t stream);
hipError_t launch_maxpool3d_bwd_h(const void *dy, const void *tap, const void *relu_src, void *dx, int dtype, int C, int D, int H, int W,
                                  int Do, int Ho, int Wo, int k, int d, hipStream_t stream);
hipError_t launch_tap3d_to_index_h(const void *tap, int32_t *idx, int C, int Do, int Ho, int Wo, int H, int W, int k, int d, int s,
                                   hipStream_t stream);
// a 3-D kernel's fp32 master as the OIHW master of the 2-D convolution over (depth tap, map) pairs; bwd = 1: of its data gradient
hipError_t launch_expand_taps3d(const float *w, float *out, int c_out, int c_in, int k, int bwd, hipStream_t stream);
hipError_t launch_maxpool3d_f32(const float *x, float *y, uint8_t *tap, int C, int D, int H, int W, int Do, int Ho, int Wo, int k,
                                int d, int s, hipStream_t stream);
// gradient of the s = 1 pool from its winner codes; relu_src (optional, like dx) zeroes the result where it is <= 0
hipError_t launch_maxpool3d_bwd_f32(const float *dy, const uint8_t *tap, const float *relu_src, float *dx, int C, int D, int H, int W,
                                    int Do, int Ho, int Wo, int k, int d, hipStream_t stream);
hipError_t launch_tap3d_to_index(const uint8_t *tap, int32_t *idx, int C, int Do, int Ho, int Wo, int H, int W, int k, int d, int s,
                                 hipStream_t stream);
// dst[(m*k + a)*k*k + r] = src[m*k*k + r] for m < maps, r < k*k
hipError_t launch_place_tap_f32(const float *src, float *dst, long maps, int k, int a, hipStream_t stream);
// dst[((o*C + c)*k + a)*k*k + r] = src[((o*k + a)*Cs + c)*k*k + r]: a gradient whose input maps are (depth tap, map) pairs;
// Cs = src_maps_per_tap (0: C) -- the 16-bit gradient carries 8*ceil(C/8) maps per tap
hipError_t launch_place_taps_f32(const float *src, float *dst, int c_out, int C, int k, hipStream_t stream, int src_maps_per_tap = 0);
// packings of a 3-D kernel [c_out][C][k][k][k] for launch_conv_f32 (see kernels_conv_f32.hip)
hipError_t launch_pack_weights3d_f32(const float *w3, float *wp, int c_out, int C, int k, int a0, int len, int flip_transpose, int rows,
                                     int n_pad, hipStream_t stream);
hipError_t launch_softmax_f32(const float *z, float *p, int n, int classes, int hw, hipStream_t stream);
// loss = -(1/P) sum log p_label, dz = (p - onehot)/P over the pixels whose label lies in 0..classes-1;
// any other label value (-1 by convention) masks the pixel (no loss, zero gradient) and P counts the
// labelled pixels only.  partial must hold softmax_loss_partials(n*hw) floats.
int softmax_loss_partials(long pixels);
// counts[0..*ncounts) = partial counts of the pixels whose label lies in 0..classes-1 (counts: softmax_loss_partials(pixels) ints)
hipError_t launch_label_count(const int32_t *labels, long pixels, int classes, int *counts, int *ncounts, hipStream_t stream);
// dz16 (optional, with dtype16 = 1 bf16 / 2 fp16): the gradient once more in the 16-bit octet layout [n][1][hw][8]; only where
// softmax_loss_writes_octets(classes, hw) says so (hipErrorInvalidValue otherwise: convert dz instead)
bool softmax_loss_writes_octets(int classes, int hw);
hipError_t launch_softmax_loss_f32(const float *z, const int32_t *labels, float *dz, float *loss,
                                   float *partial, int n, int classes, int hw, hipStream_t stream, void *dz16 = nullptr, int dtype16 = 0);
// g = dw + wd*w; v = mu*v + lr*g; w -= v   (v may be nullptr when mu = 0)
hipError_t launch_sgd_f32(float *w, const float *dw, float *v, long count, float lr, float mu,
                          float wd, hipStream_t stream);
// the same update for up to BATCH_MAX tensors in one launch (the parameters of a net are many small tensors)
constexpr int BATCH_MAX = 32;
struct SgdBatch {
    float *w[BATCH_MAX];
    const float *dw[BATCH_MAX];
    float *v[BATCH_MAX];          // nullptr entries: no momentum buffer
    long count[BATCH_MAX];
    int n;
};
hipError_t launch_sgd_batch_f32(const SgdBatch &b, float lr, float mu, float wd, hipStream_t stream);
// bias shared by the four taps of an up-convolution: gradient = sum of the taps' gradients db4[t*c_out + o]; the new
// value goes to each tap's copy and, if given, four times into b_stacked[4*c_out] (the stacked 1x1 form's bias)
hipError_t launch_up_bias_sgd_f32(float *b0, float *b1, float *b2, float *b3, float *b_stacked, const float *db4, float *v, int c_out, float lr,
                                  float mu, float wd, hipStream_t stream);
// out[b, o_off + c, y, x] = in[b, c, y + oy, x + ox] for c < maps (crop-and-place, MergeCrop halves)
hipError_t launch_crop_copy_f32(const float *in, float *out, int n, int maps, int hi, int wi,
                                int out_maps, int o_off, int ho, int wo, int oy, int ox,
                                hipStream_t stream);
// expand tap codes into flat offsets inside the input plane
hipError_t launch_tap_to_index(const uint8_t *tap, int32_t *idx, int planes, int Ho, int Wo, int W,
                               int k, int d, int s, hipStream_t stream);
hipError_t launch_relu_mask_f32(float *g, const float *act, long count, hipStream_t stream);
// backward pieces of the U-Net / USK-Net (see kernels_misc.hip): pool with s = k, d = 1; the four interleaved
// sub-images of a 2h x 2w tensor as 4*maps maps of h x w; placing a tensor into a window of a larger one
hipError_t launch_maxpool_stride_bwd_f32(const float *dy, const uint8_t *tap, float *dx, int planes, int H, int W, int Ho, int Wo,
                                         int k, int accumulate, hipStream_t stream);
hipError_t launch_space_to_depth2_f32(const float *in, float *out, int n, int in_maps, int maps, int h, int w, hipStream_t stream);
hipError_t launch_place_f32(const float *in, float *out, int n, int in_maps, int c_off, int maps, int hi, int wi, int ho, int wo,
                            int oy, int ox, hipStream_t stream);
hipError_t launch_fill_f32(float *p, float v, long count, hipStream_t stream);

}  // namespace sk
