// 3-D SK net (Section 5.2.2's N-dimensional layers, three dimensions): handle, shape inference, planning and
// the launch sequences of the forward and training passes.  See include/sknet.h for the contract of every
// entry point.
//
// Volumes live slice-major, [D][C][H][W]: a stack of D multi-map 2-D slices.  With that layout a 3-D
// convolution with kernel stride d is a 2-D SK convolution per output slice z whose input maps are the
// (depth tap a, map c) pairs, found in slice z + a*d.  The output slices form the "images" of one 2-D launch
// (consecutive output slices read overlapping windows of input slices, so the image stride is one slice):
//   d = 1 or k = 1: the k tapped slices are adjacent in memory, i.e. one 2-D convolution with k*C input maps;
//   d > 1, C a multiple of 16: still one launch; the kernel steps over the d - 1 slices between two taps;
//   d > 1 otherwise: one launch per depth tap, each adding to what the previous ones left in the output, the
//          last one applying bias and ReLU.
// The data gradient is the same convolution with every axis of the kernel flipped and the map roles swapped,
// applied to the output gradient padded with zeros: rows and columns are padded by the 2-D kernel's own zero
// padding, the (k-1)*d zero slices before and after are real memory (the gradient of a convolution's output is
// written into the interior of a buffer whose border slices are cleared).  The weight gradient of depth tap a
// is the 2-D weight gradient between the output gradient and the input slices shifted by a*d; with a power-of-two
// map count (or d = 1) all taps are one launch over the k*C (tap, map) input maps, else one launch per tap.
// The 2-D kernels are used unchanged; nothing here is a separate 3-D multiplication.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <new>

#include "sk_host.h"

using namespace skh;

namespace {

struct Dims3 {
    int c = 0, dz = 0, h = 0, w = 0;
    long slice() const { return (long)c * h * w; }
    long count() const { return slice() * dz; }
};

// the depth taps [a0, a0 + len) of one 3-D convolution as a 2-D convolution with len * (maps per slice) input maps
struct TapRun {
    int a0 = 0, len = 0, rows = 0;
    float *wp = nullptr;
};

struct Conv3 {
    int c_in = 0, c_out = 0, k = 1, d = 1;
    int n_pad = 0, n_pad_bwd = 0;
    std::vector<float> w, b;           // host master, [c_out][c_in][k][k][k] and [c_out]
    float *w_dev = nullptr, *b_dev = nullptr;   // device master (b_dev: n_pad entries, zero padded)
    std::vector<TapRun> fwd, bwd;      // bwd: runs over the flipped taps, for the data gradient
    void *wp16 = nullptr;              // 16-bit nets: the kernel as a 2-D convolution over k * 8*ceil(c_in/8) input maps, packed MFMA fragments
    void *wp16_bwd = nullptr;          // ... and its data gradient: a 2-D convolution over k * 8*ceil(c_out/8) maps of the zero-padded gradient
    float *exp2d = nullptr;            // fp32 staging of the two 2-D masters these are packed from
    float *dw = nullptr, *db = nullptr, *vw = nullptr, *vb = nullptr, *dw_tap = nullptr;
    // weight gradient of all depth taps in one launch: k > 1 and (d = 1, the tapped slices adjacent, or a power-of-two
    // map count, which the kernel's grouped addressing needs); 16-bit storage: whole octets per tap, where the grouped
    // form of the 16-bit gradient takes the shape
    bool wgrad_merged = false;
    long wcount() const { return (long)c_out * c_in * k * k * k; }
};

std::vector<TapRun> make_runs(int k, int d, int maps)
{
    // one run when the tapped slices are adjacent in memory, or the kernel can step over the d - 1 slices
    // between two taps
    const bool merged = d == 1 || k == 1 || sk::conv_f32_groups_supported(k, d, maps);
    std::vector<TapRun> runs;
    for (int a0 = 0; a0 < k; a0 += merged ? k : 1) {
        TapRun r;
        r.a0 = a0; r.len = merged ? k : 1;
        r.rows = round_up(r.len * maps, 16) * k * k;
        runs.push_back(r);
    }
    return runs;
}

void release_conv3(Conv3 &c)
{
    free_dev(c.w_dev); free_dev(c.b_dev);
    if (c.wp16) { (void)hipFree(c.wp16); c.wp16 = nullptr; }
    if (c.wp16_bwd) { (void)hipFree(c.wp16_bwd); c.wp16_bwd = nullptr; }
    free_dev(c.exp2d);
    for (auto &r : c.fwd) free_dev(r.wp);
    for (auto &r : c.bwd) free_dev(r.wp);
    c.bwd.clear();
    free_dev(c.dw); free_dev(c.db); free_dev(c.vw); free_dev(c.vb); free_dev(c.dw_tap);
}

// rebuild the packed forms from the device master (asynchronous)
sk_status repack_conv3(Conv3 &c, hipStream_t stream)
{
    for (auto &r : c.fwd)
        SK_HIP(sk::launch_pack_weights3d_f32(c.w_dev, r.wp, c.c_out, c.c_in, c.k, r.a0, r.len, 0, r.rows, c.n_pad, stream));
    for (auto &r : c.bwd)
        SK_HIP(sk::launch_pack_weights3d_f32(c.w_dev, r.wp, c.c_out, c.c_in, c.k, r.a0, r.len, 1, r.rows, c.n_pad_bwd, stream));
    return SK_OK;
}

sk_status upload_conv3(Conv3 &c, hipStream_t stream)
{
    SK_HIP(hipMemcpyAsync(c.w_dev, c.w.data(), sizeof(float) * c.wcount(), hipMemcpyHostToDevice, stream));
    std::vector<float> bp(c.n_pad, 0.f);
    std::memcpy(bp.data(), c.b.data(), sizeof(float) * c.c_out);
    SK_HIP(hipMemcpyAsync(c.b_dev, bp.data(), sizeof(float) * c.n_pad, hipMemcpyHostToDevice, stream));
    SK_TRY(repack_conv3(c, stream));
    SK_HIP(hipStreamSynchronize(stream));
    return SK_OK;
}

// 16-bit storage: depth tap a of input map c becomes input map a * 8*ceil(c_in/8) + c of a 2-D convolution (the maps an
// octet pads are zero), packed as the 2-D 16-bit kernels want it; with_bwd: also the data gradient's 2-D convolution
// over the (flipped depth tap, output map) pairs.  Built on the device from the device master (asynchronous).
sk_status repack_conv3_h(Conv3 &c, int dtype, bool with_bwd, hipStream_t stream)
{
    const int c8 = (c.c_in + 7) / 8, o8 = (c.c_out + 7) / 8, kk = c.k * c.k;
    const long fwd_floats = (long)c.c_out * c.k * c8 * 8 * kk, bwd_floats = (long)c.k * o8 * 8 * c.c_in * kk;
    if (!c.exp2d) SK_TRY(alloc_f(&c.exp2d, std::max(fwd_floats, bwd_floats)));
    if (!c.wp16) SK_HIP(hipMalloc(&c.wp16, sizeof(unsigned short) * (size_t)sk::packed_h_elems(c.c_out, c.k * c8, c.k)));
    SK_HIP(sk::launch_expand_taps3d(c.w_dev, c.exp2d, c.c_out, c.c_in, c.k, 0, stream));
    SK_HIP(sk::launch_pack_weights_h(c.exp2d, c.wp16, dtype, c.c_out, c.k * c8 * 8, c.k, 0, 0, stream));
    if (with_bwd) {
        if (!c.wp16_bwd) SK_HIP(hipMalloc(&c.wp16_bwd, sizeof(unsigned short) * (size_t)sk::packed_h_elems(c.c_in, c.k * o8, c.k)));
        SK_HIP(sk::launch_expand_taps3d(c.w_dev, c.exp2d, c.c_out, c.c_in, c.k, 1, stream));
        SK_HIP(sk::launch_pack_weights_h(c.exp2d, c.wp16_bwd, dtype, c.k * o8 * 8, c.c_in, c.k, 1, 0, stream));
    }
    return SK_OK;
}

sk_status upload_conv3_h(Conv3 &c, int dtype, bool with_bwd = false)
{
    SK_TRY(repack_conv3_h(c, dtype, with_bwd, nullptr));
    SK_HIP(hipStreamSynchronize(nullptr));
    return SK_OK;
}

sk_status alloc_conv3(Conv3 &c, bool training, bool needs_dgrad, bool half)
{
    release_conv3(c);
    c.n_pad = round_up(c.c_out, 16);
    c.n_pad_bwd = round_up(c.c_in, 16);
    SK_TRY(alloc_f(&c.w_dev, c.wcount()));
    SK_TRY(alloc_f(&c.b_dev, c.n_pad));
    for (auto &r : c.fwd) SK_TRY(alloc_f(&r.wp, (long)r.rows * c.n_pad));
    if (training) {
        if (needs_dgrad) {
            c.bwd = make_runs(c.k, c.d, c.c_out);
            for (auto &r : c.bwd) SK_TRY(alloc_f(&r.wp, (long)r.rows * c.n_pad_bwd));
        }
        SK_TRY(alloc_f(&c.dw, c.wcount()));
        SK_TRY(alloc_f(&c.db, c.c_out));
        SK_TRY(alloc_f(&c.vw, c.wcount()));
        SK_TRY(alloc_f(&c.vb, c.c_out));
        const int maps8 = (c.c_in + 7) / 8 * 8;
        if (half) c.wgrad_merged = c.k > 1 && sk::wgrad_h_grouped_supported(c.k * maps8, c.c_out, c.k, c.d);
        else c.wgrad_merged = c.k > 1 && (c.d == 1 || (c.c_in & (c.c_in - 1)) == 0);
        SK_TRY(alloc_f(&c.dw_tap, (long)c.c_out * (half && c.wgrad_merged ? maps8 : c.c_in) * c.k * c.k * (c.wgrad_merged ? c.k : 1)));
        SK_HIP(hipMemset(c.vw, 0, sizeof(float) * c.wcount()));
        SK_HIP(hipMemset(c.vb, 0, sizeof(float) * c.c_out));
    }
    return SK_OK;
}

}  // namespace

struct sknet3d {
    std::vector<sk_layer> layers;
    int c_in = 0, n_classes = 0, dtype = SK_F32;
    std::vector<Conv3> convs;
    std::vector<int> conv_of_layer;
    bool planned = false, training = false, forward_done = false, backward_done = false;
    int dz = 0, h = 0, w = 0;
    std::vector<Dims3> dims;       // dims[0] the volume, dims[i+1] the output of layer i
    std::vector<float *> act;      // act[0]: the training plan's copy of the volume, else unused
    std::vector<uint8_t *> tap;    // per layer: winner codes of the pools of a training plan
    bool fuse_head = false;        // last two 1x1x1 convolutions + softmax as one kernel
    float *head_w1p = nullptr, *zero_page = nullptr;
    float *gbuf[2] = {nullptr, nullptr}, *loss_partial = nullptr, *wgrad_scratch = nullptr;
    float *dz_f32 = nullptr;       // 16-bit training plans: the loss kernel's fp32 gradient of the logits
    hipStream_t last_stream = nullptr;
    bool half() const { return dtype != SK_F32; }
    const float *last_volume = nullptr;

    void release_plan()
    {
        for (auto &p : act) free_dev(p);
        act.clear();
        for (auto &t : tap) {
            if (t) (void)hipFree(t);
            t = nullptr;
        }
        tap.clear();
        free_dev(head_w1p); free_dev(zero_page); free_dev(gbuf[0]); free_dev(gbuf[1]); free_dev(loss_partial); free_dev(wgrad_scratch);
        free_dev(dz_f32);
        for (auto &c : convs) release_conv3(c);
        planned = training = forward_done = backward_done = false;
        fuse_head = false;
    }
};

namespace {

sk_status check3(const sknet3d_t *net)
{
    if (!net) return fail(SK_EINVAL, "null net handle");
    return SK_OK;
}

sk_status infer3(const sknet3d *net, int dz, int h, int w, std::vector<Dims3> &dims)
{
    if (dz < 1 || h < 1 || w < 1) return fail(SK_ESHAPE, "volume size %dx%dx%d", dz, h, w);
    Dims3 cur;
    cur.c = net->c_in; cur.dz = dz; cur.h = h; cur.w = w;
    dims.clear();
    dims.push_back(cur);
    for (size_t i = 0; i < net->layers.size(); ++i) {
        const sk_layer &l = net->layers[i];
        const int shrink = (l.k - 1) * l.d;
        if (l.kind == SK_CONV || l.s == 1) {
            cur.dz -= shrink; cur.h -= shrink; cur.w -= shrink;
        } else {
            if (cur.dz % l.k != 0 || cur.h % l.k != 0 || cur.w % l.k != 0)
                return fail(SK_ESHAPE, "layer %zu: pooling needs w mod k = 0 (map %dx%dx%d, k %d)", i, cur.dz, cur.h, cur.w, l.k);
            cur.dz /= l.k; cur.h /= l.k; cur.w /= l.k;
        }
        if (l.kind == SK_CONV) cur.c = l.c_out;
        if (cur.dz < 1 || cur.h < 1 || cur.w < 1) return fail(SK_ESHAPE, "layer %zu: map shrinks below one voxel", i);
        dims.push_back(cur);
    }
    return SK_OK;
}

// the launches of one 3-D convolution (forward, or data gradient on the zero-padded output gradient):
// x: first slice of the input, [*][maps][H][W]; y: [n_img][out_maps][OH][OW]
sk_status run_conv3(const std::vector<TapRun> &runs, const float *x, float *y, const float *bias, const float *mask, int n_img,
                    int maps, int H, int W, int out_maps, int n_pad, int k, int d, int in_off, int OH, int OW, int relu,
                    hipStream_t stream)
{
    const long slice = (long)maps * H * W;
    for (size_t r = 0; r < runs.size(); ++r) {
        const TapRun &run = runs[r];
        const bool last = r + 1 == runs.size();
        sk::ConvF32Args a{};
        a.x = x + (long)run.a0 * d * slice; a.wp = run.wp; a.bias = last ? bias : nullptr; a.mask = mask; a.y = y;
        a.n = n_img; a.c_in = run.len * maps; a.H = H; a.W = W;
        a.c_out = out_maps; a.n_pad = n_pad;
        a.k = k; a.d = d; a.in_off = in_off;
        a.Ho = OH; a.Wo = OW; a.relu = last ? relu : 0;
        a.out_maps = out_maps; a.o_off = 0; a.OH = OH; a.OW = OW;
        a.oy_mul = 1; a.oy_off = 0; a.ox_mul = 1; a.ox_off = 0;
        a.accumulate = r > 0 ? 1 : 0;
        a.x_bstride = slice;
        if (run.len > 1 && d > 1) {
            a.grp_maps = maps;
            a.grp_skip = (long)(d - 1) * slice;
        }
        SK_HIP(sk::launch_conv_f32(a, stream));
    }
    return SK_OK;
}

sk_status run_layer3(sknet3d *net, int li, hipStream_t stream)
{
    const sk_layer &l = net->layers[li];
    const Dims3 &in = net->dims[li], &out = net->dims[li + 1];
    const float *x = li == 0 ? net->last_volume : net->act[li];
    float *y = net->act[li + 1];
    if (net->half()) {
        // 16-bit storage, slice-major octet layout: act[0] holds the converted volume
        const int dt = net->dtype, c8 = (in.c + 7) / 8;
        if (l.kind == SK_MAXPOOL) {
            SK_HIP(sk::launch_maxpool3d_h(net->act[li], y, net->training ? net->tap[li] : nullptr, dt, in.c, in.dz, in.h, in.w, out.dz, out.h,
                                          out.w, l.k, l.d, l.s, stream));
            return SK_OK;
        }
        // one 2-D launch: the output slices are its images (one input slice apart), the (depth tap, octet) pairs its input octets
        const Conv3 &cv = net->convs[net->conv_of_layer[li]];
        const bool last = li == (int)net->layers.size() - 1;        // the last convolution leaves fp32 logits
        sk::ConvHArgs a{};
        a.zeros = net->zero_page;
        a.x = net->act[li]; a.wp = cv.wp16; a.bias = cv.b_dev; a.mask = nullptr; a.y = y; a.dtype = dt;
        a.n = out.dz; a.c8_in = l.k * c8; a.H = in.h; a.W = in.w;
        a.c_out = out.c; a.c8_out = (out.c + 7) / 8;
        a.k = l.k; a.d = l.d; a.in_off = 0; a.Ho = out.h; a.Wo = out.w; a.relu = l.relu; a.out_f32 = last ? 1 : 0;
        a.c8_out_total = (out.c + 7) / 8; a.o8_off = 0; a.OH = out.h; a.OW = out.w;
        a.oy_mul = 1; a.oy_off = 0; a.ox_mul = 1; a.ox_off = 0;
        a.mt = 0;
        if (l.k > 1) a.xb8 = c8;
        if (l.k > 1 && l.d > 1) { a.grp8 = c8; a.skip8 = (l.d - 1) * c8; }
        SK_HIP(sk::launch_conv_h(a, stream));
        return SK_OK;
    }
    if (l.kind == SK_MAXPOOL) {
        SK_HIP(sk::launch_maxpool3d_f32(x, y, net->tap[li], in.c, in.dz, in.h, in.w, out.dz, out.h, out.w, l.k, l.d, l.s, stream));
        return SK_OK;
    }
    const Conv3 &cv = net->convs[net->conv_of_layer[li]];
    return run_conv3(cv.fwd, x, y, cv.b_dev, nullptr, out.dz, in.c, in.h, in.w, out.c, cv.n_pad, l.k, l.d, 0, out.h, out.w, l.relu, stream);
}

// zero slices that surround the gradient of layer li's output while it serves as the input of li's data gradient
int grad_pad(const sknet3d *net, int li)
{
    const sk_layer &l = net->layers[li];
    return (l.kind == SK_CONV && li > 0) ? (l.k - 1) * l.d : 0;
}

}  // namespace

extern "C" {

sk_status sknet3d_create(const sk_layer *layers, int32_t n_layers, int32_t c_in, int32_t n_classes, sknet3d_t **out)
{
    return sknet3d_create_dtype(layers, n_layers, c_in, n_classes, SK_F32, out);
}

sk_status sknet3d_create_dtype(const sk_layer *layers, int32_t n_layers, int32_t c_in, int32_t n_classes, sk_dtype dtype, sknet3d_t **out)
{
    if (!out) return fail(SK_EINVAL, "create: out is null");
    *out = nullptr;
    if (!layers || n_layers < 1 || c_in < 1 || n_classes < 1) return fail(SK_EINVAL, "create: bad arguments");
    if (dtype != SK_F32 && dtype != SK_BF16 && dtype != SK_F16) return fail(SK_EINVAL, "create: unknown dtype");
    sknet3d *net = new (std::nothrow) sknet3d;
    if (!net) return fail(SK_ENOMEM, "create: out of host memory");
    net->c_in = c_in; net->n_classes = n_classes; net->dtype = dtype;
    int maps = c_in;
    for (int i = 0; i < n_layers; ++i) {
        const sk_layer &l = layers[i];
        sk_status bad = SK_OK;
        if (l.kind != SK_CONV && l.kind != SK_MAXPOOL) bad = fail(SK_EINVAL, "layer %d: bad kind", i);
        else if (l.k < 1 || l.d < 1) bad = fail(SK_ESHAPE, "layer %d: k and d must be >= 1", i);
        else if (l.k > 15) bad = fail(SK_EUNSUPPORTED, "layer %d: k > 15", i);
        else if (l.kind == SK_CONV && (l.s != 1 || l.c_out < 1)) bad = fail(SK_ESHAPE, "layer %d: conv needs s = 1 and c_out >= 1", i);
        else if (l.kind == SK_MAXPOOL && !(l.s == 1 || (l.s == l.k && l.d == 1)))
            bad = fail(SK_ESHAPE, "layer %d: pool needs s = 1, or s = k with d = 1", i);
        else if (maps > 65535) bad = fail(SK_EUNSUPPORTED, "layer %d: more than 65535 maps", i);
        else if (dtype != SK_F32 && l.kind == SK_CONV && !sk::conv_h_supported(l.k, l.d, l.c_out))
            bad = fail(SK_EUNSUPPORTED, "layer %d: no 16-bit convolution kernel for k = %d, d = %d, %d maps", i, l.k, l.d, l.c_out);
        if (bad != SK_OK) {
            delete net;
            return bad;
        }
        net->layers.push_back(l);
        if (l.kind == SK_CONV) {
            Conv3 c;
            c.c_in = maps; c.c_out = l.c_out; c.k = l.k; c.d = l.d;
            c.w.assign((size_t)c.wcount(), 0.f);
            c.b.assign((size_t)c.c_out, 0.f);
            c.fwd = make_runs(l.k, l.d, maps);
            net->conv_of_layer.push_back((int)net->convs.size());
            net->convs.push_back(std::move(c));
            maps = l.c_out;
        } else {
            net->conv_of_layer.push_back(-1);
        }
    }
    if (maps != n_classes) {
        delete net;
        return fail(SK_ESHAPE, "create: the last layer has %d maps but n_classes is %d", maps, n_classes);
    }
    *out = net;
    return SK_OK;
}

void sknet3d_destroy(sknet3d_t *net)
{
    if (!net) return;
    net->release_plan();
    delete net;
}

sk_status sknet3d_context(const sknet3d_t *net, int32_t *v)
{
    SK_TRY(check3(net));
    if (!v) return fail(SK_EINVAL, "context: v is null");
    int sum = 0;
    for (const auto &l : net->layers) {
        if (l.kind == SK_MAXPOOL && l.s != 1) return fail(SK_ESHAPE, "context: only defined for nets whose pools have s = 1");
        sum += (l.k - 1) * l.d;
    }
    *v = sum;
    return SK_OK;
}

sk_status sknet3d_infer_shapes(const sknet3d_t *net, int32_t dz, int32_t h, int32_t w, int32_t *dims4)
{
    SK_TRY(check3(net));
    if (!dims4) return fail(SK_EINVAL, "infer_shapes: dims is null");
    std::vector<Dims3> dims;
    SK_TRY(infer3(net, dz, h, w, dims));
    for (size_t i = 0; i < dims.size(); ++i) {
        dims4[4 * i] = dims[i].c; dims4[4 * i + 1] = dims[i].dz; dims4[4 * i + 2] = dims[i].h; dims4[4 * i + 3] = dims[i].w;
    }
    return SK_OK;
}

sk_status sknet3d_num_convs(const sknet3d_t *net, int32_t *count)
{
    SK_TRY(check3(net));
    if (!count) return fail(SK_EINVAL, "num_convs: count is null");
    *count = (int32_t)net->convs.size();
    return SK_OK;
}

sk_status sknet3d_conv_shape(const sknet3d_t *net, int32_t conv_idx, int32_t *shape5)
{
    SK_TRY(check3(net));
    if (!shape5 || conv_idx < 0 || conv_idx >= (int)net->convs.size()) return fail(SK_EINVAL, "conv_shape: bad arguments");
    const Conv3 &c = net->convs[conv_idx];
    shape5[0] = c.c_out; shape5[1] = c.c_in; shape5[2] = shape5[3] = shape5[4] = c.k;
    return SK_OK;
}

sk_status sknet3d_set_weights(sknet3d_t *net, int32_t conv_idx, const float *w_host, const float *b_host)
{
    SK_TRY(check3(net));
    if (!w_host || conv_idx < 0 || conv_idx >= (int)net->convs.size()) return fail(SK_EINVAL, "set_weights: bad arguments");
    Conv3 &c = net->convs[conv_idx];
    std::memcpy(c.w.data(), w_host, sizeof(float) * c.wcount());
    if (b_host) std::memcpy(c.b.data(), b_host, sizeof(float) * c.c_out);
    if (!net->planned) return SK_OK;
    if (net->last_stream) SK_HIP(hipStreamSynchronize(net->last_stream));
    if (!b_host)   // keep the device's current biases (an SGD step may have changed them)
        SK_HIP(hipMemcpy(c.b.data(), c.b_dev, sizeof(float) * c.c_out, hipMemcpyDeviceToHost));
    SK_TRY(upload_conv3(c, nullptr));
    if (net->half()) SK_TRY(upload_conv3_h(c, net->dtype, c.wp16_bwd != nullptr));
    if (net->fuse_head && conv_idx == (int)net->convs.size() - 2) {
        SK_HIP(sk::launch_pack_head_w1(c.w_dev, net->head_w1p, net->dtype, c.c_out, c.c_in, nullptr));
        SK_HIP(hipStreamSynchronize(nullptr));
    }
    return SK_OK;
}

sk_status sknet3d_get_weights(sknet3d_t *net, int32_t conv_idx, float *w_host, float *b_host)
{
    SK_TRY(check3(net));
    if (conv_idx < 0 || conv_idx >= (int)net->convs.size()) return fail(SK_EINVAL, "get_weights: bad index");
    Conv3 &c = net->convs[conv_idx];
    if (net->planned) {   // the device holds the current values
        if (net->last_stream) SK_HIP(hipStreamSynchronize(net->last_stream));
        SK_HIP(hipMemcpy(c.w.data(), c.w_dev, sizeof(float) * c.wcount(), hipMemcpyDeviceToHost));
        SK_HIP(hipMemcpy(c.b.data(), c.b_dev, sizeof(float) * c.c_out, hipMemcpyDeviceToHost));
    }
    if (w_host) std::memcpy(w_host, c.w.data(), sizeof(float) * c.wcount());
    if (b_host) std::memcpy(b_host, c.b.data(), sizeof(float) * c.c_out);
    return SK_OK;
}

sk_status sknet3d_plan(sknet3d_t *net, int32_t dz, int32_t h, int32_t w, int32_t mode)
{
    SK_TRY(check3(net));
    if (mode < 0 || mode > 2) return fail(SK_EINVAL, "plan: mode must be 0 (inference), 1 (training) or 2 (inference, every layer kept)");
    const bool training = mode == 1;
    std::vector<Dims3> dims;
    SK_TRY(infer3(net, dz, h, w, dims));
    const int L = (int)net->layers.size();
    const bool half = net->half();
    for (int i = 0; i <= L; ++i)
        if (dims[i].dz > 65535 || dims[i].h > 65535 || dims[i].count() >= (1L << 40))
            return fail(SK_EUNSUPPORTED, "plan: volume too large");
    if (training)
        for (int i = 0; i < L; ++i) {
            const sk_layer &l = net->layers[i];
            if (l.kind == SK_MAXPOOL && l.s != 1) return fail(SK_EUNSUPPORTED, "plan: training needs pools with s = 1 (layer %d)", i);
            if (l.kind == SK_MAXPOOL && l.k > 6) return fail(SK_EUNSUPPORTED, "plan: training needs pools with k <= 6 (layer %d)", i);
        }
    // keep the host masters (a planned net's masters may have been updated on the device)
    if (net->planned)
        for (int i = 0; i < (int)net->convs.size(); ++i) SK_TRY(sknet3d_get_weights(net, i, nullptr, nullptr));
    net->release_plan();
    net->dz = dz; net->h = h; net->w = w;
    net->dims = dims;
    net->act.assign(L + 1, nullptr);
    net->tap.assign(L, nullptr);
    net->fuse_head = mode == 0 && L >= 2 && net->layers[L - 2].kind == SK_CONV && net->layers[L - 1].kind == SK_CONV &&
                     net->layers[L - 2].k == 1 && net->layers[L - 1].k == 1 && net->layers[L - 2].relu && !net->layers[L - 1].relu &&
                     sk::head_supported(net->dtype, dims[L - 2].c, net->layers[L - 2].c_out, net->layers[L - 1].c_out);
    sk_status st = SK_OK;
    long max_grad = 0;   // largest gradient buffer: an activation plus the zero slices around it
    size_t scratch = 0;
    for (int i = (training || half) ? 0 : 1; i <= L && st == SK_OK; ++i) {
        if (net->fuse_head && i >= L - 1) continue;
        // 16-bit storage: octets (counted in floats), but for the logits of a last convolution, which stay fp32
        const bool f32 = !half || (i == L && net->layers[L - 1].kind == SK_CONV);
        st = alloc_f(&net->act[i], f32 ? dims[i].count() : (long)dims[i].dz * ((dims[i].c + 7) / 8) * dims[i].h * dims[i].w * 4);
    }
    if (st == SK_OK && half) st = alloc_zero_page(&net->zero_page);
    for (int i = 0; i < L && st == SK_OK && training; ++i) {
        const sk_layer &l = net->layers[i];
        // (16-bit storage: error maps in the slice-major octet layout, counted in floats; winner codes one byte per element of it)
        auto slice_floats = [&](const Dims3 &dm) { return half ? (long)((dm.c + 7) / 8) * dm.h * dm.w * 4 : dm.slice(); };
        const long padded = (dims[i + 1].dz + 2L * grad_pad(net, i)) * slice_floats(dims[i + 1]);
        if (padded > max_grad) max_grad = padded;
        if (dims[i].dz * slice_floats(dims[i]) > max_grad) max_grad = dims[i].dz * slice_floats(dims[i]);
        if (l.kind == SK_MAXPOOL) {
            const size_t tap_bytes = half ? (size_t)dims[i + 1].dz * slice_floats(dims[i + 1]) * 2 : (size_t)dims[i + 1].count();
            hipError_t e = hipMalloc(reinterpret_cast<void **>(&net->tap[i]), tap_bytes);
            if (e != hipSuccess) st = fail(SK_ENOMEM, "plan: winner codes: %s", hipGetErrorString(e));
        } else {
            // one launch over all depth taps (k * C input maps) or one per tap: the larger need
            size_t s = std::max(sk::wgrad_f32_scratch_floats(l.c_out, dims[i].c, l.k), sk::wgrad_f32_scratch_floats(l.c_out, l.k * dims[i].c, l.k));
            if (half) s = std::max(s, sk::wgrad_f32_scratch_floats(l.c_out, l.k * ((dims[i].c + 7) / 8 * 8), l.k));
            if (s > scratch) scratch = s;
        }
    }
    for (int i = 0; i < L && st == SK_OK; ++i) {
        if (net->layers[i].kind != SK_CONV) continue;
        Conv3 &c = net->convs[net->conv_of_layer[i]];
        st = alloc_conv3(c, training, i > 0, half);
        if (st == SK_OK) st = upload_conv3(c, nullptr);
        if (st == SK_OK && half) st = upload_conv3_h(c, net->dtype, training && i > 0);
        if (st == SK_OK && half && training && i > 0 && !sk::conv_h_supported(c.k, c.d, c.c_in))
            st = fail(SK_EUNSUPPORTED, "plan: the data gradient of layer %d is not built for 16-bit storage", i);
    }
    if (st == SK_OK && net->fuse_head) {
        Conv3 &c1 = net->convs[net->conv_of_layer[L - 2]];
        st = alloc_f(&net->head_w1p, (sk::head_w1_packed_bytes(net->dtype, c1.c_in, c1.c_out) + 3) / 4);
        if (st == SK_OK) {
            hipError_t e = sk::launch_pack_head_w1(c1.w_dev, net->head_w1p, net->dtype, c1.c_out, c1.c_in, nullptr);
            if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
            if (e != hipSuccess) st = fail(SK_EDEVICE, "plan: packing the head weights failed: %s", hipGetErrorString(e));
        }
    }
    if (st == SK_OK && training) {
        st = alloc_f(&net->gbuf[0], max_grad);
        if (st == SK_OK) st = alloc_f(&net->gbuf[1], max_grad);
        if (st == SK_OK) st = alloc_f(&net->loss_partial, sk::softmax_loss_partials(dims[L].count() / dims[L].c));
        if (st == SK_OK) st = alloc_f(&net->wgrad_scratch, (long)scratch);
        if (st == SK_OK && half) st = alloc_f(&net->dz_f32, dims[L].count());
        if (st == SK_OK && half && net->layers[L - 1].kind != SK_CONV) st = fail(SK_EUNSUPPORTED, "plan: a 16-bit 3-D net must end in a convolution");
    }
    if (st != SK_OK) {
        net->release_plan();
        return st;
    }
    net->planned = true;
    net->training = training;
    st = warm_up(dims[0].count(), dims[L].count(), training ? dims[L].count() / dims[L].c : 0,
                 [&](const float *vol, float *prob) { return sknet3d_forward(net, vol, prob, nullptr); },
                 [&](const int32_t *lab, float *loss) { return sknet3d_backward(net, lab, loss, nullptr); });
    net->forward_done = net->backward_done = false;
    net->last_volume = nullptr;
    if (st != SK_OK) net->release_plan();
    return st;
}

sk_status sknet3d_forward(sknet3d_t *net, const float *volume_dev, float *prob_dev, void *hip_stream)
{
    SK_TRY(check3(net));
    if (!volume_dev || !prob_dev) return fail(SK_EINVAL, "forward: null buffer");
    if (!net->planned) return fail(SK_ESTATE, "forward: call sknet3d_plan first");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    net->last_stream = stream;
    net->last_volume = volume_dev;
    if (net->training && !net->half()) {   // the backward pass reads the volume again: keep a copy (16-bit plans convert it into act[0] anyway)
        SK_HIP(hipMemcpyAsync(net->act[0], volume_dev, sizeof(float) * net->dims[0].count(), hipMemcpyDeviceToDevice, stream));
        net->last_volume = net->act[0];
    }
    const int L = (int)net->layers.size();
    if (net->half()) {
        const Dims3 &d0 = net->dims[0];
        SK_HIP(sk::launch_pad_pack_h(volume_dev, net->act[0], net->dtype, d0.dz, d0.c, d0.h, d0.w, 0, 0, d0.h, d0.w, 0, stream));
    }
    for (int i = 0; i < (net->fuse_head ? L - 2 : L); ++i) SK_TRY(run_layer3(net, i, stream));
    const Dims3 &o = net->dims[L];
    if (net->fuse_head) {
        const Conv3 &c1 = net->convs[net->conv_of_layer[L - 2]], &c2 = net->convs[net->conv_of_layer[L - 1]];
        const Dims3 &in = net->dims[L - 2];
        sk::HeadArgs a{};
        a.x = (L - 2 == 0 && !net->half()) ? volume_dev : net->act[L - 2];
        a.w1p = net->head_w1p; a.b1 = c1.b_dev; a.w2 = c2.w_dev; a.b2 = c2.b_dev;
        a.prob = prob_dev; a.dtype = net->dtype; a.n = in.dz; a.c_in = in.c; a.H = in.h; a.W = in.w;
        a.hidden = c1.c_out; a.classes = c2.c_out;
        SK_HIP(sk::launch_head_fused(a, stream));
    } else {
        if (net->half() && net->layers[L - 1].kind != SK_CONV) return fail(SK_EUNSUPPORTED, "forward: a 16-bit 3-D net must end in a convolution");
        SK_HIP(sk::launch_softmax_f32(net->act[L], prob_dev, o.dz, o.c, o.h * o.w, stream));
    }
    net->forward_done = true;
    net->backward_done = false;
    return SK_OK;
}

// The backward pass in 16-bit storage: error maps in the slice-major octet layout (fp32 sums in every kernel, fp32 weight
// gradients).  A convolution's weight gradient is one 2-D launch per depth tap (the input slices shifted by a*d against
// the output gradient); its data gradient is ONE 2-D launch over the (flipped depth tap, map) pairs of the gradient, which
// sits between (k-1)d cleared slices, with the ReLU mask of the layer below in the epilogue.
static sk_status backward3_h(sknet3d *net, const int32_t *labels_dev, float *loss_dev, hipStream_t stream)
{
    const int L = (int)net->layers.size(), dt = net->dtype;
    const Dims3 &o = net->dims[L];
    auto slice_floats = [](const Dims3 &dm) { return (long)((dm.c + 7) / 8) * dm.h * dm.w * 4; };
    float *gcur = net->gbuf[0], *gnext = net->gbuf[1];
    {
        float *dz16 = gcur + (long)grad_pad(net, L - 1) * slice_floats(o);
        const bool masked = net->layers[L - 1].relu != 0;
        const bool direct = !masked && sk::softmax_loss_writes_octets(o.c, o.h * o.w);
        SK_HIP(sk::launch_softmax_loss_f32(net->act[L], labels_dev, net->dz_f32, loss_dev, net->loss_partial, o.dz, o.c, o.h * o.w, stream,
                                           direct ? dz16 : nullptr, direct ? dt : 0));
        if (masked) SK_HIP(sk::launch_relu_mask_f32(net->dz_f32, net->act[L], o.count(), stream));
        if (!direct) SK_HIP(sk::launch_pad_pack_h(net->dz_f32, dz16, dt, o.dz, o.c, o.h, o.w, 0, 0, o.h, o.w, 0, stream));
    }
    for (int li = L - 1; li >= 0; --li) {
        const sk_layer &l = net->layers[li];
        const Dims3 &in = net->dims[li], &out = net->dims[li + 1];
        const int pad = grad_pad(net, li);
        const long in_slice = slice_floats(in), out_slice = slice_floats(out);
        const float *g = gcur + (long)pad * out_slice;        // gradient of this layer's output
        const float *relu_src = (li > 0 && net->layers[li - 1].kind == SK_CONV && net->layers[li - 1].relu) ? net->act[li] : nullptr;
        float *dst = li > 0 ? gnext + (long)grad_pad(net, li - 1) * in_slice : nullptr;
        if (l.kind == SK_CONV) {
            Conv3 &c = net->convs[net->conv_of_layer[li]];
            if (c.wgrad_merged) {
                // all depth taps in one launch: the (tap, octet) pairs are the input octets, as in the forward pass
                const int i8 = (in.c + 7) / 8;
                SK_HIP(sk::launch_wgrad_h_grouped(net->act[li], g, c.dw_tap, c.db, net->wgrad_scratch, dt, out.dz, l.k * i8 * 8, in.h, in.w, c.c_out,
                                                  l.k, l.d, i8, l.d > 1 ? i8 * 8 : 0, (l.d - 1) * i8, stream));
                SK_HIP(sk::launch_place_taps_f32(c.dw_tap, c.dw, c.c_out, c.c_in, l.k, stream, i8 * 8));
            } else {
                for (int a = 0; a < l.k; ++a) {
                    SK_HIP(sk::launch_wgrad_h(net->act[li] + (long)a * l.d * in_slice, g, c.dw_tap, a + 1 == l.k ? c.db : nullptr,
                                              net->wgrad_scratch, dt, out.dz, in.c, in.h, in.w, c.c_out, l.k, l.d, stream, 0, net->zero_page));
                    SK_HIP(sk::launch_place_tap_f32(c.dw_tap, c.dw, (long)c.c_out * c.c_in, l.k, a, stream));
                }
            }
            if (li == 0) break;   // nothing below needs the volume's gradient
            if (pad > 0) {
                SK_HIP(sk::launch_fill_f32(gcur, 0.f, (long)pad * out_slice, stream));
                SK_HIP(sk::launch_fill_f32(gcur + (long)(pad + out.dz) * out_slice, 0.f, (long)pad * out_slice, stream));
            }
            const int o8 = (out.c + 7) / 8;
            sk::ConvHArgs a{};
            a.zeros = net->zero_page;
            a.x = gcur; a.wp = c.wp16_bwd; a.bias = nullptr; a.mask = relu_src; a.y = dst; a.dtype = dt;
            a.n = in.dz; a.c8_in = l.k * o8; a.H = out.h; a.W = out.w;
            a.c_out = in.c; a.c8_out = (in.c + 7) / 8;
            a.k = l.k; a.d = l.d; a.in_off = (l.k - 1) * l.d; a.Ho = in.h; a.Wo = in.w; a.relu = 0; a.out_f32 = 0;
            a.c8_out_total = (in.c + 7) / 8; a.o8_off = 0; a.OH = in.h; a.OW = in.w;
            a.oy_mul = 1; a.oy_off = 0; a.ox_mul = 1; a.ox_off = 0;
            a.mt = 0;
            if (l.k > 1) a.xb8 = o8;
            if (l.k > 1 && l.d > 1) { a.grp8 = o8; a.skip8 = (l.d - 1) * o8; }
            SK_HIP(sk::launch_conv_h(a, stream));
        } else {
            if (li == 0) break;
            SK_HIP(sk::launch_maxpool3d_bwd_h(g, net->tap[li], relu_src, dst, dt, in.c, in.dz, in.h, in.w, out.dz, out.h, out.w, l.k, l.d, stream));
        }
        float *t = gcur; gcur = gnext; gnext = t;
    }
    return SK_OK;
}

sk_status sknet3d_backward(sknet3d_t *net, const int32_t *labels_dev, float *loss_dev, void *hip_stream)
{
    SK_TRY(check3(net));
    if (!net->planned || !net->training) return fail(SK_ESTATE, "backward: needs a training plan");
    if (!net->forward_done) return fail(SK_ESTATE, "backward: run sknet3d_forward first");
    if (!labels_dev || !loss_dev) return fail(SK_EINVAL, "backward: null buffer");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    net->last_stream = stream;
    const int L = (int)net->layers.size();
    const Dims3 &o = net->dims[L];
    float *gcur = net->gbuf[0], *gnext = net->gbuf[1];
    if (net->half()) {
        SK_TRY(backward3_h(net, labels_dev, loss_dev, stream));
        net->backward_done = true;
        return SK_OK;
    }
    {
        float *dz = gcur + (long)grad_pad(net, L - 1) * o.slice();
        SK_HIP(sk::launch_softmax_loss_f32(net->act[L], labels_dev, dz, loss_dev, net->loss_partial, o.dz, o.c, o.h * o.w, stream));
        if (net->layers[L - 1].kind == SK_CONV && net->layers[L - 1].relu) SK_HIP(sk::launch_relu_mask_f32(dz, net->act[L], o.count(), stream));
    }
    for (int li = L - 1; li >= 0; --li) {
        const sk_layer &l = net->layers[li];
        const Dims3 &in = net->dims[li], &out = net->dims[li + 1];
        const int pad = grad_pad(net, li);
        const float *g = gcur + (long)pad * out.slice();       // gradient of this layer's output
        // ReLU of the layer below acts on this layer's input
        const float *relu_src = (li > 0 && net->layers[li - 1].kind == SK_CONV && net->layers[li - 1].relu) ? net->act[li] : nullptr;
        float *dst = li > 0 ? gnext + (long)grad_pad(net, li - 1) * in.slice() : nullptr;
        if (l.kind == SK_CONV) {
            Conv3 &c = net->convs[net->conv_of_layer[li]];
            if (c.wgrad_merged) {
                // all depth taps in one launch: the (tap, map) pairs are the input maps, as in the forward pass
                SK_HIP(sk::launch_wgrad_f32_grouped(net->act[li], g, c.dw_tap, c.db, net->wgrad_scratch, out.dz, l.k * in.c, in.h, in.w,
                                                    c.c_out, l.k, l.d, in.slice(), l.d > 1 ? in.c : 0, (long)(l.d - 1) * in.slice(), stream));
                SK_HIP(sk::launch_place_taps_f32(c.dw_tap, c.dw, c.c_out, c.c_in, l.k, stream));
            } else {
                for (int a = 0; a < l.k; ++a) {   // depth tap a: the input slices shifted by a*d against the output gradient
                    SK_HIP(sk::launch_wgrad_f32(net->act[li] + (long)a * l.d * in.slice(), g, c.dw_tap, a + 1 == l.k ? c.db : nullptr,
                                                net->wgrad_scratch, out.dz, in.c, in.h, in.w, c.c_out, l.k, l.d, stream));
                    SK_HIP(sk::launch_place_tap_f32(c.dw_tap, c.dw, (long)c.c_out * c.c_in, l.k, a, stream));
                }
            }
            if (li == 0) break;   // nothing below needs the volume's gradient
            if (pad > 0) {
                SK_HIP(sk::launch_fill_f32(gcur, 0.f, (long)pad * out.slice(), stream));
                SK_HIP(sk::launch_fill_f32(gcur + (long)(pad + out.dz) * out.slice(), 0.f, (long)pad * out.slice(), stream));
            }
            const bool one = c.bwd.size() == 1;
            SK_TRY(run_conv3(c.bwd, gcur, dst, nullptr, one ? relu_src : nullptr, in.dz, out.c, out.h, out.w, in.c, c.n_pad_bwd, l.k,
                             l.d, (l.k - 1) * l.d, in.h, in.w, 0, stream));
            if (!one && relu_src) SK_HIP(sk::launch_relu_mask_f32(dst, relu_src, in.count(), stream));
        } else {
            if (li == 0) break;
            SK_HIP(sk::launch_maxpool3d_bwd_f32(g, net->tap[li], relu_src, dst, in.c, in.dz, in.h, in.w, out.dz, out.h, out.w, l.k, l.d,
                                                stream));
        }
        float *t = gcur; gcur = gnext; gnext = t;
    }
    net->backward_done = true;
    return SK_OK;
}

sk_status sknet3d_sgd_step(sknet3d_t *net, float lr, float momentum, float weight_decay, void *hip_stream)
{
    SK_TRY(check3(net));
    if (!net->planned || !net->training || !net->backward_done) return fail(SK_ESTATE, "sgd_step: needs a backward pass on a training plan");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    net->last_stream = stream;
    sk::SgdBatch sb{};
    for (auto &c : net->convs) {
        if (sb.n + 2 > sk::BATCH_MAX) {
            SK_HIP(sk::launch_sgd_batch_f32(sb, lr, momentum, weight_decay, stream));
            sb = sk::SgdBatch{};
        }
        sb.w[sb.n] = c.w_dev; sb.dw[sb.n] = c.dw; sb.v[sb.n] = momentum != 0.f ? c.vw : nullptr; sb.count[sb.n] = c.wcount(); ++sb.n;
        sb.w[sb.n] = c.b_dev; sb.dw[sb.n] = c.db; sb.v[sb.n] = momentum != 0.f ? c.vb : nullptr; sb.count[sb.n] = c.c_out; ++sb.n;
    }
    if (sb.n > 0) SK_HIP(sk::launch_sgd_batch_f32(sb, lr, momentum, weight_decay, stream));
    for (auto &c : net->convs) SK_TRY(repack_conv3(c, stream));
    if (net->half())
        for (auto &c : net->convs) SK_TRY(repack_conv3_h(c, net->dtype, c.wp16_bwd != nullptr, stream));
    return SK_OK;
}

sk_status sknet3d_get_grad(sknet3d_t *net, int32_t conv_idx, float *dw_host, float *db_host)
{
    SK_TRY(check3(net));
    if (conv_idx < 0 || conv_idx >= (int)net->convs.size()) return fail(SK_EINVAL, "get_grad: bad index");
    if (!net->backward_done) return fail(SK_ESTATE, "get_grad: no backward pass yet");
    Conv3 &c = net->convs[conv_idx];
    SK_HIP(hipStreamSynchronize(net->last_stream));
    if (dw_host) SK_HIP(hipMemcpy(dw_host, c.dw, sizeof(float) * c.wcount(), hipMemcpyDeviceToHost));
    if (db_host) SK_HIP(hipMemcpy(db_host, c.db, sizeof(float) * c.c_out, hipMemcpyDeviceToHost));
    return SK_OK;
}

sk_status sknet3d_get_activation(sknet3d_t *net, int32_t layer_idx, float *dchw_host)
{
    SK_TRY(check3(net));
    if (!dchw_host || layer_idx < 0 || layer_idx >= (int)net->layers.size()) return fail(SK_EINVAL, "get_activation: bad arguments");
    if (!net->forward_done) return fail(SK_ESTATE, "get_activation: no forward pass yet");
    if (net->fuse_head && layer_idx >= (int)net->layers.size() - 2)
        return fail(SK_ESTATE, "get_activation: this plan fuses the last two layers; plan with mode 2 to keep them");
    const Dims3 &dm = net->dims[layer_idx + 1];
    if (net->half() && !(layer_idx == (int)net->layers.size() - 1 && net->layers[layer_idx].kind == SK_CONV)) {
        float *tmp = nullptr;
        SK_TRY(alloc_f(&tmp, dm.count()));
        hipError_t e = sk::launch_unpack_h(net->act[layer_idx + 1], tmp, net->dtype, dm.dz, dm.c, dm.h, dm.w, net->last_stream);
        if (e == hipSuccess) e = hipStreamSynchronize(net->last_stream);
        if (e == hipSuccess) e = hipMemcpy(dchw_host, tmp, sizeof(float) * dm.count(), hipMemcpyDeviceToHost);
        free_dev(tmp);
        if (e != hipSuccess) return fail(SK_EDEVICE, "get_activation: %s", hipGetErrorString(e));
        return SK_OK;
    }
    SK_HIP(hipStreamSynchronize(net->last_stream));
    SK_HIP(hipMemcpy(dchw_host, net->act[layer_idx + 1], sizeof(float) * dm.count(), hipMemcpyDeviceToHost));
    return SK_OK;
}

sk_status sknet3d_get_pool_argmax(sknet3d_t *net, int32_t pool_idx, int32_t *idx_host)
{
    SK_TRY(check3(net));
    if (!idx_host || pool_idx < 0) return fail(SK_EINVAL, "get_pool_argmax: bad arguments");
    if (!net->planned || !net->training || !net->forward_done) return fail(SK_ESTATE, "get_pool_argmax: needs a forward pass on a training plan");
    int li = -1, seen = 0;
    for (int i = 0; i < (int)net->layers.size(); ++i)
        if (net->layers[i].kind == SK_MAXPOOL && seen++ == pool_idx) li = i;
    if (li < 0) return fail(SK_EINVAL, "get_pool_argmax: the net has no pool number %d", pool_idx);
    const sk_layer &l = net->layers[li];
    const Dims3 &in = net->dims[li], &out = net->dims[li + 1];
    if ((long)in.dz * in.h * in.w > 0x7fffffffL) return fail(SK_EUNSUPPORTED, "get_pool_argmax: offsets exceed 32 bits");
    int32_t *tmp = nullptr;
    SK_HIP(hipMalloc(reinterpret_cast<void **>(&tmp), sizeof(int32_t) * (size_t)out.count()));
    hipError_t e = net->half() ? sk::launch_tap3d_to_index_h(net->tap[li], tmp, out.c, out.dz, out.h, out.w, in.h, in.w, l.k, l.d, l.s, net->last_stream)
                               : sk::launch_tap3d_to_index(net->tap[li], tmp, out.c, out.dz, out.h, out.w, in.h, in.w, l.k, l.d, l.s, net->last_stream);
    if (e == hipSuccess) e = hipStreamSynchronize(net->last_stream);
    if (e == hipSuccess) e = hipMemcpy(idx_host, tmp, sizeof(int32_t) * (size_t)out.count(), hipMemcpyDeviceToHost);
    (void)hipFree(tmp);
    if (e != hipSuccess) return fail(SK_EDEVICE, "get_pool_argmax: %s", hipGetErrorString(e));
    return SK_OK;
}

}  // extern "C"
