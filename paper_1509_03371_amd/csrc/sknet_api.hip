// Host side of libsknet: handles, Algorithm 1, shape inference, workspace planning and the
// per-layer launch sequences.  See include/sknet.h for the contract of every entry point.
#include <hip/hip_runtime.h>

#include <mutex>
#include <new>

#include "sk_host.h"

using namespace skh;

// Scratch of sknet_backward_noalloc: the partial results of one backward pass (the loss kernel's partial sums and
// counts, then the private copies and bias partials of one weight gradient at a time).  One array per GPU, held
// from the moment the library's code is loaded on that GPU until the process ends.  Host code never uses this
// name as an address: it asks the runtime for the array's device address once per device (static_scratch below).
constexpr size_t kStaticScratchFloats = (size_t)8 << 20;          // 32 MiB
constexpr size_t kStaticLossFloats = 4096;                         // its first part: the loss partials
static __device__ __align__(256) float scratch[kStaticScratchFloats];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float *g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device, looked up on first use there
sk_status static_scratch(float **out)
{
    int dev = -1;
    SK_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(SK_EDEVICE, "device ordinal %d is beyond the %d this library keeps scratch for", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        SK_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(SK_EDEVICE, "hipGetSymbolAddress returned no address for the static scratch");
        g_scratch_ptr[dev] = static_cast<float *>(p);
    }
    *out = g_scratch_ptr[dev];
    return SK_OK;
}
}  // namespace

// ================================================================================ SK-Net handle
struct sknet {
    std::vector<sk_layer> layers;
    int c_in = 0, n_classes = 0, dtype = 0, pad_mode = 0;
    std::vector<ConvParams> convs;
    std::vector<int> conv_of_layer;   // layer -> conv index or -1
    // plan
    bool planned = false;
    int n = 0, h = 0, w = 0, pad = 0, training = 0;
    int pad_top = 0, pad_left = 0;
    std::vector<Dims> dims;           // dims[0] padded image, dims[i+1] output of layer i
    std::vector<float *> act;         // same indexing
    std::vector<uint8_t *> tap;       // per layer (pools on a training plan), else nullptr
    bool image_direct = false;        // 16-bit inference plans: the first layer reads the caller's image (no padded copy is made)
    float *gbuf[2] = {nullptr, nullptr};
    float *loss_partial = nullptr, *wgrad_scratch = nullptr;
    // forward schedule of the plan: kind 0 = pad / convert, 1 = layer `arg`, 2 = softmax, 3 = fused head
    struct Step { int kind, arg; };
    std::vector<Step> steps;
    bool fuse_head = false;           // inference plans: last two 1x1 convs + softmax run as one kernel
    // 16-bit inference plans: an SK pool (k = 2, s = 1, the d of the convolution in front of it) runs inside its two
    // neighbours -- the convolution stores max(Y[y], Y[y + d]) (vpool[layer] = 1, its buffer then holds H - d rows of
    // W columns), the layer after the pool reads max(X[x], X[x + d]) (pending[layer] = d; the fused head: pending_head)
    std::vector<int> vpool, pending;
    int pending_head = 0;
    bool kept(int layer) const        // is the output of `layer` in memory in the form the layer defines?
    {
        if (fuse_head && layer >= (int)layers.size() - 2) return false;
        if (vpool.empty()) return true;
        if (vpool[layer]) return false;
        return !(layer > 0 && vpool[layer - 1]);
    }
    float *head_w1p = nullptr;
    float *logits_f32 = nullptr;      // 16-bit nets: fp32 logits when the last layer is a pool; else alias of act[L]
    float *dz_f32 = nullptr;          // 16-bit training: fp32 gradient of the logits before it is packed
    float *zero_page = nullptr;       // 16-bit nets: zeros the convolution reads for samples outside the image
    bool half() const { return dtype != SK_F32; }
    bool forward_done = false, backward_done = false;
    hipStream_t last_stream = nullptr;
    const float *last_image = nullptr;
    float *last_prob = nullptr;

    void release_plan()
    {
        for (auto &p : act) free_dev(p);
        act.clear();
        for (auto &t : tap) {
            if (t) (void)hipFree(t);
            t = nullptr;
        }
        tap.clear();
        free_dev(gbuf[0]); free_dev(gbuf[1]); free_dev(loss_partial); free_dev(wgrad_scratch);
        free_dev(logits_f32); free_dev(dz_f32); free_dev(head_w1p); free_dev(zero_page);
        steps.clear();
        vpool.clear(); pending.clear(); pending_head = 0;
        fuse_head = false;
        for (auto &c : convs) release_conv(c);
        planned = forward_done = backward_done = false;
    }
};

namespace {

// sizes of every map for an h x w image; shared by infer_shapes and plan
sk_status infer(const sknet *net, int h, int w, int pad, std::vector<Dims> &dims, int *pt, int *pl)
{
    int v = 0;
    bool stride1 = true;
    for (const auto &l : net->layers) {
        v += (l.k - 1) * l.d;
        if (l.kind == SK_MAXPOOL && l.s != 1) stride1 = false;
    }
    Dims cur;
    cur.c = net->c_in; cur.h = h; cur.w = w;
    int top = 0, left = 0;
    if (pad) {
        if (!stride1) return fail(SK_ESHAPE, "context padding is only defined for nets whose pools have s = 1");
        top = left = (v + 1) / 2;
        const int bottom = v / 2;
        const int limit_h = net->pad_mode == 0 ? h - 1 : h, limit_w = net->pad_mode == 0 ? w - 1 : w;
        if (top > limit_h || top > limit_w || bottom > limit_h)
            return fail(SK_ESHAPE, "mirror border %d does not fit a %dx%d image", top, h, w);
        cur.h = h + v; cur.w = w + v;
    }
    if (h < 1 || w < 1) return fail(SK_ESHAPE, "image size %dx%d", h, w);
    dims.clear();
    dims.push_back(cur);
    for (size_t i = 0; i < net->layers.size(); ++i) {
        const sk_layer &l = net->layers[i];
        const int shrink = (l.k - 1) * l.d;
        if (l.kind == SK_CONV || l.s == 1) {
            cur.h -= shrink; cur.w -= shrink;
        } else {   // down-sampling pool, s = k, d = 1
            if (cur.h % l.k != 0 || cur.w % l.k != 0)
                return fail(SK_ESHAPE, "layer %zu: pooling needs w mod k = 0 (map %dx%d, k %d)", i, cur.h, cur.w, l.k);
            cur.h /= l.k; cur.w /= l.k;
        }
        if (l.kind == SK_CONV) cur.c = l.c_out;
        if (cur.h < 1 || cur.w < 1)
            return fail(SK_ESHAPE, "layer %zu: map shrinks below one pixel", i);
        dims.push_back(cur);
    }
    if (pt) *pt = top;
    if (pl) *pl = left;
    return SK_OK;
}

sk_status check_net(const sknet_t *net)
{
    if (!net) return fail(SK_EINVAL, "null net handle");
    return SK_OK;
}

// forward step `step`: 0 = pad/copy, 1..L = layers, L+1 = softmax
sk_status run_forward_step(sknet *net, int step_idx, hipStream_t stream)
{
    const int L = (int)net->layers.size();
    const bool half = net->half();
    const sknet::Step st = net->steps[step_idx];
    if (st.kind == 3) {   // fused head on the input of layer L-2
        const ConvParams &c1 = net->convs[net->conv_of_layer[L - 2]], &c2 = net->convs[net->conv_of_layer[L - 1]];
        const Dims &in = net->dims[L - 2];
        sk::HeadArgs a{};
        a.x = net->pending_head ? net->act[L - 3] : net->act[L - 2];    // a pending pool: the buffer of the convolution before it
        a.hd = net->pending_head;
        a.w1p = net->head_w1p; a.b1 = c1.b_dev; a.w2 = c2.w_dev; a.b2 = c2.b_dev;
        a.prob = net->last_prob; a.dtype = net->dtype; a.n = net->n; a.c_in = in.c; a.H = in.h; a.W = in.w;
        a.hidden = c1.c_out; a.classes = c2.c_out;
        SK_HIP(sk::launch_head_fused(a, stream));
        return SK_OK;
    }
    const int step = st.kind == 0 ? 0 : (st.kind == 1 ? st.arg + 1 : L + 1);
    if (step == 0) {
        const Dims &d0 = net->dims[0];
        if (half && net->image_direct) return SK_OK;   // the first layer pads and converts the image itself
        if (half)   // mirror padding fused into the conversion to the 16-bit octet layout
            SK_HIP(sk::launch_pad_pack_h(net->last_image, net->act[0], net->dtype, net->n, net->c_in, net->h, net->w,
                                         net->pad ? net->pad_top : 0, net->pad ? net->pad_left : 0, d0.h, d0.w,
                                         net->pad_mode, stream));
        else if (net->pad)
            SK_HIP(sk::launch_mirror_pad_f32(net->last_image, net->act[0], net->n * net->c_in, net->h, net->w,
                                             net->pad_top, net->pad_left, d0.h, d0.w, net->pad_mode, stream));
        else
            SK_HIP(hipMemcpyAsync(net->act[0], net->last_image, sizeof(float) * d0.count(net->n),
                                  hipMemcpyDeviceToDevice, stream));
        return SK_OK;
    }
    if (step <= L) {
        const int li = step - 1;
        const sk_layer &l = net->layers[li];
        const Dims &in = net->dims[li], &out = net->dims[li + 1];
        if (l.kind == SK_CONV) {
            const ConvParams &c = net->convs[net->conv_of_layer[li]];
            if (half) {
                const int hd = net->pending[li];
                sk::ConvHArgs a = conv_h_args(c, net->dtype, hd ? net->act[li - 1] : net->act[li], net->n, in, l.d, l.relu, net->act[li + 1], out,
                                              li == L - 1, net->zero_page);   // the last conv writes fp32 logits
                a.hd = hd;
                if (li == 0 && net->image_direct) {
                    a.x = nullptr;
                    a.img = net->last_image; a.img_h = net->h; a.img_w = net->w;
                    a.pad_top = net->pad ? net->pad_top : 0; a.pad_left = net->pad ? net->pad_left : 0; a.pad_mode = net->pad_mode;
                }
                if (net->vpool[li]) {
                    a.vpool = 1;
                    a.OH = out.h - l.d;
                }
                SK_HIP(sk::launch_conv_h(a, stream));
            } else {
                sk::ConvF32Args a = conv_args(c, net->act[li], net->n, in, l.d, l.relu, net->act[li + 1], out);
                SK_HIP(sk::launch_conv_f32(a, stream));
            }
        } else if (half) {
            SK_HIP(sk::launch_maxpool_h(net->act[li], net->act[li + 1], net->tap[li], net->dtype,
                                        (long)net->n * ((in.c + 7) / 8), in.h, in.w, out.h, out.w, l.k, l.d, l.s, stream));
        } else {
            SK_HIP(sk::launch_maxpool_f32(net->act[li], net->act[li + 1], net->tap[li], net->n * in.c, in.h, in.w,
                                          out.h, out.w, l.k, l.d, l.s, stream));
        }
        return SK_OK;
    }
    const Dims &o = net->dims[L];
    const float *logits = net->act[L];
    if (half && net->layers[L - 1].kind != SK_CONV) {
        SK_HIP(sk::launch_unpack_h(net->act[L], net->logits_f32, net->dtype, net->n, o.c, o.h, o.w, stream));
        logits = net->logits_f32;
    }
    SK_HIP(sk::launch_softmax_f32(logits, net->last_prob, net->n, o.c, o.h * o.w, stream));
    return SK_OK;
}

// does layer i (0-based) store its output as fp32 NCHW?  (always for fp32 nets; for 16-bit nets
// only the last layer when it is a conv: it writes the fp32 logits)
bool stored_f32(const sknet *net, int i)
{
    return !net->half() || (i == (int)net->layers.size() - 1 && net->layers[i].kind == SK_CONV);
}

}  // namespace

// ================================================================================ host-only helpers
extern "C" {

const char *sknet_last_error(void) { return g_last_error.c_str(); }

int64_t sknet_conv_flops(int64_t f_in, int64_t f_out, int64_t k, int64_t w_out)
{
    return f_out * w_out * w_out * (2 * f_in * k * k - 1);
}

// Algorithm 1 (Section 3.3.1) in two passes.  Pass 1 walks the patch-sized maps of the sliding-window net and
// applies the algorithm's checks; what it records per layer is the map size in front of the layer and the
// product of the pooling strides met since the last inner product -- the kernel stride the layer must take so
// that its taps fall on the samples the sliding-window layer would have seen.  Pass 2 writes the SK layers
// and checks that a full-patch input survives them (every SK layer shrinks its map by (k-1)*d).
sk_status sknet_convert_sw(const sw_layer *sw, int32_t n, int32_t w0_sw, sk_layer *sk_out, int32_t *n_out)
{
    if (!sw || !sk_out || !n_out || n < 1 || w0_sw < 1) return fail(SK_EINVAL, "convert_sw: bad arguments");
    std::vector<int> patch_before(n), stride_product(n);
    int patch = w0_sw, pooled = 1;
    for (int i = 0; i < n; ++i) {
        const sw_layer &l = sw[i];
        patch_before[i] = patch;
        stride_product[i] = pooled;
        switch (l.kind) {
        case 0:
            if (l.k < 1) return fail(SK_ESHAPE, "layer %d: k < 1", i);
            patch -= l.k - 1;
            break;
        case 1:
            if (l.k < 1 || l.k != l.s || patch % l.k != 0)
                return fail(SK_ESHAPE, "layer %d: pooling needs w mod k = 0 and k = s (w=%d k=%d s=%d)", i, patch, l.k, l.s);
            patch /= l.k;
            pooled *= l.k;
            break;
        case 2:            // the inner product consumes the whole patch; behind it every map is 1 x 1 again
            patch = 1;
            pooled = 1;
            break;
        default:
            if (l.k > 1) return fail(SK_ESHAPE, "layer %d: only element-wise layers (k = 1) convert unchanged", i);
        }
        if (patch < 1) return fail(SK_ESHAPE, "layer %d: map shrinks below one pixel", i);
    }
    if (pooled != 1) return fail(SK_ESHAPE, "kernel stride is %d after the last layer; it must be 1", pooled);
    int dense = w0_sw, count = 0;
    for (int i = 0; i < n; ++i) {
        const sw_layer &l = sw[i];
        if (l.kind > 2 || l.kind < 0) continue;                      // element-wise layers are not SK layers
        sk_layer o{};
        o.kind = l.kind == 1 ? SK_MAXPOOL : SK_CONV;
        o.k = l.kind == 2 ? patch_before[i] : l.k;                   // an inner product is a convolution over the whole map
        o.d = stride_product[i];
        o.s = 1;
        if (o.kind == SK_CONV) { o.c_out = l.c_out; o.relu = l.relu; }
        dense -= (o.k - 1) * o.d;
        if (dense < 1) return fail(SK_ESHAPE, "layer %d: map shrinks below one pixel", i);
        sk_out[count++] = o;
    }
    *n_out = count;
    return SK_OK;
}

// ================================================================================ SK-Net
sk_status sknet_create(const sk_layer *layers, int32_t n_layers, int32_t c_in, int32_t n_classes,
                       sk_dtype dtype, int32_t pad_mode, sknet_t **out)
{
    if (!out) return fail(SK_EINVAL, "create: out is null");
    *out = nullptr;
    if (!layers || n_layers < 1 || c_in < 1 || n_classes < 1) return fail(SK_EINVAL, "create: bad arguments");
    if (pad_mode != 0 && pad_mode != 1) return fail(SK_EINVAL, "create: pad_mode must be 0 or 1");
    if (dtype != SK_F32 && dtype != SK_BF16 && dtype != SK_F16) return fail(SK_EINVAL, "create: bad dtype");
    sknet *net = new (std::nothrow) sknet;
    if (!net) return fail(SK_ENOMEM, "create: out of host memory");
    net->c_in = c_in; net->n_classes = n_classes; net->dtype = dtype; net->pad_mode = pad_mode;
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
        else if (dtype != SK_F32 && l.kind == SK_CONV && !sk::conv_h_supported(l.k, l.d))
            bad = fail(SK_EUNSUPPORTED, "layer %d: 16-bit convolutions are built for k = 1..8 and 10, with a staged tile of at most 192 columns (k <= 4) or 256 (larger k)", i);
        else if (dtype != SK_F32 && l.kind == SK_CONV && !sk::conv_h_supported(l.k, l.d, l.c_out))
            bad = fail(SK_EUNSUPPORTED, "layer %d: a 16-bit %dx%d convolution to %d maps at d = %d does not fit the LDS tile", i, l.k, l.k, l.c_out, l.d);
        if (bad != SK_OK) {
            delete net;
            return bad;
        }
        net->layers.push_back(l);
        if (l.kind == SK_CONV) {
            ConvParams c;
            c.c_in = maps; c.c_out = l.c_out; c.k = l.k;
            c.w.assign((size_t)c.wcount(), 0.f);
            c.b.assign((size_t)c.c_out, 0.f);
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

void sknet_destroy(sknet_t *net)
{
    if (!net) return;
    net->release_plan();
    delete net;
}

sk_status sknet_context(const sknet_t *net, int32_t *v)
{
    SK_TRY(check_net(net));
    if (!v) return fail(SK_EINVAL, "context: v is null");
    int sum = 0;
    for (const auto &l : net->layers) {
        if (l.kind == SK_MAXPOOL && l.s != 1) return fail(SK_ESHAPE, "context is only defined when every pool has s = 1");
        sum += (l.k - 1) * l.d;
    }
    *v = sum;
    return SK_OK;
}

sk_status sknet_infer_shapes(const sknet_t *net, int32_t h, int32_t w, int32_t pad, int32_t *dims)
{
    SK_TRY(check_net(net));
    if (!dims) return fail(SK_EINVAL, "infer_shapes: dims is null");
    std::vector<Dims> d;
    SK_TRY(infer(net, h, w, pad, d, nullptr, nullptr));
    for (size_t i = 0; i < d.size(); ++i) {
        dims[3 * i] = d[i].c; dims[3 * i + 1] = d[i].h; dims[3 * i + 2] = d[i].w;
    }
    return SK_OK;
}

sk_status sknet_num_convs(const sknet_t *net, int32_t *count)
{
    SK_TRY(check_net(net));
    if (!count) return fail(SK_EINVAL, "num_convs: count is null");
    *count = (int32_t)net->convs.size();
    return SK_OK;
}

sk_status sknet_conv_shape(const sknet_t *net, int32_t conv_idx, int32_t *shape4)
{
    SK_TRY(check_net(net));
    if (!shape4 || conv_idx < 0 || conv_idx >= (int)net->convs.size()) return fail(SK_EINVAL, "conv_shape: bad index");
    const ConvParams &c = net->convs[conv_idx];
    shape4[0] = c.c_out; shape4[1] = c.c_in; shape4[2] = c.k; shape4[3] = c.k;
    return SK_OK;
}

sk_status sknet_set_weights(sknet_t *net, int32_t conv_idx, const float *w_host, const float *b_host)
{
    SK_TRY(check_net(net));
    if (!w_host || conv_idx < 0 || conv_idx >= (int)net->convs.size()) return fail(SK_EINVAL, "set_weights: bad arguments");
    ConvParams &c = net->convs[conv_idx];
    std::memcpy(c.w.data(), w_host, sizeof(float) * c.wcount());
    if (b_host) std::memcpy(c.b.data(), b_host, sizeof(float) * c.c_out);
    if (net->planned) {
        SK_TRY(upload_conv(c, net->training, net->last_stream, net->dtype));
        const int L = (int)net->layers.size();
        if (net->fuse_head && conv_idx == net->conv_of_layer[L - 2]) {
            SK_HIP(sk::launch_pack_head_w1(c.w_dev, net->head_w1p, net->dtype, c.c_out, c.c_in, net->last_stream));
            SK_HIP(hipStreamSynchronize(net->last_stream));
        }
    }
    return SK_OK;
}

sk_status sknet_get_weights(sknet_t *net, int32_t conv_idx, float *w_host, float *b_host)
{
    SK_TRY(check_net(net));
    if (conv_idx < 0 || conv_idx >= (int)net->convs.size()) return fail(SK_EINVAL, "get_weights: bad index");
    ConvParams &c = net->convs[conv_idx];
    if (net->planned) {   // the device copy is the one SGD updates
        SK_HIP(hipStreamSynchronize(net->last_stream));
        SK_HIP(hipMemcpy(c.w.data(), c.w_dev, sizeof(float) * c.wcount(), hipMemcpyDeviceToHost));
        std::vector<float> bp(c.n_pad);
        SK_HIP(hipMemcpy(bp.data(), c.b_dev, sizeof(float) * c.n_pad, hipMemcpyDeviceToHost));
        std::memcpy(c.b.data(), bp.data(), sizeof(float) * c.c_out);
    }
    if (w_host) std::memcpy(w_host, c.w.data(), sizeof(float) * c.wcount());
    if (b_host) std::memcpy(b_host, c.b.data(), sizeof(float) * c.c_out);
    return SK_OK;
}

sk_status sknet_plan(sknet_t *net, int32_t n, int32_t h, int32_t w, int32_t pad, int32_t mode)
{
    SK_TRY(check_net(net));
    if (n < 1) return fail(SK_EINVAL, "plan: n must be >= 1");
    if (mode < 0 || mode > 3)
        return fail(SK_EINVAL, "plan: mode must be 0 (inference), 1 (training), 2 (inference, every layer kept) or 3 (training, head in one kernel)");
    const int training = mode == 1 || mode == 3;
    std::vector<Dims> dims;
    int pt = 0, pl = 0;
    SK_TRY(infer(net, h, w, pad, dims, &pt, &pl));
    const int L = (int)net->layers.size();
    if (training)
        for (int i = 0; i < L; ++i)
            if (net->layers[i].kind == SK_MAXPOOL && net->layers[i].s != 1)
                return fail(SK_EUNSUPPORTED, "plan: training through a down-sampling pool is not built");
    if (training && net->dtype != SK_F32)
        for (int i = 0; i < L; ++i)
            if (net->layers[i].kind == SK_CONV && net->layers[i].k > 4)
                return fail(SK_EUNSUPPORTED, "plan: the 16-bit kernels for k > 4 (layer %d: %dx%d) are forward only; train in fp32", i, net->layers[i].k, net->layers[i].k);
    if (training && net->dtype != SK_F32)
        for (int i = 1; i < L; ++i)      // data gradients: the GEMM's output maps are the layer's input maps (the first layer needs none)
            if (net->layers[i].kind == SK_CONV && !sk::conv_h_supported(net->layers[i].k, net->layers[i].d, dims[i].c))
                return fail(SK_EUNSUPPORTED, "plan: the 16-bit data gradient of layer %d (%dx%d, d = %d, %d input maps) does not fit the LDS tile",
                            i, net->layers[i].k, net->layers[i].k, net->layers[i].d, dims[i].c);
    // keep the host masters (a planned net's masters may have been updated on the device)
    if (net->planned)
        for (int i = 0; i < (int)net->convs.size(); ++i) SK_TRY(sknet_get_weights(net, i, nullptr, nullptr));
    net->release_plan();
    net->n = n; net->h = h; net->w = w; net->pad = pad ? 1 : 0; net->training = training ? 1 : 0;
    net->pad_top = pt; net->pad_left = pl;
    net->dims = dims;
    net->act.assign(L + 1, nullptr);
    net->tap.assign(L, nullptr);
    long max_count = 0;   // largest activation, in floats (16-bit tensors counted in floats as well)
    sk_status st = SK_OK;
    const bool half = net->half();
    net->fuse_head = false;
    if (mode == 0 && L >= 2 && net->layers[L - 2].kind == SK_CONV && net->layers[L - 1].kind == SK_CONV &&
        net->layers[L - 2].k == 1 && net->layers[L - 1].k == 1 && net->layers[L - 2].relu && !net->layers[L - 1].relu &&
        sk::head_supported(net->dtype, dims[L - 2].c, net->layers[L - 2].c_out, net->layers[L - 1].c_out))
        net->fuse_head = true;
    if (mode == 3) {
        // the two 1x1 layers and the loss run as one kernel in both directions: their hidden maps are never stored
        const bool shape_ok = L >= 2 && net->layers[L - 2].kind == SK_CONV && net->layers[L - 1].kind == SK_CONV && net->layers[L - 2].k == 1 &&
                              net->layers[L - 1].k == 1 && net->layers[L - 2].relu && !net->layers[L - 1].relu;
        if (!shape_ok || !half || !sk::head_train_supported(net->dtype, dims[L - 2].c, net->layers[L - 2].c_out, net->layers[L - 1].c_out))
            return fail(SK_EUNSUPPORTED, "plan: mode 3 needs 16-bit storage and a net that ends in 1x1 conv + ReLU, 1x1 conv with at most 48 input maps, "
                                         "208 hidden maps and 4 classes");
        if (L >= 3 && net->layers[L - 3].kind == SK_CONV && net->layers[L - 3].relu)
            return fail(SK_EUNSUPPORTED, "plan: mode 3 needs a pool (or a convolution without ReLU) in front of the head");
        net->fuse_head = true;
    }
    net->vpool.assign(L, 0);
    net->pending.assign(L, 0);
    net->pending_head = 0;
    if (mode == 0 && half) {
        // walk forward; `carry` is the pool distance the next layer still has to apply to its input
        int carry = 0;
        for (int i = 0; i < L; ++i) {
            const sk_layer &l = net->layers[i];
            if (l.kind != SK_CONV) { carry = 0; continue; }
            net->pending[i] = carry;
            carry = 0;
            if (net->fuse_head && i >= L - 2) continue;
            if (i + 2 >= L || !l.relu) continue;
            const sk_layer &pl = net->layers[i + 1], &nl = net->layers[i + 2];
            if (pl.kind != SK_MAXPOOL || pl.k != 2 || pl.s != 1 || pl.d != l.d || nl.kind != SK_CONV) continue;
            const bool self_ok = sk::conv_h_pool_fusable(l.k, l.d, l.c_out, (dims[i].c + 7) / 8, dims[i + 1].h, net->pending[i]);
            bool next_ok;
            if (net->fuse_head && i + 2 == L - 2)
                next_ok = sk::head_takes_pending_pool(net->dtype, dims[L - 2].c, net->layers[L - 1].c_out, l.d);
            else
                next_ok = sk::conv_h_pool_fusable(nl.k, nl.d, nl.c_out, (dims[i + 2].c + 7) / 8, dims[i + 3].h, l.d);
            if (!self_ok || !next_ok) continue;
            net->vpool[i] = 1;
            carry = l.d;
            if (net->fuse_head && i + 2 == L - 2) net->pending_head = l.d;
            ++i;                                       // the pool is spoken for
        }
    }
    // inference plans whose first layer runs on the one-input-map kernel: that kernel reads the caller's image itself
    net->image_direct = false;
    if (mode == 0 && half && net->c_in == 1 && net->layers[0].kind == SK_CONV) {
        const ConvParams &c0 = net->convs[net->conv_of_layer[0]];
        sk::ConvHArgs a0 = conv_h_args(c0, net->dtype, nullptr, n, dims[0], net->layers[0].d, net->layers[0].relu, nullptr, dims[1], L == 1, nullptr);
        if (net->vpool[0]) { a0.vpool = 1; a0.OH = dims[1].h - net->layers[0].d; }
        net->image_direct = sk::conv_h_reads_image(a0);
    }
    net->steps.clear();
    net->steps.push_back({0, 0});
    for (int i = 0; i < (net->fuse_head ? L - 2 : L); ++i)
        if (!(i > 0 && net->vpool[i - 1])) net->steps.push_back({1, i});
    net->steps.push_back({net->fuse_head ? 3 : 2, 0});
    for (int i = 0; i <= L && st == SK_OK; ++i) {
        if (net->fuse_head && i >= L - 1) continue;   // hidden maps and logits never leave the head kernel
        if (i >= 2 && net->vpool[i - 2]) continue;    // the output of a pool that runs inside its neighbours
        const bool f32 = (i == 0) ? !half : stored_f32(net, i - 1);
        const long count = f32 ? dims[i].count(n) : octet_floats(n, dims[i]);
        st = alloc_f(&net->act[i], count);
        if (count > max_count) max_count = count;
    }
    if (st == SK_OK && half && net->layers[L - 1].kind != SK_CONV) st = alloc_f(&net->logits_f32, dims[L].count(n));
    if (st == SK_OK && half) st = alloc_zero_page(&net->zero_page);
    size_t scratch = 0;
    for (int i = 0; i < L && st == SK_OK; ++i) {
        const sk_layer &l = net->layers[i];
        if (l.kind == SK_MAXPOOL && training) {
            const size_t bytes = half ? (size_t)n * ((dims[i + 1].c + 7) / 8) * dims[i + 1].h * dims[i + 1].w * 8
                                      : (size_t)dims[i + 1].count(n);
            hipError_t e = hipMalloc(reinterpret_cast<void **>(&net->tap[i]), bytes);
            if (e != hipSuccess) st = fail(SK_ENOMEM, "plan: hipMalloc of a pool mask failed: %s", hipGetErrorString(e));
        }
        if (l.kind == SK_CONV) {
            ConvParams &c = net->convs[net->conv_of_layer[i]];
            st = alloc_conv(c, training != 0, net->dtype);
            if (st == SK_OK) st = upload_conv(c, training != 0, nullptr, net->dtype);
            const size_t s = sk::wgrad_f32_scratch_floats(c.c_out, c.c_in, c.k);
            if (s > scratch) scratch = s;
        }
    }
    if (training && net->fuse_head) scratch = std::max(scratch, sk::head_train_scratch_floats(dims[L - 2].c, net->layers[L - 2].c_out));
    if (st == SK_OK && net->fuse_head) {
        ConvParams &c1 = net->convs[net->conv_of_layer[L - 2]];
        st = alloc_f(&net->head_w1p, (sk::head_w1_packed_bytes(net->dtype, c1.c_in, c1.c_out) + 3) / 4);
        if (st == SK_OK) {
            hipError_t e = sk::launch_pack_head_w1(c1.w_dev, net->head_w1p, net->dtype, c1.c_out, c1.c_in, nullptr);
            if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
            if (e != hipSuccess) st = fail(SK_EDEVICE, "plan: packing the head weights failed: %s", hipGetErrorString(e));
        }
    }
    if (st == SK_OK && training) {
        float *unused = nullptr;
        st = static_scratch(&unused);        // sknet_backward_noalloc's scratch: its address on this device is looked up here
    }
    if (st == SK_OK && training) {
        st = alloc_f(&net->gbuf[0], max_count);
        if (st == SK_OK) st = alloc_f(&net->gbuf[1], max_count);
        if (st == SK_OK) st = alloc_f(&net->loss_partial, sk::softmax_loss_partials((long)n * dims[L].h * dims[L].w));
        if (st == SK_OK) st = alloc_f(&net->wgrad_scratch, (long)scratch);
        if (st == SK_OK && half) st = alloc_f(&net->dz_f32, dims[L].count(n));
    }
    if (st != SK_OK) {
        std::string keep = g_last_error;
        net->release_plan();
        g_last_error = keep;
        return st;
    }
    net->planned = true;
    net->last_stream = nullptr;
    st = warm_up((long)n * net->c_in * h * w, dims[L].count(n), training ? (long)n * dims[L].h * dims[L].w : 0,
                 [&](const float *img, float *prob) { return sknet_forward(net, img, prob, nullptr); },
                 [&](const int32_t *lab, float *loss) { return sknet_backward(net, lab, loss, nullptr); });
    net->forward_done = net->backward_done = false;
    net->last_image = nullptr; net->last_prob = nullptr;
    if (st != SK_OK) {
        std::string keep = g_last_error;
        net->release_plan();
        g_last_error = keep;
    }
    return st;
}

sk_status sknet_forward(sknet_t *net, const float *image_dev, float *prob_dev, void *hip_stream)
{
    SK_TRY(check_net(net));
    if (!net->planned) return fail(SK_ESTATE, "forward: call sknet_plan first");
    if (!image_dev || !prob_dev) return fail(SK_EINVAL, "forward: null buffer");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    net->last_stream = stream;
    net->last_image = image_dev;
    net->last_prob = prob_dev;
    net->backward_done = false;
    for (int s = 0; s < (int)net->steps.size(); ++s) SK_TRY(run_forward_step(net, s, stream));
    net->forward_done = true;
    return SK_OK;
}

// Backward step of layer li: gcur holds the layer's error map, gnext receives the error map of the layer below
// (with that layer's ReLU mask applied).  parts: bit 0 = the weight and bias gradient of a convolution, bit 1 = the
// gradient of the layer's input (data gradient or pool scatter; never for layer 0, whose input is the image).
static sk_status backward_layer(sknet_t *net, int li, float *gcur, float *gnext, int parts, hipStream_t stream, float *wgrad_scratch,
                                size_t wgrad_cap)
{
    const int n = net->n, dt = net->dtype;
    const bool half = net->half();
    const sk_layer &l = net->layers[li];
    const Dims &in = net->dims[li], &out = net->dims[li + 1];
    // ReLU of the layer below acts on this layer's input: fuse its mask into whatever
    // kernel produces the gradient of that input
    const float *relu_src = (li > 0 && net->layers[li - 1].kind == SK_CONV && net->layers[li - 1].relu) ? net->act[li] : nullptr;
    if (l.kind == SK_CONV) {
        ConvParams &c = net->convs[net->conv_of_layer[li]];
        if (parts & 1) {
            if (half)
                SK_HIP(sk::launch_wgrad_h(net->act[li], gcur, c.dw, c.db, wgrad_scratch, dt, n, in.c, in.h, in.w, c.c_out, c.k, l.d, stream,
                                          wgrad_cap, net->zero_page));
            else
                SK_HIP(sk::launch_wgrad_f32(net->act[li], gcur, c.dw, c.db, wgrad_scratch, n, in.c, in.h, in.w, c.c_out, c.k, l.d, stream,
                                            wgrad_cap));
        }
        if (li == 0 || !(parts & 2)) return SK_OK;   // nothing below layer 0 needs the image gradient
        if (half) {
            sk::ConvHArgs a{};
            a.x = gcur; a.wp = c.wp16_bwd; a.bias = nullptr; a.mask = relu_src; a.y = gnext; a.dtype = dt; a.zeros = net->zero_page;
            a.n = n; a.c8_in = (out.c + 7) / 8; a.H = out.h; a.W = out.w;
            a.c_out = in.c; a.c8_out = (in.c + 7) / 8;
            a.k = c.k; a.d = l.d; a.in_off = (c.k - 1) * l.d; a.Ho = in.h; a.Wo = in.w; a.relu = 0; a.out_f32 = 0;
            a.c8_out_total = (in.c + 7) / 8; a.o8_off = 0; a.OH = in.h; a.OW = in.w;
            a.oy_mul = 1; a.oy_off = 0; a.ox_mul = 1; a.ox_off = 0;
            SK_HIP(sk::launch_conv_h(a, stream));
        } else {
            sk::ConvF32Args a{};
            a.x = gcur; a.wp = c.wp_bwd; a.bias = nullptr; a.mask = relu_src; a.y = gnext;
            a.n = n; a.c_in = out.c; a.H = out.h; a.W = out.w;
            a.c_out = in.c; a.n_pad = c.n_pad_bwd;
            a.k = c.k; a.d = l.d; a.in_off = (c.k - 1) * l.d;
            a.Ho = in.h; a.Wo = in.w; a.relu = 0;
            a.out_maps = in.c; a.o_off = 0; a.OH = in.h; a.OW = in.w;
            a.oy_mul = 1; a.oy_off = 0; a.ox_mul = 1; a.ox_off = 0;
            SK_HIP(sk::launch_conv_f32(a, stream));
        }
        return SK_OK;
    }
    if (li == 0 || !(parts & 2)) return SK_OK;
    if (half)
        SK_HIP(sk::launch_maxpool_bwd_h(gcur, net->tap[li], relu_src, gnext, dt, (long)n * ((in.c + 7) / 8), in.h, in.w, out.h, out.w, l.k,
                                        l.d, stream));
    else
        SK_HIP(sk::launch_maxpool_bwd_f32(gcur, net->tap[li], relu_src, gnext, n * in.c, in.h, in.w, out.h, out.w, l.k, l.d, stream));
    return SK_OK;
}

// The backward pass from the loss down to layer stop_layer (0 = all of it).  With stop_layer > 0 the walk
// ends before layer stop_layer's own step and *grad_at_stop receives the buffer that holds the gradient of
// the loss with respect to that layer's output (after the layer's own ReLU mask), in the storage layout
// of the activations; the weight gradients of the layers below are then not computed.
//
// The partial results of the pass -- the loss kernel's per-workgroup sums and counts, the private copies of
// each weight gradient and the bias partials -- go to loss_partial and wgrad_scratch; wgrad_cap = 0: the
// plan's own buffer (sized for the fastest launch), else the floats wgrad_scratch holds.
static sk_status backward_impl(sknet_t *net, const int32_t *labels_dev, float *loss_dev, hipStream_t stream, int stop_layer,
                               float **grad_at_stop, float *loss_partial, float *wgrad_scratch, size_t wgrad_cap)
{
    const int L = (int)net->layers.size(), n = net->n;
    const Dims &o = net->dims[L];
    float *gcur = net->gbuf[0], *gnext = net->gbuf[1];
    const bool half = net->half();
    const int dt = net->dtype;
    int top = L - 1;                                   // the layer the walk starts at
    if (net->fuse_head) {
        // loss, both 1x1 layers' gradients and the gradient of the head's input in one kernel
        if (grad_at_stop && stop_layer > L - 3) return fail(SK_EUNSUPPORTED, "this plan keeps no gradient inside the head (plan with mode 1)");
        const ConvParams &c1 = net->convs[net->conv_of_layer[L - 2]], &c2 = net->convs[net->conv_of_layer[L - 1]];
        const Dims &in = net->dims[L - 2];
        const long pixels = (long)n * o.h * o.w;
        int *counts = reinterpret_cast<int *>(loss_partial);
        sk::HeadTrainArgs a{};
        SK_HIP(sk::launch_label_count(labels_dev, pixels, o.c, counts, &a.ncounts, stream));
        a.x = net->act[L - 2]; a.w1p = net->head_w1p; a.w1 = c1.w_dev; a.b1 = c1.b_dev; a.w2 = c2.w_dev; a.b2 = c2.b_dev;
        a.labels = labels_dev; a.counts = counts; a.dx = L > 2 ? gcur : nullptr; a.scratch = wgrad_scratch;
        a.dw1 = c1.dw; a.db1 = c1.db; a.dw2 = c2.dw; a.db2 = c2.db; a.loss = loss_dev;
        a.dtype = dt; a.n = n; a.c_in = in.c; a.plane = in.h * in.w; a.hidden = c1.c_out; a.classes = c2.c_out;
        SK_HIP(sk::launch_head_train_bwd(a, wgrad_cap ? wgrad_cap : sk::head_train_scratch_floats(in.c, c1.c_out), stream));
        top = L - 3;
    } else {
        const float *logits = (half && net->layers[L - 1].kind != SK_CONV) ? net->logits_f32 : net->act[L];
        float *dz = half ? net->dz_f32 : gcur;
        const bool masked = net->layers[L - 1].kind == SK_CONV && net->layers[L - 1].relu;
        // 16-bit nets: the loss kernel also writes the gradient in the octet layout the layers below read (when it can)
        const bool direct = half && !masked && sk::softmax_loss_writes_octets(o.c, o.h * o.w);
        SK_HIP(sk::launch_softmax_loss_f32(logits, labels_dev, dz, loss_dev, loss_partial, n, o.c, o.h * o.w, stream, direct ? gcur : nullptr,
                                           direct ? dt : 0));
        if (masked) SK_HIP(sk::launch_relu_mask_f32(dz, net->act[L], o.count(n), stream));
        if (half && !direct) SK_HIP(sk::launch_pad_pack_h(dz, gcur, dt, n, o.c, o.h, o.w, 0, 0, o.h, o.w, 0, stream));
    }
    for (int li = top; li >= 0; --li) {
        if (grad_at_stop && li == stop_layer) {
            *grad_at_stop = gcur;
            return SK_OK;
        }
        SK_TRY(backward_layer(net, li, gcur, gnext, 3, stream, wgrad_scratch, wgrad_cap));
        if (li == 0) break;
        float *t = gcur; gcur = gnext; gnext = t;
    }
    return SK_OK;
}

sk_status sknet_backward(sknet_t *net, const int32_t *labels_dev, float *loss_dev, void *hip_stream)
{
    SK_TRY(check_net(net));
    if (!net->planned || !net->training) return fail(SK_ESTATE, "backward: needs a training plan");
    if (!net->forward_done) return fail(SK_ESTATE, "backward: run sknet_forward first");
    if (!labels_dev || !loss_dev) return fail(SK_EINVAL, "backward: null buffer");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    net->last_stream = stream;
    SK_TRY(backward_impl(net, labels_dev, loss_dev, stream, 0, nullptr, net->loss_partial, net->wgrad_scratch, 0));
    net->backward_done = true;
    return SK_OK;
}

sk_status sknet_backward_noalloc(sknet_t *net, const int32_t *labels_dev, float *loss_dev, void *hip_stream)
{
    SK_TRY(check_net(net));
    if (!net->planned || !net->training) return fail(SK_ESTATE, "backward_noalloc: needs a training plan");
    if (!net->forward_done) return fail(SK_ESTATE, "backward_noalloc: run sknet_forward first");
    if (!labels_dev || !loss_dev) return fail(SK_EINVAL, "backward_noalloc: null buffer");
    // sizes first: the loss partials and one private copy of the largest gradient (plus its bias partials) must fit
    const int L = (int)net->layers.size();
    const size_t loss_floats = (size_t)sk::softmax_loss_partials((long)net->n * net->dims[L].h * net->dims[L].w);
    if (loss_floats > kStaticLossFloats)
        return fail(SK_EUNSUPPORTED, "backward_noalloc: the loss needs %zu floats of scratch, the static buffer keeps %zu for it", loss_floats,
                    kStaticLossFloats);
    const size_t cap = kStaticScratchFloats - kStaticLossFloats;
    if (net->fuse_head && sk::head_train_scratch_floats(net->dims[L - 2].c, net->layers[L - 2].c_out) / 512 > cap)
        return fail(SK_EUNSUPPORTED, "backward_noalloc: the head's sums do not fit the static buffer");
    for (const auto &c : net->convs) {
        const size_t need = sk::wgrad_min_scratch_floats(c.c_out, c.c_in, c.k);
        if (need > cap)
            return fail(SK_EUNSUPPORTED,
                        "backward_noalloc: the %d x %d x %dx%d weight gradient needs %zu floats of scratch, the static buffer holds %zu "
                        "(use sknet_backward, whose scratch belongs to the plan)", c.c_out, c.c_in, c.k, c.k, need, cap);
    }
    float *base = nullptr;
    SK_TRY(static_scratch(&base));
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    net->last_stream = stream;
    // nothing in the scratch has to start at zero: every kernel writes all the partials that its reduction reads
    SK_TRY(backward_impl(net, labels_dev, loss_dev, stream, 0, nullptr, base, base + kStaticLossFloats, cap));
    net->backward_done = true;
    return SK_OK;
}

sk_status sknet_get_activation_grad(sknet_t *net, int32_t layer_idx, const int32_t *labels_dev, float *nchw_host)
{
    SK_TRY(check_net(net));
    const int L = (int)net->layers.size();
    if (!nchw_host || !labels_dev || layer_idx < 0 || layer_idx >= L) return fail(SK_EINVAL, "get_activation_grad: bad arguments");
    if (!net->planned || !net->training || !net->forward_done)
        return fail(SK_ESTATE, "get_activation_grad: needs a forward pass on a training plan");
    hipStream_t stream = net->last_stream;
    float *loss = nullptr, *g = nullptr, *tmp = nullptr;
    SK_TRY(alloc_f(&loss, 1));
    // the walk overwrites the weight gradients of the layers it passes: a later get_grad needs a new backward
    net->backward_done = false;
    sk_status st = backward_impl(net, labels_dev, loss, stream, layer_idx, &g, net->loss_partial, net->wgrad_scratch, 0);
    const Dims &dm = net->dims[layer_idx + 1];
    const long count = dm.count(net->n);
    hipError_t e = hipSuccess;
    if (st == SK_OK && layer_idx == L - 1 && net->half()) g = net->dz_f32;   // the logits' gradient is kept in fp32 beside its packed copy
    const bool f32 = !net->half() || layer_idx == L - 1;
    if (st == SK_OK && !f32) {
        st = alloc_f(&tmp, count);
        if (st == SK_OK) e = sk::launch_unpack_h(g, tmp, net->dtype, net->n, dm.c, dm.h, dm.w, stream);
    }
    if (st == SK_OK && e == hipSuccess) e = hipStreamSynchronize(stream);
    if (st == SK_OK && e == hipSuccess) e = hipMemcpy(nchw_host, f32 ? g : tmp, sizeof(float) * (size_t)count, hipMemcpyDeviceToHost);
    free_dev(loss); free_dev(tmp);
    if (st != SK_OK) return st;
    if (e != hipSuccess) return fail(SK_EDEVICE, "get_activation_grad: %s", hipGetErrorString(e));
    return SK_OK;
}

sk_status sknet_sgd_step(sknet_t *net, float lr, float momentum, float weight_decay, void *hip_stream)
{
    SK_TRY(check_net(net));
    if (!net->planned || !net->training || !net->backward_done)
        return fail(SK_ESTATE, "sgd_step: needs a backward pass on a training plan");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    net->last_stream = stream;
    // one launch updates every weight and bias tensor, a second rebuilds every packed form
    // (a net is a dozen small tensors: one launch each would cost more than the work)
    const int nc = (int)net->convs.size();
    if (2 * nc > sk::BATCH_MAX) {
        for (auto &c : net->convs) {
            SK_HIP(sk::launch_sgd_f32(c.w_dev, c.dw, momentum != 0.f ? c.vw : nullptr, c.wcount(), lr, momentum, weight_decay, stream));
            SK_HIP(sk::launch_sgd_f32(c.b_dev, c.db, momentum != 0.f ? c.vb : nullptr, c.c_out, lr, momentum, weight_decay, stream));
            SK_TRY(repack_conv(c, true, net->dtype, stream));
        }
        return SK_OK;
    }
    sk::SgdBatch sb{};
    sk::PackF32Job pf[sk::BATCH_MAX];
    sk::PackHJob ph[sk::BATCH_MAX];
    int np = 0;
    for (auto &c : net->convs) {
        sb.w[sb.n] = c.w_dev; sb.dw[sb.n] = c.dw; sb.v[sb.n] = momentum != 0.f ? c.vw : nullptr; sb.count[sb.n] = c.wcount(); ++sb.n;
        sb.w[sb.n] = c.b_dev; sb.dw[sb.n] = c.db; sb.v[sb.n] = momentum != 0.f ? c.vb : nullptr; sb.count[sb.n] = c.c_out; ++sb.n;
        if (net->dtype == SK_F32) {
            pf[np++] = {c.w_dev, c.wp_fwd, c.c_out, c.c_in, c.k, 0, c.rows_fwd, c.n_pad};
            if (c.wp_bwd) pf[np++] = {c.w_dev, c.wp_bwd, c.c_out, c.c_in, c.k, 1, c.rows_bwd, c.n_pad_bwd};
        } else {
            ph[np++] = {c.w_dev, c.wp16_fwd, c.c_out, c.c_in, c.k, 0, c.mt16};
            if (c.wp16_bwd) ph[np++] = {c.w_dev, c.wp16_bwd, c.c_out, c.c_in, c.k, 1, 0};
        }
    }
    SK_HIP(sk::launch_sgd_batch_f32(sb, lr, momentum, weight_decay, stream));
    if (net->dtype == SK_F32) SK_HIP(sk::launch_pack_weights_f32_batch(pf, np, stream));
    else SK_HIP(sk::launch_pack_weights_h_batch(ph, np, net->dtype, stream));
    if (net->fuse_head) {
        const ConvParams &c1 = net->convs[net->conv_of_layer[(int)net->layers.size() - 2]];
        SK_HIP(sk::launch_pack_head_w1(c1.w_dev, net->head_w1p, net->dtype, c1.c_out, c1.c_in, stream));
    }
    return SK_OK;
}

sk_status sknet_get_grad(sknet_t *net, int32_t conv_idx, float *dw_host, float *db_host)
{
    SK_TRY(check_net(net));
    if (conv_idx < 0 || conv_idx >= (int)net->convs.size()) return fail(SK_EINVAL, "get_grad: bad index");
    if (!net->backward_done) return fail(SK_ESTATE, "get_grad: no backward pass yet");
    ConvParams &c = net->convs[conv_idx];
    SK_HIP(hipStreamSynchronize(net->last_stream));
    if (dw_host) SK_HIP(hipMemcpy(dw_host, c.dw, sizeof(float) * c.wcount(), hipMemcpyDeviceToHost));
    if (db_host) SK_HIP(hipMemcpy(db_host, c.db, sizeof(float) * c.c_out, hipMemcpyDeviceToHost));
    return SK_OK;
}

sk_status sknet_get_activation(sknet_t *net, int32_t layer_idx, float *nchw_host)
{
    SK_TRY(check_net(net));
    if (!nchw_host || layer_idx < -1 || layer_idx >= (int)net->layers.size()) return fail(SK_EINVAL, "get_activation: bad arguments");
    if (!net->forward_done) return fail(SK_ESTATE, "get_activation: no forward pass yet");
    if (layer_idx >= 0 && !net->kept(layer_idx))
        return fail(SK_ESTATE, "get_activation: this plan fuses layer %d with its neighbours; plan with mode 2 to keep every layer", layer_idx);
    SK_HIP(hipStreamSynchronize(net->last_stream));
    const int i = layer_idx + 1;
    const Dims &dm = net->dims[i];
    const bool f32 = (i == 0) ? !net->half() : stored_f32(net, i - 1);
    if (f32) {
        SK_HIP(hipMemcpy(nchw_host, net->act[i], sizeof(float) * dm.count(net->n), hipMemcpyDeviceToHost));
        return SK_OK;
    }
    float *tmp = nullptr;   // widen the 16-bit octet layout to fp32 NCHW on the device first
    SK_TRY(alloc_f(&tmp, dm.count(net->n)));
    hipError_t e = sk::launch_unpack_h(net->act[i], tmp, net->dtype, net->n, dm.c, dm.h, dm.w, net->last_stream);
    if (e == hipSuccess) e = hipStreamSynchronize(net->last_stream);
    if (e == hipSuccess) e = hipMemcpy(nchw_host, tmp, sizeof(float) * dm.count(net->n), hipMemcpyDeviceToHost);
    (void)hipFree(tmp);
    if (e != hipSuccess) return fail(SK_EDEVICE, "get_activation: %s", hipGetErrorString(e));
    return SK_OK;
}

sk_status sknet_get_pool_argmax(sknet_t *net, int32_t pool_idx, int32_t *idx_host)
{
    SK_TRY(check_net(net));
    if (!idx_host || pool_idx < 0) return fail(SK_EINVAL, "get_pool_argmax: bad arguments");
    if (!net->forward_done || !net->training) return fail(SK_ESTATE, "get_pool_argmax: needs a forward pass on a training plan");
    int li = -1, seen = 0;
    for (int i = 0; i < (int)net->layers.size(); ++i)
        if (net->layers[i].kind == SK_MAXPOOL && seen++ == pool_idx) { li = i; break; }
    if (li < 0) return fail(SK_EINVAL, "get_pool_argmax: the net has no pool %d", pool_idx);
    const sk_layer &l = net->layers[li];
    const Dims &in = net->dims[li], &out = net->dims[li + 1];
    const long count = out.count(net->n);
    int32_t *tmp = nullptr;
    SK_HIP(hipMalloc(reinterpret_cast<void **>(&tmp), sizeof(int32_t) * (size_t)count));
    hipError_t e = net->half()
                       ? sk::launch_tap_to_index_h(net->tap[li], tmp, net->n, out.c, out.h, out.w, in.w, l.k, l.d, l.s, net->last_stream)
                       : sk::launch_tap_to_index(net->tap[li], tmp, net->n * out.c, out.h, out.w, in.w, l.k, l.d, l.s, net->last_stream);
    if (e == hipSuccess) e = hipStreamSynchronize(net->last_stream);
    if (e == hipSuccess) e = hipMemcpy(idx_host, tmp, sizeof(int32_t) * (size_t)count, hipMemcpyDeviceToHost);
    (void)hipFree(tmp);
    if (e != hipSuccess) return fail(SK_EDEVICE, "get_pool_argmax: %s", hipGetErrorString(e));
    return SK_OK;
}

sk_status sknet_num_steps(const sknet_t *net, int32_t *count)
{
    SK_TRY(check_net(net));
    if (!count) return fail(SK_EINVAL, "num_steps: count is null");
    if (!net->planned) return fail(SK_ESTATE, "num_steps: call sknet_plan first");
    *count = (int32_t)net->steps.size();
    return SK_OK;
}

sk_status sknet_step_name(const sknet_t *net, int32_t step, char *name, int32_t cap)
{
    SK_TRY(check_net(net));
    if (!net->planned) return fail(SK_ESTATE, "step_name: call sknet_plan first");
    if (!name || cap < 1 || step < 0 || step >= (int)net->steps.size()) return fail(SK_EINVAL, "step_name: bad arguments");
    const sknet::Step st = net->steps[step];
    if (st.kind == 0) snprintf(name, cap, "pad");
    else if (st.kind == 2) snprintf(name, cap, "softmax");
    else if (st.kind == 3) snprintf(name, cap, "head_fused");
    else {
        const sk_layer &l = net->layers[st.arg];
        if (l.kind == SK_CONV)
            snprintf(name, cap, "conv%d_k%d_d%d_o%d%s%s", st.arg, l.k, l.d, l.c_out, net->pending[st.arg] ? "_hpool" : "", net->vpool[st.arg] ? "_vpool" : "");
        else snprintf(name, cap, "pool%d_k%d_d%d_s%d", st.arg, l.k, l.d, l.s);
    }
    return SK_OK;
}

sk_status sknet_time_step(sknet_t *net, int32_t step, int32_t iters, void *hip_stream, float *avg_ms)
{
    SK_TRY(check_net(net));
    if (!avg_ms || iters < 1 || step < 0 || step >= (int)net->steps.size()) return fail(SK_EINVAL, "time_step: bad arguments");
    if (!net->forward_done) return fail(SK_ESTATE, "time_step: run sknet_forward first");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipEvent_t e0, e1;
    SK_HIP(hipEventCreate(&e0));
    SK_HIP(hipEventCreate(&e1));
    sk_status st = run_forward_step(net, step, stream);   // warm-up
    hipError_t e = hipEventRecord(e0, stream);
    for (int i = 0; i < iters && st == SK_OK; ++i) st = run_forward_step(net, step, stream);
    if (e == hipSuccess) e = hipEventRecord(e1, stream);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (st != SK_OK) return st;
    if (e != hipSuccess) return fail(SK_EDEVICE, "time_step: %s", hipGetErrorString(e));
    *avg_ms = ms / (float)iters;
    return SK_OK;
}

sk_status sknet_time_backward_step(sknet_t *net, const int32_t *labels_dev, int32_t layer_idx, int32_t part, int32_t iters, void *hip_stream,
                                   float *avg_ms)
{
    SK_TRY(check_net(net));
    const int L = (int)net->layers.size();
    if (!avg_ms || !labels_dev || iters < 1 || part < 0 || part > 2 || (part != 2 && (layer_idx < 0 || layer_idx >= L)))
        return fail(SK_EINVAL, "time_backward_step: bad arguments");
    if (!net->planned || !net->training || !net->forward_done) return fail(SK_ESTATE, "time_backward_step: needs a forward pass on a training plan");
    if (part == 0 && net->layers[layer_idx].kind != SK_CONV) return fail(SK_EINVAL, "time_backward_step: layer %d has no weights", layer_idx);
    if (part == 1 && layer_idx == 0) return fail(SK_EINVAL, "time_backward_step: layer 0 has no input gradient");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    net->last_stream = stream;
    net->backward_done = false;                // the walk overwrites weight gradients
    float *loss = nullptr, *g = nullptr;
    SK_TRY(alloc_f(&loss, 1));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    sk_status st = e == hipSuccess ? SK_OK : fail(SK_EDEVICE, "time_backward_step: %s", hipGetErrorString(e));
    // the error map of the layer (part 2: the loss alone, which is the walk down to the last layer)
    const int li = part == 2 ? (net->fuse_head ? L - 3 : L - 1) : layer_idx;     // (a head in one kernel: the loss part is that kernel)
    if (st == SK_OK) st = backward_impl(net, labels_dev, loss, stream, li, &g, net->loss_partial, net->wgrad_scratch, 0);
    float *other = g == net->gbuf[0] ? net->gbuf[1] : net->gbuf[0];
    auto once = [&]() -> sk_status {
        if (part == 2) return backward_impl(net, labels_dev, loss, stream, li, &g, net->loss_partial, net->wgrad_scratch, 0);
        return backward_layer(net, li, g, other, part == 0 ? 1 : 2, stream, net->wgrad_scratch, 0);
    };
    if (st == SK_OK) st = once();              // warm-up
    if (st == SK_OK) e = hipEventRecord(e0, stream);
    for (int i = 0; i < iters && st == SK_OK; ++i) st = once();
    if (st == SK_OK && e == hipSuccess) e = hipEventRecord(e1, stream);
    if (st == SK_OK && e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (st == SK_OK && e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    free_dev(loss);
    if (st != SK_OK) return st;
    if (e != hipSuccess) return fail(SK_EDEVICE, "time_backward_step: %s", hipGetErrorString(e));
    *avg_ms = ms / (float)iters;
    return SK_OK;
}

}  // extern "C"
