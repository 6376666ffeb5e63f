// U-Net forward (paper Section 3.4 and its configuration table) on the same kernels as the SK
// net: 3x3 convolutions are the SK convolution at d = 1, the 2x2 stride-2 up-convolution is four
// 1x1 convolutions whose outputs interleave, MergeCrop is the up path written in place plus a
// crop-and-place copy of the skip maps.  The USK-Net (Section 3.5 and its configuration table) is
// the same engine with another layer list: one contracting step, the SK layer sequence at d = 1, 2,
// 4, 8 on the half-resolution maps, one expanding step.  See include/sknet.h for the contract.
#include <algorithm>
#include <map>
#include <new>
#include <set>

#include "sk_host.h"

using namespace skh;

namespace {

struct UpParams {
    int c_in = 0, c_out = 0;
    std::vector<float> w, b;        // host master [c_in][c_out][2][2], [c_out]
    float *w_dev = nullptr;         // same layout on the device
    ConvParams tap[4];              // per (a, b): a 1x1 convolution with weight W1[o][c] = w[c][o][a][b]
    // training: the four taps as ONE 1x1 convolution with 4*c_out output maps (map t*c_out + o = tap t of
    // map o, t = 2a + b); its data- and weight-gradient kernels serve the up-convolution's backward
    ConvParams cat;
};

struct Stage {
    std::string name;
    Dims dims;
    float *buf = nullptr;
    int buf_c = 0;                  // maps of the buffer the stage lives in (> dims.c for the up path inside a merged buffer)
};

}  // namespace

struct unet {
    int arch = 0;                            // 0 = U-Net, 1 = USK-Net
    int c_in = 0, n_classes = 0, depth = 0, base = 0;
    int dtype = SK_F32;                      // storage type of activations and packed weights
    // parameters in forward order; kind 0 = conv (index into convs), 1 = up-convolution (index into ups)
    struct Param { std::string name; int kind; int idx; };
    std::vector<Param> params;
    std::vector<ConvParams> convs;
    std::vector<UpParams> ups;
    // plan
    bool training = false, backward_done = false;
    int merge_backward = 0;                            // MergeCrop's backward: 0 = into the up path only, 1 = into the skip map as well
    float *image_copy = nullptr;                       // training: the image of the last forward pass (the first layer's weight gradient reads it)
    std::map<const float *, float *> grad_of;          // training: gradient buffer of every activation buffer
    std::vector<uint8_t *> taps;                       // training: winner codes, one entry per op (pools only)
    float *loss_partial = nullptr, *wgrad_scratch = nullptr, *s2d = nullptr;
    float *dz16 = nullptr;                             // 16-bit training: the loss gradient in the octet layout (the last conv's dY)
    std::set<const float *> relu_out;                  // buffers written by a convolution with ReLU
    bool planned = false, forward_done = false;
    int n = 0, h_in = 0, w_in = 0;
    std::vector<float *> buffers;            // every device activation buffer, for release
    struct Op {
        int kind;                            // 0 conv, 1 pool, 2 up-convolution, 3 crop copy, 4 image -> octet layout
        int param;                           // conv / up index
        int relu;
        const float *src;                    // nullptr = the caller's image
        float *dst;
        Dims in, out;                        // out.c = maps of the destination buffer
        int o_off, crop;                     // map offset in dst; crop offset for kind 3
        int src_maps;
        int k, d, s;                         // pool window / spacing / stride; d also the conv's kernel stride
    };
    std::vector<Op> ops;
    std::vector<Stage> stages;
    float *logits = nullptr;                 // fp32 NCHW in every storage type
    float *zero_page = nullptr;              // 16-bit types: zeros the convolution reads for samples outside the image
    float *unpack_tmp = nullptr;             // 16-bit types: fp32 staging for unet_get_activation
    long unpack_tmp_floats = 0;
    Dims out_dims;
    hipStream_t last_stream = nullptr;

    void release_plan()
    {
        for (auto &p : buffers) free_dev(p);
        buffers.clear();
        free_dev(unpack_tmp); free_dev(zero_page);
        unpack_tmp_floats = 0;
        for (auto &kv : grad_of) { float *g = kv.second; free_dev(g); }
        grad_of.clear();
        for (auto &t : taps)
            if (t) { (void)hipFree(t); t = nullptr; }
        taps.clear();
        free_dev(loss_partial); free_dev(wgrad_scratch); free_dev(s2d); free_dev(image_copy); free_dev(dz16);
        relu_out.clear();
        ops.clear();
        stages.clear();
        for (auto &c : convs) release_conv(c);
        for (auto &u : ups) {
            free_dev(u.w_dev);
            for (auto &t : u.tap) release_conv(t);
            release_conv(u.cat);
        }
        planned = forward_done = backward_done = false;
    }
};

namespace {

sk_status check(const unet_t *net)
{
    if (!net) return fail(SK_EINVAL, "null U-Net handle");
    return SK_OK;
}

// spatial sizes: every level two valid 3x3 convs, then a k = s = 2 pool; mirrored on the way up
// the SK part of the USK-Net: (conv?, f_out multiple of base, k, d)
struct UskCore { bool conv; int f_mul, k, d; const char *name; };
const UskCore kUskCore[] = {{true, 2, 6, 1, "conv3"}, {false, 0, 2, 1, "pool2"}, {true, 2, 4, 2, "conv4"}, {false, 0, 2, 2, "pool3"},
                            {true, 2, 4, 4, "conv5"}, {false, 0, 2, 4, "pool4"}, {true, 8, 8, 8, "ip1"}, {true, 4, 1, 1, "ip2"}};

sk_status walk_sizes_usk(int h, int w, int *ho, int *wo)
{
    h -= 4; w -= 4;
    if (h < 2 || w < 2) return fail(SK_ESHAPE, "USK-Net: map vanishes before the pooling step");
    if (h % 2 || w % 2) return fail(SK_ESHAPE, "USK-Net: pooling needs an even map (got %dx%d)", h, w);
    h /= 2; w /= 2;
    for (const auto &l : kUskCore) {
        h -= (l.k - 1) * l.d; w -= (l.k - 1) * l.d;
        if (h < 1 || w < 1) return fail(SK_ESHAPE, "USK-Net: map vanishes at %s", l.name);
    }
    h = 2 * h - 4; w = 2 * w - 4;
    if (h < 1 || w < 1) return fail(SK_ESHAPE, "USK-Net: map vanishes on the expanding step");
    *ho = h; *wo = w;
    return SK_OK;
}

sk_status walk_sizes(const unet *net, int h, int w, int *ho, int *wo)
{
    if (net->arch == 1) return walk_sizes_usk(h, w, ho, wo);
    for (int i = 0; i <= net->depth; ++i) {
        h -= 4; w -= 4;
        if (h < 1 || w < 1) return fail(SK_ESHAPE, "U-Net: map vanishes at level %d", i);
        if (i < net->depth) {
            if (h % 2 || w % 2) return fail(SK_ESHAPE, "U-Net: pooling needs an even map at level %d (got %dx%d)", i, h, w);
            h /= 2; w /= 2;
        }
    }
    for (int i = net->depth - 1; i >= 0; --i) {
        h = 2 * h - 4; w = 2 * w - 4;
        if (h < 1 || w < 1) return fail(SK_ESHAPE, "U-Net: map vanishes on the expanding path at level %d", i);
    }
    *ho = h; *wo = w;
    return SK_OK;
}

sk_status upload_up(UpParams &u, int dtype)
{
    for (int a = 0; a < 2; ++a)
        for (int b = 0; b < 2; ++b) {
            ConvParams &t = u.tap[a * 2 + b];
            t.c_in = u.c_in; t.c_out = u.c_out; t.k = 1;
            t.w.resize((size_t)u.c_in * u.c_out);
            for (int c = 0; c < u.c_in; ++c)
                for (int o = 0; o < u.c_out; ++o)
                    t.w[(size_t)o * u.c_in + c] = u.w[(((size_t)c * u.c_out + o) * 2 + a) * 2 + b];
            t.b = u.b;
            SK_TRY(upload_conv(t, false, nullptr, dtype));
        }
    if (u.cat.w_dev) {                 // the stacked form: one launch in the fp32 forward pass, and the backward pass
        u.cat.w.resize((size_t)4 * u.c_out * u.c_in);
        u.cat.b.resize((size_t)4 * u.c_out);
        for (int t = 0; t < 4; ++t) {
            std::memcpy(u.cat.w.data() + (size_t)t * u.c_out * u.c_in, u.tap[t].w.data(), sizeof(float) * u.c_out * u.c_in);
            std::memcpy(u.cat.b.data() + (size_t)t * u.c_out, u.b.data(), sizeof(float) * u.c_out);
        }
        SK_TRY(upload_conv(u.cat, u.cat.wp_bwd != nullptr || u.cat.wp16_bwd != nullptr, nullptr, dtype));
    }
    return SK_OK;
}

}  // namespace

extern "C" {

sk_status unet_create(int32_t c_in, int32_t n_classes, int32_t depth, int32_t base_ch, sk_dtype dtype, unet_t **out)
{
    if (!out) return fail(SK_EINVAL, "unet_create: out is null");
    *out = nullptr;
    if (c_in < 1 || n_classes < 1 || depth < 1 || depth > 6 || base_ch < 1) return fail(SK_EINVAL, "unet_create: bad arguments");
    if (dtype != SK_F32 && dtype != SK_BF16 && dtype != SK_F16) return fail(SK_EINVAL, "unet_create: unknown dtype %d", (int)dtype);
    if (dtype != SK_F32 && base_ch % 8 != 0)
        return fail(SK_EUNSUPPORTED, "unet_create: the 16-bit layout keeps maps in groups of 8, base_ch must be a multiple of 8");
    unet *net = new (std::nothrow) unet;
    if (!net) return fail(SK_ENOMEM, "unet_create: out of host memory");
    net->c_in = c_in; net->n_classes = n_classes; net->depth = depth; net->base = base_ch; net->dtype = dtype;
    auto add_conv = [&](const std::string &name, int fi, int fo, int k) {
        ConvParams c;
        c.c_in = fi; c.c_out = fo; c.k = k;
        c.w.assign((size_t)c.wcount(), 0.f);
        c.b.assign((size_t)fo, 0.f);
        net->params.push_back({name, 0, (int)net->convs.size()});
        net->convs.push_back(std::move(c));
    };
    int f = c_in;
    for (int i = 0; i <= depth; ++i) {
        const int ch = base_ch << i;
        add_conv("down" + std::to_string(i) + "a", f, ch, 3);
        add_conv("down" + std::to_string(i) + "b", ch, ch, 3);
        f = ch;
    }
    for (int i = depth - 1; i >= 0; --i) {
        const int ch = base_ch << i;
        UpParams u;
        u.c_in = 2 * ch; u.c_out = ch;
        u.w.assign((size_t)u.c_in * u.c_out * 4, 0.f);
        u.b.assign((size_t)ch, 0.f);
        net->params.push_back({"up" + std::to_string(i), 1, (int)net->ups.size()});
        net->ups.push_back(std::move(u));
        add_conv("dec" + std::to_string(i) + "a", 2 * ch, ch, 3);
        add_conv("dec" + std::to_string(i) + "b", ch, ch, 3);
    }
    add_conv("head", base_ch, n_classes, 1);
    *out = net;
    return SK_OK;
}

sk_status usknet_create(int32_t c_in, int32_t n_classes, int32_t base_ch, sk_dtype dtype, unet_t **out)
{
    if (!out) return fail(SK_EINVAL, "usknet_create: out is null");
    *out = nullptr;
    if (c_in < 1 || n_classes < 1 || base_ch < 1) return fail(SK_EINVAL, "usknet_create: bad arguments");
    if (dtype != SK_F32 && dtype != SK_BF16 && dtype != SK_F16) return fail(SK_EINVAL, "usknet_create: unknown dtype %d", (int)dtype);
    if (dtype != SK_F32 && base_ch % 8 != 0)
        return fail(SK_EUNSUPPORTED, "usknet_create: the 16-bit layout keeps maps in groups of 8, base_ch must be a multiple of 8");
    unet *net = new (std::nothrow) unet;
    if (!net) return fail(SK_ENOMEM, "usknet_create: out of host memory");
    net->arch = 1; net->c_in = c_in; net->n_classes = n_classes; net->depth = 1; net->base = base_ch; net->dtype = dtype;
    auto add_conv = [&](const std::string &name, int fi, int fo, int k) {
        ConvParams c;
        c.c_in = fi; c.c_out = fo; c.k = k;
        c.w.assign((size_t)c.wcount(), 0.f);
        c.b.assign((size_t)fo, 0.f);
        net->params.push_back({name, 0, (int)net->convs.size()});
        net->convs.push_back(std::move(c));
    };
    add_conv("conv1", c_in, base_ch, 3);
    add_conv("conv2", base_ch, base_ch, 3);
    int f = base_ch;
    for (const auto &l : kUskCore)
        if (l.conv) {
            add_conv(l.name, f, l.f_mul * base_ch, l.k);
            f = l.f_mul * base_ch;
        }
    UpParams u;
    u.c_in = f; u.c_out = 2 * base_ch;
    u.w.assign((size_t)u.c_in * u.c_out * 4, 0.f);
    u.b.assign((size_t)u.c_out, 0.f);
    net->params.push_back({"up1", 1, 0});
    net->ups.push_back(std::move(u));
    add_conv("conv7", 3 * base_ch, 2 * base_ch, 3);
    add_conv("conv8", 2 * base_ch, base_ch, 3);
    add_conv("ip3", base_ch, n_classes, 1);
    *out = net;
    return SK_OK;
}

void unet_destroy(unet_t *net)
{
    if (!net) return;
    net->release_plan();
    delete net;
}

sk_status unet_num_params(const unet_t *net, int32_t *count)
{
    SK_TRY(check(net));
    if (!count) return fail(SK_EINVAL, "unet_num_params: count is null");
    *count = (int32_t)net->params.size();
    return SK_OK;
}

sk_status unet_param_shape(const unet_t *net, int32_t idx, int32_t *shape4)
{
    SK_TRY(check(net));
    if (!shape4 || idx < 0 || idx >= (int)net->params.size()) return fail(SK_EINVAL, "unet_param_shape: bad index");
    const auto &p = net->params[idx];
    if (p.kind == 0) {
        const ConvParams &c = net->convs[p.idx];
        shape4[0] = c.c_out; shape4[1] = c.c_in; shape4[2] = c.k; shape4[3] = c.k;
    } else {
        const UpParams &u = net->ups[p.idx];
        shape4[0] = u.c_in; shape4[1] = u.c_out; shape4[2] = 2; shape4[3] = 2;
    }
    return SK_OK;
}

sk_status unet_param_kind(const unet_t *net, int32_t idx, int32_t *kind)
{
    SK_TRY(check(net));
    if (!kind || idx < 0 || idx >= (int)net->params.size()) return fail(SK_EINVAL, "unet_param_kind: bad index");
    *kind = net->params[idx].kind;
    return SK_OK;
}

sk_status unet_set_weights(unet_t *net, int32_t idx, const float *w_host, const float *b_host)
{
    SK_TRY(check(net));
    if (!w_host || idx < 0 || idx >= (int)net->params.size()) return fail(SK_EINVAL, "unet_set_weights: bad arguments");
    const auto &p = net->params[idx];
    if (p.kind == 0) {
        ConvParams &c = net->convs[p.idx];
        std::memcpy(c.w.data(), w_host, sizeof(float) * c.wcount());
        if (b_host) std::memcpy(c.b.data(), b_host, sizeof(float) * c.c_out);
        if (net->planned) SK_TRY(upload_conv(c, net->training, net->last_stream, net->dtype));
    } else {
        UpParams &u = net->ups[p.idx];
        std::memcpy(u.w.data(), w_host, sizeof(float) * u.w.size());
        if (b_host) std::memcpy(u.b.data(), b_host, sizeof(float) * u.c_out);
        if (net->planned) SK_TRY(upload_up(u, net->dtype));
    }
    return SK_OK;
}

sk_status unet_output_size(const unet_t *net, int32_t h_in, int32_t w_in, int32_t *h_out, int32_t *w_out)
{
    SK_TRY(check(net));
    if (!h_out || !w_out) return fail(SK_EINVAL, "unet_output_size: null output");
    return walk_sizes(net, h_in, w_in, h_out, w_out);
}

static sk_status sync_masters(unet_t *net);

static sk_status plan_impl(unet_t *net, int32_t n, int32_t h_in, int32_t w_in, bool training)
{
    SK_TRY(check(net));
    if (n < 1) return fail(SK_EINVAL, "unet_plan: n must be >= 1");
    int ho, wo;
    SK_TRY(walk_sizes(net, h_in, w_in, &ho, &wo));
    SK_TRY(sync_masters(net));             // a trained net keeps its weights across plans
    net->release_plan();
    net->n = n; net->h_in = h_in; net->w_in = w_in; net->training = training;
    sk_status st = SK_OK;
    const bool half = net->dtype != SK_F32;
    // activation buffers: fp32 NCHW, or the 16-bit octet layout (sized in floats either way)
    auto new_buf = [&](const Dims &d) -> float * {
        float *p = nullptr;
        if (st == SK_OK) st = alloc_f(&p, half ? octet_floats(n, d) : d.count(n));
        if (p) net->buffers.push_back(p);
        if (half && d.count(n) > net->unpack_tmp_floats) net->unpack_tmp_floats = d.count(n);
        return p;
    };
    auto conv_op = [&](int conv_idx, int relu, const float *src, const Dims &in, float *dst, const Dims &out, int d = 1) {
        unet::Op op{};
        op.kind = 0; op.param = conv_idx; op.relu = relu; op.src = src; op.dst = dst; op.in = in; op.out = out; op.d = d;
        net->ops.push_back(op);
    };
    auto pool_op = [&](const float *src, const Dims &in, float *dst, const Dims &out, int k, int d, int s) {
        unet::Op op{};
        op.kind = 1; op.src = src; op.dst = dst; op.in = in; op.out = out; op.k = k; op.d = d; op.s = s;
        net->ops.push_back(op);
    };
    int ci = 0;   // running conv index
    Dims cur;
    cur.c = net->c_in; cur.h = h_in; cur.w = w_in;
    const float *src = nullptr;
    if (half) {                              // the caller's fp32 image goes to the octet layout first
        float *packed = new_buf(cur);
        unet::Op op{};
        op.kind = 4; op.src = nullptr; op.dst = packed; op.in = cur; op.out = cur;
        net->ops.push_back(op);
        src = packed;
    }
    if (net->arch == 1) {
        // USK-Net: conv1, conv2 | pool k2 s2 | SK core at half resolution | up-convolution into the
        // merged buffer, conv2's maps cropped in behind it | conv7, conv8
        const int b0 = net->base;
        Dims a = {b0, cur.h - 2, cur.w - 2}, b = {b0, cur.h - 4, cur.w - 4};
        float *ba = new_buf(a), *bb = new_buf(b);
        conv_op(ci++, 1, src, cur, ba, a);
        conv_op(ci++, 1, ba, a, bb, b);
        net->stages.push_back({"conv2", b, bb, b.c});
        Dims p = {b0, b.h / 2, b.w / 2};
        float *bp = new_buf(p);
        pool_op(bb, b, bp, p, 2, 1, 2);
        net->stages.push_back({"pool1", p, bp, p.c});
        cur = p; src = bp;
        for (const auto &l : kUskCore) {
            Dims o = {l.conv ? l.f_mul * b0 : cur.c, cur.h - (l.k - 1) * l.d, cur.w - (l.k - 1) * l.d};
            float *bo = new_buf(o);
            if (l.conv) conv_op(ci++, 1, src, cur, bo, o, l.d);
            else pool_op(src, cur, bo, o, l.k, l.d, 1);
            net->stages.push_back({l.name, o, bo, o.c});
            cur = o; src = bo;
        }
        Dims merged = {3 * b0, 2 * cur.h, 2 * cur.w};
        float *bm = new_buf(merged);
        unet::Op up{};
        up.kind = 2; up.param = 0; up.src = src; up.dst = bm; up.in = cur; up.out = merged; up.o_off = 0;
        net->ops.push_back(up);
        Dims upd = {2 * b0, merged.h, merged.w};
        net->stages.push_back({"up1", upd, bm, merged.c});
        unet::Op cp{};
        cp.kind = 3; cp.src = bb; cp.dst = bm; cp.in = b; cp.out = merged; cp.o_off = 2 * b0;
        cp.crop = (b.h - merged.h) / 2; cp.src_maps = b0;
        if (b.h < merged.h || b.w < merged.w) st = fail(SK_ESHAPE, "USK-Net: skip map smaller than the up path");
        net->ops.push_back(cp);
        Dims c7 = {2 * b0, merged.h - 2, merged.w - 2}, c8 = {b0, merged.h - 4, merged.w - 4};
        float *b7 = new_buf(c7), *b8 = new_buf(c8);
        conv_op(ci++, 1, bm, merged, b7, c7);
        conv_op(ci++, 1, b7, c7, b8, c8);
        net->stages.push_back({"conv8", c8, b8, c8.c});
        cur = c8; src = b8;
    } else {
        std::vector<Dims> skip_dims;
        std::vector<const float *> skip_buf;
        for (int i = 0; i <= net->depth && st == SK_OK; ++i) {
            const int ch = net->base << i;
            Dims a = {ch, cur.h - 2, cur.w - 2}, b = {ch, cur.h - 4, cur.w - 4};
            float *ba = new_buf(a), *bb = new_buf(b);
            conv_op(ci++, 1, src, cur, ba, a);
            conv_op(ci++, 1, ba, a, bb, b);
            net->stages.push_back({"down" + std::to_string(i), b, bb, b.c});
            cur = b; src = bb;
            if (i < net->depth) {
                skip_dims.push_back(b);
                skip_buf.push_back(bb);
                Dims p = {ch, b.h / 2, b.w / 2};
                float *bp = new_buf(p);
                pool_op(bb, b, bp, p, 2, 1, 2);
                cur = p; src = bp;
            }
        }
        int ui = 0;
        for (int i = net->depth - 1; i >= 0 && st == SK_OK; --i) {
            const int ch = net->base << i;
            Dims merged = {2 * ch, 2 * cur.h, 2 * cur.w};
            float *bm = new_buf(merged);
            unet::Op up{};
            up.kind = 2; up.param = ui++; up.src = src; up.dst = bm; up.in = cur; up.out = merged; up.o_off = 0;
            net->ops.push_back(up);
            Dims upd = {ch, merged.h, merged.w};
            net->stages.push_back({"up" + std::to_string(i), upd, bm, merged.c});
            unet::Op cp{};
            cp.kind = 3; cp.src = skip_buf[i]; cp.dst = bm; cp.in = skip_dims[i]; cp.out = merged; cp.o_off = ch;
            cp.crop = (skip_dims[i].h - merged.h) / 2; cp.src_maps = ch;
            if (skip_dims[i].h < merged.h || skip_dims[i].w < merged.w) st = fail(SK_ESHAPE, "U-Net: skip map smaller than the up path at level %d", i);
            net->ops.push_back(cp);
            Dims a = {ch, merged.h - 2, merged.w - 2}, b = {ch, merged.h - 4, merged.w - 4};
            float *ba = new_buf(a), *bb = new_buf(b);
            conv_op(ci++, 1, bm, merged, ba, a);
            conv_op(ci++, 1, ba, a, bb, b);
            net->stages.push_back({"dec" + std::to_string(i), b, bb, b.c});
            cur = b; src = bb;
        }
    }
    if (st == SK_OK) {
        Dims z = {net->n_classes, cur.h, cur.w};
        if (st == SK_OK) st = alloc_f(&net->logits, z.count(n));
        if (net->logits) net->buffers.push_back(net->logits);
        conv_op(ci++, 0, src, cur, net->logits, z);
        net->stages.push_back({"logits", z, net->logits, z.c});
        net->out_dims = z;
    }
    if (half) {
        // map tiles per workgroup that suit each layer's output size (the deep levels are small)
        for (const auto &op : net->ops) {
            if (op.kind == 0) {
                ConvParams &c = net->convs[op.param];
                c.mt16 = sk::conv_h_pick_mode(c.c_out, c.c_in, c.k, op.d, n, op.out.h, op.out.w);
            } else if (op.kind == 2) {
                for (auto &t : net->ups[op.param].tap) t.mt16 = sk::conv_h_pick_mt(net->ups[op.param].c_out, 1, n, op.in.h, op.in.w);
                net->ups[op.param].cat.mt16 = sk::conv_h_pick_mt(4 * net->ups[op.param].c_out, 1, n, op.in.h, op.in.w);
            }
        }
    }
    if (half)
        for (const auto &op : net->ops)
            if (st == SK_OK && op.kind == 0 && !sk::conv_h_supported(net->convs[op.param].k, op.d, net->convs[op.param].c_out))
                st = fail(SK_EUNSUPPORTED, "a %dx%d convolution at d = %d to %d maps is not built for 16-bit storage", net->convs[op.param].k,
                          net->convs[op.param].k, op.d, net->convs[op.param].c_out);
    for (auto &c : net->convs) {
        if (st != SK_OK) break;
        if (st == SK_OK) st = alloc_conv(c, training, net->dtype);
        if (st == SK_OK) st = upload_conv(c, training, nullptr, net->dtype);
    }
    for (auto &u : net->ups) {
        if (st != SK_OK) break;
        for (auto &t : u.tap) {
            t.c_in = u.c_in; t.c_out = u.c_out; t.k = 1;
            if (st == SK_OK) st = alloc_conv(t, false, net->dtype);
        }
        {
            u.cat.c_in = u.c_in; u.cat.c_out = 4 * u.c_out; u.cat.k = 1;
            u.cat.w.assign((size_t)4 * u.c_out * u.c_in, 0.f);
            u.cat.b.assign((size_t)4 * u.c_out, 0.f);
            if (st == SK_OK) st = alloc_conv(u.cat, training, net->dtype);
        }
        if (st == SK_OK) st = upload_up(u, net->dtype);
    }
    if (st == SK_OK && half) st = alloc_f(&net->unpack_tmp, net->unpack_tmp_floats);
    if (st == SK_OK && half) st = alloc_zero_page(&net->zero_page);
    if (st == SK_OK && training) {
        // a gradient buffer per activation buffer, winner codes per pool, scratch of the loss and the weight gradients
        for (float *bufp : net->buffers) {
            if (st != SK_OK) break;
            long floats = 0;
            for (const auto &op : net->ops)
                if (op.dst == bufp) floats = std::max(floats, half && bufp != net->logits ? octet_floats(n, op.out) : op.out.count(n));
            float *g = nullptr;
            st = alloc_f(&g, floats);
            if (g) net->grad_of[bufp] = g;
        }
        net->taps.assign(net->ops.size(), nullptr);
        size_t scratch = 0;
        long s2d_floats = 0;
        for (size_t i = 0; i < net->ops.size() && st == SK_OK; ++i) {
            const auto &op = net->ops[i];
            if (op.kind == 1) {
                if (op.s != 1 && !(op.s == op.k && op.d == 1)) st = fail(SK_EUNSUPPORTED, "training: pool needs s = 1, or s = k with d = 1");
                // one byte per element, in the layout of the pool's output
                const size_t tap_bytes = half ? (size_t)octet_floats(n, op.out) * 2 : (size_t)op.out.count(n);
                hipError_t e = st == SK_OK ? hipMalloc(reinterpret_cast<void **>(&net->taps[i]), tap_bytes) : hipSuccess;
                if (e != hipSuccess) st = fail(SK_ENOMEM, "plan: hipMalloc of a pool mask failed: %s", hipGetErrorString(e));
            } else if (op.kind == 0) {
                const ConvParams &c = net->convs[op.param];
                scratch = std::max(scratch, sk::wgrad_f32_scratch_floats(c.c_out, c.c_in, c.k));
                if (op.relu) net->relu_out.insert(op.dst);
                if (half && op.src != net->ops[0].dst && !sk::conv_h_supported(c.k, op.d, c.c_in))
                    st = fail(SK_EUNSUPPORTED, "training: the data gradient of a %dx%d convolution at d = %d to %d maps is not built for 16-bit storage",
                              c.k, c.k, op.d, c.c_in);
            } else if (op.kind == 2) {
                const UpParams &u = net->ups[op.param];
                scratch = std::max(scratch, sk::wgrad_f32_scratch_floats(4 * u.c_out, u.c_in, 1));
                s2d_floats = std::max(s2d_floats, (long)n * 4 * u.c_out * op.in.h * op.in.w);
            }
        }
        if (st == SK_OK) st = alloc_f(&net->wgrad_scratch, (long)scratch);
        if (st == SK_OK) st = alloc_f(&net->s2d, s2d_floats);
        if (st == SK_OK) st = alloc_f(&net->image_copy, (long)n * net->c_in * h_in * w_in);
        if (st == SK_OK && half) st = alloc_f(&net->dz16, octet_floats(n, net->out_dims));
        if (st == SK_OK) st = alloc_f(&net->loss_partial, sk::softmax_loss_partials((long)n * net->out_dims.h * net->out_dims.w));
    }
    if (st != SK_OK) {
        std::string keep = g_last_error;
        net->release_plan();
        g_last_error = keep;
        return st;
    }
    net->planned = true;
    st = warm_up((long)n * net->c_in * h_in * w_in, net->out_dims.count(n), training ? (long)n * net->out_dims.h * net->out_dims.w : 0,
                 [&](const float *img, float *prob) { return unet_forward(net, img, prob, nullptr); },
                 [&](const int32_t *lab, float *loss) { return unet_backward(net, lab, loss, nullptr); });
    net->forward_done = net->backward_done = false;
    if (st != SK_OK) {
        std::string keep = g_last_error;
        net->release_plan();
        g_last_error = keep;
    }
    return st;
}

sk_status unet_set_merge_backward(unet_t *net, int32_t mode)
{
    SK_TRY(check(net));
    if (mode != 0 && mode != 1) return fail(SK_EINVAL, "unet_set_merge_backward: mode must be 0 (up path only) or 1 (skip map as well)");
    net->merge_backward = mode;
    return SK_OK;
}

sk_status unet_plan(unet_t *net, int32_t n, int32_t h_in, int32_t w_in) { return plan_impl(net, n, h_in, w_in, false); }

sk_status unet_plan_training(unet_t *net, int32_t n, int32_t h_in, int32_t w_in) { return plan_impl(net, n, h_in, w_in, true); }

sk_status unet_forward(unet_t *net, const float *image_dev, float *prob_dev, void *hip_stream)
{
    SK_TRY(check(net));
    if (!net->planned) return fail(SK_ESTATE, "unet_forward: call unet_plan first");
    if (!image_dev || !prob_dev) return fail(SK_EINVAL, "unet_forward: null buffer");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    net->last_stream = stream;
    const int n = net->n;
    const int dt = net->dtype;
    for (size_t opi = 0; opi < net->ops.size(); ++opi) {
        const auto &op = net->ops[opi];
        const float *src = op.src ? op.src : image_dev;
        if (dt != SK_F32) {
            // 16-bit storage: the same sequence on the octet layout
            if (op.kind == 4) {
                SK_HIP(sk::launch_pad_pack_h(image_dev, op.dst, dt, n, op.in.c, op.in.h, op.in.w, 0, 0, op.in.h, op.in.w, 0, stream));
            } else if (op.kind == 0) {
                const ConvParams &c = net->convs[op.param];
                const bool to_logits = op.dst == net->logits;     // the last conv leaves fp32 NCHW
                sk::ConvHArgs a = conv_h_args(c, dt, src, n, op.in, op.d, op.relu, op.dst, op.out, to_logits, net->zero_page);
                SK_HIP(sk::launch_conv_h(a, stream));
            } else if (op.kind == 1) {
                SK_HIP(sk::launch_maxpool_h(src, op.dst, net->training ? net->taps[opi] : nullptr, dt, (long)n * ((op.in.c + 7) / 8), op.in.h, op.in.w,
                                            op.out.h, op.out.w, op.k, op.d, op.s, stream));
            } else if (op.kind == 2) {
                const UpParams &u = net->ups[op.param];
                if (u.c_out % 16 == 0) {
                    // one 1x1 convolution to 4*c_out maps; the epilogue puts tap t of map o at (2y + t/2, 2x + t%2)
                    Dims lowres = {4 * u.c_out, op.in.h, op.in.w};
                    sk::ConvHArgs a = conv_h_args(u.cat, dt, src, n, op.in, 1, 0, op.dst, lowres, false, net->zero_page);
                    a.c8_out_total = (op.out.c + 7) / 8; a.o8_off = 0; a.OH = op.out.h; a.OW = op.out.w;
                    a.oy_mul = 2; a.oy_off = 0; a.ox_mul = 2; a.ox_off = 0; a.tap_maps = u.c_out;
                    SK_HIP(sk::launch_conv_h(a, stream));
                } else {
                    for (int t = 0; t < 4; ++t) {
                        Dims lowres = {u.c_out, op.in.h, op.in.w};
                        sk::ConvHArgs a = conv_h_args(u.tap[t], dt, src, n, op.in, 1, 0, op.dst, lowres, false, net->zero_page);
                        a.c8_out_total = (op.out.c + 7) / 8; a.o8_off = 0; a.OH = op.out.h; a.OW = op.out.w;
                        a.oy_mul = 2; a.oy_off = t / 2; a.ox_mul = 2; a.ox_off = t % 2;
                        SK_HIP(sk::launch_conv_h(a, stream));
                    }
                }
            } else {
                SK_HIP(sk::launch_crop_copy_h(src, op.dst, n, op.src_maps / 8, op.in.h, op.in.w, (op.out.c + 7) / 8, op.o_off / 8,
                                              op.out.h, op.out.w, op.crop, (op.in.w - op.out.w) / 2, stream));
            }
            continue;
        }
        if (op.kind == 0) {
            const ConvParams &c = net->convs[op.param];
            sk::ConvF32Args a = conv_args(c, src, n, op.in, op.d, op.relu, op.dst, op.out);
            SK_HIP(sk::launch_conv_f32(a, stream));
        } else if (op.kind == 1) {
            SK_HIP(sk::launch_maxpool_f32(src, op.dst, net->training ? net->taps[opi] : nullptr, n * op.in.c, op.in.h, op.in.w, op.out.h, op.out.w,
                                          op.k, op.d, op.s, stream));
        } else if (op.kind == 2) {
            const UpParams &u = net->ups[op.param];
            if (u.c_out % 16 == 0) {
                // one 1x1 convolution to 4*c_out maps; the epilogue puts tap t of map o at (2y + t/2, 2x + t%2)
                Dims lowres = {4 * u.c_out, op.in.h, op.in.w};
                sk::ConvF32Args a = conv_args(u.cat, src, n, op.in, 1, 0, op.dst, lowres);
                a.out_maps = op.out.c; a.OH = op.out.h; a.OW = op.out.w;
                a.oy_mul = 2; a.oy_off = 0; a.ox_mul = 2; a.ox_off = 0; a.tap_maps = u.c_out;
                SK_HIP(sk::launch_conv_f32(a, stream));
            } else {
                for (int t = 0; t < 4; ++t) {
                    Dims lowres = {u.c_out, op.in.h, op.in.w};
                    sk::ConvF32Args a = conv_args(u.tap[t], src, n, op.in, 1, 0, op.dst, lowres);
                    a.out_maps = op.out.c; a.OH = op.out.h; a.OW = op.out.w;
                    a.oy_mul = 2; a.oy_off = t / 2; a.ox_mul = 2; a.ox_off = t % 2;
                    SK_HIP(sk::launch_conv_f32(a, stream));
                }
            }
        } else {
            SK_HIP(sk::launch_crop_copy_f32(src, op.dst, n, op.src_maps, op.in.h, op.in.w, op.out.c, op.o_off,
                                            op.out.h, op.out.w, op.crop, (op.in.w - op.out.w) / 2, stream));
        }
    }
    SK_HIP(sk::launch_softmax_f32(net->logits, prob_dev, n, net->out_dims.c, net->out_dims.h * net->out_dims.w, stream));
    if (net->training && dt == SK_F32)          // (16-bit plans keep the image in their first buffer, in the octet layout)
        SK_HIP(hipMemcpyAsync(net->image_copy, image_dev, sizeof(float) * (size_t)n * net->c_in * net->h_in * net->w_in,
                              hipMemcpyDeviceToDevice, stream));
    net->forward_done = true;
    net->backward_done = false;
    return SK_OK;
}

// The backward pass on the 16-bit octet layout: the same walk as the fp32 one below, with 16-bit error maps (fp32
// sums inside every kernel, fp32 weight gradients).  The ReLU mask of a convolution's output is applied by whichever
// kernel writes the last contribution to that map's gradient (data gradient, pool gradient or up-convolution gradient).
static sk_status backward_h(unet_t *net, const int32_t *labels_dev, float *loss_dev, hipStream_t stream)
{
    const int n = net->n, dt = net->dtype;
    const Dims &o = net->out_dims;
    const bool direct = sk::softmax_loss_writes_octets(o.c, o.h * o.w);
    SK_HIP(sk::launch_softmax_loss_f32(net->logits, labels_dev, net->grad_of[net->logits], loss_dev, net->loss_partial, n, o.c, o.h * o.w,
                                       stream, direct ? net->dz16 : nullptr, direct ? dt : 0));
    if (!direct) SK_HIP(sk::launch_pad_pack_h(net->grad_of[net->logits], net->dz16, dt, n, o.c, o.h, o.w, 0, 0, o.h, o.w, 0, stream));
    std::set<const float *> written;          // gradient buffers that already hold a contribution
    written.insert(net->logits);
    const float *image16 = net->ops[0].dst;   // the image in the octet layout: needs no gradient
    auto relu_of = [&](const float *buf) -> const float * { return net->relu_out.count(buf) ? buf : nullptr; };
    for (size_t opi = net->ops.size(); opi-- > 1;) {
        const auto &op = net->ops[opi];
        float *gsrc = op.src != image16 ? net->grad_of[op.src] : nullptr;
        if (op.kind == 0) {
            ConvParams &c = net->convs[op.param];
            const float *g = op.dst == net->logits ? net->dz16 : net->grad_of[op.dst];
            SK_HIP(sk::launch_wgrad_h(op.src, g, c.dw, c.db, net->wgrad_scratch, dt, n, op.in.c, op.in.h, op.in.w, c.c_out, c.k, op.d, stream, 0,
                                      net->zero_page));
            if (!gsrc) continue;
            if (written.count(op.src)) return fail(SK_EUNSUPPORTED, "unet_backward: a map that feeds a convolution and another layer");
            sk::ConvHArgs a{};
            a.x = g; a.wp = c.wp16_bwd; a.bias = nullptr; a.mask = relu_of(op.src); a.y = gsrc; a.dtype = dt; a.zeros = net->zero_page;
            a.n = n; a.c8_in = (op.out.c + 7) / 8; a.H = op.out.h; a.W = op.out.w;
            a.c_out = op.in.c; a.c8_out = (op.in.c + 7) / 8;
            a.k = c.k; a.d = op.d; a.in_off = (c.k - 1) * op.d; a.Ho = op.in.h; a.Wo = op.in.w; a.relu = 0; a.out_f32 = 0;
            a.c8_out_total = (op.in.c + 7) / 8; a.o8_off = 0; a.OH = op.in.h; a.OW = op.in.w;
            a.oy_mul = 1; a.oy_off = 0; a.ox_mul = 1; a.ox_off = 0;
            SK_HIP(sk::launch_conv_h(a, stream));
            written.insert(op.src);
        } else if (op.kind == 1) {
            const float *g = net->grad_of[op.dst];
            const int acc = written.count(op.src) ? 1 : 0;
            const long planes8 = (long)n * ((op.in.c + 7) / 8);
            if (op.s == 1) {
                if (acc) return fail(SK_EUNSUPPORTED, "unet_backward: a map that feeds a stride-1 pool and another layer");
                SK_HIP(sk::launch_maxpool_bwd_h(g, net->taps[opi], relu_of(op.src), gsrc, dt, planes8, op.in.h, op.in.w, op.out.h, op.out.w, op.k,
                                                op.d, stream));
            } else {
                SK_HIP(sk::launch_maxpool_stride_bwd_h(g, net->taps[opi], relu_of(op.src), gsrc, dt, planes8, op.in.h, op.in.w, op.out.h, op.out.w,
                                                       op.k, acc, stream));
            }
            written.insert(op.src);
        } else if (op.kind == 2) {
            UpParams &u = net->ups[op.param];
            const float *gm = net->grad_of[op.dst];       // gradient of the merged buffer: the up path is its first c_out maps
            SK_HIP(sk::launch_space_to_depth2_h(gm, net->s2d, n, (op.out.c + 7) / 8, u.c_out / 8, op.in.h, op.in.w, stream));
            SK_HIP(sk::launch_wgrad_h(op.src, net->s2d, u.cat.dw, u.cat.db, net->wgrad_scratch, dt, n, u.c_in, op.in.h, op.in.w, 4 * u.c_out, 1, 1,
                                      stream, 0, net->zero_page));
            if (written.count(op.src)) return fail(SK_EUNSUPPORTED, "unet_backward: a map that feeds an up-convolution and another layer");
            sk::ConvHArgs a{};
            a.x = net->s2d; a.wp = u.cat.wp16_bwd; a.bias = nullptr; a.mask = relu_of(op.src); a.y = gsrc; a.dtype = dt; a.zeros = net->zero_page;
            a.n = n; a.c8_in = 4 * u.c_out / 8; a.H = op.in.h; a.W = op.in.w;
            a.c_out = u.c_in; a.c8_out = (u.c_in + 7) / 8;
            a.k = 1; a.d = 1; a.in_off = 0; a.Ho = op.in.h; a.Wo = op.in.w; a.relu = 0; a.out_f32 = 0;
            a.c8_out_total = (u.c_in + 7) / 8; a.o8_off = 0; a.OH = op.in.h; a.OW = op.in.w;
            a.oy_mul = 1; a.oy_off = 0; a.ox_mul = 1; a.ox_off = 0;
            SK_HIP(sk::launch_conv_h(a, stream));
            written.insert(op.src);
        } else if (op.kind == 3) {
            if (!net->merge_backward) continue;    // backwarding enabled for the up path only
            if (written.count(op.src)) return fail(SK_EUNSUPPORTED, "unet_backward: MergeCrop must be the last consumer of its skip map");
            // (the pool that also reads the skip map adds its gradient afterwards and applies the map's ReLU mask to the sum)
            SK_HIP(sk::launch_place_h(net->grad_of[op.dst], gsrc, n, op.src_maps / 8, op.in.h, op.in.w, (op.out.c + 7) / 8, op.o_off / 8,
                                      op.out.h, op.out.w, op.crop, (op.in.w - op.out.w) / 2, stream));
            written.insert(op.src);
        }
    }
    return SK_OK;
}

// Gradient of the (optionally masked) mean softmax loss with respect to every parameter: the
// forward ops in reverse order.  Conv: ReLU mask, weight/bias gradient, data gradient (the forward
// kernel with flipped, transposed weights and zero padding).  Pool: to the recorded winner.
// Up-convolution: the gradient's four interleaved sub-images stacked as 4*c_out maps turn it into a 1x1
// convolution, whose weight and data gradients are the up-convolution's.  MergeCrop (Section 5.3.1):
// the up path's maps go back to the up-convolution; the skip map takes its gradient from the pool it
// also feeds and nothing from MergeCrop (merge_backward 0, the section's rule for these nets), or
// (merge_backward 1, the exact derivative) MergeCrop's skip maps are also copied into the centre
// window of the skip gradient, zero elsewhere, and the pool's gradient is added to them.
sk_status unet_backward(unet_t *net, const int32_t *labels_dev, float *loss_dev, void *hip_stream)
{
    SK_TRY(check(net));
    if (!net->planned || !net->training) return fail(SK_ESTATE, "unet_backward: needs a training plan (unet_plan_training)");
    if (!net->forward_done) return fail(SK_ESTATE, "unet_backward: no forward pass yet");
    if (!labels_dev || !loss_dev) return fail(SK_EINVAL, "unet_backward: null buffer");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    net->last_stream = stream;
    const int n = net->n;
    const Dims &o = net->out_dims;
    if (net->dtype != SK_F32) {
        SK_TRY(backward_h(net, labels_dev, loss_dev, stream));
        net->backward_done = true;
        return SK_OK;
    }
    SK_HIP(sk::launch_softmax_loss_f32(net->logits, labels_dev, net->grad_of[net->logits], loss_dev, net->loss_partial, n, o.c,
                                       o.h * o.w, stream));
    std::set<const float *> written;          // gradient buffers that already hold a contribution
    written.insert(net->logits);
    for (size_t opi = net->ops.size(); opi-- > 0;) {
        const auto &op = net->ops[opi];
        float *gsrc = op.src ? net->grad_of[op.src] : nullptr;
        if (op.kind == 0) {
            ConvParams &c = net->convs[op.param];
            float *g = net->grad_of[op.dst];
            if (op.relu) SK_HIP(sk::launch_relu_mask_f32(g, op.dst, op.out.count(n), stream));
            const float *x = op.src ? op.src : net->image_copy;
            SK_HIP(sk::launch_wgrad_f32(x, g, c.dw, c.db, net->wgrad_scratch, n, op.in.c, op.in.h, op.in.w, c.c_out, c.k, op.d, stream));
            if (!op.src) continue;                 // the image needs no gradient
            if (written.count(op.src)) return fail(SK_EUNSUPPORTED, "unet_backward: a map that feeds a convolution and another layer");
            sk::ConvF32Args a{};
            a.x = g; a.wp = c.wp_bwd; a.bias = nullptr; a.mask = nullptr; a.y = gsrc;
            a.n = n; a.c_in = op.out.c; a.H = op.out.h; a.W = op.out.w;
            a.c_out = op.in.c; a.n_pad = c.n_pad_bwd;
            a.k = c.k; a.d = op.d; a.in_off = (c.k - 1) * op.d;
            a.Ho = op.in.h; a.Wo = op.in.w; a.relu = 0;
            a.out_maps = op.in.c; a.o_off = 0; a.OH = op.in.h; a.OW = op.in.w;
            a.oy_mul = 1; a.oy_off = 0; a.ox_mul = 1; a.ox_off = 0;
            SK_HIP(sk::launch_conv_f32(a, stream));
            written.insert(op.src);
        } else if (op.kind == 1) {
            const float *g = net->grad_of[op.dst];
            const int acc = written.count(op.src) ? 1 : 0;
            if (op.s == 1) {
                if (acc) return fail(SK_EUNSUPPORTED, "unet_backward: a map that feeds a stride-1 pool and another layer");
                SK_HIP(sk::launch_maxpool_bwd_f32(g, net->taps[opi], nullptr, gsrc, n * op.in.c, op.in.h, op.in.w, op.out.h, op.out.w,
                                                  op.k, op.d, stream));
            } else {
                SK_HIP(sk::launch_maxpool_stride_bwd_f32(g, net->taps[opi], gsrc, n * op.in.c, op.in.h, op.in.w, op.out.h, op.out.w,
                                                         op.k, acc, stream));
            }
            written.insert(op.src);
        } else if (op.kind == 2) {
            UpParams &u = net->ups[op.param];
            const float *gm = net->grad_of[op.dst];       // gradient of the merged buffer: the up path is its first c_out maps
            SK_HIP(sk::launch_space_to_depth2_f32(gm, net->s2d, n, op.out.c, u.c_out, op.in.h, op.in.w, stream));
            SK_HIP(sk::launch_wgrad_f32(op.src, net->s2d, u.cat.dw, u.cat.db, net->wgrad_scratch, n, u.c_in, op.in.h, op.in.w,
                                        4 * u.c_out, 1, 1, stream));
            if (written.count(op.src)) return fail(SK_EUNSUPPORTED, "unet_backward: a map that feeds an up-convolution and another layer");
            sk::ConvF32Args a{};
            a.x = net->s2d; a.wp = u.cat.wp_bwd; a.bias = nullptr; a.mask = nullptr; a.y = gsrc;
            a.n = n; a.c_in = 4 * u.c_out; a.H = op.in.h; a.W = op.in.w;
            a.c_out = u.c_in; a.n_pad = u.cat.n_pad_bwd;
            a.k = 1; a.d = 1; a.in_off = 0;
            a.Ho = op.in.h; a.Wo = op.in.w; a.relu = 0;
            a.out_maps = u.c_in; a.o_off = 0; a.OH = op.in.h; a.OW = op.in.w;
            a.oy_mul = 1; a.oy_off = 0; a.ox_mul = 1; a.ox_off = 0;
            SK_HIP(sk::launch_conv_f32(a, stream));
            written.insert(op.src);
        } else if (op.kind == 3) {
            if (!net->merge_backward) continue;    // backwarding enabled for the up path only
            const float *gm = net->grad_of[op.dst];
            if (written.count(op.src)) return fail(SK_EUNSUPPORTED, "unet_backward: MergeCrop must be the last consumer of its skip map");
            SK_HIP(sk::launch_fill_f32(gsrc, 0.f, (long)n * op.src_maps * op.in.h * op.in.w, stream));
            SK_HIP(sk::launch_place_f32(gm, gsrc, n, op.out.c, op.o_off, op.src_maps, op.out.h, op.out.w, op.in.h, op.in.w, op.crop,
                                        (op.in.w - op.out.w) / 2, stream));
            written.insert(op.src);
        }
    }
    net->backward_done = true;
    return SK_OK;
}

sk_status unet_get_grad(unet_t *net, int32_t idx, float *dw_host, float *db_host)
{
    SK_TRY(check(net));
    if (idx < 0 || idx >= (int)net->params.size()) return fail(SK_EINVAL, "unet_get_grad: bad index");
    if (!net->backward_done) return fail(SK_ESTATE, "unet_get_grad: no backward pass yet");
    SK_HIP(hipStreamSynchronize(net->last_stream));
    const auto &p = net->params[idx];
    if (p.kind == 0) {
        ConvParams &c = net->convs[p.idx];
        if (dw_host) SK_HIP(hipMemcpy(dw_host, c.dw, sizeof(float) * c.wcount(), hipMemcpyDeviceToHost));
        if (db_host) SK_HIP(hipMemcpy(db_host, c.db, sizeof(float) * c.c_out, hipMemcpyDeviceToHost));
        return SK_OK;
    }
    // up-convolution: the stacked 1x1 gradient [t*c_out + o][c] back to [c][o][a][b]; the bias is shared by the four taps
    UpParams &u = net->ups[p.idx];
    std::vector<float> dw((size_t)4 * u.c_out * u.c_in), db((size_t)4 * u.c_out);
    SK_HIP(hipMemcpy(dw.data(), u.cat.dw, sizeof(float) * dw.size(), hipMemcpyDeviceToHost));
    SK_HIP(hipMemcpy(db.data(), u.cat.db, sizeof(float) * db.size(), hipMemcpyDeviceToHost));
    if (dw_host)
        for (int c = 0; c < u.c_in; ++c)
            for (int o2 = 0; o2 < u.c_out; ++o2)
                for (int t = 0; t < 4; ++t)
                    dw_host[((size_t)c * u.c_out + o2) * 4 + t] = dw[((size_t)t * u.c_out + o2) * u.c_in + c];
    if (db_host)
        for (int o2 = 0; o2 < u.c_out; ++o2)
            db_host[o2] = (db[o2] + db[u.c_out + o2]) + (db[2 * u.c_out + o2] + db[3 * u.c_out + o2]);
    return SK_OK;
}

// device masters -> host masters (after SGD steps the device copies are the current ones)
static sk_status sync_masters(unet_t *net)
{
    if (!net->planned || !net->training) return SK_OK;
    if (net->last_stream) SK_HIP(hipStreamSynchronize(net->last_stream));
    for (auto &c : net->convs) {
        SK_HIP(hipMemcpy(c.w.data(), c.w_dev, sizeof(float) * c.wcount(), hipMemcpyDeviceToHost));
        SK_HIP(hipMemcpy(c.b.data(), c.b_dev, sizeof(float) * c.c_out, hipMemcpyDeviceToHost));
    }
    for (auto &u : net->ups) {
        std::vector<float> cat((size_t)4 * u.c_out * u.c_in);
        SK_HIP(hipMemcpy(cat.data(), u.cat.w_dev, sizeof(float) * cat.size(), hipMemcpyDeviceToHost));
        for (int c = 0; c < u.c_in; ++c)
            for (int o2 = 0; o2 < u.c_out; ++o2)
                for (int t = 0; t < 4; ++t) u.w[((size_t)c * u.c_out + o2) * 4 + t] = cat[((size_t)t * u.c_out + o2) * u.c_in + c];
        SK_HIP(hipMemcpy(u.b.data(), u.tap[0].b_dev, sizeof(float) * u.c_out, hipMemcpyDeviceToHost));
    }
    return SK_OK;
}

sk_status unet_sgd_step(unet_t *net, float lr, float momentum, float weight_decay, void *hip_stream)
{
    SK_TRY(check(net));
    if (!net->planned || !net->training || !net->backward_done) return fail(SK_ESTATE, "unet_sgd_step: needs a backward pass on a training plan");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    net->last_stream = stream;
    // every weight and bias tensor (the up-convolutions in their stacked 1x1 form), BATCH_MAX per launch
    sk::SgdBatch sb{};
    auto push = [&](float *w, const float *dw, float *v, long count) -> sk_status {
        sb.w[sb.n] = w; sb.dw[sb.n] = dw; sb.v[sb.n] = momentum != 0.f ? v : nullptr; sb.count[sb.n] = count;
        if (++sb.n == sk::BATCH_MAX) {
            SK_HIP(sk::launch_sgd_batch_f32(sb, lr, momentum, weight_decay, stream));
            sb.n = 0;
        }
        return SK_OK;
    };
    for (auto &c : net->convs) {
        SK_TRY(push(c.w_dev, c.dw, c.vw, c.wcount()));
        SK_TRY(push(c.b_dev, c.db, c.vb, c.c_out));
    }
    for (auto &u : net->ups) SK_TRY(push(u.cat.w_dev, u.cat.dw, u.cat.vw, u.cat.wcount()));
    if (sb.n > 0) SK_HIP(sk::launch_sgd_batch_f32(sb, lr, momentum, weight_decay, stream));
    // the packed forms of every tensor, BATCH_MAX per launch (training plans are fp32)
    sk::PackF32Job jobs[sk::BATCH_MAX];
    int nj = 0;
    auto pack = [&](const ConvParams &c, bool bwd) -> sk_status {
        for (int f = 0; f < (bwd && c.wp_bwd ? 2 : 1); ++f) {
            jobs[nj++] = f == 0 ? sk::PackF32Job{c.w_dev, c.wp_fwd, c.c_out, c.c_in, c.k, 0, c.rows_fwd, c.n_pad}
                                : sk::PackF32Job{c.w_dev, c.wp_bwd, c.c_out, c.c_in, c.k, 1, c.rows_bwd, c.n_pad_bwd};
            if (nj == sk::BATCH_MAX) {
                SK_HIP(sk::launch_pack_weights_f32_batch(jobs, nj, stream));
                nj = 0;
            }
        }
        return SK_OK;
    };
    for (auto &u : net->ups) {
        // the shared bias (its momentum lives in the stacked form's first c_out entries), then the taps' weights
        SK_HIP(sk::launch_up_bias_sgd_f32(u.tap[0].b_dev, u.tap[1].b_dev, u.tap[2].b_dev, u.tap[3].b_dev, u.cat.b_dev, u.cat.db,
                                          momentum != 0.f ? u.cat.vb : nullptr, u.c_out, lr, momentum, weight_decay, stream));
        // (the per-tap weights are only launched where the stacked form is not: map counts off the 16-map tile)
        if (u.c_out % 16 != 0)
            for (int t = 0; t < 4; ++t)
                SK_HIP(hipMemcpyAsync(u.tap[t].w_dev, u.cat.w_dev + (size_t)t * u.c_out * u.c_in, sizeof(float) * u.c_out * u.c_in,
                                      hipMemcpyDeviceToDevice, stream));
    }
    if (net->dtype != SK_F32) {
        // 16-bit plans: the forward and data-gradient packings in the storage type
        sk::PackHJob hj[sk::BATCH_MAX];
        int nh = 0;
        auto pack_h = [&](const ConvParams &c, bool bwd) -> sk_status {
            for (int f = 0; f < (bwd && c.wp16_bwd ? 2 : 1); ++f) {
                hj[nh++] = f == 0 ? sk::PackHJob{c.w_dev, c.wp16_fwd, c.c_out, c.c_in, c.k, 0, c.mt16}
                                  : sk::PackHJob{c.w_dev, c.wp16_bwd, c.c_out, c.c_in, c.k, 1, 0};
                if (nh == sk::BATCH_MAX) {
                    SK_HIP(sk::launch_pack_weights_h_batch(hj, nh, net->dtype, stream));
                    nh = 0;
                }
            }
            return SK_OK;
        };
        for (auto &u : net->ups) {
            if (u.c_out % 16 != 0)
                for (int t = 0; t < 4; ++t) SK_TRY(pack_h(u.tap[t], false));
            SK_TRY(pack_h(u.cat, true));
        }
        for (auto &c : net->convs) SK_TRY(pack_h(c, true));
        if (nh > 0) SK_HIP(sk::launch_pack_weights_h_batch(hj, nh, net->dtype, stream));
        return SK_OK;
    }
    for (auto &u : net->ups) {
        if (u.c_out % 16 != 0)
            for (int t = 0; t < 4; ++t) SK_TRY(pack(u.tap[t], false));
        SK_TRY(pack(u.cat, true));
    }
    for (auto &c : net->convs) SK_TRY(pack(c, true));
    if (nj > 0) SK_HIP(sk::launch_pack_weights_f32_batch(jobs, nj, stream));
    return SK_OK;
}

sk_status unet_get_weights(unet_t *net, int32_t idx, float *w_host, float *b_host)
{
    SK_TRY(check(net));
    if (idx < 0 || idx >= (int)net->params.size()) return fail(SK_EINVAL, "unet_get_weights: bad index");
    SK_TRY(sync_masters(net));
    const auto &p = net->params[idx];
    if (p.kind == 0) {
        const ConvParams &c = net->convs[p.idx];
        if (w_host) std::memcpy(w_host, c.w.data(), sizeof(float) * c.wcount());
        if (b_host) std::memcpy(b_host, c.b.data(), sizeof(float) * c.c_out);
    } else {
        const UpParams &u = net->ups[p.idx];
        if (w_host) std::memcpy(w_host, u.w.data(), sizeof(float) * u.w.size());
        if (b_host) std::memcpy(b_host, u.b.data(), sizeof(float) * u.c_out);
    }
    return SK_OK;
}

sk_status unet_get_activation(unet_t *net, const char *stage, float *nchw_host, int32_t *dims3)
{
    SK_TRY(check(net));
    if (!stage) return fail(SK_EINVAL, "unet_get_activation: stage is null");
    if (!net->planned) return fail(SK_ESTATE, "unet_get_activation: call unet_plan first");
    for (const auto &s : net->stages) {
        if (s.name != stage) continue;
        if (dims3) { dims3[0] = s.dims.c; dims3[1] = s.dims.h; dims3[2] = s.dims.w; }
        if (!nchw_host) return SK_OK;
        if (!net->forward_done) return fail(SK_ESTATE, "unet_get_activation: no forward pass yet");
        SK_HIP(hipStreamSynchronize(net->last_stream));
        // the up path occupies the first maps of the merged buffer: copy image by image
        const int buf_c = s.buf_c;
        const float *src = s.buf;
        if (net->dtype != SK_F32 && s.buf != net->logits) {      // widen the octet layout to fp32 NCHW first
            SK_HIP(sk::launch_unpack_h(s.buf, net->unpack_tmp, net->dtype, net->n, buf_c, s.dims.h, s.dims.w, net->last_stream));
            SK_HIP(hipStreamSynchronize(net->last_stream));
            src = net->unpack_tmp;
        }
        const size_t img = (size_t)s.dims.c * s.dims.h * s.dims.w;
        for (int b = 0; b < net->n; ++b)
            SK_HIP(hipMemcpy(nchw_host + b * img, src + (size_t)b * buf_c * s.dims.h * s.dims.w,
                             sizeof(float) * img, hipMemcpyDeviceToHost));
        return SK_OK;
    }
    return fail(SK_EINVAL, "unet_get_activation: unknown stage '%s'", stage);
}

}  // extern "C"
