// 3-D SK net forward (Section 5.2.2's N-dimensional layers, three dimensions): handle, shape inference,
// planning and the launch sequence.  See include/sknet.h for the contract of every entry point.
//
// Volumes live slice-major, [D][C][H][W]: a stack of D multi-map 2-D slices.  With that layout a 3-D
// convolution with kernel stride d is a 2-D SK convolution per output slice z whose input maps are the
// (depth tap a, map c) pairs, found in slice z + a*d.  The output slices form the "images" of one 2-D launch
// (consecutive output slices read overlapping windows of input slices, so the image stride is one slice):
//   d = 1 or k = 1: the k tapped slices are adjacent in memory, i.e. one 2-D convolution with k*C input maps;
//   d > 1, C a multiple of 16: still one launch; the kernel steps over the d - 1 slices between two taps;
//   d > 1 otherwise: one launch per depth tap, each adding to what the previous ones left in the output, the
//          last one applying bias and ReLU.
// The 2-D kernels are used unchanged; nothing here is a separate 3-D multiplication.
#include <hip/hip_runtime.h>

#include <new>

#include "sk_host.h"

using namespace skh;

namespace {

struct Dims3 {
    int c = 0, dz = 0, h = 0, w = 0;
    long count() const { return (long)c * dz * h * w; }
};

// the depth taps [a0, a0 + len) of one 3-D convolution as a 2-D convolution with len*C input maps
struct TapRun {
    int a0 = 0, len = 0;
    ConvParams p;
};

struct Conv3 {
    int c_in = 0, c_out = 0, k = 1, d = 1;
    std::vector<float> w, b;   // host master, [c_out][c_in][k][k][k] and [c_out]
    std::vector<TapRun> runs;
    long wcount() const { return (long)c_out * c_in * k * k * k; }
};

// 2-D weights of a run: map (a - a0)*C + c of the 2-D convolution is depth tap a of map c
void fill_run_weights(const Conv3 &cv, TapRun &r, bool last)
{
    const int k = cv.k, C = cv.c_in;
    ConvParams &p = r.p;
    p.w.assign((size_t)p.wcount(), 0.f);
    for (int o = 0; o < cv.c_out; ++o)
        for (int a = 0; a < r.len; ++a)
            for (int c = 0; c < C; ++c)
                std::memcpy(&p.w[(((size_t)o * p.c_in) + (size_t)a * C + c) * k * k],
                            &cv.w[((((size_t)o * C + c) * k) + r.a0 + a) * k * k], sizeof(float) * k * k);
    p.b.assign((size_t)cv.c_out, 0.f);
    if (last) p.b = cv.b;
}

}  // namespace

struct sknet3d {
    std::vector<sk_layer> layers;
    int c_in = 0, n_classes = 0;
    std::vector<Conv3> convs;
    std::vector<int> conv_of_layer;
    bool planned = false, forward_done = false;
    int dz = 0, h = 0, w = 0;
    std::vector<Dims3> dims;       // dims[0] the volume, dims[i+1] the output of layer i
    std::vector<float *> act;      // act[0] unused (the caller's volume is read in place)
    bool fuse_head = false;        // last two 1x1x1 convolutions + softmax as one kernel
    float *head_w1p = nullptr;
    hipStream_t last_stream = nullptr;
    const float *last_volume = nullptr;

    void release_plan()
    {
        for (auto &p : act) free_dev(p);
        act.clear();
        free_dev(head_w1p);
        for (auto &c : convs)
            for (auto &r : c.runs) release_conv(r.p);
        planned = forward_done = false;
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

sk_status run_layer3(sknet3d *net, int li, hipStream_t stream)
{
    const sk_layer &l = net->layers[li];
    const Dims3 &in = net->dims[li], &out = net->dims[li + 1];
    const float *x = li == 0 ? net->last_volume : net->act[li];
    float *y = net->act[li + 1];
    if (l.kind == SK_MAXPOOL) {
        SK_HIP(sk::launch_maxpool3d_f32(x, y, in.c, in.dz, in.h, in.w, out.dz, out.h, out.w, l.k, l.d, l.s, stream));
        return SK_OK;
    }
    Conv3 &cv = net->convs[net->conv_of_layer[li]];
    const long slice = (long)in.c * in.h * in.w;
    for (size_t r = 0; r < cv.runs.size(); ++r) {
        const TapRun &run = cv.runs[r];
        const bool last = r + 1 == cv.runs.size();
        Dims in2, out2;
        in2.c = run.len * in.c; in2.h = in.h; in2.w = in.w;
        out2.c = out.c; out2.h = out.h; out2.w = out.w;
        sk::ConvF32Args a = conv_args(run.p, x + (long)run.a0 * l.d * slice, out.dz, in2, l.d, last ? l.relu : 0, y, out2);
        a.bias = last ? run.p.b_dev : nullptr;
        a.accumulate = r > 0 ? 1 : 0;
        a.x_bstride = slice;
        if (run.len > 1 && l.d > 1) {
            a.grp_maps = in.c;
            a.grp_skip = (long)(l.d - 1) * slice;
        }
        SK_HIP(sk::launch_conv_f32(a, stream));
    }
    return SK_OK;
}

}  // namespace

extern "C" {

sk_status sknet3d_create(const sk_layer *layers, int32_t n_layers, int32_t c_in, int32_t n_classes, sknet3d_t **out)
{
    if (!out) return fail(SK_EINVAL, "create: out is null");
    *out = nullptr;
    if (!layers || n_layers < 1 || c_in < 1 || n_classes < 1) return fail(SK_EINVAL, "create: bad arguments");
    sknet3d *net = new (std::nothrow) sknet3d;
    if (!net) return fail(SK_ENOMEM, "create: out of host memory");
    net->c_in = c_in; net->n_classes = n_classes;
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
            // one run when the tapped slices are adjacent in memory, or the kernel can step over the d - 1
            // slices between two taps
            const bool adjacent = l.d == 1 || l.k == 1 || sk::conv_f32_groups_supported(l.k, l.d, maps);
            for (int a0 = 0; a0 < l.k; a0 += adjacent ? l.k : 1) {
                TapRun r;
                r.a0 = a0; r.len = adjacent ? l.k : 1;
                r.p.c_in = r.len * maps; r.p.c_out = l.c_out; r.p.k = l.k;
                c.runs.push_back(std::move(r));
            }
            for (size_t r = 0; r < c.runs.size(); ++r) fill_run_weights(c, c.runs[r], r + 1 == c.runs.size());
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
    for (size_t r = 0; r < c.runs.size(); ++r) {
        fill_run_weights(c, c.runs[r], r + 1 == c.runs.size());
        if (net->planned) SK_TRY(upload_conv(c.runs[r].p, false, nullptr));
    }
    if (net->planned && net->fuse_head && conv_idx == (int)net->convs.size() - 2) {
        ConvParams &c1 = c.runs[0].p;
        SK_HIP(sk::launch_pack_head_w1(c1.w_dev, net->head_w1p, SK_F32, c1.c_out, c1.c_in, nullptr));
        SK_HIP(hipStreamSynchronize(nullptr));
    }
    return SK_OK;
}

sk_status sknet3d_plan(sknet3d_t *net, int32_t dz, int32_t h, int32_t w, int32_t mode)
{
    SK_TRY(check3(net));
    if (mode != 0 && mode != 2) return fail(SK_EINVAL, "plan: mode must be 0 (inference) or 2 (inference, every layer kept)");
    std::vector<Dims3> dims;
    SK_TRY(infer3(net, dz, h, w, dims));
    const int L = (int)net->layers.size();
    for (int i = 0; i <= L; ++i)
        if (dims[i].dz > 65535 || dims[i].h > 65535 || dims[i].count() >= (1L << 40))
            return fail(SK_EUNSUPPORTED, "plan: volume too large");
    net->release_plan();
    net->dz = dz; net->h = h; net->w = w;
    net->dims = dims;
    net->act.assign(L + 1, nullptr);
    net->fuse_head = mode == 0 && L >= 2 && net->layers[L - 2].kind == SK_CONV && net->layers[L - 1].kind == SK_CONV &&
                     net->layers[L - 2].k == 1 && net->layers[L - 1].k == 1 && net->layers[L - 2].relu && !net->layers[L - 1].relu &&
                     sk::head_supported(SK_F32, dims[L - 2].c, net->layers[L - 2].c_out, net->layers[L - 1].c_out);
    sk_status st = SK_OK;
    for (int i = 1; i <= L && st == SK_OK; ++i) {
        if (net->fuse_head && i >= L - 1) continue;
        st = alloc_f(&net->act[i], dims[i].count());
    }
    for (auto &c : net->convs)
        for (auto &r : c.runs) {
            if (st == SK_OK) st = alloc_conv(r.p, false);
            if (st == SK_OK) st = upload_conv(r.p, false, nullptr);
        }
    if (st == SK_OK && net->fuse_head) {
        ConvParams &c1 = net->convs[net->conv_of_layer[L - 2]].runs[0].p;
        st = alloc_f(&net->head_w1p, (sk::head_w1_packed_bytes(SK_F32, c1.c_in, c1.c_out) + 3) / 4);
        if (st == SK_OK) {
            hipError_t e = sk::launch_pack_head_w1(c1.w_dev, net->head_w1p, SK_F32, c1.c_out, c1.c_in, nullptr);
            if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
            if (e != hipSuccess) st = fail(SK_EDEVICE, "plan: packing the head weights failed: %s", hipGetErrorString(e));
        }
    }
    if (st != SK_OK) {
        net->release_plan();
        return st;
    }
    net->planned = true;
    return SK_OK;
}

sk_status sknet3d_forward(sknet3d_t *net, const float *volume_dev, float *prob_dev, void *hip_stream)
{
    SK_TRY(check3(net));
    if (!volume_dev || !prob_dev) return fail(SK_EINVAL, "forward: null buffer");
    if (!net->planned) return fail(SK_ESTATE, "forward: call sknet3d_plan first");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    net->last_stream = stream;
    net->last_volume = volume_dev;
    const int L = (int)net->layers.size();
    for (int i = 0; i < (net->fuse_head ? L - 2 : L); ++i) SK_TRY(run_layer3(net, i, stream));
    const Dims3 &o = net->dims[L];
    if (net->fuse_head) {
        const ConvParams &c1 = net->convs[net->conv_of_layer[L - 2]].runs[0].p, &c2 = net->convs[net->conv_of_layer[L - 1]].runs[0].p;
        const Dims3 &in = net->dims[L - 2];
        sk::HeadArgs a{};
        a.x = L - 2 == 0 ? volume_dev : net->act[L - 2];
        a.w1p = net->head_w1p; a.b1 = c1.b_dev; a.w2 = c2.w_dev; a.b2 = c2.b_dev;
        a.prob = prob_dev; a.dtype = SK_F32; a.n = in.dz; a.c_in = in.c; a.H = in.h; a.W = in.w;
        a.hidden = c1.c_out; a.classes = c2.c_out;
        SK_HIP(sk::launch_head_fused(a, stream));
    } else {
        SK_HIP(sk::launch_softmax_f32(net->act[L], prob_dev, o.dz, o.c, o.h * o.w, stream));
    }
    net->forward_done = true;
    return SK_OK;
}

sk_status sknet3d_get_activation(sknet3d_t *net, int32_t layer_idx, float *dchw_host)
{
    SK_TRY(check3(net));
    if (!dchw_host || layer_idx < 0 || layer_idx >= (int)net->layers.size()) return fail(SK_EINVAL, "get_activation: bad arguments");
    if (!net->forward_done) return fail(SK_ESTATE, "get_activation: no forward pass yet");
    if (net->fuse_head && layer_idx >= (int)net->layers.size() - 2)
        return fail(SK_ESTATE, "get_activation: this plan fuses the last two layers; plan with mode 2 to keep them");
    SK_HIP(hipStreamSynchronize(net->last_stream));
    SK_HIP(hipMemcpy(dchw_host, net->act[layer_idx + 1], sizeof(float) * net->dims[layer_idx + 1].count(), hipMemcpyDeviceToHost));
    return SK_OK;
}

}  // extern "C"
