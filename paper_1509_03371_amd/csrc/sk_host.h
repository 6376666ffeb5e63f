// Host-side helpers shared by the SK-Net and U-Net entry points of libsknet (internal).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/sknet.h"
#include "sk_kernels.h"

namespace skh {

inline thread_local std::string g_last_error;

inline sk_status fail(sk_status code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    g_last_error = buf;
    return code;
}

#define SK_HIP(expr)                                                                             \
    do {                                                                                         \
        hipError_t e_ = (expr);                                                                  \
        if (e_ != hipSuccess)                                                                    \
            return fail(e_ == hipErrorOutOfMemory ? SK_ENOMEM : SK_EDEVICE, "%s failed: %s", #expr, \
                        hipGetErrorString(e_));                                                  \
    } while (0)

#define SK_TRY(expr)                    \
    do {                                \
        sk_status s_ = (expr);          \
        if (s_ != SK_OK) return s_;     \
    } while (0)

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

struct Dims {
    int c = 0, h = 0, w = 0;
    long count(int n) const { return (long)n * c * h * w; }
};

// One convolution's parameters: fp32 master copy on the host and on the device, the packed
// forms the kernels read, gradients and momentum.
struct ConvParams {
    int c_in = 0, c_out = 0, k = 1;
    std::vector<float> w, b;   // host master, OIHW and [c_out]
    float *w_dev = nullptr, *b_dev = nullptr;   // b_dev has n_pad entries (zero padded)
    float *wp_fwd = nullptr, *wp_bwd = nullptr;       // fp32 packings
    float *wp16_fwd = nullptr, *wp16_bwd = nullptr;   // 16-bit packings (typed loosely; see kernels_conv_h.hip)
    float *dw = nullptr, *db = nullptr, *vw = nullptr, *vb = nullptr;
    int mt16 = 0;                         // 16-bit forward packing: map tiles per workgroup (0 = default)
    int n_pad = 0, rows_fwd = 0;          // forward packing: [rows_fwd][n_pad]
    int n_pad_bwd = 0, rows_bwd = 0;      // data-gradient packing: [rows_bwd][n_pad_bwd]
    long wcount() const { return (long)c_out * c_in * k * k; }
};

inline void free_dev(float *&p)
{
    if (p) (void)hipFree(p);
    p = nullptr;
}

inline void release_conv(ConvParams &c)
{
    free_dev(c.w_dev); free_dev(c.b_dev); free_dev(c.wp_fwd); free_dev(c.wp_bwd);
    free_dev(c.wp16_fwd); free_dev(c.wp16_bwd);
    free_dev(c.dw); free_dev(c.db); free_dev(c.vw); free_dev(c.vb);
}

inline sk_status alloc_f(float **p, long count)
{
    *p = nullptr;
    if (count <= 0) count = 1;
    SK_HIP(hipMalloc(reinterpret_cast<void **>(p), sizeof(float) * (size_t)count));
    return SK_OK;
}

// rebuild the packed forms of one conv from its device master weights (asynchronous)
inline sk_status repack_conv(ConvParams &c, bool training, int dtype, hipStream_t stream)
{
    if (dtype == SK_F32) {
        SK_HIP(sk::launch_pack_weights_f32(c.w_dev, c.wp_fwd, c.c_out, c.c_in, c.k, 0, c.rows_fwd, c.n_pad, stream));
        if (training && c.wp_bwd)
            SK_HIP(sk::launch_pack_weights_f32(c.w_dev, c.wp_bwd, c.c_out, c.c_in, c.k, 1, c.rows_bwd, c.n_pad_bwd, stream));
    } else {
        SK_HIP(sk::launch_pack_weights_h(c.w_dev, c.wp16_fwd, dtype, c.c_out, c.c_in, c.k, 0, c.mt16, stream));
        if (training && c.wp16_bwd)
            SK_HIP(sk::launch_pack_weights_h(c.w_dev, c.wp16_bwd, dtype, c.c_out, c.c_in, c.k, 1, 0, stream));
    }
    return SK_OK;
}

// upload master weights and rebuild the packed forms (synchronous on `stream`)
inline sk_status upload_conv(ConvParams &c, bool training, hipStream_t stream, int dtype = SK_F32)
{
    SK_HIP(hipMemcpyAsync(c.w_dev, c.w.data(), sizeof(float) * c.wcount(), hipMemcpyHostToDevice, stream));
    std::vector<float> bp(c.n_pad, 0.f);
    std::memcpy(bp.data(), c.b.data(), sizeof(float) * c.c_out);
    SK_HIP(hipMemcpyAsync(c.b_dev, bp.data(), sizeof(float) * c.n_pad, hipMemcpyHostToDevice, stream));
    SK_TRY(repack_conv(c, training, dtype, stream));
    SK_HIP(hipStreamSynchronize(stream));
    return SK_OK;
}

inline sk_status alloc_conv(ConvParams &c, bool training, int dtype = SK_F32)
{
    release_conv(c);
    c.n_pad = round_up(c.c_out, 16);
    c.rows_fwd = round_up(c.c_in, 16) * c.k * c.k;
    c.n_pad_bwd = round_up(c.c_in, 16);
    c.rows_bwd = round_up(c.c_out, 16) * c.k * c.k;
    SK_TRY(alloc_f(&c.w_dev, c.wcount()));
    SK_TRY(alloc_f(&c.b_dev, c.n_pad));
    if (dtype == SK_F32) {
        SK_TRY(alloc_f(&c.wp_fwd, (long)c.rows_fwd * c.n_pad));
        if (training) SK_TRY(alloc_f(&c.wp_bwd, (long)c.rows_bwd * c.n_pad_bwd));
    } else {   // 16-bit elements, allocated in floats
        SK_TRY(alloc_f(&c.wp16_fwd, (sk::packed_h_elems(c.c_out, (c.c_in + 7) / 8, c.k, c.mt16) + 1) / 2));
        if (training) SK_TRY(alloc_f(&c.wp16_bwd, (sk::packed_h_elems(c.c_in, (c.c_out + 7) / 8, c.k) + 1) / 2));
    }
    if (training) {
        SK_TRY(alloc_f(&c.dw, c.wcount()));
        SK_TRY(alloc_f(&c.db, c.c_out));
        SK_TRY(alloc_f(&c.vw, c.wcount()));
        SK_TRY(alloc_f(&c.vb, c.c_out));
        SK_HIP(hipMemset(c.vw, 0, sizeof(float) * c.wcount()));
        SK_HIP(hipMemset(c.vb, 0, sizeof(float) * c.c_out));
    }
    return SK_OK;
}

// element counts on the 16-bit octet layout, expressed in floats (what alloc_f takes)
inline long octet_floats(int n, const Dims &d) { return (long)n * ((d.c + 7) / 8) * d.h * d.w * 4; }

// One pass of a freshly planned net over zero inputs on the null stream, so that whatever a first launch sets
// up (kernel attributes, code loading) has happened when the plan call returns: forward and backward then only
// enqueue kernels, also when the caller records its very first call into a HIP graph.  fwd(image, prob) and
// bwd(labels, loss) run the planned passes; bwd is skipped when label_count is 0.
template <class Fwd, class Bwd>
inline sk_status warm_up(long image_floats, long prob_floats, long label_count, Fwd fwd, Bwd bwd)
{
    float *img = nullptr, *prob = nullptr, *lab = nullptr, *loss = nullptr;
    sk_status st = alloc_f(&img, image_floats);
    if (st == SK_OK) st = alloc_f(&prob, prob_floats);
    if (st == SK_OK && label_count > 0) st = alloc_f(&lab, label_count);
    if (st == SK_OK && label_count > 0) st = alloc_f(&loss, 1);
    hipError_t e = hipSuccess;
    if (st == SK_OK) e = hipMemset(img, 0, sizeof(float) * (size_t)image_floats);
    if (st == SK_OK && e == hipSuccess && lab) e = hipMemset(lab, 0, sizeof(int32_t) * (size_t)label_count);   // every pixel of class 0
    if (st == SK_OK && e != hipSuccess) st = fail(SK_EDEVICE, "plan: clearing the warm-up buffers failed: %s", hipGetErrorString(e));
    if (st == SK_OK) st = fwd(img, prob);
    if (st == SK_OK && lab) st = bwd(reinterpret_cast<const int32_t *>(lab), loss);
    e = hipDeviceSynchronize();
    if (st == SK_OK && e != hipSuccess) st = fail(SK_EDEVICE, "plan: the warm-up pass failed: %s", hipGetErrorString(e));
    free_dev(img); free_dev(prob); free_dev(lab); free_dev(loss);
    return st;
}

// the page of zeros the 16-bit convolution reads for samples outside the image; part of a plan
inline sk_status alloc_zero_page(float **p)
{
    SK_TRY(alloc_f(p, sk::CONV_H_ZERO_BYTES / 4));
    SK_HIP(hipMemset(*p, 0, sk::CONV_H_ZERO_BYTES));
    return SK_OK;
}

inline sk::ConvHArgs conv_h_args(const ConvParams &c, int dtype, const void *x, int n, const Dims &in, int d, int relu,
                                 void *y, const Dims &out, bool out_f32, const void *zeros)
{
    sk::ConvHArgs a{};
    a.zeros = zeros;
    a.x = x; a.wp = c.wp16_fwd; a.bias = c.b_dev; a.mask = nullptr; a.y = y; a.dtype = dtype;
    a.n = n; a.c8_in = (in.c + 7) / 8; a.H = in.h; a.W = in.w;
    a.c_out = c.c_out; a.c8_out = (c.c_out + 7) / 8;
    a.k = c.k; a.d = d; a.in_off = 0; a.Ho = out.h; a.Wo = out.w; a.relu = relu; a.out_f32 = out_f32 ? 1 : 0;
    a.c8_out_total = (out.c + 7) / 8; a.o8_off = 0; a.OH = out.h; a.OW = out.w;
    a.oy_mul = 1; a.oy_off = 0; a.ox_mul = 1; a.ox_off = 0;
    a.mt = c.mt16;
    a.single_map = c.c_in == 1 ? 1 : 0;
    return a;
}

inline sk::ConvF32Args conv_args(const ConvParams &c, const float *x, int n, const Dims &in, int d, int relu,
                          float *y, const Dims &out)
{
    sk::ConvF32Args a{};
    a.x = x; a.wp = c.wp_fwd; a.bias = c.b_dev; a.mask = nullptr; a.y = y;
    a.n = n; a.c_in = in.c; a.H = in.h; a.W = in.w;
    a.c_out = c.c_out; a.n_pad = c.n_pad;
    a.k = c.k; a.d = d; a.in_off = 0;
    a.Ho = out.h; a.Wo = out.w; a.relu = relu;
    a.out_maps = out.c; a.o_off = 0; a.OH = out.h; a.OW = out.w;
    a.oy_mul = 1; a.oy_off = 0; a.ox_mul = 1; a.ox_off = 0;
    return a;
}


}  // namespace skh
