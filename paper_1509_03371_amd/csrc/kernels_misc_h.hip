// HBM-bound layers on the 16-bit octet layout ([n][ceil(C/8)][H][W][8] bf16 or fp16): conversion
// from / to fp32 NCHW (with the mirror padding of Section 1.3 fused into the conversion of the
// image), max pooling with kernel stride (forward with winner codes, gather-form backward) and the
// bias gradient.  One 16-byte unit (8 maps of one pixel) per thread, pixels fastest, so a wavefront
// moves 1 KB of consecutive addresses per access.  Comparisons are done on the exactly widened
// fp32 values, so pooling is bit-exact in both formats.
#include "sk_kernels.h"

namespace sk {

typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
typedef unsigned int uint2v __attribute__((ext_vector_type(2)));

static inline int grid_for(long total, int block = 256, int cap = 1 << 20)
{
    long b = (total + block - 1) / block;
    if (b < 1) b = 1;
    return (int)(b < cap ? b : cap);
}

template <int DT> __device__ __forceinline__ float up16(unsigned u);
template <> __device__ __forceinline__ float up16<1>(unsigned u) { return __uint_as_float(u << 16); }
template <> __device__ __forceinline__ float up16<2>(unsigned u) { return (float)__builtin_bit_cast(_Float16, (unsigned short)u); }
template <int DT> __device__ __forceinline__ unsigned down16(float f);
template <> __device__ __forceinline__ unsigned down16<1>(float f) { return __builtin_bit_cast(unsigned short, static_cast<__bf16>(f)); }
template <> __device__ __forceinline__ unsigned down16<2>(float f) { return __builtin_bit_cast(unsigned short, static_cast<_Float16>(f)); }

__device__ __forceinline__ unsigned elem16(const uint4v &u, int e) { return (u[e >> 1] >> ((e & 1) * 16)) & 0xffffu; }

__device__ __forceinline__ int mirror_index_h(int t, int len, int mode)
{
    if (len == 1) return 0;
    if (mode == 0) {
        const int period = 2 * (len - 1);
        t %= period;
        if (t < 0) t += period;
        return t < len ? t : period - t;
    }
    const int period = 2 * len;
    t %= period;
    if (t < 0) t += period;
    return t < len ? t : period - 1 - t;
}

// out[b][o][y][x][e] = in[b][8o+e][m(y-top)][m(x-left)] rounded to nearest even (0 for maps >= c)
template <int DT>
__global__ void pad_pack_h_kernel(const float *in, uint4v *out, int n, int c, int h, int w, int top, int left,
                                  int ho, int wo, int mode)
{
    const int c8 = (c + 7) / 8;
    const long total = (long)n * c8 * ho * wo;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const int x = (int)(q % wo);
        long t = q / wo;
        const int y = (int)(t % ho);
        t /= ho;
        const int o = (int)(t % c8);
        const long b = t / c8;
        const int sy = (top | left) ? mirror_index_h(y - top, h, mode) : y;
        const int sx = (top | left) ? mirror_index_h(x - left, w, mode) : x;
        unsigned hv[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int ch = o * 8 + e;
            hv[e] = ch < c ? down16<DT>(in[((b * c + ch) * h + sy) * (long)w + sx]) : 0u;
        }
        out[q] = uint4v{hv[0] | (hv[1] << 16), hv[2] | (hv[3] << 16), hv[4] | (hv[5] << 16), hv[6] | (hv[7] << 16)};
    }
}

hipError_t launch_pad_pack_h(const float *in, void *out, int dtype, int n, int c, int h, int w, int top, int left,
                             int ho, int wo, int mode, hipStream_t stream)
{
    const long total = (long)n * ((c + 7) / 8) * ho * wo;
    if (dtype == 1)
        hipLaunchKernelGGL(pad_pack_h_kernel<1>, dim3(grid_for(total)), dim3(256), 0, stream, in, static_cast<uint4v *>(out), n, c, h, w, top, left, ho, wo, mode);
    else
        hipLaunchKernelGGL(pad_pack_h_kernel<2>, dim3(grid_for(total)), dim3(256), 0, stream, in, static_cast<uint4v *>(out), n, c, h, w, top, left, ho, wo, mode);
    return hipGetLastError();
}

template <int DT>
__global__ void unpack_h_kernel(const uint4v *in, float *out, int n, int c, int h, int w)
{
    const int c8 = (c + 7) / 8;
    const long plane = (long)h * w, total = (long)n * c8 * plane;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const long pix = q % plane;
        const long t = q / plane;
        const int o = (int)(t % c8);
        const long b = t / c8;
        const uint4v u = in[q];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (o * 8 + e < c) out[(b * c + o * 8 + e) * plane + pix] = up16<DT>(elem16(u, e));
    }
}

hipError_t launch_unpack_h(const void *in, float *out, int dtype, int n, int c, int h, int w, hipStream_t stream)
{
    const long total = (long)n * ((c + 7) / 8) * h * w;
    if (dtype == 1)
        hipLaunchKernelGGL(unpack_h_kernel<1>, dim3(grid_for(total)), dim3(256), 0, stream, static_cast<const uint4v *>(in), out, n, c, h, w);
    else
        hipLaunchKernelGGL(unpack_h_kernel<2>, dim3(grid_for(total)), dim3(256), 0, stream, static_cast<const uint4v *>(in), out, n, c, h, w);
    return hipGetLastError();
}

// ---- max pooling with kernel stride d and layer stride s (Section 5.2.1) on octets --------------------
// grid: x = column blocks, y = output row, z = plane (image x octet); no index division
template <int DT>
__global__ void maxpool_h_kernel(const uint4v *x, uint4v *y, uint2v *tap, int H, int W, int Ho, int Wo,
                                 int k, int d, int s)
{
    const int xx = blockIdx.x * blockDim.x + threadIdx.x, yy = blockIdx.y;
    if (xx >= Wo) return;
    const long p = blockIdx.z;
    const uint4v *src = x + (p * H + (long)s * yy) * W + (long)s * xx;
    const uint4v first = src[0];
    float best[8];
    unsigned bits[8], code[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        bits[e] = elem16(first, e);
        best[e] = up16<DT>(bits[e]);
        code[e] = 0;
    }
    for (int i = 0; i < k; ++i)
        for (int j = 0; j < k; ++j) {
            const uint4v u = src[(long)i * d * W + j * d];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const unsigned b16 = elem16(u, e);
                const float v = up16<DT>(b16);
                if (v > best[e]) {          // strictly greater: the first maximum wins
                    best[e] = v;
                    bits[e] = b16;
                    code[e] = i * k + j;
                }
            }
        }
    const long q = (p * Ho + yy) * Wo + xx;
    y[q] = uint4v{bits[0] | (bits[1] << 16), bits[2] | (bits[3] << 16), bits[4] | (bits[5] << 16), bits[6] | (bits[7] << 16)};
    if (tap)
        tap[q] = uint2v{code[0] | (code[1] << 8) | (code[2] << 16) | (code[3] << 24),
                        code[4] | (code[5] << 8) | (code[6] << 16) | (code[7] << 24)};
}

// k = 2, s = 1 (every SK pool of the paper): window (y, x) is {h[y], h[y + d]} where h[r] is the
// first maximum of X[r][x], X[r][x + d].  A thread walks one column down the rows y0, y0 + d,
// y0 + 2d, ... of one residue class mod d, so each h is formed once and serves both windows it
// belongs to, and a block reads every input row it needs exactly once (no second workgroup, on
// another XCD with another L2, fetches the same rows again).  grid: x = column blocks,
// y = residue class x segments of M chain links, z = plane.  Winner codes follow the row-major
// scan: 0,1 for row y, 2,3 for row y + d, strictly-greater replaces.
template <int DT>
__device__ __forceinline__ void row_first_max(const uint4v a, const uint4v b, uint4v &h, unsigned &hc)
{
    hc = 0u;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        unsigned m = 0u;
        if (up16<DT>(b[w] & 0xffffu) > up16<DT>(a[w] & 0xffffu)) { m |= 0x0000ffffu; hc |= 1u << (2 * w); }
        if (up16<DT>(b[w] >> 16) > up16<DT>(a[w] >> 16)) { m |= 0xffff0000u; hc |= 1u << (2 * w + 1); }
        h[w] = (a[w] & ~m) | (b[w] & m);
    }
}

template <int DT, bool TAP>
__global__ void __launch_bounds__(256) maxpool2_chain_h_kernel(const uint4v *__restrict__ x, uint4v *__restrict__ y,
                                                               uint2v *__restrict__ tap, int H, int W, int Ho, int Wo,
                                                               int d, int M, int nseg)
{
    const int xx = blockIdx.x * 256 + threadIdx.x;
    const int phase = blockIdx.y / nseg, seg = blockIdx.y - phase * nseg;
    if (xx >= Wo || phase >= Ho) return;
    const int links = (Ho - phase + d - 1) / d;           // windows of this residue class
    const int m0 = seg * M, m1 = min(links, m0 + M);
    if (m0 >= m1) return;
    const long p = blockIdx.z;
    const long rstep = (long)d * W;
    const uint4v *src = x + (p * H + phase + (long)m0 * d) * W + xx;
    uint4v *dst = y + (p * Ho + phase + (long)m0 * d) * Wo + xx;
    uint2v *tdst = TAP ? tap + (p * Ho + phase + (long)m0 * d) * Wo + xx : nullptr;
    const long ostep = (long)d * Wo;
    uint4v h;
    unsigned hc;
    row_first_max<DT>(src[0], src[d], h, hc);
    constexpr int U = 4;
    for (int m = m0; m < m1; m += U) {
        uint4v a[U], b[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {                     // all loads of the group first
            const bool live = m + u < m1;
            const uint4v *r = src + (live ? (long)(u + 1) * rstep : 0);
            a[u] = r[0];
            b[u] = r[d];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (m + u >= m1) break;
            uint4v h2;
            unsigned hc2;
            row_first_max<DT>(a[u], b[u], h2, hc2);
            uint4v o;
            unsigned c_lo = 0u, c_hi = 0u;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                unsigned msk = 0u;
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    const int e = 2 * w + hh;
                    const unsigned v1 = hh ? (h[w] >> 16) : (h[w] & 0xffffu), v2 = hh ? (h2[w] >> 16) : (h2[w] & 0xffffu);
                    const bool lower = up16<DT>(v2) > up16<DT>(v1);
                    if (lower) msk |= hh ? 0xffff0000u : 0x0000ffffu;
                    if (TAP) {
                        const unsigned code = lower ? 2u + ((hc2 >> e) & 1u) : ((hc >> e) & 1u);
                        if (e < 4) c_lo |= code << (8 * e); else c_hi |= code << (8 * (e - 4));
                    }
                }
                o[w] = (h[w] & ~msk) | (h2[w] & msk);
            }
            dst[(long)u * ostep] = o;
            if (TAP) tdst[(long)u * ostep] = uint2v{c_lo, c_hi};
            h = h2;
            hc = hc2;
        }
        src += (long)U * rstep;
        dst += (long)U * ostep;
        if (TAP) tdst += (long)U * ostep;
    }
}

hipError_t launch_maxpool_h(const void *x, void *y, void *tap, int dtype, long planes8, int H, int W, int Ho, int Wo,
                            int k, int d, int s, hipStream_t stream)
{
    if (Ho > 65535 || planes8 > 65535) return hipErrorInvalidValue;
    if (k == 2 && s == 1 && Ho == H - d && Wo == W - d) {
        const int M = 32, links = (Ho + d - 1) / d, nseg = (links + M - 1) / M;
        if ((long)d * nseg <= 65535) {
            const dim3 grid((Wo + 255) / 256, (unsigned)(d * nseg), (unsigned)planes8);
            const uint4v *xi = static_cast<const uint4v *>(x);
            uint4v *yo = static_cast<uint4v *>(y);
            uint2v *tp = static_cast<uint2v *>(tap);
            if (dtype == 1) {
                if (tap) hipLaunchKernelGGL((maxpool2_chain_h_kernel<1, true>), grid, dim3(256), 0, stream, xi, yo, tp, H, W, Ho, Wo, d, M, nseg);
                else hipLaunchKernelGGL((maxpool2_chain_h_kernel<1, false>), grid, dim3(256), 0, stream, xi, yo, tp, H, W, Ho, Wo, d, M, nseg);
            } else {
                if (tap) hipLaunchKernelGGL((maxpool2_chain_h_kernel<2, true>), grid, dim3(256), 0, stream, xi, yo, tp, H, W, Ho, Wo, d, M, nseg);
                else hipLaunchKernelGGL((maxpool2_chain_h_kernel<2, false>), grid, dim3(256), 0, stream, xi, yo, tp, H, W, Ho, Wo, d, M, nseg);
            }
            return hipGetLastError();
        }
    }
    const dim3 grid((Wo + 255) / 256, Ho, (unsigned)planes8);
    if (dtype == 1)
        hipLaunchKernelGGL(maxpool_h_kernel<1>, grid, dim3(256), 0, stream, static_cast<const uint4v *>(x),
                           static_cast<uint4v *>(y), static_cast<uint2v *>(tap), H, W, Ho, Wo, k, d, s);
    else
        hipLaunchKernelGGL(maxpool_h_kernel<2>, grid, dim3(256), 0, stream, static_cast<const uint4v *>(x),
                           static_cast<uint4v *>(y), static_cast<uint2v *>(tap), H, W, Ho, Wo, k, d, s);
    return hipGetLastError();
}

// ---- 3-D max pooling on the slice-major octet layout [D][C8][H][W][8] (Section 5.2.2) -----------------------
// Y[z][o8][y][x] = max over the k^3 taps X[s z + a d][o8][s y + i d][s x + j d]; tap (optional, laid out like y, one
// byte per element): the winner's code (a k + i) k + j, the first maximum in that scan order.
// grid: x = column blocks, y = output row, z = (output slice, octet)
template <int DT>
__global__ void maxpool3d_h_kernel(const uint4v *x, uint4v *y, uint2v *tap, int C8, int H, int W, int Ho, int Wo, int k, int d, int s)
{
    const int xx = blockIdx.x * blockDim.x + threadIdx.x, yy = blockIdx.y;
    if (xx >= Wo) return;
    const int zo = blockIdx.z / C8, o8 = blockIdx.z - zo * C8;
    const long plane = (long)H * W;
    const uint4v *src = x + ((long)s * zo * C8 + o8) * plane + (long)s * yy * W + (long)s * xx;
    const uint4v first = src[0];
    float best[8];
    unsigned bits[8], code[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        bits[e] = elem16(first, e);
        best[e] = up16<DT>(bits[e]);
        code[e] = 0;
    }
    for (int a = 0; a < k; ++a)
        for (int i = 0; i < k; ++i)
            for (int j = 0; j < k; ++j) {
                const uint4v u = src[(long)a * d * C8 * plane + (long)i * d * W + j * d];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const unsigned b16 = elem16(u, e);
                    const float v = up16<DT>(b16);
                    if (v > best[e]) {          // strictly greater: the first maximum wins
                        best[e] = v;
                        bits[e] = b16;
                        code[e] = (a * k + i) * k + j;
                    }
                }
            }
    const long q = ((long)blockIdx.z * Ho + yy) * Wo + xx;
    y[q] = uint4v{bits[0] | (bits[1] << 16), bits[2] | (bits[3] << 16), bits[4] | (bits[5] << 16), bits[6] | (bits[7] << 16)};
    if (tap)
        tap[q] = uint2v{code[0] | (code[1] << 8) | (code[2] << 16) | (code[3] << 24),
                        code[4] | (code[5] << 8) | (code[6] << 16) | (code[7] << 24)};
}

// Gather form of the 3-D pool gradient (s = 1) on the slice-major octet layout: input unit (z, u, v) of octet o8 collects,
// per map, dY of the windows whose recorded winner it is; fp32 sums, rounded once; relu_src as in the 2-D kernel.
// grid: x = column blocks, y = input row, z = (input slice, octet)
template <int DT>
__global__ void maxpool3d_bwd_h_kernel(const uint4v *__restrict__ dy, const uint2v *__restrict__ tap, const uint4v *__restrict__ relu_src,
                                       uint4v *__restrict__ dx, int C8, int H, int W, int Do, int Ho, int Wo, int k, int d)
{
    const int v = blockIdx.x * blockDim.x + threadIdx.x, u = blockIdx.y;
    if (v >= W) return;
    const int z = blockIdx.z / C8, o8 = blockIdx.z - z * C8;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    for (int a = 0; a < k; ++a) {
        const int zo = z - a * d;
        if (zo < 0 || zo >= Do) continue;
        for (int i = 0; i < k; ++i) {
            const int yo = u - i * d;
            if (yo < 0 || yo >= Ho) continue;
            for (int j = 0; j < k; ++j) {
                const int xo = v - j * d;
                if (xo < 0 || xo >= Wo) continue;
                const long o = (((long)zo * C8 + o8) * Ho + yo) * Wo + xo;
                const uint2v c = tap[o];
                const uint4v g = dy[o];
                const unsigned want = (unsigned)((a * k + i) * k + j);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const unsigned code = (c[e >> 2] >> ((e & 3) * 8)) & 0xffu;
                    if (code == want) acc[e] += up16<DT>(elem16(g, e));
                }
            }
        }
    }
    const long q = ((long)blockIdx.z * H + u) * W + v;
    uint4v rs = uint4v{0u, 0u, 0u, 0u};
    if (relu_src) rs = relu_src[q];
    unsigned hv[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float t = acc[e];
        if (relu_src && !(up16<DT>(elem16(rs, e)) > 0.f)) t = 0.f;
        hv[e] = down16<DT>(t);
    }
    dx[q] = uint4v{hv[0] | (hv[1] << 16), hv[2] | (hv[3] << 16), hv[4] | (hv[5] << 16), hv[6] | (hv[7] << 16)};
}

hipError_t launch_maxpool3d_bwd_h(const void *dy, const void *tap, const void *relu_src, void *dx, int dtype, int C, int D, int H, int W,
                                  int Do, int Ho, int Wo, int k, int d, hipStream_t stream)
{
    const int C8 = (C + 7) / 8;
    if (H > 65535 || (long)D * C8 > 65535 || (dtype != 1 && dtype != 2) || k < 1 || k > 6) return hipErrorInvalidValue;
    if (Do != D - (k - 1) * d || Ho != H - (k - 1) * d || Wo != W - (k - 1) * d || Do < 1 || Ho < 1 || Wo < 1) return hipErrorInvalidValue;
    const dim3 grid((W + 255) / 256, H, (unsigned)(D * C8));
    const uint4v *g = static_cast<const uint4v *>(dy), *rs = static_cast<const uint4v *>(relu_src);
    const uint2v *tp = static_cast<const uint2v *>(tap);
    uint4v *out = static_cast<uint4v *>(dx);
    if (dtype == 1) hipLaunchKernelGGL(maxpool3d_bwd_h_kernel<1>, grid, dim3(256), 0, stream, g, tp, rs, out, C8, H, W, Do, Ho, Wo, k, d);
    else hipLaunchKernelGGL(maxpool3d_bwd_h_kernel<2>, grid, dim3(256), 0, stream, g, tp, rs, out, C8, H, W, Do, Ho, Wo, k, d);
    return hipGetLastError();
}

// winner codes of a 3-D pool on the octet layout -> flat offsets ((z_in*H + y_in)*W + x_in) inside the map's input
// volume, int32 [Do][C][Ho][Wo] (for the parity accessor)
__global__ void tap3d_to_index_h_kernel(const uint2v *tap, int32_t *idx, int C, int Do, int Ho, int Wo, int H, int W, int k, int d, int s,
                                        long total)
{
    const int C8 = (C + 7) / 8;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const int xo = (int)(q % Wo);
        long t = q / Wo;
        const int yo = (int)(t % Ho);
        t /= Ho;
        const int c = (int)(t % C), zo = (int)(t / C);
        const uint2v w = tap[(((long)zo * C8 + (c >> 3)) * Ho + yo) * Wo + xo];
        const int e = c & 7;
        const int code = (int)((w[e >> 2] >> ((e & 3) * 8)) & 0xffu);
        const int j = code % k, i = (code / k) % k, a = code / (k * k);
        idx[q] = (int32_t)((((long)s * zo + a * d) * H + s * yo + i * d) * W + s * xo + j * d);
    }
}

hipError_t launch_tap3d_to_index_h(const void *tap, int32_t *idx, int C, int Do, int Ho, int Wo, int H, int W, int k, int d, int s,
                                   hipStream_t stream)
{
    const long total = (long)C * Do * Ho * Wo;
    hipLaunchKernelGGL(tap3d_to_index_h_kernel, dim3(grid_for(total)), dim3(256), 0, stream, static_cast<const uint2v *>(tap), idx, C, Do, Ho, Wo,
                       H, W, k, d, s, total);
    return hipGetLastError();
}

// A 3-D kernel [o][c][a][i][j] (fp32 master) as the OIHW master of the 2-D convolution that computes it on the slice-major
// octet layout.  Forward (bwd = 0): out[o][a * C8*8 + c][i][j] = w[o][c][a][i][j] (c_out x k*C8*8 maps; the maps an octet pads
// stay zero).  Data gradient (bwd = 1): out[a' * O8*8 + o][c][i][j] = w[o][c][k-1-a'][i][j] (k*O8*8 x c_in maps), which the
// 2-D data-gradient packing then flips in the plane and transposes.
__global__ void expand_taps3d_kernel(const float *__restrict__ w, float *__restrict__ out, int c_out, int c_in, int k, int bwd, long total)
{
    const int kk = k * k, C8 = (c_in + 7) / 8 * 8, O8 = (c_out + 7) / 8 * 8;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const int r = (int)(q % kk);
        long t = q / kk;
        float v = 0.f;
        if (!bwd) {
            const int m = (int)(t % (k * C8)), o = (int)(t / (k * C8));
            const int a = m / C8, c = m - a * C8;
            if (c < c_in) v = w[(((long)o * c_in + c) * k + a) * kk + r];
        } else {
            const int c = (int)(t % c_in), m = (int)(t / c_in);
            const int a = m / O8, o = m - a * O8;
            if (o < c_out) v = w[(((long)o * c_in + c) * k + (k - 1 - a)) * kk + r];
        }
        out[q] = v;
    }
}

hipError_t launch_expand_taps3d(const float *w, float *out, int c_out, int c_in, int k, int bwd, hipStream_t stream)
{
    if (c_out < 1 || c_in < 1 || k < 1) return hipErrorInvalidValue;
    const long total = bwd ? (long)k * ((c_out + 7) / 8 * 8) * c_in * k * k : (long)c_out * k * ((c_in + 7) / 8 * 8) * k * k;
    hipLaunchKernelGGL(expand_taps3d_kernel, dim3(grid_for(total)), dim3(256), 0, stream, w, out, c_out, c_in, k, bwd, total);
    return hipGetLastError();
}

hipError_t launch_maxpool3d_h(const void *x, void *y, void *tap, int dtype, int C, int D, int H, int W, int Do, int Ho, int Wo, int k, int d,
                              int s, hipStream_t stream)
{
    const int C8 = (C + 7) / 8;
    if (Ho > 65535 || (long)Do * C8 > 65535 || (dtype != 1 && dtype != 2) || D < 1) return hipErrorInvalidValue;
    const dim3 grid((Wo + 255) / 256, Ho, (unsigned)(Do * C8));
    if (dtype == 1)
        hipLaunchKernelGGL(maxpool3d_h_kernel<1>, grid, dim3(256), 0, stream, static_cast<const uint4v *>(x), static_cast<uint4v *>(y),
                           static_cast<uint2v *>(tap), C8, H, W, Ho, Wo, k, d, s);
    else
        hipLaunchKernelGGL(maxpool3d_h_kernel<2>, grid, dim3(256), 0, stream, static_cast<const uint4v *>(x), static_cast<uint4v *>(y),
                           static_cast<uint2v *>(tap), C8, H, W, Ho, Wo, k, d, s);
    return hipGetLastError();
}

// MergeCrop's second operand on octets (Section 5.3.1): dst[b][o8_off + o][y][x] = src[b][o][y + cy][x + cx]
__global__ void crop_copy_h_kernel(const uint4v *__restrict__ src, uint4v *__restrict__ dst, int n, int c8, int Hs, int Ws,
                                   int c8_total, int o8_off, int H, int W, int cy, int cx)
{
    const long plane = (long)H * W, total = (long)n * c8 * plane;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const long pix = q % plane, t = q / plane;
        const int x = (int)(pix % W), y = (int)(pix / W);
        const int o = (int)(t % c8);
        const long b = t / c8;
        dst[((b * c8_total + o8_off + o) * H + y) * W + x] = src[((b * c8 + o) * Hs + y + cy) * Ws + x + cx];
    }
}

hipError_t launch_crop_copy_h(const void *src, void *dst, int n, int c8, int Hs, int Ws, int c8_total, int o8_off,
                              int H, int W, int cy, int cx, hipStream_t stream)
{
    if (cy < 0 || cx < 0 || cy + H > Hs || cx + W > Ws || o8_off < 0 || o8_off + c8 > c8_total) return hipErrorInvalidValue;
    const long total = (long)n * c8 * H * W;
    hipLaunchKernelGGL(crop_copy_h_kernel, dim3(grid_for(total)), dim3(256), 0, stream, static_cast<const uint4v *>(src),
                       static_cast<uint4v *>(dst), n, c8, Hs, Ws, c8_total, o8_off, H, W, cy, cx);
    return hipGetLastError();
}

// Gather form of the pool gradient (s = 1): input unit (u, v) collects, per map, dY of the windows
// whose recorded winner it is.  Sums are formed in fp32 and rounded once.  relu_src (optional,
// same shape as dx) zeroes the result where the layer below produced a non-positive value.
// K > 0: compile-time kernel size, the K*K code and gradient octets fetched together (windows outside the
// output read unit 0 and are discarded); K = 0: any k.
template <int DT, int K>
__global__ void maxpool_bwd_h_kernel(const uint4v *__restrict__ dy, const uint2v *__restrict__ tap, const uint4v *__restrict__ relu_src,
                                     uint4v *__restrict__ dx, int H, int W, int Ho, int Wo, int k, int d)
{
    const int v = blockIdx.x * blockDim.x + threadIdx.x, u = blockIdx.y;
    if (v >= W) return;
    const long p = blockIdx.z;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    if constexpr (K > 0) {
        long o[K * K];
        bool ok[K * K];
#pragma unroll
        for (int t = 0; t < K * K; ++t) {
            const int yy = u - (t / K) * d, xx = v - (t % K) * d;
            ok[t] = yy >= 0 && yy < Ho && xx >= 0 && xx < Wo;
            o[t] = ok[t] ? (p * Ho + yy) * Wo + xx : 0;
        }
        uint2v c[K * K];
        uint4v g[K * K];
#pragma unroll
        for (int t = 0; t < K * K; ++t) c[t] = tap[o[t]];
#pragma unroll
        for (int t = 0; t < K * K; ++t) g[t] = dy[o[t]];
#pragma unroll
        for (int t = 0; t < K * K; ++t)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const unsigned code = (c[t][e >> 2] >> ((e & 3) * 8)) & 0xffu;
                acc[e] += (ok[t] && code == (unsigned)t) ? up16<DT>(elem16(g[t], e)) : 0.f;
            }
    } else
    for (int i = 0; i < k; ++i) {
        const int yy = u - i * d;
        if (yy < 0 || yy >= Ho) continue;
        for (int j = 0; j < k; ++j) {
            const int xx = v - j * d;
            if (xx < 0 || xx >= Wo) continue;
            const long o = (p * Ho + yy) * Wo + xx;
            const uint2v c = tap[o];
            const uint4v g = dy[o];
            const unsigned want = i * k + j;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const unsigned code = (c[e >> 2] >> ((e & 3) * 8)) & 0xffu;
                if (code == want) acc[e] += up16<DT>(elem16(g, e));
            }
        }
    }
    const long q = (p * H + u) * W + v;
    unsigned hv[8];
    uint4v rs = uint4v{0u, 0u, 0u, 0u};
    if (relu_src) rs = relu_src[q];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float a = acc[e];
        if (relu_src && !(up16<DT>(elem16(rs, e)) > 0.f)) a = 0.f;
        hv[e] = down16<DT>(a);
    }
    dx[q] = uint4v{hv[0] | (hv[1] << 16), hv[2] | (hv[3] << 16), hv[4] | (hv[5] << 16), hv[6] | (hv[7] << 16)};
}

hipError_t launch_maxpool_bwd_h(const void *dy, const void *tap, const void *relu_src, void *dx, int dtype,
                                long planes8, int H, int W, int Ho, int Wo, int k, int d, hipStream_t stream)
{
    if (H > 65535 || planes8 > 65535) return hipErrorInvalidValue;
    const dim3 grid((W + 255) / 256, H, (unsigned)planes8);
    const uint4v *g = static_cast<const uint4v *>(dy), *rs = static_cast<const uint4v *>(relu_src);
    const uint2v *tp = static_cast<const uint2v *>(tap);
    uint4v *out = static_cast<uint4v *>(dx);
    if (dtype == 1 && k == 2) hipLaunchKernelGGL((maxpool_bwd_h_kernel<1, 2>), grid, dim3(256), 0, stream, g, tp, rs, out, H, W, Ho, Wo, k, d);
    else if (dtype == 1) hipLaunchKernelGGL((maxpool_bwd_h_kernel<1, 0>), grid, dim3(256), 0, stream, g, tp, rs, out, H, W, Ho, Wo, k, d);
    else if (k == 2) hipLaunchKernelGGL((maxpool_bwd_h_kernel<2, 2>), grid, dim3(256), 0, stream, g, tp, rs, out, H, W, Ho, Wo, k, d);
    else hipLaunchKernelGGL((maxpool_bwd_h_kernel<2, 0>), grid, dim3(256), 0, stream, g, tp, rs, out, H, W, Ho, Wo, k, d);
    return hipGetLastError();
}

// Gradient of a pool with layer stride s = k at d = 1 (the U-Net pools, Section 3.4): the windows do not overlap, input
// unit (u, v) belongs to window (u / k, v / k) and takes that window's dY where it is the recorded winner; units beyond
// the last window get zero.  acc != 0: added to what dx holds (another consumer of the same map wrote first).  relu_src
// as in the gather form above (applied to the sum).
template <int DT>
__global__ void maxpool_stride_bwd_h_kernel(const uint4v *__restrict__ dy, const uint2v *__restrict__ tap, const uint4v *__restrict__ relu_src,
                                            uint4v *__restrict__ dx, int H, int W, int Ho, int Wo, int k, int acc)
{
    const int v = blockIdx.x * blockDim.x + threadIdx.x, u = blockIdx.y;
    if (v >= W) return;
    const long p = blockIdx.z;
    const int yy = u / k, xx = v / k;
    const unsigned want = (unsigned)((u - yy * k) * k + (v - xx * k));
    const long q = (p * H + u) * W + v;
    float a[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] = 0.f;
    if (yy < Ho && xx < Wo) {
        const long o = (p * Ho + yy) * Wo + xx;
        const uint2v c = tap[o];
        const uint4v g = dy[o];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const unsigned code = (c[e >> 2] >> ((e & 3) * 8)) & 0xffu;
            if (code == want) a[e] = up16<DT>(elem16(g, e));
        }
    }
    if (acc) {
        const uint4v old = dx[q];
#pragma unroll
        for (int e = 0; e < 8; ++e) a[e] += up16<DT>(elem16(old, e));
    }
    uint4v rs = uint4v{0u, 0u, 0u, 0u};
    if (relu_src) rs = relu_src[q];
    unsigned hv[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float t = a[e];
        if (relu_src && !(up16<DT>(elem16(rs, e)) > 0.f)) t = 0.f;
        hv[e] = down16<DT>(t);
    }
    dx[q] = uint4v{hv[0] | (hv[1] << 16), hv[2] | (hv[3] << 16), hv[4] | (hv[5] << 16), hv[6] | (hv[7] << 16)};
}

hipError_t launch_maxpool_stride_bwd_h(const void *dy, const void *tap, const void *relu_src, void *dx, int dtype, long planes8, int H, int W,
                                       int Ho, int Wo, int k, int acc, hipStream_t stream)
{
    if (H > 65535 || planes8 > 65535 || k < 1 || (dtype != 1 && dtype != 2) || Ho * k > H || Wo * k > W) return hipErrorInvalidValue;
    const dim3 grid((W + 255) / 256, H, (unsigned)planes8);
    const uint4v *g = static_cast<const uint4v *>(dy), *rs = static_cast<const uint4v *>(relu_src);
    const uint2v *tp = static_cast<const uint2v *>(tap);
    uint4v *out = static_cast<uint4v *>(dx);
    if (dtype == 1) hipLaunchKernelGGL(maxpool_stride_bwd_h_kernel<1>, grid, dim3(256), 0, stream, g, tp, rs, out, H, W, Ho, Wo, k, acc);
    else hipLaunchKernelGGL(maxpool_stride_bwd_h_kernel<2>, grid, dim3(256), 0, stream, g, tp, rs, out, H, W, Ho, Wo, k, acc);
    return hipGetLastError();
}

// Backward of the 2x2 stride-2 up-convolution (Section 3.4), first step: the gradient of the merged buffer's first c8
// octets (the up path; the buffer has c8_total octets of 2h x 2w) as four interleaved sub-images stacked along the maps:
// out[b][t * c8 + o][y][x] = in[b][o][2y + t/2][2x + t%2].  Bits are moved, nothing is rounded.
__global__ void space_to_depth2_h_kernel(const uint4v *__restrict__ in, uint4v *__restrict__ out, int n, int c8_total, int c8, int h, int w)
{
    const long plane = (long)h * w, total = (long)n * 4 * c8 * plane;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const long pix = q % plane, r = q / plane;
        const int x = (int)(pix % w), y = (int)(pix / w);
        const int o4 = (int)(r % (4 * c8)), t = o4 / c8, o = o4 - t * c8;
        const long b = r / (4 * c8);
        out[q] = in[((b * c8_total + o) * (2 * h) + 2 * y + (t >> 1)) * (2L * w) + 2 * x + (t & 1)];
    }
}

hipError_t launch_space_to_depth2_h(const void *in, void *out, int n, int c8_total, int c8, int h, int w, hipStream_t stream)
{
    if (n < 1 || c8 < 1 || c8 > c8_total || h < 1 || w < 1) return hipErrorInvalidValue;
    const long total = (long)n * 4 * c8 * h * w;
    hipLaunchKernelGGL(space_to_depth2_h_kernel, dim3(grid_for(total)), dim3(256), 0, stream, static_cast<const uint4v *>(in),
                       static_cast<uint4v *>(out), n, c8_total, c8, h, w);
    return hipGetLastError();
}

// MergeCrop's backward into the skip map (Section 5.3.1, when enabled): dst [n][c8][Hd][Wd] takes octets o8_off .. of
// src [n][c8_total][Hs][Ws] in its centre window (offset cy, cx) and zero elsewhere
__global__ void place_h_kernel(const uint4v *__restrict__ src, uint4v *__restrict__ dst, int n, int c8, int Hd, int Wd, int c8_total,
                               int o8_off, int Hs, int Ws, int cy, int cx)
{
    const long plane = (long)Hd * Wd, total = (long)n * c8 * plane;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const long pix = q % plane, r = q / plane;
        const int x = (int)(pix % Wd) - cx, y = (int)(pix / Wd) - cy;
        const int o = (int)(r % c8);
        const long b = r / c8;
        uint4v v = uint4v{0u, 0u, 0u, 0u};
        if (x >= 0 && x < Ws && y >= 0 && y < Hs) v = src[((b * c8_total + o8_off + o) * Hs + y) * Ws + x];
        dst[q] = v;
    }
}

hipError_t launch_place_h(const void *src, void *dst, int n, int c8, int Hd, int Wd, int c8_total, int o8_off, int Hs, int Ws, int cy,
                          int cx, hipStream_t stream)
{
    if (cy < 0 || cx < 0 || cy + Hs > Hd || cx + Ws > Wd || o8_off < 0 || o8_off + c8 > c8_total || n < 1) return hipErrorInvalidValue;
    const long total = (long)n * c8 * Hd * Wd;
    hipLaunchKernelGGL(place_h_kernel, dim3(grid_for(total)), dim3(256), 0, stream, static_cast<const uint4v *>(src), static_cast<uint4v *>(dst),
                       n, c8, Hd, Wd, c8_total, o8_off, Hs, Ws, cy, cx);
    return hipGetLastError();
}

// winner codes on the octet layout -> flat input offsets, int32 NCHW (for the parity accessor)
__global__ void tap_to_index_h_kernel(const uint2v *tap, int32_t *idx, int n, int c, int Ho, int Wo, int W, int k, int d, int s)
{
    const int c8 = (c + 7) / 8;
    const long plane = (long)Ho * Wo, total = (long)n * c8 * plane;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const long pix = q % plane;
        const int xx = (int)(pix % Wo), yy = (int)(pix / Wo);
        const long t = q / plane;
        const int o = (int)(t % c8);
        const long b = t / c8;
        const uint2v cd = tap[q];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (o * 8 + e >= c) continue;
            const int code = (cd[e >> 2] >> ((e & 3) * 8)) & 0xff, i = code / k, j = code - i * k;
            idx[(b * c + o * 8 + e) * plane + pix] = (s * yy + i * d) * W + s * xx + j * d;
        }
    }
}

hipError_t launch_tap_to_index_h(const void *tap, int32_t *idx, int n, int c, int Ho, int Wo, int W, int k, int d, int s,
                                 hipStream_t stream)
{
    const long total = (long)n * ((c + 7) / 8) * Ho * Wo;
    hipLaunchKernelGGL(tap_to_index_h_kernel, dim3(grid_for(total)), dim3(256), 0, stream, static_cast<const uint2v *>(tap), idx, n, c, Ho, Wo, W, k, d, s);
    return hipGetLastError();
}

// db[o] = sum over images and pixels of dY (octet layout), in two stages with a fixed summation
// order: workgroup (s, octet) sums slice s of the pixels of its octet over all images into
// part[(8*octet + e) * slices + s]; wgrad_reduce_kernel (kernels_wgrad_f32.hip) adds the slices.
template <int DT>
__global__ void __launch_bounds__(256) bias_grad_h_kernel(const uint4v *__restrict__ dy, float *__restrict__ part, int n, int c,
                                                          long plane, int slices)
{
    __shared__ float sh[4][8];
    const int c8 = (c + 7) / 8, o = blockIdx.y, sl = blockIdx.x;
    const long per = (plane + slices - 1) / slices, q0 = sl * per, q1 = q0 + per < plane ? q0 + per : plane;
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = 0.f;
    for (int b = 0; b < n; ++b) {
        const uint4v *src = dy + ((long)b * c8 + o) * plane;
        for (long q = q0 + threadIdx.x; q < q1; q += 256) {
            const uint4v u = src[q];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += up16<DT>(elem16(u, e));
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        for (int off = 32; off > 0; off >>= 1) v[e] += __shfl_down(v[e], off, 64);
        if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6][e] = v[e];
    }
    __syncthreads();
    if (threadIdx.x < 8)
        part[(long)(o * 8 + threadIdx.x) * slices + sl] = sh[0][threadIdx.x] + sh[1][threadIdx.x] + sh[2][threadIdx.x] + sh[3][threadIdx.x];
}

hipError_t launch_bias_grad_h(const void *dy, float *part, int dtype, int n, int c, long plane, int slices, hipStream_t stream)
{
    const dim3 grid(slices, (c + 7) / 8);
    if (dtype == 1)
        hipLaunchKernelGGL(bias_grad_h_kernel<1>, grid, dim3(256), 0, stream, static_cast<const uint4v *>(dy), part, n, c, plane, slices);
    else
        hipLaunchKernelGGL(bias_grad_h_kernel<2>, grid, dim3(256), 0, stream, static_cast<const uint4v *>(dy), part, n, c, plane, slices);
    return hipGetLastError();
}

}  // namespace sk
