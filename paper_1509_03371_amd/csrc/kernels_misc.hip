// HBM-bound layers of the SK-Net / U-Net path for gfx950: mirror padding, max pooling with
// kernel stride (forward with tap codes, gather-form backward), per-pixel softmax and softmax
// loss, SGD, crop-and-place copy.  One element per thread, x fastest, so that a 64-lane
// wavefront reads and writes consecutive addresses.
#include "sk_kernels.h"

namespace sk {

static inline int grid_for(long total, int block = 256, int cap = 1 << 20)
{
    long b = (total + block - 1) / block;
    if (b < 1) b = 1;
    return (int)(b < cap ? b : cap);
}

// ---- mirror padding (Section 1.3) ---------------------------------------------------------------
__device__ __forceinline__ int mirror_index(int t, int len, int mode)
{
    if (len == 1) return 0;
    if (mode == 0) {                       // reflect: ... 2 1 | 0 1 2 ... L-1 | L-2 L-3 ...
        const int period = 2 * (len - 1);
        t %= period;
        if (t < 0) t += period;
        return t < len ? t : period - t;
    }
    const int period = 2 * len;            // symmetric: ... 1 0 | 0 1 ... L-1 | L-1 L-2 ...
    t %= period;
    if (t < 0) t += period;
    return t < len ? t : period - 1 - t;
}

__global__ void mirror_pad_f32_kernel(const float *in, float *out, int planes, int h, int w, int top,
                                      int left, int ho, int wo, int mode)
{
    const long total = (long)planes * ho * wo;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const int x = (int)(q % wo);
        const long t = q / wo;
        const int y = (int)(t % ho);
        const long p = t / ho;
        out[q] = in[(p * h + mirror_index(y - top, h, mode)) * w + mirror_index(x - left, w, mode)];
    }
}

hipError_t launch_mirror_pad_f32(const float *in, float *out, int planes, int h, int w, int top,
                                 int left, int ho, int wo, int mode, hipStream_t stream)
{
    const long total = (long)planes * ho * wo;
    hipLaunchKernelGGL(mirror_pad_f32_kernel, dim3(grid_for(total)), dim3(256), 0, stream, in, out,
                       planes, h, w, top, left, ho, wo, mode);
    return hipGetLastError();
}

// ---- max pooling with kernel stride d and layer stride s (Section 5.2.1) --------------------------
// grid: x = column blocks, y = output row, z = plane; no index division on the hot path
__global__ void maxpool_f32_kernel(const float *x, float *y, uint8_t *tap, int H, int W, int Ho, int Wo, int k, int d, int s)
{
    const int xx = blockIdx.x * blockDim.x + threadIdx.x, yy = blockIdx.y;
    if (xx >= Wo) return;
    const long p = blockIdx.z;
    const float *src = x + (p * H + (long)s * yy) * W + (long)s * xx;
    float best = src[0];
    int code = 0;
    for (int i = 0; i < k; ++i)
        for (int j = 0; j < k; ++j) {
            const float v = src[(long)i * d * W + j * d];
            if (v > best) {            // strictly greater: the first maximum wins
                best = v;
                code = i * k + j;
            }
        }
    const long q = (p * Ho + yy) * Wo + xx;
    y[q] = best;
    if (tap) tap[q] = (uint8_t)code;
}

// k = 2, s = 1 (every SK pool of the paper): window (y, x) is {h[y], h[y + d]} where h[r] is the
// first maximum of X[r][x], X[r][x + d].  A thread walks one column down the rows y0, y0 + d,
// y0 + 2d, ... of one residue class mod d, so each h is formed once and serves both windows it
// belongs to, and a block reads every input row it needs exactly once.  grid: x = column blocks,
// y = residue class x segments of M chain links, z = plane.  Winner codes follow the row-major
// scan (0,1 for row y; 2,3 for row y + d), strictly-greater replaces.
template <bool TAP>
__global__ void __launch_bounds__(256) maxpool2_chain_f32_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                                 uint8_t *__restrict__ tap, int H, int W, int Ho, int Wo,
                                                                 int d, int M, int nseg)
{
    const int xx = blockIdx.x * 256 + threadIdx.x;
    const int phase = blockIdx.y / nseg, seg = blockIdx.y - phase * nseg;
    if (xx >= Wo || phase >= Ho) return;
    const int links = (Ho - phase + d - 1) / d;
    const int m0 = seg * M, m1 = min(links, m0 + M);
    if (m0 >= m1) return;
    const long p = blockIdx.z;
    const long rstep = (long)d * W, ostep = (long)d * Wo;
    const float *src = x + (p * H + phase + (long)m0 * d) * W + xx;
    float *dst = y + (p * Ho + phase + (long)m0 * d) * Wo + xx;
    uint8_t *tdst = TAP ? tap + (p * Ho + phase + (long)m0 * d) * Wo + xx : nullptr;
    float h = src[0];
    int hc = 0;
    {
        const float b = src[d];
        if (b > h) { h = b; hc = 1; }
    }
    constexpr int U = 8;
    for (int m = m0; m < m1; m += U) {
        float a[U], b[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {                     // all loads of the group first
            const float *r = src + (m + u < m1 ? (long)(u + 1) * rstep : 0);
            a[u] = r[0];
            b[u] = r[d];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (m + u >= m1) break;
            float h2 = a[u];
            int hc2 = 0;
            if (b[u] > h2) { h2 = b[u]; hc2 = 1; }
            const bool lower = h2 > h;
            dst[(long)u * ostep] = lower ? h2 : h;
            if (TAP) tdst[(long)u * ostep] = (uint8_t)(lower ? 2 + hc2 : hc);
            h = h2;
            hc = hc2;
        }
        src += (long)U * rstep;
        dst += (long)U * ostep;
        if (TAP) tdst += (long)U * ostep;
    }
}

hipError_t launch_maxpool_f32(const float *x, float *y, uint8_t *tap, int planes, int H, int W,
                              int Ho, int Wo, int k, int d, int s, hipStream_t stream)
{
    if (Ho > 65535 || planes > 65535) return hipErrorInvalidValue;
    if (k == 2 && s == 1 && Ho == H - d && Wo == W - d) {
        const int M = 32, links = (Ho + d - 1) / d, nseg = (links + M - 1) / M;
        if ((long)d * nseg <= 65535) {
            const dim3 grid((Wo + 255) / 256, (unsigned)(d * nseg), (unsigned)planes);
            if (tap) hipLaunchKernelGGL(maxpool2_chain_f32_kernel<true>, grid, dim3(256), 0, stream, x, y, tap, H, W, Ho, Wo, d, M, nseg);
            else hipLaunchKernelGGL(maxpool2_chain_f32_kernel<false>, grid, dim3(256), 0, stream, x, y, tap, H, W, Ho, Wo, d, M, nseg);
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL(maxpool_f32_kernel, dim3((Wo + 255) / 256, Ho, planes), dim3(256), 0, stream, x, y, tap,
                       H, W, Ho, Wo, k, d, s);
    return hipGetLastError();
}

// ---- 3-D max pooling with kernel stride d and layer stride s on the slice-major layout (Section 5.2.2) ----
// X[D][C][H][W] -> Y[Do][C][Ho][Wo], Y[z,c,y,x] = max_{a,i,j<k} X[s*z + a*d, c, s*y + i*d, s*x + j*d].
// Taps are scanned in the order (a, i, j) and only a strictly greater value replaces the incumbent, so the
// first maximum wins; tap (optional, laid out like y) receives the winner's code (a*k + i)*k + j.
// grid: x = (output slice, column block), y = output row, z = map
__global__ void __launch_bounds__(256) maxpool3d_f32_kernel(const float *__restrict__ x, float *__restrict__ y, uint8_t *__restrict__ tap,
                                                            int C, int H, int W, int Ho, int Wo, int k, int d, int s, int xblocks)
{
    const int zo = blockIdx.x / xblocks, xb = blockIdx.x - zo * xblocks;
    const int xx = xb * 256 + threadIdx.x, yy = blockIdx.y, c = blockIdx.z;
    if (xx >= Wo) return;
    const long plane = (long)H * W;
    const float *src = x + (((long)s * zo * C + c) * H + (long)s * yy) * W + (long)s * xx;
    float best = src[0];
    int code = 0;
    for (int a = 0; a < k; ++a) {
        const float *sl = src + (long)a * d * C * plane;
        for (int i = 0; i < k; ++i)
            for (int j = 0; j < k; ++j) {
                const float v = sl[(long)i * d * W + j * d];
                if (v > best) {
                    best = v;
                    code = (a * k + i) * k + j;
                }
            }
    }
    const long q = (((long)zo * C + c) * Ho + yy) * Wo + xx;
    y[q] = best;
    if (tap) tap[q] = (uint8_t)code;
}

// k = 2, s = 1 (the SK pools of a converted net): a thread owns one output column of one map and walks down
// the slices z0, z0 + d, z0 + 2d, ... of one residue class mod d.  The 2x2 in-slice maximum q[z] of slice z
// serves the windows of the outputs z - d and z, so each is formed once: four loads per output, not eight.
// Winner codes follow the (a, i, j) scan: 0..3 inside slice z, 4..7 inside slice z + d, which only wins
// when strictly greater.
// A workgroup takes 256 consecutive positions of the Ho x Wo plane (rows of 136 outputs would leave half of a
// 256-thread row block idle).  grid: x = (residue class and chain segment, plane block), y = map
template <bool TAP>
__global__ void __launch_bounds__(256) maxpool3d_k2_chain_f32_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                                     uint8_t *__restrict__ tap, int C, int H, int W, int Do, int Ho,
                                                                     int Wo, int d, int M, int nseg, int pblocks)
{
    const int chain = blockIdx.x / pblocks, pb = blockIdx.x - chain * pblocks;
    const int phase = chain / nseg, seg = chain - phase * nseg;
    const int pos = pb * 256 + threadIdx.x, c = blockIdx.y;
    if (pos >= Ho * Wo || phase >= Do) return;
    const int yy = pos / Wo, xx = pos - yy * Wo;
    const int links = (Do - phase + d - 1) / d;
    const int m0 = seg * M, m1 = min(links, m0 + M);
    if (m0 >= m1) return;
    const long plane = (long)H * W, zstep = (long)d * C * plane, ostep = (long)d * C * Ho * Wo;
    const float *src = x + (((long)(phase + m0 * d) * C + c) * H + yy) * W + xx;
    const long o0 = (((long)(phase + m0 * d) * C + c) * Ho + yy) * Wo + xx;
    float *dst = y + o0;
    uint8_t *tdst = TAP ? tap + o0 : nullptr;
    const long dn = (long)d * W;
    int qc = 0;
    auto quad = [&](const float *p, int &code) {
        const float a = p[0], b = p[d], e = p[dn], f = p[dn + d];
        float best = a;
        code = 0;
        if (b > best) { best = b; code = 1; }
        if (e > best) { best = e; code = 2; }
        if (f > best) { best = f; code = 3; }
        return best;
    };
    float q = quad(src, qc);
    for (int m = m0; m < m1; ++m) {
        src += zstep;
        int qc2;
        const float q2 = quad(src, qc2);
        const bool lower = q2 > q;
        *dst = lower ? q2 : q;
        if (TAP) {
            *tdst = (uint8_t)(lower ? 4 + qc2 : qc);
            tdst += ostep;
        }
        dst += ostep;
        q = q2;
        qc = qc2;
    }
}

hipError_t launch_maxpool3d_f32(const float *x, float *y, uint8_t *tap, int C, int D, int H, int W, int Do, int Ho, int Wo, int k,
                                int d, int s, hipStream_t stream)
{
    if (C < 1 || C > 65535 || Ho < 1 || Ho > 65535 || Do < 1 || Wo < 1 || k < 1 || (tap && k > 6)) return hipErrorInvalidValue;
    if ((long)s * (Do - 1) + (long)(k - 1) * d >= D || (long)s * (Ho - 1) + (long)(k - 1) * d >= H ||
        (long)s * (Wo - 1) + (long)(k - 1) * d >= W)
        return hipErrorInvalidValue;
    const int xblocks = (Wo + 255) / 256;
    if (k == 2 && s == 1) {
        const int M = 16, links = (Do + d - 1) / d, nseg = (links + M - 1) / M;
        const long plane = (long)Ho * Wo, pblocks = (plane + 255) / 256;
        const long gx = (long)d * nseg * pblocks;
        if (gx <= 0x7fffffffL && plane <= 0x7fffffffL) {
            if (tap)
                hipLaunchKernelGGL(maxpool3d_k2_chain_f32_kernel<true>, dim3((unsigned)gx, C), dim3(256), 0, stream, x, y, tap, C, H, W,
                                   Do, Ho, Wo, d, M, nseg, (int)pblocks);
            else
                hipLaunchKernelGGL(maxpool3d_k2_chain_f32_kernel<false>, dim3((unsigned)gx, C), dim3(256), 0, stream, x, y, tap, C, H, W,
                                   Do, Ho, Wo, d, M, nseg, (int)pblocks);
            return hipGetLastError();
        }
    }
    if ((long)Do * xblocks > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(maxpool3d_f32_kernel, dim3((unsigned)(Do * xblocks), Ho, C), dim3(256), 0, stream, x, y, tap, C, H, W, Ho, Wo, k,
                       d, s, xblocks);
    return hipGetLastError();
}

// Gather form of the 3-D pool gradient (s = 1): input sample (z, u, v) can only have won the windows whose
// output sits at (z - a*d, u - i*d, v - j*d); it collects dY from those whose recorded code is (a*k + i)*k + j.
// relu_src (optional, laid out like dx): the result is zeroed where relu_src <= 0.  No atomics.
// K > 0: compile-time kernel size; the K^3 winner codes and gradients are then fetched unconditionally (addresses
// of windows outside the output clamped to element 0) so that all loads are in flight together instead of one
// dependent load per branch.  K = 0: any k, plain loops.
// grid: x = (input slice, block of 256 consecutive positions of the H x W plane), y = map
template <int K>
__global__ void __launch_bounds__(256) maxpool3d_bwd_f32_kernel(const float *__restrict__ dy, const uint8_t *__restrict__ tap,
                                                                const float *__restrict__ relu_src, float *__restrict__ dx, int C,
                                                                int H, int W, int Do, int Ho, int Wo, int k, int d, int pblocks)
{
    const int z = blockIdx.x / pblocks, pb = blockIdx.x - z * pblocks;
    const int pos = pb * 256 + threadIdx.x, c = blockIdx.y;
    if (pos >= H * W) return;
    const int u = pos / W, v = pos - u * W;
    float sum = 0.f;
    if constexpr (K > 0) {
        long q[K * K * K];
        bool ok[K * K * K];
#pragma unroll
        for (int t = 0; t < K * K * K; ++t) {
            const int a = t / (K * K), i = (t / K) % K, j = t % K;
            const int zo = z - a * d, yo = u - i * d, xo = v - j * d;
            ok[t] = zo >= 0 && zo < Do && yo >= 0 && yo < Ho && xo >= 0 && xo < Wo;
            q[t] = ok[t] ? (((long)zo * C + c) * Ho + yo) * Wo + xo : 0;
        }
        uint8_t code[K * K * K];
        float g[K * K * K];
#pragma unroll
        for (int t = 0; t < K * K * K; ++t) code[t] = tap[q[t]];
#pragma unroll
        for (int t = 0; t < K * K * K; ++t) g[t] = dy[q[t]];
#pragma unroll
        for (int t = 0; t < K * K * K; ++t) sum += (ok[t] && code[t] == (uint8_t)t) ? g[t] : 0.f;
    } else {
        for (int a = 0; a < k; ++a) {
            const int zo = z - a * d;
            if (zo < 0 || zo >= Do) continue;
            for (int i = 0; i < k; ++i) {
                const int yo = u - i * d;
                if (yo < 0 || yo >= Ho) continue;
                for (int j = 0; j < k; ++j) {
                    const int xo = v - j * d;
                    if (xo < 0 || xo >= Wo) continue;
                    const long qq = (((long)zo * C + c) * Ho + yo) * Wo + xo;
                    if (tap[qq] == (uint8_t)((a * k + i) * k + j)) sum += dy[qq];
                }
            }
        }
    }
    const long p = (((long)z * C + c) * H + u) * W + v;
    if (relu_src && !(relu_src[p] > 0.f)) sum = 0.f;
    dx[p] = sum;
}

hipError_t launch_maxpool3d_bwd_f32(const float *dy, const uint8_t *tap, const float *relu_src, float *dx, int C, int D, int H, int W,
                                    int Do, int Ho, int Wo, int k, int d, hipStream_t stream)
{
    if (C < 1 || C > 65535 || H < 1 || H > 65535 || k < 1 || k > 6) return hipErrorInvalidValue;
    if (Do != D - (k - 1) * d || Ho != H - (k - 1) * d || Wo != W - (k - 1) * d || Do < 1 || Ho < 1 || Wo < 1) return hipErrorInvalidValue;
    const long pblocks = ((long)H * W + 255) / 256;
    if ((long)H * W > 0x7fffffffL || (long)D * pblocks > 0x7fffffffL) return hipErrorInvalidValue;
    if (k == 2)
        hipLaunchKernelGGL(maxpool3d_bwd_f32_kernel<2>, dim3((unsigned)(D * pblocks), C), dim3(256), 0, stream, dy, tap, relu_src, dx, C,
                           H, W, Do, Ho, Wo, k, d, (int)pblocks);
    else
        hipLaunchKernelGGL(maxpool3d_bwd_f32_kernel<0>, dim3((unsigned)(D * pblocks), C), dim3(256), 0, stream, dy, tap, relu_src, dx, C,
                           H, W, Do, Ho, Wo, k, d, (int)pblocks);
    return hipGetLastError();
}

// winner codes of a 3-D pool -> flat offsets ((z_in*H + y_in)*W + x_in) inside the map's input volume
__global__ void tap3d_to_index_kernel(const uint8_t *tap, int32_t *idx, int C, int Do, int Ho, int Wo, int H, int W, int k, int d, int s,
                                      long total)
{
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const int xo = (int)(q % Wo);
        long t = q / Wo;
        const int yo = (int)(t % Ho);
        t /= Ho;
        const int zo = (int)(t / C);
        const int code = tap[q];
        const int j = code % k, i = (code / k) % k, a = code / (k * k);
        idx[q] = (int32_t)((((long)s * zo + a * d) * H + s * yo + i * d) * W + s * xo + j * d);
    }
}

hipError_t launch_tap3d_to_index(const uint8_t *tap, int32_t *idx, int C, int Do, int Ho, int Wo, int H, int W, int k, int d, int s,
                                 hipStream_t stream)
{
    const long total = (long)C * Do * Ho * Wo;
    hipLaunchKernelGGL(tap3d_to_index_kernel, dim3(grid_for(total)), dim3(256), 0, stream, tap, idx, C, Do, Ho, Wo, H, W, k, d, s, total);
    return hipGetLastError();
}

// dst[(m*k + a)*kk + r] = src[m*kk + r]: the gradient of depth tap a, [maps][k][k], into the 3-D gradient [maps][k][k][k]
__global__ void place_tap_f32_kernel(const float *src, float *dst, long maps, int k, int a)
{
    const int kk = k * k;
    const long total = maps * kk;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const long m = q / kk;
        const int r = (int)(q - m * kk);
        dst[(m * k + a) * kk + r] = src[q];
    }
}

__global__ void place_taps_f32_kernel(const float *src, float *dst, int c_out, int C, int k, int Cs)
{
    const int kk = k * k;
    const long total = (long)c_out * C * k * kk;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const int r = (int)(q % kk);
        long t = q / kk;
        const int c = (int)(t % C);
        t /= C;
        const int a = (int)(t % k), o = (int)(t / k);
        dst[(((long)o * C + c) * k + a) * kk + r] = src[(((long)o * k + a) * Cs + c) * kk + r];
    }
}

hipError_t launch_place_taps_f32(const float *src, float *dst, int c_out, int C, int k, hipStream_t stream, int src_maps_per_tap)
{
    const int Cs = src_maps_per_tap > 0 ? src_maps_per_tap : C;
    if (Cs < C) return hipErrorInvalidValue;
    hipLaunchKernelGGL(place_taps_f32_kernel, dim3(grid_for((long)c_out * C * k * k * k)), dim3(256), 0, stream, src, dst, c_out, C, k, Cs);
    return hipGetLastError();
}

hipError_t launch_place_tap_f32(const float *src, float *dst, long maps, int k, int a, hipStream_t stream)
{
    hipLaunchKernelGGL(place_tap_f32_kernel, dim3(grid_for(maps * k * k)), dim3(256), 0, stream, src, dst, maps, k, a);
    return hipGetLastError();
}

// Gather form of the pool gradient: input sample (u, v) can only have won the windows whose
// output sits at (u - i*d, v - j*d); it collects dY from those whose recorded tap is (i, j).
// No atomics, so the result does not depend on scheduling.
// K > 0: compile-time kernel size, the K*K codes and gradients fetched together (windows outside the output read
// element 0 and are discarded); K = 0: any k
template <int K>
__global__ void maxpool_bwd_f32_kernel(const float *__restrict__ dy, const uint8_t *__restrict__ tap, const float *__restrict__ relu_src,
                                       float *__restrict__ dx, int H, int W, int Ho, int Wo, int k, int d)
{
    const int v = blockIdx.x * blockDim.x + threadIdx.x, u = blockIdx.y;
    if (v >= W) return;
    const long p = blockIdx.z;
    float acc = 0.f;
    if constexpr (K > 0) {
        long o[K * K];
        bool ok[K * K];
#pragma unroll
        for (int t = 0; t < K * K; ++t) {
            const int yy = u - (t / K) * d, xx = v - (t % K) * d;
            ok[t] = yy >= 0 && yy < Ho && xx >= 0 && xx < Wo;
            o[t] = ok[t] ? (p * Ho + yy) * Wo + xx : 0;
        }
        uint8_t code[K * K];
        float g[K * K];
#pragma unroll
        for (int t = 0; t < K * K; ++t) code[t] = tap[o[t]];
#pragma unroll
        for (int t = 0; t < K * K; ++t) g[t] = dy[o[t]];
#pragma unroll
        for (int t = 0; t < K * K; ++t) acc += (ok[t] && code[t] == (uint8_t)t) ? g[t] : 0.f;
    } else {
        for (int i = 0; i < k; ++i) {
            const int yy = u - i * d;
            if (yy < 0 || yy >= Ho) continue;
            for (int j = 0; j < k; ++j) {
                const int xx = v - j * d;
                if (xx < 0 || xx >= Wo) continue;
                const long o = (p * Ho + yy) * Wo + xx;
                if (tap[o] == i * k + j) acc += dy[o];
            }
        }
    }
    const long q = (p * H + u) * W + v;
    if (relu_src && !(relu_src[q] > 0.f)) acc = 0.f;
    dx[q] = acc;
}

hipError_t launch_maxpool_bwd_f32(const float *dy, const uint8_t *tap, const float *relu_src,
                                  float *dx, int planes, int H, int W, int Ho, int Wo, int k, int d,
                                  hipStream_t stream)
{
    if (H > 65535 || planes > 65535) return hipErrorInvalidValue;
    const dim3 grid((W + 255) / 256, H, planes);
    if (k == 2) hipLaunchKernelGGL(maxpool_bwd_f32_kernel<2>, grid, dim3(256), 0, stream, dy, tap, relu_src, dx, H, W, Ho, Wo, k, d);
    else hipLaunchKernelGGL(maxpool_bwd_f32_kernel<0>, grid, dim3(256), 0, stream, dy, tap, relu_src, dx, H, W, Ho, Wo, k, d);
    return hipGetLastError();
}

__global__ void tap_to_index_kernel(const uint8_t *tap, int32_t *idx, int planes, int Ho, int Wo, int W,
                                    int k, int d, int s)
{
    const long total = (long)planes * Ho * Wo;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const int xx = (int)(q % Wo);
        const int yy = (int)((q / Wo) % Ho);
        const int code = tap[q], i = code / k, j = code - i * k;
        idx[q] = (s * yy + i * d) * W + s * xx + j * d;
    }
}

hipError_t launch_tap_to_index(const uint8_t *tap, int32_t *idx, int planes, int Ho, int Wo, int W,
                               int k, int d, int s, hipStream_t stream)
{
    const long total = (long)planes * Ho * Wo;
    hipLaunchKernelGGL(tap_to_index_kernel, dim3(grid_for(total)), dim3(256), 0, stream, tap, idx, planes,
                       Ho, Wo, W, k, d, s);
    return hipGetLastError();
}

// ---- per-pixel softmax over the class maps ----------------------------------------------------------
__global__ void softmax_f32_kernel(const float *z, float *p, int n, int classes, int hw)
{
    const long total = (long)n * hw;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const long b = q / hw, pix = q - b * hw;
        const float *zp = z + b * classes * hw + pix;
        float m = zp[0];
        for (int c = 1; c < classes; ++c) m = fmaxf(m, zp[(long)c * hw]);
        float sum = 0.f;
        for (int c = 0; c < classes; ++c) sum += expf(zp[(long)c * hw] - m);
        const float inv = 1.f / sum;
        float *pp = p + b * classes * hw + pix;
        for (int c = 0; c < classes; ++c) pp[(long)c * hw] = expf(zp[(long)c * hw] - m) * inv;
    }
}

// Four consecutive pixels per thread (16-byte loads and stores), the exponentials kept in registers: the kernel
// moves 8 bytes per pixel and class and does nothing else, so access width and instruction count are what it has.
typedef float float4v __attribute__((ext_vector_type(4)));
template <int CLS>
__global__ void __launch_bounds__(256) softmax_f32_v4_kernel(const float *__restrict__ z, float *__restrict__ p, int n, int hw4)
{
    const long total = (long)n * hw4;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const long b = q / hw4, g4 = q - b * hw4;
        const float4v *zp = reinterpret_cast<const float4v *>(z) + b * CLS * hw4 + g4;
        float4v e[CLS];
#pragma unroll
        for (int c = 0; c < CLS; ++c) e[c] = zp[(long)c * hw4];
        float4v m = e[0];
#pragma unroll
        for (int c = 1; c < CLS; ++c)
#pragma unroll
            for (int t = 0; t < 4; ++t) m[t] = fmaxf(m[t], e[c][t]);
        float4v sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < CLS; ++c)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                e[c][t] = expf(e[c][t] - m[t]);
                sum[t] += e[c][t];
            }
        float4v inv;
#pragma unroll
        for (int t = 0; t < 4; ++t) inv[t] = 1.f / sum[t];
        float4v *pp = reinterpret_cast<float4v *>(p) + b * CLS * hw4 + g4;
#pragma unroll
        for (int c = 0; c < CLS; ++c) pp[(long)c * hw4] = e[c] * inv;
    }
}

hipError_t launch_softmax_f32(const float *z, float *p, int n, int classes, int hw, hipStream_t stream)
{
    const bool vec = hw % 4 == 0 && classes >= 2 && classes <= 4 && (reinterpret_cast<uintptr_t>(z) | reinterpret_cast<uintptr_t>(p)) % 16 == 0;
    if (vec) {
        const dim3 grid(grid_for((long)n * (hw / 4)));
        if (classes == 2) hipLaunchKernelGGL(softmax_f32_v4_kernel<2>, grid, dim3(256), 0, stream, z, p, n, hw / 4);
        else if (classes == 3) hipLaunchKernelGGL(softmax_f32_v4_kernel<3>, grid, dim3(256), 0, stream, z, p, n, hw / 4);
        else hipLaunchKernelGGL(softmax_f32_v4_kernel<4>, grid, dim3(256), 0, stream, z, p, n, hw / 4);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(softmax_f32_kernel, dim3(grid_for((long)n * hw)), dim3(256), 0, stream, z, p, n,
                       classes, hw);
    return hipGetLastError();
}

// ---- softmax loss (Section 4.3): mean over all pixels of -log p_label, and its gradient ----------------
constexpr int LOSS_BLOCK = 256;
constexpr int LOSS_MAX_BLOCKS = 2048;

static int loss_blocks(long pixels)
{
    long b = (pixels + LOSS_BLOCK - 1) / LOSS_BLOCK;
    return (int)(b < LOSS_MAX_BLOCKS ? (b < 1 ? 1 : b) : LOSS_MAX_BLOCKS);
}

// floats of scratch the loss needs: one partial sum and one partial count of labelled pixels per workgroup
int softmax_loss_partials(long pixels) { return 2 * loss_blocks(pixels); }

__device__ __forceinline__ float block_sum(float v, float *sh)
{
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) sh[wave] = v;
    __syncthreads();
    float r = 0.f;
    if (threadIdx.x == 0)
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) r += sh[w];
    __syncthreads();
    return r;   // valid on thread 0
}

// A pixel whose label lies outside 0..classes-1 (-1 by convention) is masked out of the error map
// (Section 4.2's label masking): no loss, zero gradient, and the normaliser P counts the labelled
// pixels only.  P must be known before the first gradient is written, so the labelled pixels are
// counted first (integer partial counts, one per workgroup), and every workgroup of the loss kernel
// adds up those few counts for itself.
__global__ void label_count_kernel(const int32_t *labels, long total, int classes, int *counts)
{
    __shared__ int sh[LOSS_BLOCK / 64];
    int local = 0;
    if (total % 4 == 0 && reinterpret_cast<uintptr_t>(labels) % 16 == 0) {          // four labels per load
        typedef int int4l __attribute__((ext_vector_type(4)));
        const int4l *l4 = reinterpret_cast<const int4l *>(labels);
        for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total / 4; q += (long)gridDim.x * blockDim.x) {
            const int4l lab = l4[q];
#pragma unroll
            for (int t = 0; t < 4; ++t) local += (lab[t] >= 0 && lab[t] < classes) ? 1 : 0;
        }
    } else {
        for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
            const int lab = labels[q];
            local += (lab >= 0 && lab < classes) ? 1 : 0;
        }
    }
    for (int off = 32; off > 0; off >>= 1) local += __shfl_down(local, off, 64);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = local;
    __syncthreads();
    if (threadIdx.x == 0) {
        int s = 0;
        for (int w = 0; w < LOSS_BLOCK / 64; ++w) s += sh[w];
        counts[blockIdx.x] = s;
    }
}

// total of the partial counts, computed by the whole workgroup (exact: integers) and returned to every thread
__device__ __forceinline__ long labelled_pixels(const int *counts, int nblocks)
{
    __shared__ long cnt_sh[LOSS_BLOCK / 64];
    long local = 0;
    for (int q = threadIdx.x; q < nblocks; q += blockDim.x) local += counts[q];
    for (int off = 32; off > 0; off >>= 1) local += __shfl_down(local, off, 64);
    if ((threadIdx.x & 63) == 0) cnt_sh[threadIdx.x >> 6] = local;
    __syncthreads();
    long kept = 0;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) kept += cnt_sh[w];
    return kept;
}

__global__ void softmax_loss_f32_kernel(const float *z, const int32_t *labels, float *dz, float *partial, const int *counts,
                                        int n, int classes, int hw)
{
    __shared__ float sh[LOSS_BLOCK / 64];
    const long total = (long)n * hw;
    const long kept = labelled_pixels(counts, gridDim.x);
    const float invP = 1.f / (float)(kept > 0 ? kept : 1);
    float local = 0.f;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const long b = q / hw, pix = q - b * hw;
        const float *zp = z + b * classes * hw + pix;
        float *gp = dz + b * classes * hw + pix;
        const int lab = labels[q];
        if (lab < 0 || lab >= classes) {
            for (int c = 0; c < classes; ++c) gp[(long)c * hw] = 0.f;
            continue;
        }
        float m = zp[0];
        for (int c = 1; c < classes; ++c) m = fmaxf(m, zp[(long)c * hw]);
        float sum = 0.f;
        for (int c = 0; c < classes; ++c) sum += expf(zp[(long)c * hw] - m);
        local -= zp[(long)lab * hw] - m - logf(sum);
        const float inv = 1.f / sum;
        for (int c = 0; c < classes; ++c)
            gp[(long)c * hw] = (expf(zp[(long)c * hw] - m) * inv - (c == lab ? 1.f : 0.f)) * invP;
    }
    const float s = block_sum(local, sh);
    if (threadIdx.x == 0) partial[blockIdx.x] = s;
}

// The same, four consecutive pixels per thread, 16-byte accesses.  dz16 (optional): the gradient once more in the
// 16-bit octet layout [n][1][hw][8] (classes 0..CLS-1 of a pixel in the first elements of its 16 bytes, zeros behind),
// which is what the 16-bit layers below read -- written here instead of by a conversion pass over dz.
typedef unsigned int uint4w __attribute__((ext_vector_type(4)));
typedef int int4w __attribute__((ext_vector_type(4)));
template <int CLS, int DT>
__global__ void __launch_bounds__(LOSS_BLOCK) softmax_loss_f32_v4_kernel(const float *__restrict__ z, const int32_t *__restrict__ labels,
                                                                          float *__restrict__ dz, uint4w *__restrict__ dz16,
                                                                          float *__restrict__ partial, const int *__restrict__ counts, int n, int hw4)
{
    __shared__ float sh[LOSS_BLOCK / 64];
    const long total = (long)n * hw4;
    const long kept = labelled_pixels(counts, gridDim.x);
    const float invP = 1.f / (float)(kept > 0 ? kept : 1);
    float local = 0.f;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const long b = q / hw4, g4 = q - b * hw4;
        const float4v *zp = reinterpret_cast<const float4v *>(z) + b * CLS * hw4 + g4;
        const int4w lab = reinterpret_cast<const int4w *>(labels)[q];
        float4v e[CLS];
#pragma unroll
        for (int c = 0; c < CLS; ++c) e[c] = zp[(long)c * hw4];
        float4v g[CLS];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const bool ok = lab[t] >= 0 && lab[t] < CLS;
            float m = e[0][t];
#pragma unroll
            for (int c = 1; c < CLS; ++c) m = fmaxf(m, e[c][t]);
            float sum = 0.f, zl = 0.f, ex[CLS];
#pragma unroll
            for (int c = 0; c < CLS; ++c) {
                ex[c] = expf(e[c][t] - m);
                sum += ex[c];
                zl = c == lab[t] ? e[c][t] : zl;
            }
            if (ok) local -= zl - m - logf(sum);
            const float inv = 1.f / sum;
#pragma unroll
            for (int c = 0; c < CLS; ++c) g[c][t] = ok ? (ex[c] * inv - (c == lab[t] ? 1.f : 0.f)) * invP : 0.f;
        }
        float4v *gp = reinterpret_cast<float4v *>(dz) + b * CLS * hw4 + g4;
#pragma unroll
        for (int c = 0; c < CLS; ++c) gp[(long)c * hw4] = g[c];
        if constexpr (DT != 0) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                unsigned short h[4] = {0, 0, 0, 0};
#pragma unroll
                for (int c = 0; c < CLS; ++c) {
                    if constexpr (DT == 1) h[c] = __builtin_bit_cast(unsigned short, static_cast<__bf16>(g[c][t]));
                    else h[c] = __builtin_bit_cast(unsigned short, static_cast<_Float16>(g[c][t]));
                }
                dz16[4 * q + t] = uint4w{(unsigned)h[0] | ((unsigned)h[1] << 16), (unsigned)h[2] | ((unsigned)h[3] << 16), 0u, 0u};
            }
        }
    }
    const float s = block_sum(local, sh);
    if (threadIdx.x == 0) partial[blockIdx.x] = s;
}

__global__ void loss_finish_kernel(const float *partial, const int *counts, int count, float *loss)
{
    __shared__ float sh[LOSS_BLOCK / 64];
    float v = 0.f;
    for (int q = threadIdx.x; q < count; q += blockDim.x) v += partial[q];
    const float s = block_sum(v, sh);
    const long kept = labelled_pixels(counts, count);
    if (threadIdx.x == 0) *loss = s / (float)(kept > 0 ? kept : 1);
}

hipError_t launch_label_count(const int32_t *labels, long pixels, int classes, int *counts, int *ncounts, hipStream_t stream)
{
    const int blocks = loss_blocks(pixels);
    hipLaunchKernelGGL(label_count_kernel, dim3(blocks), dim3(LOSS_BLOCK), 0, stream, labels, pixels, classes, counts);
    *ncounts = blocks;
    return hipGetLastError();
}

template <int DT>
static void launch_loss_v4(int classes, int blocks, hipStream_t stream, const float *z, const int32_t *labels, float *dz, void *dz16, float *partial,
                           const int *counts, int n, int hw4)
{
    uint4w *o = static_cast<uint4w *>(dz16);
    if (classes == 2) hipLaunchKernelGGL((softmax_loss_f32_v4_kernel<2, DT>), dim3(blocks), dim3(LOSS_BLOCK), 0, stream, z, labels, dz, o, partial, counts, n, hw4);
    else if (classes == 3) hipLaunchKernelGGL((softmax_loss_f32_v4_kernel<3, DT>), dim3(blocks), dim3(LOSS_BLOCK), 0, stream, z, labels, dz, o, partial, counts, n, hw4);
    else hipLaunchKernelGGL((softmax_loss_f32_v4_kernel<4, DT>), dim3(blocks), dim3(LOSS_BLOCK), 0, stream, z, labels, dz, o, partial, counts, n, hw4);
}

// can launch_softmax_loss_f32 write the 16-bit octet copy of the gradient itself?  (else the caller converts dz)
bool softmax_loss_writes_octets(int classes, int hw) { return hw % 4 == 0 && classes >= 2 && classes <= 4; }

hipError_t launch_softmax_loss_f32(const float *z, const int32_t *labels, float *dz, float *loss,
                                   float *partial, int n, int classes, int hw, hipStream_t stream, void *dz16, int dtype16)
{
    const long pixels = (long)n * hw;
    const int blocks = loss_blocks(pixels);
    int *counts = reinterpret_cast<int *>(partial + blocks);
    hipLaunchKernelGGL(label_count_kernel, dim3(blocks), dim3(LOSS_BLOCK), 0, stream, labels, pixels, classes, counts);
    const bool aligned = (reinterpret_cast<uintptr_t>(z) | reinterpret_cast<uintptr_t>(dz) | reinterpret_cast<uintptr_t>(labels)) % 16 == 0;
    if (dz16 && !(softmax_loss_writes_octets(classes, hw) && aligned && (dtype16 == 1 || dtype16 == 2))) return hipErrorInvalidValue;
    if (softmax_loss_writes_octets(classes, hw) && aligned) {
        if (!dz16) launch_loss_v4<0>(classes, blocks, stream, z, labels, dz, nullptr, partial, counts, n, hw / 4);
        else if (dtype16 == 1) launch_loss_v4<1>(classes, blocks, stream, z, labels, dz, dz16, partial, counts, n, hw / 4);
        else launch_loss_v4<2>(classes, blocks, stream, z, labels, dz, dz16, partial, counts, n, hw / 4);
        hipLaunchKernelGGL(loss_finish_kernel, dim3(1), dim3(LOSS_BLOCK), 0, stream, partial, counts, blocks, loss);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(softmax_loss_f32_kernel, dim3(blocks), dim3(LOSS_BLOCK), 0, stream, z, labels, dz,
                       partial, counts, n, classes, hw);
    hipLaunchKernelGGL(loss_finish_kernel, dim3(1), dim3(LOSS_BLOCK), 0, stream, partial, counts, blocks, loss);
    return hipGetLastError();
}

// ---- SGD ---------------------------------------------------------------------------------------------
__global__ void sgd_f32_kernel(float *w, const float *dw, float *v, long count, float lr, float mu, float wd)
{
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < count; q += (long)gridDim.x * blockDim.x) {
        const float g = dw[q] + wd * w[q];
        const float vel = (v ? mu * v[q] : 0.f) + lr * g;
        if (v) v[q] = vel;
        w[q] -= vel;
    }
}

hipError_t launch_sgd_f32(float *w, const float *dw, float *v, long count, float lr, float mu, float wd,
                          hipStream_t stream)
{
    hipLaunchKernelGGL(sgd_f32_kernel, dim3(grid_for(count, 256, 1024)), dim3(256), 0, stream, w, dw, v,
                       count, lr, mu, wd);
    return hipGetLastError();
}

// one launch for all parameter tensors of a net.  Workgroups are dealt out in proportion to the tensors' sizes
// (SGD_CHUNK elements each; start[t] = first workgroup of tensor t), so the largest tensor does not finish alone;
// a thread updates four float4 when the tensor's three arrays are 16-byte aligned.
constexpr int SGD_CHUNK = 4096;
struct SgdBatchDev { SgdBatch b; int start[BATCH_MAX + 1]; };

// new velocity of one element (momentum mu, weight decay wd); the weight moves by minus this
__device__ __forceinline__ float sgd_velocity(float w, float dw, float v_old, float lr, float mu, float wd)
{
    return mu * v_old + lr * (dw + wd * w);
}

__global__ void __launch_bounds__(256) sgd_batch_f32_kernel(SgdBatchDev d, float lr, float mu, float wd)
{
    int t = 0;
    while (t + 1 < d.b.n && (int)blockIdx.x >= d.start[t + 1]) ++t;
    float *w = d.b.w[t], *v = d.b.v[t];
    const float *dw = d.b.dw[t];
    const long count = d.b.count[t], q0 = (long)((int)blockIdx.x - d.start[t]) * SGD_CHUNK;
    const bool vec = ((reinterpret_cast<size_t>(w) | reinterpret_cast<size_t>(dw) | reinterpret_cast<size_t>(v)) & 15) == 0;
    if (vec && q0 + SGD_CHUNK <= count) {
        float4v wv[4], gv[4], vv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const long q = q0 + (u * 256 + threadIdx.x) * 4;
            wv[u] = *reinterpret_cast<const float4v *>(w + q);
            gv[u] = *reinterpret_cast<const float4v *>(dw + q);
            if (v) vv[u] = *reinterpret_cast<const float4v *>(v + q);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const long q = q0 + (u * 256 + threadIdx.x) * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float vel = sgd_velocity(wv[u][i], gv[u][i], v ? vv[u][i] : 0.f, lr, mu, wd);
                vv[u][i] = vel;
                wv[u][i] -= vel;
            }
            *reinterpret_cast<float4v *>(w + q) = wv[u];
            if (v) *reinterpret_cast<float4v *>(v + q) = vv[u];
        }
        return;
    }
    for (long q = q0 + threadIdx.x; q < q0 + SGD_CHUNK && q < count; q += 256) {
        const float vel = sgd_velocity(w[q], dw[q], v ? v[q] : 0.f, lr, mu, wd);
        if (v) v[q] = vel;
        w[q] -= vel;
    }
}

hipError_t launch_sgd_batch_f32(const SgdBatch &b, float lr, float mu, float wd, hipStream_t stream)
{
    if (b.n < 1 || b.n > BATCH_MAX) return hipErrorInvalidValue;
    SgdBatchDev d;
    d.b = b;
    long blocks = 0;
    for (int t = 0; t < b.n; ++t) {
        d.start[t] = (int)blocks;
        blocks += (b.count[t] + SGD_CHUNK - 1) / SGD_CHUNK;
        if (b.count[t] < 0 || blocks > 0x7fffffffL) return hipErrorInvalidValue;
    }
    for (int t = b.n; t <= BATCH_MAX; ++t) d.start[t] = (int)blocks;
    if (blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(sgd_batch_f32_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, d, lr, mu, wd);
    return hipGetLastError();
}

// SGD on the bias of a 2x2 up-convolution, which its four taps share: the gradient is the sum of the four
// taps' bias gradients (db4[t*c_out + o]); the new value goes to each tap's own copy.
__global__ void up_bias_sgd_f32_kernel(float *b0, float *b1, float *b2, float *b3, float *b_stacked, const float *db4, float *v, int c_out,
                                       float lr, float mu, float wd)
{
    const int o = blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= c_out) return;
    const float g = (db4[o] + db4[c_out + o]) + (db4[2 * c_out + o] + db4[3 * c_out + o]) + wd * b0[o];
    const float vel = (v ? mu * v[o] : 0.f) + lr * g;
    if (v) v[o] = vel;
    const float nb = b0[o] - vel;
    b0[o] = nb; b1[o] = nb; b2[o] = nb; b3[o] = nb;
    if (b_stacked) {
#pragma unroll
        for (int t = 0; t < 4; ++t) b_stacked[t * c_out + o] = nb;
    }
}

hipError_t launch_up_bias_sgd_f32(float *b0, float *b1, float *b2, float *b3, float *b_stacked, const float *db4, float *v, int c_out, float lr,
                                  float mu, float wd, hipStream_t stream)
{
    hipLaunchKernelGGL(up_bias_sgd_f32_kernel, dim3((c_out + 255) / 256), dim3(256), 0, stream, b0, b1, b2, b3, b_stacked, db4, v, c_out, lr, mu,
                       wd);
    return hipGetLastError();
}

// ---- crop-and-place copy (the two halves of MergeCrop, Section 5.3.1) -----------------------------------
__global__ void crop_copy_f32_kernel(const float *in, float *out, int n, int maps, int hi, int wi,
                                     int out_maps, int o_off, int ho, int wo, int oy, int ox)
{
    const long total = (long)n * maps * ho * wo;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const int x = (int)(q % wo);
        long t = q / wo;
        const int y = (int)(t % ho);
        t /= ho;
        const int c = (int)(t % maps);
        const long b = t / maps;
        out[((b * out_maps + o_off + c) * ho + y) * wo + x] = in[((b * maps + c) * hi + y + oy) * wi + x + ox];
    }
}

hipError_t launch_crop_copy_f32(const float *in, float *out, int n, int maps, int hi, int wi,
                                int out_maps, int o_off, int ho, int wo, int oy, int ox,
                                hipStream_t stream)
{
    const long total = (long)n * maps * ho * wo;
    hipLaunchKernelGGL(crop_copy_f32_kernel, dim3(grid_for(total)), dim3(256), 0, stream, in, out, n, maps,
                       hi, wi, out_maps, o_off, ho, wo, oy, ox);
    return hipGetLastError();
}

// g[q] = act[q] > 0 ? g[q] : 0   (ReLU backward where no producer kernel could fuse it)
__global__ void relu_mask_f32_kernel(float *g, const float *act, long count)
{
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < count; q += (long)gridDim.x * blockDim.x)
        if (!(act[q] > 0.f)) g[q] = 0.f;
}

hipError_t launch_relu_mask_f32(float *g, const float *act, long count, hipStream_t stream)
{
    hipLaunchKernelGGL(relu_mask_f32_kernel, dim3(grid_for(count)), dim3(256), 0, stream, g, act, count);
    return hipGetLastError();
}

// ---- backward pieces of the U-Net / USK-Net (Sections 3.4, 5.3.1) ---------------------------------------
// Pool with stride s = k at d = 1: the windows do not overlap, so input sample (u, v) belongs to the one
// window (u / k, v / k) and receives its dY if the recorded tap is (u % k, v % k).  Samples right of /
// below the last window receive nothing.  accumulate adds to what dX holds (a map that also feeds a
// skip connection).
__global__ void maxpool_sk_eq_s_bwd_f32_kernel(const float *dy, const uint8_t *tap, float *dx, int H, int W, int Ho, int Wo,
                                               int k, int accumulate)
{
    const int v = blockIdx.x * blockDim.x + threadIdx.x, u = blockIdx.y;
    if (v >= W) return;
    const long p = blockIdx.z;
    const int yy = u / k, xx = v / k;
    float g = 0.f;
    if (yy < Ho && xx < Wo) {
        const long q = (p * Ho + yy) * Wo + xx;
        if (tap[q] == (uint8_t)((u - yy * k) * k + (v - xx * k))) g = dy[q];
    }
    const long o = (p * H + u) * W + v;
    dx[o] = accumulate ? dx[o] + g : g;
}

hipError_t launch_maxpool_stride_bwd_f32(const float *dy, const uint8_t *tap, float *dx, int planes, int H, int W, int Ho, int Wo,
                                         int k, int accumulate, hipStream_t stream)
{
    hipLaunchKernelGGL(maxpool_sk_eq_s_bwd_f32_kernel, dim3((W + 255) / 256, H, planes), dim3(256), 0, stream, dy, tap, dx, H, W, Ho,
                       Wo, k, accumulate);
    return hipGetLastError();
}

// out[b][t*maps + o][y][x] = in[b][o][2y + a][2x + c], t = 2a + c: the four interleaved sub-images of the
// first `maps` maps of a tensor with in_maps maps and 2h x 2w pixels, stacked as 4*maps maps of h x w (the
// gradient of a 2x2 stride-2 up-convolution seen as a 1x1 convolution with four times the output maps).
__global__ void space_to_depth2_f32_kernel(const float *in, float *out, int n, int in_maps, int maps, int h, int w)
{
    const long total = (long)n * 4 * maps * h * w;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const int x = (int)(q % w);
        long r = q / w;
        const int y = (int)(r % h); r /= h;
        const int o = (int)(r % maps); r /= maps;
        const int t = (int)(r % 4);
        const long b = r / 4;
        out[q] = in[((b * in_maps + o) * (2L * h) + 2 * y + (t >> 1)) * (2L * w) + 2 * x + (t & 1)];
    }
}

hipError_t launch_space_to_depth2_f32(const float *in, float *out, int n, int in_maps, int maps, int h, int w, hipStream_t stream)
{
    const long total = (long)n * 4 * maps * h * w;
    hipLaunchKernelGGL(space_to_depth2_f32_kernel, dim3(grid_for(total, 256, 8192)), dim3(256), 0, stream, in, out, n, in_maps, maps, h, w);
    return hipGetLastError();
}

// out[b][c][y + oy][x + ox] = in[b][c_off + c][y][x] for c < maps (MergeCrop backward into the skip map:
// the cropped-away border keeps whatever out held -- the caller clears it first)
__global__ void place_f32_kernel(const float *in, float *out, int n, int in_maps, int c_off, int maps, int hi, int wi, int ho, int wo,
                                 int oy, int ox)
{
    const long total = (long)n * maps * hi * wi;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const int x = (int)(q % wi);
        long r = q / wi;
        const int y = (int)(r % hi); r /= hi;
        const int c = (int)(r % maps);
        const long b = r / maps;
        out[((b * maps + c) * ho + y + oy) * wo + x + ox] = in[((b * in_maps + c_off + c) * hi + y) * wi + x];
    }
}

hipError_t launch_place_f32(const float *in, float *out, int n, int in_maps, int c_off, int maps, int hi, int wi, int ho, int wo,
                            int oy, int ox, hipStream_t stream)
{
    const long total = (long)n * maps * hi * wi;
    hipLaunchKernelGGL(place_f32_kernel, dim3(grid_for(total, 256, 8192)), dim3(256), 0, stream, in, out, n, in_maps, c_off, maps, hi, wi,
                       ho, wo, oy, ox);
    return hipGetLastError();
}

__global__ void fill_f32_kernel(float *p, float v, long count)
{
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < count; q += (long)gridDim.x * blockDim.x) p[q] = v;
}

hipError_t launch_fill_f32(float *p, float v, long count, hipStream_t stream)
{
    hipLaunchKernelGGL(fill_f32_kernel, dim3(grid_for(count, 256, 4096)), dim3(256), 0, stream, p, v, count);
    return hipGetLastError();
}

}  // namespace sk
