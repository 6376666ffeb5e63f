// Weight and bias gradient of the SK convolution (gfx950): MFMA 16x16x4 fp32 for fp32 storage,
// MFMA 16x16x32 bf16 / fp16 for 16-bit storage (second kernel below); fp32 accumulation in both.
//
//   dW[o][c][i][j] = sum_{b,y,x} dY[b,o,y,x] * X[b,c,y+i*d,x+j*d]        db[o] = sum dY[b,o,y,x]
//
// GEMM view: the paper's forward GEMM (Section 5.5) transposed: M = f_out, N = f_in*k*k, and the
// reduction runs over all output pixels.  The result is tiny (f_out x f_in*k*k) and the reduction
// is huge, so the pixels are split over a persistent grid: each workgroup walks over row segments
// (one output row, 64 columns), stages that segment of dY for all output maps and the k input
// rows it touches for all input maps in LDS, and accumulates a private copy of dW in MFMA
// accumulators.  The copies are written to scratch and summed by a second kernel in a fixed order,
// so the result is reproducible (no float atomics).
//
// MFMA roles: A[m = output map][kk = pixel] = dY, B[kk = pixel][n = (c,i,j)] = X shifted by the
// tap, D[m][n] = dW laid out exactly as OIHW.  Wave w of a workgroup owns MB row tiles (16 output
// maps each) times NB column tiles (16 (c,i,j) triples each); blockIdx.y selects further groups.
#include <algorithm>
#include <type_traits>

#include "sk_kernels.h"

namespace sk {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int WG_SEG = 64;          // output pixels per segment
constexpr int WG_DYP = WG_SEG + 4;  // LDS pitch of a dY row
constexpr int WG_MAX_BLOCKS = 512;

typedef unsigned int uint4v __attribute__((ext_vector_type(4)));

template <int DT> __device__ __forceinline__ float up16(unsigned u);
template <> __device__ __forceinline__ float up16<0>(unsigned u) { return __uint_as_float(u); }
template <> __device__ __forceinline__ float up16<1>(unsigned u) { return __uint_as_float(u << 16); }
template <> __device__ __forceinline__ float up16<2>(unsigned u) { return (float)__builtin_bit_cast(_Float16, (unsigned short)u); }
// a staged operand (fp32 as it is, 16-bit storage widened) as the MFMA's fp32 input
template <int DT> __device__ __forceinline__ float staged(float f) { return f; }
template <int DT> __device__ __forceinline__ float staged(unsigned short u) { return up16<DT>((unsigned)u); }

struct WgradArgs {
    const void *x, *dy;     // fp32 NCHW planar (DT = 0) or 16-bit octet layout (DT = 1 bf16, 2 fp16)
    float *scratch;
    int n, c_in, H, W, c_out, k, d, Ho, Wo;
    int MTo, NTk;          // 16-wide tiles over output maps / over (c,i,j)
    int xsegs, total_segs;
    int xpitch;            // LDS pitch of an input row
    // fp32 storage only: distance in floats between the inputs of consecutive images (0 = c_in*H*W), and input maps
    // in groups of 2^grp_shift consecutive planes with grp_skip more floats between groups (the depth taps of a 3-D
    // convolution: see launch_conv_f32); grp_shift = 31: no groups
    long x_bstride, grp_skip;
    int grp_shift;
    // transposing-read 16-bit kernel only, in octet planes: consecutive images start xb8 planes apart (default: the
    // octets of c_in), and the input octets come in groups of grp8 with skip8 more planes between groups (the depth
    // taps of a 3-D convolution on slice-major volumes: slices as overlapping images)
    int xb8, grp8, skip8;
    // 16-bit matrix path: bias_part != nullptr makes the kernel sum dY over the pixels as well (one more MFMA per map tile
    // against a fragment of ones) and write bias_part[map * gridDim.x + blockIdx.x]
    float *bias_part;
};

template <int MB, int NB, int DT>
// (fp32 storage with at most 16 tiles per wave: compiled for two waves per SIMD, i.e. two workgroups per CU)
__global__ __launch_bounds__(256, (DT == 0 && MB * NB <= 16) ? 2 : 1) void wgrad_f32_kernel(WgradArgs a)
{
    extern __shared__ float smem[];
    const int k = a.k, d = a.d, K = a.c_in * k * k;
    const int m_rows = a.MTo * 16;
    // staged operands: fp32, or (16-bit storage types) the raw 16-bit values, widened when they are read
    // for the MFMA -- half the LDS, so two workgroups fit a CU and one stages while the other multiplies
    typedef typename std::conditional<DT == 0, float, unsigned short>::type stage_t;
    // LDS holds what this workgroup's tile group needs: the dY rows of its MB map tiles and (fp32
    // storage) the input maps its NB*4 column tiles touch -- a 1024 x 9216 gradient is split over
    // many groups, and no group could hold all maps
    stage_t *dys = reinterpret_cast<stage_t *>(smem);    // [MB*16][WG_DYP]
    stage_t *xs = dys + MB * 16 * WG_DYP;                // [maps of the group * k][xpitch]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l16 = lane & 15, g = lane >> 4;
    const int PW = WG_SEG + (k - 1) * d;

    // tile groups: blockIdx.y = mgroup * ngroups + ngroup
    const int ngroups = (a.NTk + 4 * NB - 1) / (4 * NB);
    const int mgroup = blockIdx.y / ngroups, ngroup = blockIdx.y - mgroup * ngroups;
    const int mo0 = mgroup * MB;
    // input maps this group's columns (c,i,j) belong to; 16-bit storage stages whole octets and keeps all maps
    const int c_lo = DT == 0 ? (ngroup * NB * 64) / (k * k) : 0;
    int c_hi = DT == 0 ? ((ngroup + 1) * NB * 64 - 1) / (k * k) : a.c_in - 1;
    c_hi = c_hi < a.c_in - 1 ? c_hi : a.c_in - 1;
    const int cw = c_hi - c_lo + 1;
    // column tiles of this wave: nk = (ngroup*NB + q)*4 + wave
    int xoff[NB];
#pragma unroll
    for (int q = 0; q < NB; ++q) {
        const int nk = (ngroup * NB + q) * 4 + wave;
        const int cij = nk * 16 + l16;
        int off = 0;
        if (nk < a.NTk && cij < K) {
            const int c = cij / (k * k), r = cij - c * k * k, i = r / k, j = r - i * k;
            off = ((c - c_lo) * k + i) * a.xpitch + j * d;
        }
        xoff[q] = off + g;
    }
    floatx4 acc[MB][NB];
#pragma unroll
    for (int m = 0; m < MB; ++m)
#pragma unroll
        for (int q = 0; q < NB; ++q) acc[m][q] = floatx4{0.f, 0.f, 0.f, 0.f};

    const long xplane = (long)a.H * a.W, yplane = (long)a.Ho * a.Wo;
    // fp32 storage: the loads of a segment are issued in batches (every load of a batch before its first
    // value is written to LDS: one row after the other, each load's latency is paid in full, and with
    // hundreds of rows per segment that was most of the kernel), and the first batch of the NEXT segment
    // -- this wave's dY rows and SU input rows -- is issued before the MFMA loop and held in registers.
    constexpr int SU = MB * NB <= 16 ? 8 : 16, SV = 3;   // input rows per wave and batch, 64-column groups per row (PW <= 192)
    constexpr int DYU = 4 * MB;               // dY rows per wave
    float pdy[DT == 0 ? DYU : 1], px[DT == 0 ? SU : 1][DT == 0 ? SV : 1];
    const int xrows = cw * k;
    auto load_dy = [&](int b, int y, int x0) {
        const float *dyp = static_cast<const float *>(a.dy);
        const int xl = x0 + lane < a.Wo ? x0 + lane : a.Wo - 1;
#pragma unroll
        for (int u = 0; u < DYU; ++u) {
            const int row = mo0 * 16 + wave + 4 * u;
            const int rc = row < a.c_out ? row : a.c_out - 1;
            pdy[u] = dyp[((long)b * a.c_out + rc) * yplane + (long)y * a.Wo + xl];
        }
    };
    auto store_dy = [&](int x0) {
#pragma unroll
        for (int u = 0; u < DYU; ++u) {
            const int row = mo0 * 16 + wave + 4 * u;            // < (mo0 + MB) * 16
            dys[(row - mo0 * 16) * WG_DYP + lane] = (row < a.c_out && x0 + lane < a.Wo) ? pdy[u] : 0.f;
        }
    };
    auto load_x = [&](int bat, int b, int y, int x0) {
        const float *xp = static_cast<const float *>(a.x);
#pragma unroll
        for (int u = 0; u < SU; ++u) {
            int row = wave + 4 * (bat * SU + u);
            row = row < xrows ? row : xrows - 1;
            const int c = c_lo + row / k, i = row - (row / k) * k;
            const float *src = xp + (long)b * a.x_bstride + (long)c * xplane + (long)(c >> a.grp_shift) * a.grp_skip + (long)(y + i * d) * a.W;
#pragma unroll
            for (int sv = 0; sv < SV; ++sv) {
                const int xc = lane + 64 * sv;
                px[u][sv] = src[x0 + xc < a.W ? x0 + xc : a.W - 1];
            }
        }
    };
    auto store_x = [&](int bat, int x0) {
#pragma unroll
        for (int u = 0; u < SU; ++u) {
            const int row = wave + 4 * (bat * SU + u);
            if (row >= xrows) break;                             // uniform
#pragma unroll
            for (int sv = 0; sv < SV; ++sv) {
                const int xc = lane + 64 * sv;
                if (xc < PW) xs[row * a.xpitch + xc] = (x0 + xc < a.W) ? px[u][sv] : 0.f;
            }
        }
    };
    auto locate = [&](int seg, int &b, int &y, int &x0) {
        const int xs_i = seg % a.xsegs, t = seg / a.xsegs;
        y = t % a.Ho;
        b = t / a.Ho;
        x0 = xs_i * WG_SEG;
    };
    const int nbat = (xrows + 4 * SU - 1) / (4 * SU);
    int pb = 0, py = 0, px0 = 0;              // position of the segment whose first batch is in registers
    if constexpr (DT == 0) {
        if ((int)blockIdx.x < a.total_segs) {
            locate(blockIdx.x, pb, py, px0);
            load_dy(pb, py, px0);
            load_x(0, pb, py, px0);
        }
    }
    for (int seg = blockIdx.x; seg < a.total_segs; seg += gridDim.x) {
        const int xs_i = seg % a.xsegs;
        const int t = seg / a.xsegs;
        const int y = t % a.Ho, b = t / a.Ho;
        const int x0 = xs_i * WG_SEG;
        __syncthreads();
        if constexpr (DT == 0) {
            store_dy(x0);
            store_x(0, x0);
            for (int bat = 1; bat < nbat; ++bat) {
                load_x(bat, b, y, x0);
                store_x(bat, x0);
            }
        } else {
            // 16-bit octet layout: one 16-byte load brings 8 maps of a pixel; widen to fp32 in LDS
            const uint4v *dyp = static_cast<const uint4v *>(a.dy), *xp = static_cast<const uint4v *>(a.x);
            const int c8o = (a.c_out + 7) / 8, c8i = (a.c_in + 7) / 8;
            const int xl = x0 + lane < a.Wo ? x0 + lane : a.Wo - 1;
            const int oc_end = (mo0 + MB) * 2 < a.MTo * 2 ? (mo0 + MB) * 2 : a.MTo * 2;
#pragma unroll 2
            for (int oc = mo0 * 2 + wave; oc < oc_end; oc += 4) {
                const int occ = oc < c8o ? oc : c8o - 1;
                const uint4v u = dyp[((long)b * c8o + occ) * yplane + (long)y * a.Wo + xl];
                const bool ok = oc < c8o && x0 + lane < a.Wo;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    dys[(oc * 8 + e - mo0 * 16) * WG_DYP + lane] = ok ? (unsigned short)((u[e >> 1] >> ((e & 1) * 16)) & 0xffffu) : (unsigned short)0;
            }
            for (int rid = wave; rid < c8i * k; rid += 4) {
                const int oc = rid / k, i = rid - oc * k;
                const uint4v *src = xp + ((long)b * c8i + oc) * xplane + (long)(y + i * d) * a.W;
#pragma unroll 3
                for (int xc = lane; xc < PW; xc += 64) {
                    const int gx = x0 + xc < a.W ? x0 + xc : a.W - 1;
                    const uint4v u = src[gx];
                    const bool ok = x0 + xc < a.W;
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        xs[((oc * 8 + e) * k + i) * a.xpitch + xc] = ok ? (unsigned short)((u[e >> 1] >> ((e & 1) * 16)) & 0xffffu) : (unsigned short)0;
                }
            }
        }
        __syncthreads();
        if constexpr (DT == 0) {
            const int nseg = seg + gridDim.x;
            if (nseg < a.total_segs) {                           // in flight while this segment is multiplied
                locate(nseg, pb, py, px0);
                load_dy(pb, py, px0);
                load_x(0, pb, py, px0);
            }
        }
#pragma unroll 2
        for (int p = 0; p < WG_SEG; p += 4) {
            float av[MB];
#pragma unroll
            for (int m = 0; m < MB; ++m) {
                av[m] = (mo0 + m < a.MTo) ? staged<DT>(dys[(m * 16 + l16) * WG_DYP + p + g]) : 0.f;
            }
#pragma unroll
            for (int q = 0; q < NB; ++q) {
                const float bv = staged<DT>(xs[xoff[q] + p]);
#pragma unroll
                for (int m = 0; m < MB; ++m)
                    acc[m][q] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[m], bv, acc[m][q], 0, 0, 0);
            }
        }
    }
    // private copy -> scratch[blockIdx.x][o][cij]  (o < MTo*16, cij < NTk*16)
    const long ncols = (long)a.NTk * 16;
    float *dst = a.scratch + (long)blockIdx.x * m_rows * ncols;
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        if (mo0 + m >= a.MTo) continue;
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const int nk = (ngroup * NB + q) * 4 + wave;
            if (nk >= a.NTk) continue;
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4)
                dst[((long)(mo0 + m) * 16 + 4 * g + r4) * ncols + nk * 16 + l16] = acc[m][q][r4];
        }
    }
}

// ------------------------------------------------------------------------------------------------
// The same gradient on the 16-bit matrix path (MFMA 16x16x32, bf16 or fp16 operands, fp32
// accumulation) for 16-bit storage.  The contraction runs over pixels, so a lane must supply 8
// consecutive pixels of ONE map -- the octet layout holds 8 maps of one pixel -- and the staging
// loop is where the transposition happens: it scatters every loaded octet into map-major LDS rows
// (pixels contiguous), exactly as the fp32-path kernel above does.  An A fragment (dY) is then one
// aligned 16-byte LDS read; a B fragment (X shifted by tap column j) starts j*d elements into its
// row, so its alignment is that of j*d: RB = 16, 8, 4 or 2 bytes per read for d % 8 == 0 (and 1x1
// kernels), d % 4 == 0, d % 2 == 0, odd d (eight 2-byte reads per fragment: still far fewer cycles
// than the fp32 matrix path).
typedef __bf16 bf16x8v __attribute__((ext_vector_type(8)));
typedef _Float16 halfx8v __attribute__((ext_vector_type(8)));
typedef unsigned int uint2v __attribute__((ext_vector_type(2)));
template <int DT> __device__ __forceinline__ floatx4 mfma32(uint4v a, uint4v b, floatx4 c);
template <> __device__ __forceinline__ floatx4 mfma32<1>(uint4v a, uint4v b, floatx4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8v, a), __builtin_bit_cast(bf16x8v, b), c, 0, 0, 0);
}
template <> __device__ __forceinline__ floatx4 mfma32<2>(uint4v a, uint4v b, floatx4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(halfx8v, a), __builtin_bit_cast(halfx8v, b), c, 0, 0, 0);
}
// 8 consecutive 16-bit elements from LDS, starting `off` elements into the 4-byte aligned array `base`; base + off is
// aligned to RB bytes.  RB = 2 (odd kernel strides, 3x3 kernels at d = 1): five aligned 4-byte reads and a funnel
// shift by 0 or 16 bits per lane instead of eight 2-byte reads.
template <int RB> __device__ __forceinline__ uint4v lds_read8(const unsigned short *base, int off)
{
    const unsigned short *p = base + off;
    if constexpr (RB == 16) return *reinterpret_cast<const uint4v *>(p);
    else if constexpr (RB == 8) {
        const uint2v lo = *reinterpret_cast<const uint2v *>(p), hi = *reinterpret_cast<const uint2v *>(p + 4);
        return uint4v{lo[0], lo[1], hi[0], hi[1]};
    } else if constexpr (RB == 4) {
        const unsigned *q = reinterpret_cast<const unsigned *>(p);
        return uint4v{q[0], q[1], q[2], q[3]};
    } else {
        const unsigned *q = reinterpret_cast<const unsigned *>(base) + (off >> 1);
        const unsigned sh = (unsigned)(off & 1) * 16u;
        const unsigned w0 = q[0], w1 = q[1], w2 = q[2], w3 = q[3], w4 = q[4];
        return uint4v{__builtin_amdgcn_alignbit(w1, w0, sh), __builtin_amdgcn_alignbit(w2, w1, sh), __builtin_amdgcn_alignbit(w3, w2, sh),
                      __builtin_amdgcn_alignbit(w4, w3, sh)};
    }
}

constexpr int WG_DYH = WG_SEG + 8;   // LDS pitch (elements) of a dY row: rows stay 16-byte aligned

// Staging is what this kernel's time goes to (a segment is only 72 MFMAs per wave), so the global
// loads of the next segment -- this wave's dY octets and the first batch of its input rows -- are
// issued before the MFMA loop and sit in registers until the next trip writes them to LDS; a net
// with more input rows than one batch holds (XU row ids per wave) loads the rest in place.
template <int MB, int NB, int DT, int RB>
__global__ __launch_bounds__(256) void wgrad_h_kernel(WgradArgs a)
{
    constexpr int DYL = (2 * MB + 3) / 4;   // dY octet loads per wave and segment
    constexpr int XU = 6, XV = 2;           // input loads per wave and batch: XU row ids x XV groups of 64 columns
    extern __shared__ uint4v smem16[];
    const int k = a.k, d = a.d, K = a.c_in * k * k;
    const int m_rows = a.MTo * 16;
    // a tile group stages what it multiplies: the dY rows of its MB map tiles and the input octets its columns touch
    unsigned short *dys = reinterpret_cast<unsigned short *>(smem16);   // [MB*16][WG_DYH]
    unsigned short *xs = dys + MB * 16 * WG_DYH;                         // [8*(octets of the group)*k][xpitch]
    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int PW = WG_SEG + (k - 1) * d;        // <= 64 * XV (checked by the launcher)

    const int ngroups = (a.NTk + 4 * NB - 1) / (4 * NB);
    const int mgroup = blockIdx.y / ngroups, ngroup = blockIdx.y - mgroup * ngroups;
    const int mo0 = mgroup * MB;
    // input octets of this group's columns (c, i, j) = cij: [oc0, oc0 + noct)
    const int cij_lo = ngroup * NB * 4 * 16;
    int cij_hi = cij_lo + NB * 4 * 16 - 1;
    cij_hi = cij_hi < K - 1 ? cij_hi : K - 1;
    const int oc0 = cij_lo / (k * k) / 8, noct = cij_hi / (k * k) / 8 - oc0 + 1;
    int xoff[NB];
#pragma unroll
    for (int q = 0; q < NB; ++q) {
        const int nk = (ngroup * NB + q) * 4 + wave;
        const int cij = nk * 16 + l16;
        int off = 0;
        if (nk < a.NTk && cij < K) {
            const int c = cij / (k * k), r = cij - c * k * k, i = r / k, j = r - i * k;
            off = ((c - oc0 * 8) * k + i) * a.xpitch + j * d;
        }
        xoff[q] = off + 8 * g;
    }
    floatx4 acc[MB][NB];
#pragma unroll
    for (int m = 0; m < MB; ++m)
#pragma unroll
        for (int q = 0; q < NB; ++q) acc[m][q] = floatx4{0.f, 0.f, 0.f, 0.f};
    // bias gradient: map tile m of this workgroup is summed by wave m (MB <= 4) in the column group 0 blocks
    const bool sum_dy = a.bias_part != nullptr && ngroup == 0 && wave < MB && mo0 + wave < a.MTo;
    floatx4 bacc = floatx4{0.f, 0.f, 0.f, 0.f};
    const unsigned one2 = DT == 1 ? 0x3F803F80u : 0x3C003C00u;      // two ones in the storage type
    const uint4v ones = uint4v{one2, one2, one2, one2};

    const long xplane = (long)a.H * a.W, yplane = (long)a.Ho * a.Wo;
    const uint4v *dyp = static_cast<const uint4v *>(a.dy), *xp = static_cast<const uint4v *>(a.x);
    const int c8o = (a.c_out + 7) / 8, c8i = (a.c_in + 7) / 8;
    const int oc_end = (mo0 + MB) * 2 < a.MTo * 2 ? (mo0 + MB) * 2 : a.MTo * 2;
    const int nrid = noct * k;                                  // (input octet, kernel row) pairs to stage
    const int nbat = (nrid + 4 * XU - 1) / (4 * XU);
    const int kxp = k * a.xpitch;                               // LDS distance between the 8 maps of an octet

    uint4v pdy[DYL], px[XU][XV];
    // all addresses are clamped into the tensors; what lies outside is replaced by zero when it is stored
    auto load_dy = [&](int b, int y, int x0) {
        const int xl = x0 + lane < a.Wo ? x0 + lane : a.Wo - 1;
#pragma unroll
        for (int t = 0; t < DYL; ++t) {
            const int oc = mo0 * 2 + wave + 4 * t;
            const int occ = oc < c8o ? oc : c8o - 1;
            pdy[t] = dyp[((long)b * c8o + occ) * yplane + (long)y * a.Wo + xl];
        }
    };
    auto load_x = [&](int bat, int b, int y, int x0) {
#pragma unroll
        for (int u = 0; u < XU; ++u) {
            const int rid = wave + 4 * (bat * XU + u);
            const int ridc = rid < nrid ? rid : nrid - 1;
            const int ocr = ridc / k, i = ridc - ocr * k;
            int oc = oc0 + ocr;
            oc = oc < c8i ? oc : c8i - 1;
            const uint4v *src = xp + ((long)b * a.xb8 + oc + (oc / a.grp8) * a.skip8) * xplane + (long)(y + i * d) * a.W;
#pragma unroll
            for (int v = 0; v < XV; ++v) {
                const int xc = lane + 64 * v;
                px[u][v] = src[x0 + xc < a.W ? x0 + xc : a.W - 1];
            }
        }
    };
    auto scatter = [&](unsigned short *dst, int stride, uint4v u, bool ok) {
        if (!ok) u = uint4v{0u, 0u, 0u, 0u};
#pragma unroll
        for (int e = 0; e < 8; ++e) dst[e * stride] = (unsigned short)((u[e >> 1] >> ((e & 1) * 16)) & 0xffffu);
    };
    auto store_dy = [&](int x0) {
#pragma unroll
        for (int t = 0; t < DYL; ++t) {
            const int oc = mo0 * 2 + wave + 4 * t;
            if (oc < oc_end) scatter(dys + (oc - mo0 * 2) * 8 * WG_DYH + lane, WG_DYH, pdy[t], oc < c8o && x0 + lane < a.Wo);
        }
    };
    auto store_x = [&](int bat, int x0) {
#pragma unroll
        for (int u = 0; u < XU; ++u) {
            const int rid = wave + 4 * (bat * XU + u);
            if (rid >= nrid) continue;                          // uniform
            const int oc = rid / k, i = rid - oc * k;                 // octet relative to the group's first
            unsigned short *row = xs + (oc * 8 * k + i) * a.xpitch;
#pragma unroll
            for (int v = 0; v < XV; ++v) {
                const int xc = lane + 64 * v;
                if (xc < PW) scatter(row + xc, kxp, px[u][v], x0 + xc < a.W && oc0 + oc < c8i);
            }
        }
    };
    auto locate = [&](int seg, int &b, int &y, int &x0) {
        const int xs_i = seg % a.xsegs, t = seg / a.xsegs;
        y = t % a.Ho;
        b = t / a.Ho;
        x0 = xs_i * WG_SEG;
    };

    int seg = blockIdx.x, b = 0, y = 0, x0 = 0;
    if (seg < a.total_segs) {
        locate(seg, b, y, x0);
        load_dy(b, y, x0);
        load_x(0, b, y, x0);
    }
    for (; seg < a.total_segs; seg += gridDim.x) {
        __syncthreads();                                        // the previous segment's MFMAs have read LDS
        store_dy(x0);
        store_x(0, x0);
        for (int bat = 1; bat < nbat; ++bat) {
            load_x(bat, b, y, x0);
            store_x(bat, x0);
        }
        __syncthreads();
        const int nseg = seg + gridDim.x;
        if (nseg < a.total_segs) {                              // in flight while this segment is multiplied
            locate(nseg, b, y, x0);
            load_dy(b, y, x0);
            load_x(0, b, y, x0);
        }
#pragma unroll
        for (int p = 0; p < WG_SEG; p += 32) {
            uint4v av[MB];
#pragma unroll
            for (int m = 0; m < MB; ++m) {
                const int row = m * 16 + l16;
                av[m] = uint4v{0u, 0u, 0u, 0u};
                if (mo0 + m < a.MTo) av[m] = *reinterpret_cast<const uint4v *>(dys + row * WG_DYH + p + 8 * g);
            }
#pragma unroll
            for (int q = 0; q < NB; ++q) {
                const uint4v bv = lds_read8<RB>(xs, xoff[q] + p);
#pragma unroll
                for (int m = 0; m < MB; ++m) acc[m][q] = mfma32<DT>(av[m], bv, acc[m][q]);
            }
            if (sum_dy) {                                        // wave-uniform
                uint4v aw = av[0];
#pragma unroll
                for (int m = 1; m < MB; ++m) aw = wave == m ? av[m] : aw;
                bacc = mfma32<DT>(aw, ones, bacc);
            }
        }
    }
    if (sum_dy && l16 == 0) {                                   // every column of bacc holds the same sums
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const int o = (mo0 + wave) * 16 + 4 * g + r4;
            if (o < a.c_out) a.bias_part[(long)o * gridDim.x + blockIdx.x] = bacc[r4];
        }
    }
    const long ncols = (long)a.NTk * 16;
    float *dst = a.scratch + (long)blockIdx.x * m_rows * ncols;
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        if (mo0 + m >= a.MTo) continue;
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const int nk = (ngroup * NB + q) * 4 + wave;
            if (nk >= a.NTk) continue;
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4)
                dst[((long)(mo0 + m) * 16 + 4 * g + r4) * ncols + nk * 16 + l16] = acc[m][q][r4];
        }
    }
}

// ---- 16 input maps or more: operands staged as octets, fragments by the transposing LDS read ---------------------------
// The segment kernel above scatters every loaded octet into eight map-major LDS rows (eight 2-byte writes) so that a
// fragment -- 8 consecutive pixels of one map -- is a plain read, and reads it in pieces of whatever alignment the tap
// offset j*d leaves.  Here an octet goes to LDS as it is (ONE 16-byte write: [row][pixel][8 maps]) and ds_read_b64_tr_b16
// does the transposition on the way out: of a group of 16 lanes, lane 4r + q addresses pixel r, maps 4q..4q+3, and lane
// 4q + e receives map 4q + e of pixels 0..3.  A tile of 16 GEMM columns is then 16 consecutive input maps (two octets) at
// ONE tap (i, j) -- column tile nk = (map pair, i, j), against 16 consecutive (c, i, j) in the kernel above -- and a tap's
// offset moves whole 16-byte pixels, so there are no alignment classes.  The private copies have the columns in that
// order; the reduction maps them back (tr_k2).  Tiles over the output maps, tile groups, persistent workgroups, the bias
// sums on the matrix unit and the prefetch of the next segment are those of the kernel above.
typedef short short4tr __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4v read_frag_tr(const char *lds_base, unsigned off_lo, unsigned off_hi)
{
    typedef short4tr __attribute__((address_space(3))) *lds_s4;
    const short4tr lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(lds_base + off_lo));
    const short4tr hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(lds_base + off_hi));
    const uint2v l2 = __builtin_bit_cast(uint2v, lo), h2 = __builtin_bit_cast(uint2v, hi);
    return uint4v{l2[0], l2[1], h2[0], h2[1]};
}

constexpr int WG_TRP = WG_SEG + 4;      // LDS pitch (16-byte units) of a dY octet row: row starts alternate between the two halves of the banks

template <int MB, int NB, int DT>
__global__ __launch_bounds__(256) void wgrad_tr_h_kernel(WgradArgs a)
{
    constexpr int DYL = (2 * MB + 3) / 4;   // dY octet loads per wave and segment
    constexpr int XU = 6, XV = 2;           // input loads per wave and batch: XU row ids x XV groups of 64 columns
    extern __shared__ uint4v smem16[];
    const int k = a.k, d = a.d, kk = k * k;
    const int m_rows = a.MTo * 16;
    uint4v *dys = smem16;                               // [2*MB octets][WG_TRP pixels]
    uint4v *xs = dys + 2 * MB * WG_TRP;                 // [(octets of the group) * k rows][xpitch pixels]
    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rr = l16 >> 2, qq = l16 & 3;              // the transposing read: this lane addresses pixel rr, map quad qq
    const int PW = WG_SEG + (k - 1) * d;                // <= 64 * XV (checked by the launcher)

    const int ngroups = (a.NTk + 4 * NB - 1) / (4 * NB);
    const int mgroup = blockIdx.y / ngroups, ngroup = blockIdx.y - mgroup * ngroups;
    const int mo0 = mgroup * MB;
    const int c8o = (a.c_out + 7) / 8, c8i = (a.c_in + 7) / 8;
    // input octets of this group's column tiles (map pair, i, j): [oc0, oc0 + noct); octets beyond the last real one are zeros
    const int nk_lo = ngroup * NB * 4;
    int nk_hi = nk_lo + NB * 4 - 1;
    nk_hi = nk_hi < a.NTk - 1 ? nk_hi : a.NTk - 1;
    const int oc0 = 2 * (nk_lo / kk), noct = 2 * (nk_hi / kk) + 2 - oc0;
    unsigned xoff[NB], aoff[MB];
#pragma unroll
    for (int q = 0; q < NB; ++q) {
        const int nk = (ngroup * NB + q) * 4 + wave;
        unsigned off = (unsigned)((8 * g + rr) * 16);
        if (nk < a.NTk) {
            const int op = nk / kk, r = nk - op * kk, i = r / k, j = r - i * k;
            off = (unsigned)((((2 * op - oc0 + (qq >> 1)) * k + i) * a.xpitch + j * d + 8 * g + rr) * 16 + (qq & 1) * 8);
        }
        xoff[q] = off;
    }
#pragma unroll
    for (int m = 0; m < MB; ++m) aoff[m] = (unsigned)(((2 * m + (qq >> 1)) * WG_TRP + 8 * g + rr) * 16 + (qq & 1) * 8);
    floatx4 acc[MB][NB];
#pragma unroll
    for (int m = 0; m < MB; ++m)
#pragma unroll
        for (int q = 0; q < NB; ++q) acc[m][q] = floatx4{0.f, 0.f, 0.f, 0.f};
    const bool sum_dy = a.bias_part != nullptr && ngroup == 0 && wave < MB && mo0 + wave < a.MTo;
    floatx4 bacc = floatx4{0.f, 0.f, 0.f, 0.f};
    const unsigned one2 = DT == 1 ? 0x3F803F80u : 0x3C003C00u;      // two ones in the storage type
    const uint4v ones = uint4v{one2, one2, one2, one2};

    const long xplane = (long)a.H * a.W, yplane = (long)a.Ho * a.Wo;
    const uint4v *dyp = static_cast<const uint4v *>(a.dy), *xp = static_cast<const uint4v *>(a.x);
    const int oc_end = 2 * MB;                                       // dY octet rows of the tile group (relative)
    // kernel rows the group's tiles use: all k, or (a group inside one map pair: kernels with more than 4*NB taps) a range
    int i_lo = 0, ni = k;
    if (nk_lo / kk == nk_hi / kk) {
        i_lo = (nk_lo % kk) / k;
        ni = (nk_hi % kk) / k - i_lo + 1;
    }
    const int nrid = noct * ni;                                      // (input octet, kernel row) pairs to stage
    const int nbat = (nrid + 4 * XU - 1) / (4 * XU);
    const uint4v zero = uint4v{0u, 0u, 0u, 0u};

    uint4v pdy[DYL], px[XU][XV];
    // all addresses are clamped into the tensors; what lies outside is replaced by zero when it is stored
    auto load_dy = [&](int b, int y, int x0) {
        const int xl = x0 + lane < a.Wo ? x0 + lane : a.Wo - 1;
#pragma unroll
        for (int t = 0; t < DYL; ++t) {
            const int oc = mo0 * 2 + wave + 4 * t;
            const int occ = oc < c8o ? oc : c8o - 1;
            pdy[t] = dyp[((long)b * c8o + occ) * yplane + (long)y * a.Wo + xl];
        }
    };
    auto load_x = [&](int bat, int b, int y, int x0) {
#pragma unroll
        for (int u = 0; u < XU; ++u) {
            const int rid = wave + 4 * (bat * XU + u);
            const int ridc = rid < nrid ? rid : nrid - 1;
            const int ocr = ridc / ni, i = i_lo + ridc - ocr * ni;
            int oc = oc0 + ocr;
            oc = oc < c8i ? oc : c8i - 1;
            const uint4v *src = xp + ((long)b * a.xb8 + oc + (oc / a.grp8) * a.skip8) * xplane + (long)(y + i * d) * a.W;
#pragma unroll
            for (int v = 0; v < XV; ++v) {
                const int xc = lane + 64 * v;
                px[u][v] = src[x0 + xc < a.W ? x0 + xc : a.W - 1];
            }
        }
    };
    auto store_dy = [&](int x0) {
#pragma unroll
        for (int t = 0; t < DYL; ++t) {
            const int rel = wave + 4 * t;
            if (rel < oc_end) dys[rel * WG_TRP + lane] = (mo0 * 2 + rel < c8o && x0 + lane < a.Wo) ? pdy[t] : zero;
        }
    };
    auto store_x = [&](int bat, int x0) {
#pragma unroll
        for (int u = 0; u < XU; ++u) {
            const int rid = wave + 4 * (bat * XU + u);
            if (rid >= nrid) continue;                          // uniform
            const int ocr = rid / ni, row = ocr * k + i_lo + rid - ocr * ni;
#pragma unroll
            for (int v = 0; v < XV; ++v) {
                const int xc = lane + 64 * v;
                if (xc < PW) xs[row * a.xpitch + xc] = (x0 + xc < a.W && oc0 + ocr < c8i) ? px[u][v] : zero;
            }
        }
    };
    auto locate = [&](int seg, int &b, int &y, int &x0) {
        const int xs_i = seg % a.xsegs, t = seg / a.xsegs;
        y = t % a.Ho;
        b = t / a.Ho;
        x0 = xs_i * WG_SEG;
    };

    const char *dys_b = reinterpret_cast<const char *>(dys), *xs_b = reinterpret_cast<const char *>(xs);
    int seg = blockIdx.x, b = 0, y = 0, x0 = 0;
    if (seg < a.total_segs) {
        locate(seg, b, y, x0);
        load_dy(b, y, x0);
        load_x(0, b, y, x0);
    }
    for (; seg < a.total_segs; seg += gridDim.x) {
        __syncthreads();                                        // the previous segment's MFMAs have read LDS
        store_dy(x0);
        store_x(0, x0);
        for (int bat = 1; bat < nbat; ++bat) {
            load_x(bat, b, y, x0);
            store_x(bat, x0);
        }
        __syncthreads();
        const int nseg = seg + gridDim.x;
        if (nseg < a.total_segs) {                              // in flight while this segment is multiplied
            locate(nseg, b, y, x0);
            load_dy(b, y, x0);
            load_x(0, b, y, x0);
        }
#pragma unroll
        for (int p = 0; p < WG_SEG; p += 32) {
            uint4v av[MB];
#pragma unroll
            for (int m = 0; m < MB; ++m) av[m] = read_frag_tr(dys_b, aoff[m] + p * 16, aoff[m] + p * 16 + 64);
#pragma unroll
            for (int q = 0; q < NB; ++q) {
                const uint4v bv = read_frag_tr(xs_b, xoff[q] + p * 16, xoff[q] + p * 16 + 64);
#pragma unroll
                for (int m = 0; m < MB; ++m) acc[m][q] = mfma32<DT>(av[m], bv, acc[m][q]);
            }
            if (sum_dy) {                                        // wave-uniform
                uint4v aw = av[0];
#pragma unroll
                for (int m = 1; m < MB; ++m) aw = wave == m ? av[m] : aw;
                bacc = mfma32<DT>(aw, ones, bacc);
            }
        }
    }
    if (sum_dy && l16 == 0) {                                   // every column of bacc holds the same sums
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const int o = (mo0 + wave) * 16 + 4 * g + r4;
            if (o < a.c_out) a.bias_part[(long)o * gridDim.x + blockIdx.x] = bacc[r4];
        }
    }
    const long ncols = (long)a.NTk * 16;
    float *dst = a.scratch + (long)blockIdx.x * m_rows * ncols;
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        if (mo0 + m >= a.MTo) continue;
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const int nk = (ngroup * NB + q) * 4 + wave;
            if (nk >= a.NTk) continue;
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4)
                dst[((long)(mo0 + m) * 16 + 4 * g + r4) * ncols + nk * 16 + l16] = acc[m][q][r4];
        }
    }
}

// The same gradient with the staged input rows kept across steps (k >= 2).
// A workgroup walks a strip -- one image, one 64-column segment, the output rows of one residue class y = r, r + d,
// r + 2d, ... -- so that consecutive steps share k - 1 of their k input rows: the rows sit in a ring of k LDS slots per
// input octet (input row y + i*d of step t in slot (t + i) mod k; a tile group inside one map pair keeps only the
// kernel rows its taps use), a step loads one new row per octet instead of k,
// and the column tiles' read offsets rotate with the step.  The steps of all strips, in strip order, are dealt out
// to the workgroups in equal contiguous ranges; the first step of a range or of a strip loads all k rows.
template <int MB, int NB, int DT>
__global__ __launch_bounds__(256, MB * NB > 36 ? 1 : 2) void wgrad_trr_h_kernel(WgradArgs a)
{
    constexpr int DYL = (2 * MB + 3) / 4;   // dY octet loads per wave and step
    constexpr int XU = 3, XV = 2;           // input loads per wave and batch: XU row ids x XV groups of 64 columns
    extern __shared__ uint4v smem16[];
    const int k = a.k, d = a.d, kk = k * k;
    const int m_rows = a.MTo * 16;
    uint4v *dys = smem16;                               // [2*MB octets][WG_TRP pixels]
    uint4v *xs = dys + 2 * MB * WG_TRP;                 // [(octets of the group) * k slots][xpitch pixels]
    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rr = l16 >> 2, qq = l16 & 3;
    const int PW = WG_SEG + (k - 1) * d;                // <= 64 * XV (checked by the launcher)

    const int ngroups = (a.NTk + 4 * NB - 1) / (4 * NB);
    const int mgroup = blockIdx.y / ngroups, ngroup = blockIdx.y - mgroup * ngroups;
    const int mo0 = mgroup * MB;
    const int c8o = (a.c_out + 7) / 8, c8i = (a.c_in + 7) / 8;
    const int nk_lo = ngroup * NB * 4;
    int nk_hi = nk_lo + NB * 4 - 1;
    nk_hi = nk_hi < a.NTk - 1 ? nk_hi : a.NTk - 1;
    const int oc0 = 2 * (nk_lo / kk), noct = 2 * (nk_hi / kk) + 2 - oc0;     // <= 4 * XU = 12 (checked by the launcher)
    // kernel rows the group's tiles use: all k, or (a group inside one map pair: kernels with more than 4*NB taps) a
    // range [i_lo, i_lo + ni); the ring holds those ni rows
    int i_lo = 0, ni = k;
    if (nk_lo / kk == nk_hi / kk) {
        i_lo = (nk_lo % kk) / k;
        ni = (nk_hi % kk) / k - i_lo + 1;
    }
    const unsigned slot_bytes = (unsigned)a.xpitch * 16;
    unsigned xoff[NB], aoff[MB];
    int iq[NB];                                         // kernel row of column tile q within the ring (wave-uniform)
#pragma unroll
    for (int q = 0; q < NB; ++q) {
        const int nk = (ngroup * NB + q) * 4 + wave;
        unsigned off = (unsigned)((8 * g + rr) * 16);
        iq[q] = 0;
        if (nk < a.NTk) {
            const int op = nk / kk, r = nk - op * kk, i = r / k, j = r - i * k;
            off = (unsigned)((((2 * op - oc0 + (qq >> 1)) * k) * a.xpitch + j * d + 8 * g + rr) * 16 + (qq & 1) * 8);
            iq[q] = i - i_lo;
        }
        xoff[q] = off;
    }
#pragma unroll
    for (int m = 0; m < MB; ++m) aoff[m] = (unsigned)(((2 * m + (qq >> 1)) * WG_TRP + 8 * g + rr) * 16 + (qq & 1) * 8);
    floatx4 acc[MB][NB];
#pragma unroll
    for (int m = 0; m < MB; ++m)
#pragma unroll
        for (int q = 0; q < NB; ++q) acc[m][q] = floatx4{0.f, 0.f, 0.f, 0.f};
    const bool sum_dy = a.bias_part != nullptr && ngroup == 0 && wave < MB && mo0 + wave < a.MTo;
    floatx4 bacc = floatx4{0.f, 0.f, 0.f, 0.f};
    const unsigned one2 = DT == 1 ? 0x3F803F80u : 0x3C003C00u;
    const uint4v ones = uint4v{one2, one2, one2, one2};

    const long xplane = (long)a.H * a.W, yplane = (long)a.Ho * a.Wo;
    const uint4v *dyp = static_cast<const uint4v *>(a.dy), *xp = static_cast<const uint4v *>(a.x);
    const int oc_end = 2 * MB;
    const int nrid = noct * ni;                                      // (input octet, kernel row) pairs of a fresh step
    const int nbat = (nrid + 4 * XU - 1) / (4 * XU);
    const uint4v zero = uint4v{0u, 0u, 0u, 0u};

    uint4v pdy[DYL], px[XU][XV];
    auto load_dy = [&](int b, int y, int x0) {
        const int xl = x0 + lane < a.Wo ? x0 + lane : a.Wo - 1;
#pragma unroll
        for (int t = 0; t < DYL; ++t) {
            const int oc = mo0 * 2 + wave + 4 * t;
            const int occ = oc < c8o ? oc : c8o - 1;
            pdy[t] = dyp[((long)b * c8o + occ) * yplane + (long)y * a.Wo + xl];
        }
    };
    // fresh: row ids run over (octet, kernel row); else over the octets, each loading its one new row (the last kernel row of the ring)
    auto load_x = [&](int bat, int b, int y, int x0, bool fresh) {
        const int lim = fresh ? nrid : noct;
#pragma unroll
        for (int u = 0; u < XU; ++u) {
            const int rid = wave + 4 * (bat * XU + u);
            const int ridc = rid < lim ? rid : lim - 1;
            const int ocr = fresh ? ridc / ni : ridc, i = fresh ? ridc - ocr * ni : ni - 1;
            int oc = oc0 + ocr;
            oc = oc < c8i ? oc : c8i - 1;
            const uint4v *src = xp + ((long)b * a.xb8 + oc + (oc / a.grp8) * a.skip8) * xplane + (long)(y + (i_lo + i) * d) * a.W;
#pragma unroll
            for (int v = 0; v < XV; ++v) {
                const int xc = lane + 64 * v;
                px[u][v] = src[x0 + xc < a.W ? x0 + xc : a.W - 1];
            }
        }
    };
    auto store_dy = [&](int x0) {
#pragma unroll
        for (int t = 0; t < DYL; ++t) {
            const int rel = wave + 4 * t;
            if (rel < oc_end) dys[rel * WG_TRP + lane] = (mo0 * 2 + rel < c8o && x0 + lane < a.Wo) ? pdy[t] : zero;
        }
    };
    auto store_x = [&](int bat, int x0, bool fresh, int rot) {
        const int lim = fresh ? nrid : noct;
#pragma unroll
        for (int u = 0; u < XU; ++u) {
            const int rid = wave + 4 * (bat * XU + u);
            if (rid >= lim) continue;                           // uniform
            const int ocr = fresh ? rid / ni : rid, i = fresh ? rid - ocr * ni : ni - 1;
            int slot = i + rot;
            slot = slot >= ni ? slot - ni : slot;
            const int row = ocr * k + slot;
#pragma unroll
            for (int v = 0; v < XV; ++v) {
                const int xc = lane + 64 * v;
                if (xc < PW) xs[row * a.xpitch + xc] = (x0 + xc < a.W && oc0 + ocr < c8i) ? px[u][v] : zero;
            }
        }
    };
    // steps of this workgroup: [g0, g1) of the strip order (image and segment, residue class, step within the class)
    const int per = (a.total_segs + (int)gridDim.x - 1) / (int)gridDim.x;
    const int g0 = (int)blockIdx.x * per;
    const int g1 = g0 + per < a.total_segs ? g0 + per : a.total_segs;
    auto class_len = [&](int r) { return r < a.Ho ? (a.Ho - r + d - 1) / d : 0; };
    int bx = 0, r = 0, t = 0;
    if (g0 < g1) {
        bx = g0 / a.Ho;
        int rem = g0 - bx * a.Ho;
        while (rem >= class_len(r)) { rem -= class_len(r); ++r; }
        t = rem;
    }
    // position of the step after (bx, r, t); fresh = it starts a strip
    auto advance = [&](int &bx_, int &r_, int &t_, bool &fresh_) {
        ++t_;
        fresh_ = false;
        if (t_ >= class_len(r_)) {
            t_ = 0; ++r_; fresh_ = true;
            if (r_ >= d || class_len(r_) == 0) { r_ = 0; ++bx_; }
        }
    };
    auto place = [&](int bx_, int r_, int t_, int &b_, int &y_, int &x0_) {
        b_ = bx_ / a.xsegs;
        x0_ = (bx_ - b_ * a.xsegs) * WG_SEG;
        y_ = r_ + t_ * d;
    };

    const char *dys_b = reinterpret_cast<const char *>(dys), *xs_b = reinterpret_cast<const char *>(xs);
    int b = 0, y = 0, x0 = 0, rot = 0;
    bool fresh = true;
    if (g0 < g1) {
        place(bx, r, t, b, y, x0);
        load_dy(b, y, x0);
        load_x(0, b, y, x0, true);
    }
    for (int gs = g0; gs < g1; ++gs) {
        __syncthreads();                                        // the previous step's MFMAs have read LDS
        store_dy(x0);
        store_x(0, x0, fresh, rot);
        if (fresh) {
            for (int bat = 1; bat < nbat; ++bat) {
                load_x(bat, b, y, x0, true);
                store_x(bat, x0, true, rot);
            }
        }
        __syncthreads();
        const int rot_now = rot;
        if (gs + 1 < g1) {                                      // in flight while this step is multiplied
            advance(bx, r, t, fresh);
            rot = fresh ? 0 : (rot + 1 == ni ? 0 : rot + 1);
            place(bx, r, t, b, y, x0);
            load_dy(b, y, x0);
            load_x(0, b, y, x0, fresh);
        }
        unsigned xo[NB];
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            int slot = iq[q] + rot_now;
            slot = slot >= ni ? slot - ni : slot;
            xo[q] = xoff[q] + (unsigned)slot * slot_bytes;
        }
#pragma unroll
        for (int p = 0; p < WG_SEG; p += 32) {
            uint4v av[MB];
#pragma unroll
            for (int m = 0; m < MB; ++m) av[m] = read_frag_tr(dys_b, aoff[m] + p * 16, aoff[m] + p * 16 + 64);
#pragma unroll
            for (int q = 0; q < NB; ++q) {
                const uint4v bv = read_frag_tr(xs_b, xo[q] + p * 16, xo[q] + p * 16 + 64);
#pragma unroll
                for (int m = 0; m < MB; ++m) acc[m][q] = mfma32<DT>(av[m], bv, acc[m][q]);
            }
            if (sum_dy) {                                        // wave-uniform
                uint4v aw = av[0];
#pragma unroll
                for (int m = 1; m < MB; ++m) aw = wave == m ? av[m] : aw;
                bacc = mfma32<DT>(aw, ones, bacc);
            }
        }
    }
    if (sum_dy && l16 == 0) {                                   // every column of bacc holds the same sums
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const int o = (mo0 + wave) * 16 + 4 * g + r4;
            if (o < a.c_out) a.bias_part[(long)o * gridDim.x + blockIdx.x] = bacc[r4];
        }
    }
    const long ncols = (long)a.NTk * 16;
    float *dst = a.scratch + (long)blockIdx.x * m_rows * ncols;
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        if (mo0 + m >= a.MTo) continue;
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const int nk = (ngroup * NB + q) * 4 + wave;
            if (nk >= a.NTk) continue;
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4)
                dst[((long)(mo0 + m) * 16 + 4 * g + r4) * ncols + nk * 16 + l16] = acc[m][q][r4];
        }
    }
}

// dW[o][cij] = sum over the private copies, and (last workgroups of the grid) db[o] = sum over the
// slices of the bias partials.  A workgroup of 256 threads sums 64 consecutive elements: wave w takes
// the copies w, w+4, w+8, ... with four running sums (copies w+4(4i+u), u = 0..3), so that sixteen
// loads per element are in flight and the grid has a few hundred workgroups even for a 48x768
// gradient; the four waves' sums are added through LDS.  The order is fixed: reproducible results.
constexpr int RED_ELEMS = 64;
__global__ void __launch_bounds__(256) wgrad_reduce_kernel(const float *__restrict__ scratch, float *__restrict__ dw, int copies, int c_out, int K,
                                                           int m_rows, int ncols, int dw_blocks, const float *__restrict__ bias_part,
                                                           float *__restrict__ db, int slices, int tr_k2)
{
    __shared__ float sh[4][RED_ELEMS];
    const int e = threadIdx.x & 63, w = threadIdx.x >> 6;
    if ((int)blockIdx.x >= dw_blocks) {
        // bias: 64 maps per workgroup, wave w adds slices w, w+4, ...; then the waves in order
        const int o = ((int)blockIdx.x - dw_blocks) * RED_ELEMS + e;
        float v = 0.f;
        if (o < c_out)
            for (int sl = w; sl < slices; sl += 4) v += bias_part[(long)o * slices + sl];
        sh[w][e] = v;
        __syncthreads();
        if (w == 0 && o < c_out) db[o] = (sh[0][e] + sh[1][e]) + (sh[2][e] + sh[3][e]);
        return;
    }
    // Elements are walked in the order the copies hold them (consecutive threads read consecutive addresses of every
    // copy).  tr_k2 = 0: copy column = (c, i, j) = the gradient's own order.  tr_k2 = k*k (copies of wgrad_tr_h_kernel):
    // copy column = ((map pair, i, j), map within the pair); columns of maps beyond c_in are skipped, and the one
    // write per element goes to dw[o][c][i][j].
    const long total = tr_k2 > 0 ? (long)c_out * ncols : (long)c_out * K, stride = (long)m_rows * ncols;
    const long qe = (long)blockIdx.x * RED_ELEMS + e;
    long q = -1;                                        // index into dw, -1: nothing to write
    int o = 0, col = 0;
    if (qe < total) {
        if (tr_k2 > 0) {
            o = (int)(qe / ncols);
            col = (int)(qe - (long)o * ncols);
            const int tile = col >> 4, pr = tile / tr_k2, r = tile - pr * tr_k2, c = pr * 16 + (col & 15);
            if (c * tr_k2 < K) q = (long)o * K + (long)c * tr_k2 + r;
        } else {
            o = (int)(qe / K);
            col = (int)(qe - (long)o * K);
            q = qe;
        }
    }
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    if (q >= 0) {
        const float *src = scratch + (long)o * ncols + col;
        int cpy = w;
        for (; cpy + 12 < copies; cpy += 16) {
            s0 += src[(cpy + 0) * stride];
            s1 += src[(cpy + 4) * stride];
            s2 += src[(cpy + 8) * stride];
            s3 += src[(cpy + 12) * stride];
        }
        for (; cpy < copies; cpy += 4) s0 += src[cpy * stride];
    }
    sh[w][e] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (w == 0 && q >= 0) dw[q] = (sh[0][e] + sh[1][e]) + (sh[2][e] + sh[3][e]);
}

// Reduction of the copies of wgrad_tr_h_kernel with 16-byte accesses on both sides.  A copy row holds, per pair of
// input octets, k*k column tiles of 16 maps: a run of 16*k*k floats that is the same stretch of dw[o] with (tap, map)
// transposed to (map, tap).  A workgroup takes `rpb` whole runs of one row: `lanes` = span / 4 threads each sum a
// float4 of every copy (the 256 / lanes thread groups share the copies out), the partial sums meet in LDS, and the
// span leaves in the gradient's own order, again as float4 per thread.  Fixed summation order.
constexpr int TRR_SPAN = 1024;     // floats of one row per workgroup at most

__global__ void __launch_bounds__(256) wgrad_tr_reduce_kernel(const float *__restrict__ scratch, float *__restrict__ dw, int copies, int c_out, int K,
                                                              int m_rows, int ncols, int k2, int rpb, int parts, int dw_blocks,
                                                              const float *__restrict__ bias_part, float *__restrict__ db, int slices)
{
    __shared__ __attribute__((aligned(16))) float sh[TRR_SPAN];
    const int t = threadIdx.x;
    if ((int)blockIdx.x >= dw_blocks) {
        // bias: 64 maps per workgroup, wave w adds slices w, w+4, ...; then the waves in order
        const int e = t & 63, w = t >> 6;
        const int o = ((int)blockIdx.x - dw_blocks) * 64 + e;
        float v = 0.f;
        if (o < c_out)
            for (int sl = w; sl < slices; sl += 4) v += bias_part[(long)o * slices + sl];
        sh[w * 64 + e] = v;
        __syncthreads();
        if (w == 0 && o < c_out) db[o] = (sh[e] + sh[64 + e]) + (sh[128 + e] + sh[192 + e]);
        return;
    }
    const int o = (int)blockIdx.x / parts, part = (int)blockIdx.x - o * parts;
    const int run_len = 16 * k2, col0 = part * rpb * run_len;
    const int span = min(rpb * run_len, ncols - col0);            // whole runs: a multiple of 16
    const int lanes = span >> 2;
    int nsplit = 256 / lanes;
    nsplit = nsplit < copies ? nsplit : copies;
    const int cw = t / lanes, tt = t - cw * lanes;
    if (cw < nsplit) {
        const long stride = (long)m_rows * ncols;
        const float *src = scratch + (long)o * ncols + col0 + 4 * tt;
        floatx4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = s0, s2 = s0, s3 = s0;
        int c = cw;
        for (; c + 3 * nsplit < copies; c += 4 * nsplit) {
            const floatx4 v0 = *reinterpret_cast<const floatx4 *>(src + (long)c * stride);
            const floatx4 v1 = *reinterpret_cast<const floatx4 *>(src + (long)(c + nsplit) * stride);
            const floatx4 v2 = *reinterpret_cast<const floatx4 *>(src + (long)(c + 2 * nsplit) * stride);
            const floatx4 v3 = *reinterpret_cast<const floatx4 *>(src + (long)(c + 3 * nsplit) * stride);
            s0 += v0;
            s1 += v1;
            s2 += v2;
            s3 += v3;
        }
        for (; c < copies; c += nsplit) s0 += *reinterpret_cast<const floatx4 *>(src + (long)c * stride);
        *reinterpret_cast<floatx4 *>(sh + cw * span + 4 * tt) = (s0 + s1) + (s2 + s3);
    }
    __syncthreads();
    if (t >= lanes) return;
    // floats 4t .. 4t+3 of the span in the gradient's order: (run, map l, tap r) sits at run*run_len + r*16 + l
    float v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = 4 * t + i, run = e / run_len, within = e - run * run_len, l = within / k2, r = within - l * k2;
        const int at = run * run_len + r * 16 + l;
        float s = sh[at];
        for (int p = 1; p < nsplit; ++p) s += sh[p * span + at];
        v[i] = s;
    }
    const int pos = col0 + 4 * t;                                   // position in dw[o]; maps beyond c_in lie at pos >= K
    float *dst = dw + (long)o * K + pos;
    if ((K & 3) == 0 && (reinterpret_cast<size_t>(dw) & 15) == 0) {
        if (pos < K) *reinterpret_cast<floatx4 *>(dst) = floatx4{v[0], v[1], v[2], v[3]};
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (pos + i < K) dst[i] = v[i];
    }
}

// Bias gradient db[o] = sum over images and pixels of dY, in two stages with a fixed summation order.
// Stage 1 (fp32 NCHW): workgroup (s, o) sums slice s of the pixels of map o over all images.
constexpr int BG_SLICES = 64;

__global__ void __launch_bounds__(256) bias_grad_kernel(const float *__restrict__ dy, float *__restrict__ part, int n, int c_out,
                                                        long plane, int slices)
{
    __shared__ float sh[4];
    const int o = blockIdx.y, sl = blockIdx.x;
    const long per = (plane + slices - 1) / slices, q0 = sl * per, q1 = q0 + per < plane ? q0 + per : plane;
    float v = 0.f;
    for (int b = 0; b < n; ++b) {
        const float *src = dy + ((long)b * c_out + o) * plane;
        for (long q = q0 + threadIdx.x; q < q1; q += 256) v += src[q];
    }
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) part[(long)o * slices + sl] = sh[0] + sh[1] + sh[2] + sh[3];
}

// Tiles per workgroup: MB map tiles x 4*NB column tiles (NB per wave).  Tiles beyond the gradient's extent are
// multiplied like the others, so the counts are chosen to leave few of them.
static void wgrad_tiling(int c_out, int c_in, int k, bool f32, int &MTo, int &NTk, int &MB, int &NB)
{
    MTo = (c_out + 15) / 16;
    NTk = (c_in * k * k + 15) / 16;
    MB = MTo == 1 ? 1 : (MTo % 3 == 0 ? 3 : 4);
    NB = NTk >= 48 ? 12 : (NTk > 4 ? 4 : 1);
    if (!f32) return;
    // fp32 storage (MFMA 16x16x4: the multiplications are a large share of the time): fewer map tiles per
    // workgroup where that saves a quarter or more of the padded tiles (2 for 32 maps, 3 for 80); a smaller gain
    // does not pay for the lower reuse of the staged input rows (13 map tiles: 4.09 ms with 4, 4.21 ms with 2)
    if (MTo > 1) {
        const int pad0 = (MTo + MB - 1) / MB * MB;
        int best = MB, pad = pad0;
        for (int cand = 4; cand >= 2; --cand) {
            const int p = (MTo + cand - 1) / cand * cand;
            if (4 * p <= 3 * pad0 && p < pad) { pad = p; best = cand; }
        }
        MB = best;
    }
    // column tiles: groups of at most 16, all of the same size (18 tiles are 2 x 12 slots, not 16 + 16; 36 are
    // 3 x 12); with three map tiles and 48 or more column tiles one group of 48 stays (the 48-map SK-Net)
    if (!(MB == 3 && NTk >= 48) && NTk > 4) {
        const int ngroups = (NTk + 15) / 16, per = (NTk + ngroups - 1) / ngroups;
        NB = (per + 3) / 4;
    }
}

// column tiles of wgrad_tr_h_kernel (16-bit storage, 16 input maps or more): (pair of input octets, i, j)
static bool wgrad_tr_applies(int c_in) { return c_in >= 16; }
static int wgrad_tr_ntk(int c_in, int k) { return (c_in + 15) / 16 * k * k; }
// input octets the column tiles of one tile group touch, at most (groups of 4*nb consecutive tiles; k*k tiles per map pair)
static int wgrad_tr_goct(int ntk, int nb, int kk)
{
    const int ngroups = (ntk + 4 * nb - 1) / (4 * nb);
    int goct = 2;
    for (int gi = 0; gi < ngroups; ++gi) {
        const int lo = gi * nb * 4, hi = std::min(lo + nb * 4, ntk) - 1;
        goct = std::max(goct, 2 * (hi / kk) + 2 - 2 * (lo / kk));
    }
    return goct;
}
// Column tiles per wave.  The kernel prefetches ONE batch of 24 (octet, kernel row) input rows while it multiplies; a
// group that needs more loads the rest in place and waits for it every segment.  So, for a gradient with many column
// tiles: the largest count whose groups stay within one batch (3x3: 9 = four map pairs exactly, 8x8: 8 = half a pair,
// 4x4: 12 = three pairs); 1x1 kernels touch a new octet pair with every tile and keep 12.
static int wgrad_tr_nb(int ntk, int k)
{
    if (ntk < 48) return ntk > 4 ? 4 : 1;
    for (int nb : {12, 9, 8, 6})
        if (wgrad_tr_goct(ntk, nb, k * k) * k <= 24) return nb;
    return 12;
}

// Private copies of a gradient.  A small gradient (one tile group: the 48x768 of the benchmark nets)
// takes one copy per resident workgroup; a large one is split over tile groups (blockIdx.y), which
// already spread it over the GPU, so it gets proportionally fewer copies -- 512 copies of a
// 1024 x 9216 gradient would be 19 GB to write and to sum.
static int wgrad_tile_groups(int MTo, int NTk, int MB, int NB)
{
    return ((MTo + MB - 1) / MB) * ((NTk + 4 * NB - 1) / (4 * NB));
}
static int wgrad_max_copies(int groups)
{
    const int c = (WG_MAX_BLOCKS + groups - 1) / groups;
    return c < 1 ? 1 : c;
}

// floats of the bias partials: one per map and per slice (the slices of bias_grad_kernel, or one per workgroup
// of the 16-bit kernel, which sums dY itself)
static size_t wgrad_bias_floats(int c_out) { return (size_t)(c_out + 15) / 16 * 16 * (WG_MAX_BLOCKS > BG_SLICES ? WG_MAX_BLOCKS : BG_SLICES); }

size_t wgrad_f32_scratch_floats(int c_out, int c_in, int k)
{
    // private dW copies (the larger of what the fp32 and the 16-bit tiling ask for), then the bias partials
    // (8 * ceil(c_out/8) maps x BG_SLICES)
    int MTo, NTk, MB, NB;
    wgrad_tiling(c_out, c_in, k, false, MTo, NTk, MB, NB);
    int copies = wgrad_max_copies(wgrad_tile_groups(MTo, NTk, MB, NB));
    wgrad_tiling(c_out, c_in, k, true, MTo, NTk, MB, NB);
    copies = std::max(copies, wgrad_max_copies(wgrad_tile_groups(MTo, NTk, MB, NB)));
    if (wgrad_tr_applies(c_in)) {            // the transposing-read kernel: its own column tiles, groups and (wider) copies
        int MT2, NT2, MB2, NB2;
        wgrad_tiling(c_out, c_in, k, false, MT2, NT2, MB2, NB2);
        NT2 = wgrad_tr_ntk(c_in, k);
        NB2 = wgrad_tr_nb(NT2, k);
        copies = std::max(copies, wgrad_max_copies(wgrad_tile_groups(MT2, NT2, MB2, NB2)));
        NTk = std::max(NTk, NT2);
    }
    const size_t segs = (size_t)copies * MTo * 16 * NTk * 16 + wgrad_bias_floats(c_out);
    return std::max(segs, wgrad_rows_h_supported(c_in, c_out, k, 1) ? wgrad_rows_h_scratch_floats(c_in, c_out) : (size_t)0);
}

template <int MB, int NB, int DT>
static hipError_t launch_wgrad_t(const WgradArgs &a, size_t smem, int blocks, hipStream_t stream)
{
    static bool attr_set = false;
    if (smem > 48 * 1024 && !attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&wgrad_f32_kernel<MB, NB, DT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int mgroups = (a.MTo + MB - 1) / MB, ngroups = (a.NTk + 4 * NB - 1) / (4 * NB);
    hipLaunchKernelGGL((wgrad_f32_kernel<MB, NB, DT>), dim3(blocks, mgroups * ngroups), dim3(256), smem, stream, a);
    return hipGetLastError();
}

template <int MB, int NB, int DT, int RB>
static hipError_t launch_wgrad_h_t(const WgradArgs &a, size_t smem, int blocks, hipStream_t stream)
{
    static bool attr_set = false;
    if (smem > 48 * 1024 && !attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&wgrad_h_kernel<MB, NB, DT, RB>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int mgroups = (a.MTo + MB - 1) / MB, ngroups = (a.NTk + 4 * NB - 1) / (4 * NB);
    hipLaunchKernelGGL((wgrad_h_kernel<MB, NB, DT, RB>), dim3(blocks, mgroups * ngroups), dim3(256), smem, stream, a);
    return hipGetLastError();
}

template <int DT, int RB>
static hipError_t launch_wgrad_h_rb(const WgradArgs &a, int MB, int NB, size_t smem, int blocks, hipStream_t stream)
{
    hipError_t e = hipErrorInvalidValue;
#define SK_WG_CASE(mb, nb) if (MB == mb && NB == nb) e = launch_wgrad_h_t<mb, nb, DT, RB>(a, smem, blocks, stream);
    SK_WG_CASE(1, 1) SK_WG_CASE(1, 4) SK_WG_CASE(1, 12)
    SK_WG_CASE(3, 1) SK_WG_CASE(3, 4) SK_WG_CASE(3, 12)
    SK_WG_CASE(4, 1) SK_WG_CASE(4, 4) SK_WG_CASE(4, 12)
#undef SK_WG_CASE
    return e;
}

template <int MB, int NB, int DT>
static hipError_t launch_wgrad_tr_t(const WgradArgs &a, size_t smem, int blocks, hipStream_t stream)
{
    static bool attr_set = false;
    if (smem > 48 * 1024 && !attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&wgrad_tr_h_kernel<MB, NB, DT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int mgroups = (a.MTo + MB - 1) / MB, ngroups = (a.NTk + 4 * NB - 1) / (4 * NB);
    hipLaunchKernelGGL((wgrad_tr_h_kernel<MB, NB, DT>), dim3(blocks, mgroups * ngroups), dim3(256), smem, stream, a);
    return hipGetLastError();
}

template <int MB, int NB, int DT>
static hipError_t launch_wgrad_trr_t(const WgradArgs &a, size_t smem, int blocks, hipStream_t stream)
{
    static bool attr_set = false;
    if (smem > 48 * 1024 && !attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&wgrad_trr_h_kernel<MB, NB, DT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int mgroups = (a.MTo + MB - 1) / MB, ngroups = (a.NTk + 4 * NB - 1) / (4 * NB);
    hipLaunchKernelGGL((wgrad_trr_h_kernel<MB, NB, DT>), dim3(blocks, mgroups * ngroups), dim3(256), smem, stream, a);
    return hipGetLastError();
}

// ring = the strip-walking kernel that keeps the staged input rows across steps
template <int DT>
static hipError_t launch_wgrad_tr(const WgradArgs &a, int MB, int NB, size_t smem, int blocks, hipStream_t stream, bool ring)
{
    hipError_t e = hipErrorInvalidValue;
#define SK_WG_CASE(mb, nb) \
    if (MB == mb && NB == nb) e = ring ? launch_wgrad_trr_t<mb, nb, DT>(a, smem, blocks, stream) : launch_wgrad_tr_t<mb, nb, DT>(a, smem, blocks, stream);
    SK_WG_CASE(1, 1) SK_WG_CASE(1, 4) SK_WG_CASE(1, 12) SK_WG_CASE(1, 6) SK_WG_CASE(1, 8) SK_WG_CASE(1, 9)
    SK_WG_CASE(3, 1) SK_WG_CASE(3, 4) SK_WG_CASE(3, 12) SK_WG_CASE(3, 6) SK_WG_CASE(3, 8) SK_WG_CASE(3, 9)
    SK_WG_CASE(4, 1) SK_WG_CASE(4, 4) SK_WG_CASE(4, 12) SK_WG_CASE(4, 6) SK_WG_CASE(4, 8) SK_WG_CASE(4, 9)
#undef SK_WG_CASE
    return e;
}

// floats of one private copy of a gradient, and of its bias partials
static size_t wgrad_copy_floats(int c_out, int c_in, int k)
{
    int ntk = (c_in * k * k + 15) / 16;
    if (wgrad_tr_applies(c_in)) ntk = std::max(ntk, wgrad_tr_ntk(c_in, k));
    return (size_t)((c_out + 15) / 16 * 16) * (size_t)ntk * 16;
}

size_t wgrad_min_scratch_floats(int c_out, int c_in, int k) { return wgrad_copy_floats(c_out, c_in, k) + wgrad_bias_floats(c_out); }

template <int DT>
static hipError_t launch_wgrad_dt(const void *x, const void *dy, float *dw, float *db, float *scratch, int n, int c_in, int H,
                                  int W, int c_out, int k, int d, hipStream_t stream, long x_bstride = 0, int grp_maps = 0,
                                  long grp_skip = 0, size_t scratch_cap = 0)
{
    WgradArgs a;
    a.x_bstride = x_bstride ? x_bstride : (long)c_in * H * W;
    a.grp_shift = 31; a.grp_skip = 0;
    a.xb8 = (c_in + 7) / 8; a.grp8 = 1 << 30; a.skip8 = 0;
    const bool grouped_h = DT != 0 && (grp_maps > 0 || x_bstride != 0);
    if (grouped_h) {
        // 16-bit storage: x_bstride and grp_skip count octet planes, grp_maps is a multiple of 8 (transposing-read kernel only)
        if (grp_maps < 0 || grp_maps % 8 != 0 || grp_skip < 0 || x_bstride < 0 || x_bstride > 0x7fffffffL || grp_skip > 0x7fffffffL ||
            (grp_maps > 0 && c_in % grp_maps != 0))
            return hipErrorInvalidValue;
        if (x_bstride > 0) a.xb8 = (int)x_bstride;
        if (grp_maps > 0) { a.grp8 = grp_maps / 8; a.skip8 = (int)grp_skip; }
        a.x_bstride = 0;
    } else if (grp_maps > 0) {
        if ((grp_maps & (grp_maps - 1)) != 0 || c_in % grp_maps != 0 || grp_skip < 0) return hipErrorInvalidValue;
        a.grp_shift = __builtin_ctz((unsigned)grp_maps);
        a.grp_skip = grp_skip;
    }
    a.x = x; a.dy = dy; a.scratch = scratch; a.bias_part = nullptr;
    a.n = n; a.c_in = c_in; a.H = H; a.W = W; a.c_out = c_out; a.k = k; a.d = d;
    a.Ho = H - (k - 1) * d; a.Wo = W - (k - 1) * d;
    if (a.Ho < 1 || a.Wo < 1) return hipErrorInvalidValue;
    int MB, NB;
    wgrad_tiling(c_out, c_in, k, DT == 0, a.MTo, a.NTk, MB, NB);
    // fp32 storage: at most 16 column tiles per workgroup keep the kernel within half the register file, so two
    // workgroups share a CU and one stages while the other multiplies; with 48 column tiles (192 accumulator
    // registers at four map tiles) only one fits.  Measured on the training steps: U-Net 22.4 -> 20.1 ms, USK-Net
    // 49.3 -> 41.8 ms.  (More tile groups mean fewer private copies, so the scratch sized for 48 still suffices;
    // with three map tiles the single 48-tile group stays faster: 4.09 against 4.38 ms on the 48-map SK-Net.)
    a.xsegs = (a.Wo + WG_SEG - 1) / WG_SEG;
    a.total_segs = a.xsegs * a.Ho * n;
    const int PW = WG_SEG + (k - 1) * d;
    // fp32 storage: a tile group stages only the maps of its own columns; fewer column tiles per group
    // when even those do not fit the LDS (1x1 kernels over many maps)
    auto f32_smem = [&](int nb) {
        const int maps = std::min(c_in, (nb * 64 + k * k - 1) / (k * k) + 1);
        return sizeof(float) * ((size_t)MB * 16 * WG_DYP + (size_t)maps * k * ((PW + 31) / 32 * 32 + 4));
    };
    if (DT == 0 && PW > 192) return hipErrorInvalidValue;            // the staging loop covers three 64-column groups per row
    if (DT == 0)
        while (NB > 1 && f32_smem(NB) > 150 * 1024) NB = NB == 12 ? 4 : NB - 1;
    // 16-bit storage (and a window of at most 128 columns): the 16-bit matrix path
    const bool h_path = DT != 0 && PW <= 128;
    // ... with 16 input maps or more: octets staged as they are, fragments by the transposing LDS read
    const bool tr_path = h_path && wgrad_tr_applies(c_in);
    if (grouped_h && !tr_path) return hipErrorInvalidValue;
    if (tr_path) {
        a.NTk = wgrad_tr_ntk(c_in, k);
        NB = wgrad_tr_nb(a.NTk, k);
    }
    a.xpitch = tr_path ? (PW + 7) / 8 * 8 + 4 : (h_path ? (PW + 7) / 8 * 8 + 8 : (PW + 31) / 32 * 32 + 4);
    // 16-bit matrix path: a tile group stages the input octets its columns touch (the most any group has)
    int goct = (c_in + 7) / 8;
    if (tr_path) {
        goct = wgrad_tr_goct(a.NTk, NB, k * k);
    } else if (h_path) {
        const int K = c_in * k * k, ngroups = (a.NTk + 4 * NB - 1) / (4 * NB);
        goct = 1;
        for (int gi = 0; gi < ngroups; ++gi) {
            const int lo = gi * NB * 64, hi = std::min(lo + NB * 64 - 1, K - 1);
            goct = std::max(goct, hi / (k * k) / 8 - lo / (k * k) / 8 + 1);
        }
    }
    const int x_rows = (DT == 0 ? c_in : goct * 8) * k;
    const size_t smem = DT == 0 ? f32_smem(NB)
                        : tr_path ? 16 * ((size_t)2 * MB * WG_TRP + (size_t)goct * k * a.xpitch)
                                  : sizeof(unsigned short) * ((size_t)MB * 16 * (h_path ? WG_DYH : WG_DYP) + (size_t)x_rows * a.xpitch);
    if (smem > 150 * 1024) return hipErrorInvalidValue;
    // as many persistent workgroups as fit on the GPU at once (more would only add private copies
    // for the reduction to read): LDS decides
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    const long per_cu = (long)(160 * 1024) / (long)(smem > 1 ? smem : 1);
    long resident = (long)cus * (per_cu < 1 ? 1 : (per_cu > 2 ? 2 : per_cu));
    // 16-bit path, few segments per workgroup (one 512^2 image): the private copies -- written once per workgroup, read
    // once by the reduction -- cost more than a second workgroup per CU hides (measured 96 + 12 -> 87 + 7 us per layer)
    if (h_path && wgrad_tile_groups(a.MTo, a.NTk, MB, NB) == 1 && a.NTk >= 48 && a.total_segs < 24L * 2 * cus && resident > cus) resident = cus;
    if (resident > WG_MAX_BLOCKS) resident = WG_MAX_BLOCKS;
    const int groups = wgrad_tile_groups(a.MTo, a.NTk, MB, NB);
    int max_copies = wgrad_max_copies(groups);
    if (scratch_cap > 0) {
        // a scratch buffer of a given size: as many private copies as it holds (fewer workgroups, same sums)
        const size_t per = wgrad_copy_floats(c_out, c_in, k), bias = wgrad_bias_floats(c_out);
        if (scratch_cap < per + bias) return hipErrorInvalidValue;
        const size_t fit = (scratch_cap - bias) / per;
        if (fit < (size_t)max_copies) max_copies = (int)fit;
    }
    long copies = (resident + groups - 1) / groups;
    if (copies > max_copies) copies = max_copies;
    const int blocks = a.total_segs < copies ? a.total_segs : (int)copies;
    float *bias_part = scratch + (size_t)max_copies * a.MTo * 16 * a.NTk * 16;
    const bool bias_in_kernel = db && h_path && MB <= 4;
    if (bias_in_kernel) a.bias_part = bias_part;
    hipError_t e = hipErrorInvalidValue;
    if constexpr (DT != 0) {
        if (tr_path) {
            // input rows kept across steps: kernels of two rows or more
            const bool ring = k >= 2 && goct <= 12;
            e = launch_wgrad_tr<DT>(a, MB, NB, smem, blocks, stream, ring);
        } else if (h_path) {
            if (k == 1 || d % 8 == 0) e = launch_wgrad_h_rb<DT, 16>(a, MB, NB, smem, blocks, stream);
            else if (d % 4 == 0) e = launch_wgrad_h_rb<DT, 8>(a, MB, NB, smem, blocks, stream);
            else if (d % 2 == 0) e = launch_wgrad_h_rb<DT, 4>(a, MB, NB, smem, blocks, stream);
            else e = launch_wgrad_h_rb<DT, 2>(a, MB, NB, smem, blocks, stream);
        }
    }
    if (!h_path) {
#define SK_WG_CASE(mb, nb) if (MB == mb && NB == nb) e = launch_wgrad_t<mb, nb, DT>(a, smem, blocks, stream);
        SK_WG_CASE(1, 1) SK_WG_CASE(1, 4) SK_WG_CASE(1, 12)
        SK_WG_CASE(3, 1) SK_WG_CASE(3, 4) SK_WG_CASE(3, 12)
        SK_WG_CASE(4, 1) SK_WG_CASE(4, 4) SK_WG_CASE(4, 12)
        if constexpr (DT == 0) {   // the tile counts only the fp32 tiling asks for
            SK_WG_CASE(1, 2) SK_WG_CASE(1, 3)
            SK_WG_CASE(2, 1) SK_WG_CASE(2, 2) SK_WG_CASE(2, 3) SK_WG_CASE(2, 4)
            SK_WG_CASE(3, 2) SK_WG_CASE(3, 3)
            SK_WG_CASE(4, 2) SK_WG_CASE(4, 3)
        }
#undef SK_WG_CASE
    }
    if (e != hipSuccess) return e;
    // stage 1 of the bias gradient into the partials behind the dW copies, then one kernel that sums
    // the copies and the partials
    if (db && !bias_in_kernel) {
        const long plane = (long)a.Ho * a.Wo;
        if constexpr (DT == 0) {
            hipLaunchKernelGGL(bias_grad_kernel, dim3(BG_SLICES, c_out), dim3(256), 0, stream, static_cast<const float *>(dy), bias_part,
                               n, c_out, plane, BG_SLICES);
            e = hipGetLastError();
        } else {
            e = launch_bias_grad_h(dy, bias_part, DT, n, c_out, plane, BG_SLICES, stream);
        }
        if (e != hipSuccess) return e;
    }
    const int K = c_in * k * k;
    const long total = (long)c_out * K;
    const long walked = tr_path ? (long)c_out * a.NTk * 16 : total;       // (the reduction walks the copies' columns)
    const int dw_blocks = (int)((walked + RED_ELEMS - 1) / RED_ELEMS), db_blocks = db ? (c_out + RED_ELEMS - 1) / RED_ELEMS : 0;
    if (tr_path && 16 * k * k <= TRR_SPAN) {
        // whole runs of 16*k*k floats per workgroup: few copies -> long spans (every thread a float4), many copies ->
        // short spans, so that the thread groups of a workgroup share the copies out
        const int k2 = k * k, run_len = 16 * k2, nruns = a.NTk / k2;
        int want_split = blocks / 4;
        want_split = want_split < 1 ? 1 : (want_split > 16 ? 16 : want_split);
        int rpb = (256 / want_split) * 4 / run_len;
        rpb = rpb < 1 ? 1 : (rpb > nruns ? nruns : rpb);
        const int parts = (nruns + rpb - 1) / rpb, tr_blocks = c_out * parts;
        hipLaunchKernelGGL(wgrad_tr_reduce_kernel, dim3(tr_blocks + db_blocks), dim3(256), 0, stream, scratch, dw, blocks, c_out, K, a.MTo * 16,
                           a.NTk * 16, k2, rpb, parts, tr_blocks, bias_part, db, bias_in_kernel ? blocks : BG_SLICES);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3(dw_blocks + db_blocks), dim3(256), 0, stream, scratch, dw, blocks, c_out, K,
                       a.MTo * 16, a.NTk * 16, dw_blocks, bias_part, db, bias_in_kernel ? blocks : BG_SLICES, tr_path ? k * k : 0);
    return hipGetLastError();
}

hipError_t launch_wgrad_f32(const float *x, const float *dy, float *dw, float *db, float *scratch,
                            int n, int c_in, int H, int W, int c_out, int k, int d,
                            hipStream_t stream, size_t scratch_cap)
{
    return launch_wgrad_dt<0>(x, dy, dw, db, scratch, n, c_in, H, W, c_out, k, d, stream, 0, 0, 0, scratch_cap);
}

hipError_t launch_wgrad_f32_grouped(const float *x, const float *dy, float *dw, float *db, float *scratch, int n, int c_in, int H,
                                    int W, int c_out, int k, int d, long x_bstride, int grp_maps, long grp_skip, hipStream_t stream)
{
    return launch_wgrad_dt<0>(x, dy, dw, db, scratch, n, c_in, H, W, c_out, k, d, stream, x_bstride, grp_maps, grp_skip);
}

// 16-bit storage, input maps in groups (the depth taps of a 3-D convolution as input maps; see WgradArgs): images start
// xb8 octet planes apart, groups of grp_maps maps (a multiple of 8, 0 = none) lie skip8 more planes apart.  Needs at
// least 16 input maps and a staged window of at most 128 columns (wgrad_h_grouped_supported).
bool wgrad_h_grouped_supported(int c_in, int c_out, int k, int d)
{
    if (!wgrad_tr_applies(c_in) || c_in % 8 != 0 || WG_SEG + (k - 1) * d > 128) return false;
    int MTo, NTk, MB, NB;
    wgrad_tiling(c_out, c_in, k, false, MTo, NTk, MB, NB);
    NTk = wgrad_tr_ntk(c_in, k);
    NB = wgrad_tr_nb(NTk, k);
    const int PW = WG_SEG + (k - 1) * d, xpitch = (PW + 7) / 8 * 8 + 4;
    return 16 * ((size_t)2 * MB * WG_TRP + (size_t)wgrad_tr_goct(NTk, NB, k * k) * k * xpitch) <= 150 * 1024;
}

hipError_t launch_wgrad_h_grouped(const void *x, const void *dy, float *dw, float *db, float *scratch, int dtype, int n, int c_in, int H, int W,
                                  int c_out, int k, int d, int xb8, int grp_maps, int skip8, hipStream_t stream, size_t scratch_cap)
{
    if (dtype != 1 && dtype != 2) return hipErrorInvalidValue;
    return dtype == 1 ? launch_wgrad_dt<1>(x, dy, dw, db, scratch, n, c_in, H, W, c_out, k, d, stream, xb8, grp_maps, skip8, scratch_cap)
                      : launch_wgrad_dt<2>(x, dy, dw, db, scratch, n, c_in, H, W, c_out, k, d, stream, xb8, grp_maps, skip8, scratch_cap);
}

// same gradient from 16-bit octet-layout activations (dtype 1 = bf16, 2 = fp16): the operands are
// staged as they are and widened to fp32 when read, the contraction runs on the fp32 MFMA path
hipError_t launch_wgrad_h(const void *x, const void *dy, float *dw, float *db, float *scratch, int dtype,
                          int n, int c_in, int H, int W, int c_out, int k, int d, hipStream_t stream, size_t scratch_cap, const void *zeros)
{
    if (zeros && (dtype == 1 || dtype == 2) && wgrad_rows_h_supported(c_in, c_out, k, d))
        return launch_wgrad_rows_h(x, dy, zeros, dw, db, scratch, scratch_cap ? scratch_cap : wgrad_f32_scratch_floats(c_out, c_in, k), dtype, n,
                                   c_in, H, W, c_out, d, stream);
    return dtype == 1 ? launch_wgrad_dt<1>(x, dy, dw, db, scratch, n, c_in, H, W, c_out, k, d, stream, 0, 0, 0, scratch_cap)
                      : launch_wgrad_dt<2>(x, dy, dw, db, scratch, n, c_in, H, W, c_out, k, d, stream, 0, 0, 0, scratch_cap);
}

}  // namespace sk
