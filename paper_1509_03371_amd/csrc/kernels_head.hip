// Fused classification head of an SK net for inference on gfx950:
//   h = ReLU(W1 x + b1)   (1x1 convolution, f_in -> hidden)
//   z = W2 h + b2         (1x1 convolution, hidden -> classes)
//   p = softmax(z)        (per pixel)
// i.e. the layers that Algorithm 1 makes out of the inner-product layers of a sliding-window net
// (ip1/ip2/ip3 + prob in the paper's SK table) when their kernel is 1x1.  Unfused, the hidden maps
// go out to HBM and come back (1800 B per pixel for 48 -> 200 -> 2 in fp32); fused, a pixel costs
// its f_in inputs and its class probabilities only.
//
// The first product runs on MFMA (A = W1 fragments kept in LDS, B = the pixels, loaded from global
// memory straight into registers, M = hidden maps, N = 16 pixels).  Its accumulator layout gives
// lane (g, l16) the hidden maps 4g..4g+3 of every 16-map tile for pixel l16, so the second product
// is a per-lane partial dot product followed by a reduction over the four lane groups; softmax and
// the store are done by lane group 0.
#include "sk_kernels.h"

namespace sk {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 halfx2 __attribute__((ext_vector_type(2)));

constexpr int HEAD_THREADS = 256;
constexpr int HEAD_MAX_CLASSES = 8;

// DT = 0: fp32 NCHW input, MFMA 16x16x4 fp32, one K step = 4 input maps.
// DT = 1/2: bf16/fp16 octet-layout input, MFMA 16x16x32, one K step = 4 input octets.
// HT hidden tiles of 16 maps, NTP pixel tiles of 16 pixels per wave and pass, CL class slots.
template <int DT, int HT, int NTP, int CL>
__global__ __launch_bounds__(HEAD_THREADS, 2) void head_fused_kernel(HeadArgs a)
{
    extern __shared__ float smem[];
    // LDS: [W1 fragments][b1: HT*16][W2: CL*HT*16][b2: CL]
    constexpr int FRAG_FLOATS = DT == 0 ? 64 : 256;       // one A fragment: 64 lanes x (4 B | 16 B)
    const int ksteps = a.ksteps;
    float *w1 = smem;
    float *b1 = w1 + HT * ksteps * FRAG_FLOATS;
    float *w2 = b1 + HT * 16;
    float *b2 = w2 + CL * HT * 16;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l16 = lane & 15, g = lane >> 4;

    for (int q = tid; q < HT * ksteps * FRAG_FLOATS; q += HEAD_THREADS) w1[q] = static_cast<const float *>(a.w1p)[q];
    for (int q = tid; q < HT * 16; q += HEAD_THREADS) b1[q] = q < a.hidden ? a.b1[q] : 0.f;
    for (int q = tid; q < CL * HT * 16; q += HEAD_THREADS) {
        const int c = q / (HT * 16), m = q - c * (HT * 16);
        w2[q] = (c < a.classes && m < a.hidden) ? a.w2[c * a.hidden + m] : 0.f;
    }
    for (int q = tid; q < CL; q += HEAD_THREADS) b2[q] = q < a.classes ? a.b2[q] : 0.f;
    __syncthreads();

    // pixel counts fit 32 bits (checked by the launcher)
    const int plane = a.H * a.W, total = a.n * plane;
    const int groups = (total + 16 * NTP - 1) / (16 * NTP);
    const int wave_id = blockIdx.x * (HEAD_THREADS / 64) + wave, wave_cnt = gridDim.x * (HEAD_THREADS / 64);
    const int c8 = (a.c_in + 7) / 8;

    for (int grp = wave_id; grp < groups; grp += wave_cnt) {
        floatx4 acc[HT][NTP];
#pragma unroll
        for (int mt = 0; mt < HT; ++mt)
#pragma unroll
            for (int pt = 0; pt < NTP; ++pt) acc[mt][pt] = floatx4{0.f, 0.f, 0.f, 0.f};
        long base[NTP];       // element offset of (image, map/octet 0, pixel) for this lane
        int pix[NTP], img[NTP];
        bool ok[NTP];
#pragma unroll
        for (int pt = 0; pt < NTP; ++pt) {
            const int p = (grp * NTP + pt) * 16 + l16;
            ok[pt] = p < total;
            const int pc = ok[pt] ? p : total - 1;
            img[pt] = pc / plane;
            pix[pt] = pc - img[pt] * plane;
            base[pt] = (long)img[pt] * (DT == 0 ? a.c_in : c8) * plane + pix[pt];
        }
        for (int ks = 0; ks < ksteps; ++ks) {
            if constexpr (DT == 0) {
                float bv[NTP];
                const int c = ks * 4 + g;
                const int cc = c < a.c_in ? c : a.c_in - 1;
#pragma unroll
                for (int pt = 0; pt < NTP; ++pt) {
                    const float v = static_cast<const float *>(a.x)[base[pt] + (long)cc * plane];
                    bv[pt] = c < a.c_in ? v : 0.f;
                }
#pragma unroll
                for (int mt = 0; mt < HT; ++mt) {
                    const float av = w1[(mt * ksteps + ks) * 64 + lane];
#pragma unroll
                    for (int pt = 0; pt < NTP; ++pt)
                        acc[mt][pt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv[pt], acc[mt][pt], 0, 0, 0);
                }
            } else {
                uint4v bv[NTP];
                const int o = ks * 4 + g;
                const int oc = o < c8 ? o : c8 - 1;
#pragma unroll
                for (int pt = 0; pt < NTP; ++pt) {
                    const uint4v v = static_cast<const uint4v *>(a.x)[base[pt] + (long)oc * plane];
                    bv[pt] = o < c8 ? v : uint4v{0u, 0u, 0u, 0u};
                }
#pragma unroll
                for (int mt = 0; mt < HT; ++mt) {
                    const uint4v av = reinterpret_cast<const uint4v *>(w1)[(mt * ksteps + ks) * 64 + lane];
#pragma unroll
                    for (int pt = 0; pt < NTP; ++pt) {
                        if constexpr (DT == 1)
                            acc[mt][pt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, bv[pt]), acc[mt][pt], 0, 0, 0);
                        else
                            acc[mt][pt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(halfx8, av), __builtin_bit_cast(halfx8, bv[pt]), acc[mt][pt], 0, 0, 0);
                    }
                }
            }
        }
        // hidden activation and second product: b1 / W2 fragments are read once per hidden tile and
        // used for every pixel tile of the pass
        float z[NTP][CL];
#pragma unroll
        for (int pt = 0; pt < NTP; ++pt)
#pragma unroll
            for (int c = 0; c < CL; ++c) z[pt][c] = 0.f;
#pragma unroll
        for (int mt = 0; mt < HT; ++mt) {
            const floatx4 bb = *reinterpret_cast<const floatx4 *>(b1 + mt * 16 + 4 * g);
            floatx4 ww[CL];
#pragma unroll
            for (int c = 0; c < CL; ++c) ww[c] = *reinterpret_cast<const floatx4 *>(w2 + (c * HT + mt) * 16 + 4 * g);
#pragma unroll
            for (int pt = 0; pt < NTP; ++pt) {
                floatx4 h = acc[mt][pt] + bb;
#pragma unroll
                for (int r = 0; r < 4; ++r) h[r] = fmaxf(h[r], 0.f);
#pragma unroll
                for (int c = 0; c < CL; ++c) z[pt][c] += h[0] * ww[c][0] + h[1] * ww[c][1] + h[2] * ww[c][2] + h[3] * ww[c][3];
            }
            // keep the compiler from hoisting the LDS reads of all hidden tiles above this point
            // (it would hold every b1 / W2 fragment in registers at once and spill)
            if (mt % 2 == 1) __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int pt = 0; pt < NTP; ++pt) {
#pragma unroll
            for (int c = 0; c < CL; ++c) {
                z[pt][c] += __shfl_xor(z[pt][c], 16, 64);
                z[pt][c] += __shfl_xor(z[pt][c], 32, 64);
                z[pt][c] += b2[c];
            }
            if (g == 0 && ok[pt]) {       // per-pixel softmax over the real classes
                float m = z[pt][0];
#pragma unroll
                for (int c = 1; c < CL; ++c)
                    if (c < a.classes) m = fmaxf(m, z[pt][c]);
                float e[CL], sum = 0.f;
#pragma unroll
                for (int c = 0; c < CL; ++c) {
                    e[c] = c < a.classes ? expf(z[pt][c] - m) : 0.f;
                    sum += e[c];
                }
                const float inv = 1.f / sum;
                float *dst = a.prob + (long)img[pt] * a.classes * plane + pix[pt];
#pragma unroll
                for (int c = 0; c < CL; ++c)
                    if (c < a.classes) dst[(long)c * plane] = e[c] * inv;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// 16-bit head with both products on MFMA 16x16x32.  The accumulator of the first product gives lane
// (g, l16) the hidden maps 4g..4g+3 of a 16-map tile for pixel l16; two such tiles, ReLU'd and
// rounded to the storage type, are exactly one lane's share (8 K values) of the B operand of a
// second MFMA whose K index runs over the 32 hidden maps of the tile pair in the order
// [tile 2p: 4g..4g+3 | tile 2p+1: 4g..4g+3] -- the W2 fragments are packed in that order, so the
// second product needs no shuffle and costs 3 VALU instructions per two hidden values (max, max,
// pack) instead of bias + max + a multiply-add per class.  b1 and b2 enter as the initial value of
// the accumulators.  Rounding h to the storage type is what the unfused path does when it stores
// the hidden layer.  Hidden tiles are processed in groups of at most GT so that four pixel tiles
// (64 pixels) share each W1 fragment read from LDS; the pixels of the next pass are loaded while
// the current one is multiplied.
// PEND > 0: the input still lacks the horizontal half of an SK pool at kernel stride PEND (see ConvHArgs::vpool): its
// rows hold W + PEND samples and pixel (y, x) is max(X[y][x], X[y][x + PEND]).  The kernel then walks the samples
// in memory order (all W + PEND of a row: the partner of sample q is sample q + PEND whatever the row), loads a
// fifth pixel tile per pass and takes the partner from the lanes PEND further on -- a row shift inside the tile,
// and the first lanes of the next tile -- instead of loading everything twice.  Samples with x >= W are computed
// and dropped.  The values are ReLU outputs, so the unsigned 16-bit order of the bit patterns is the numerical order.
template <unsigned CTRL>
__device__ __forceinline__ unsigned dpp_row_move(unsigned v)
{
    return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);   // lanes shifted in from outside the row read 0
}

template <int DT, int HT, int KSTEPS, int PEND = 0>
__global__ __launch_bounds__(HEAD_THREADS, 2) void head_fused_h_kernel(HeadArgs a)
{
    extern __shared__ float smem[];
    constexpr int NTP = 4, GT = 6, HP = (HT + 1) / 2;   // GT even: tile pairs never straddle two groups
    constexpr int NTL = PEND > 0 ? NTP + 1 : NTP;       // pixel tiles loaded per pass
    uint4v *w1 = reinterpret_cast<uint4v *>(smem);               // [HT][KSTEPS][64]
    uint4v *w2f = w1 + HT * KSTEPS * 64;                         // [HP][64]
    float *b1 = reinterpret_cast<float *>(w2f + HP * 64);        // [HT*16]
    float *b2 = b1 + HT * 16;                                    // [4]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l16 = lane & 15, g = lane >> 4;

    for (int q = tid; q < HT * KSTEPS * 64; q += HEAD_THREADS) w1[q] = static_cast<const uint4v *>(a.w1p)[q];
    for (int q = tid; q < HP * 64; q += HEAD_THREADS) {
        const int pr = q >> 6, ln = q & 63, cls = ln & 15, gg = ln >> 4;
        unsigned short v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int h = 16 * (2 * pr + (e >> 2)) + 4 * gg + (e & 3);
            const float f = (cls < a.classes && h < a.hidden) ? a.w2[cls * a.hidden + h] : 0.f;
            if constexpr (DT == 1) v[e] = __builtin_bit_cast(unsigned short, static_cast<__bf16>(f));
            else v[e] = __builtin_bit_cast(unsigned short, static_cast<_Float16>(f));
        }
        w2f[q] = uint4v{v[0] | ((unsigned)v[1] << 16), v[2] | ((unsigned)v[3] << 16), v[4] | ((unsigned)v[5] << 16), v[6] | ((unsigned)v[7] << 16)};
    }
    for (int q = tid; q < HT * 16; q += HEAD_THREADS) b1[q] = q < a.hidden ? a.b1[q] : 0.f;
    if (tid < 4) b2[tid] = tid < a.classes ? a.b2[tid] : 0.f;
    __syncthreads();

    // samples per image as the kernel walks them: the W + PEND samples of every row in memory
    const int Wm = a.W + PEND;
    const int plane = a.H * Wm, total = a.n * plane;            // fit 32 bits (checked by the launcher)
    const int out_plane = a.H * a.W;
    const int groups = (total + 16 * NTP - 1) / (16 * NTP);
    const int wave_id = blockIdx.x * (HEAD_THREADS / 64) + wave, wave_cnt = gridDim.x * (HEAD_THREADS / 64);
    const int c8 = (a.c_in + 7) / 8;
    const uint4v *xin = static_cast<const uint4v *>(a.x);

    // one division per pass: pixel tile pt + 1 starts 16 pixels after tile pt and may wrap into the
    // following image(s)
    auto load_pixels = [&](int grp, uint4v (&bv)[KSTEPS][NTL]) {
        int p = grp * (16 * NTP) + l16;
        p = p < total ? p : total - 1;
        int img = p / plane, pix = p - img * plane;
#pragma unroll
        for (int pt = 0; pt < NTL; ++pt) {
            const long base = (long)img * c8 * plane + pix;
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                const int o = ks * 4 + g;
                const uint4v v = xin[base + (long)(o < c8 ? o : c8 - 1) * plane];
                bv[ks][pt] = o < c8 ? v : uint4v{0u, 0u, 0u, 0u};
            }
            pix += 16;                                           // next tile; clamp at the very end
            while (pix >= plane && img + 1 < a.n) { pix -= plane; ++img; }
            if (pix >= plane) pix = plane - 1;
        }
    };
    // PEND: tile pt becomes the maximum of itself, itself shifted down by PEND lanes inside each row of 16 lanes,
    // and the next tile shifted up by 16 - PEND
    auto finish_pool = [&](uint4v (&bv)[KSTEPS][NTL]) {
        if constexpr (PEND > 0) {
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
                for (int pt = 0; pt < NTP; ++pt)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        unsigned v = bv[ks][pt][e];
                        const unsigned own = PEND < 16 ? dpp_row_move<0x100 + (PEND < 16 ? PEND : 1)>(v) : 0u;                  // row_shl: lane l reads lane l + PEND
                        const unsigned nxt = PEND < 16 ? dpp_row_move<0x110 + (PEND < 16 ? 16 - PEND : 1)>(bv[ks][pt + 1][e])   // row_shr: lane l reads lane l - (16 - PEND)
                                                       : bv[ks][pt + 1][e];
                        asm("v_pk_max_u16 %0, %1, %2" : "=v"(v) : "v"(v), "v"(own));
                        asm("v_pk_max_u16 %0, %1, %2" : "=v"(v) : "v"(v), "v"(nxt));
                        bv[ks][pt][e] = v;
                    }
        }
    };
    auto mfma = [](uint4v av, uint4v bvv, floatx4 c) {
        if constexpr (DT == 1) return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, bvv), c, 0, 0, 0);
        else return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(halfx8, av), __builtin_bit_cast(halfx8, bvv), c, 0, 0, 0);
    };
    // ReLU as a signed-integer max on the bit pattern (negative floats, -0 included, are negative
    // integers; one instruction, where fmaxf costs a NaN canonicalisation besides the max), then
    // both values are rounded to the storage type by one packed conversion
    auto pack2 = [](float lo, float hi) -> unsigned {
        const floatx2 r = {__int_as_float(max(__float_as_int(lo), 0)), __int_as_float(max(__float_as_int(hi), 0))};
        if constexpr (DT == 1) return __builtin_bit_cast(unsigned, __builtin_convertvector(r, bf16x2));
        else return __builtin_bit_cast(unsigned, __builtin_convertvector(r, halfx2));
    };

    uint4v bv[KSTEPS][NTL], nx[KSTEPS][NTL];
    if (wave_id < groups) load_pixels(wave_id, bv);
    for (int grp = wave_id; grp < groups; grp += wave_cnt) {
        const int nxt = grp + wave_cnt;
        load_pixels(nxt < groups ? nxt : grp, nx);               // in flight during this pass
        finish_pool(bv);
        floatx4 z[NTP];
        {
            const floatx4 zb = g == 0 ? *reinterpret_cast<const floatx4 *>(b2) : floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int pt = 0; pt < NTP; ++pt) z[pt] = zb;
        }
#pragma unroll
        for (int t0 = 0; t0 < HT; t0 += GT) {
            const int nt = HT - t0 < GT ? HT - t0 : GT;           // compile-time after unrolling
            floatx4 acc[GT][NTP];
#pragma unroll
            for (int t = 0; t < GT; ++t) {
                if (t >= nt) break;
                const floatx4 bb = *reinterpret_cast<const floatx4 *>(b1 + (t0 + t) * 16 + 4 * g);
#pragma unroll
                for (int pt = 0; pt < NTP; ++pt) acc[t][pt] = bb;
            }
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
                for (int t = 0; t < GT; ++t) {
                    if (t >= nt) break;
                    const uint4v av = w1[((t0 + t) * KSTEPS + ks) * 64 + lane];
#pragma unroll
                    for (int pt = 0; pt < NTP; ++pt) acc[t][pt] = mfma(av, bv[ks][pt], acc[t][pt]);
                    // keep the LDS reads of later tiles from being hoisted (they would spill)
                    if (t % 2 == 1) __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
            for (int t = 0; t < GT; t += 2) {
                if (t >= nt) break;
                const uint4v wv = w2f[((t0 + t) >> 1) * 64 + lane];
                const bool two = t + 1 < nt;
#pragma unroll
                for (int pt = 0; pt < NTP; ++pt) {
                    uint4v hb;
                    hb[0] = pack2(acc[t][pt][0], acc[t][pt][1]);
                    hb[1] = pack2(acc[t][pt][2], acc[t][pt][3]);
                    hb[2] = two ? pack2(acc[t + 1 < GT ? t + 1 : t][pt][0], acc[t + 1 < GT ? t + 1 : t][pt][1]) : 0u;
                    hb[3] = two ? pack2(acc[t + 1 < GT ? t + 1 : t][pt][2], acc[t + 1 < GT ? t + 1 : t][pt][3]) : 0u;
                    z[pt] = mfma(wv, hb, z[pt]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // Classes 0..3 of pixel (pt, l16) sit in lane (0, l16) of z[pt].  Lane (g, l16) fetches those
        // of pixel tile pt = g, so that all 64 lanes do one softmax each and a store instruction
        // writes 64 consecutive pixels of one class.
        {
            float zc[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                zc[c] = 0.f;
                if (c < a.classes) {                              // uniform
#pragma unroll
                    for (int pt = 0; pt < NTP; ++pt) {
                        const float v = __shfl(z[pt][c], l16, 64);
                        if (g == pt) zc[c] = v;
                    }
                }
            }
            const int p = grp * (16 * NTP) + lane;
            const int img = p / plane;
            int pix = p - img * plane;
            bool keep = p < total;
            if constexpr (PEND > 0) {                             // memory sample -> output pixel; the PEND extra samples of a row are dropped
                const int yy = pix / Wm, xx = pix - yy * Wm;
                keep = keep && xx < a.W;
                pix = yy * a.W + xx;
            }
            if (keep) {
                float m = zc[0];
#pragma unroll
                for (int c = 1; c < 4; ++c)
                    if (c < a.classes) m = fmaxf(m, zc[c]);
                float e[4], sum = 0.f;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    e[c] = c < a.classes ? __expf(zc[c] - m) : 0.f;
                    sum += e[c];
                }
                const float inv = __frcp_rn(sum);
                float *dst = a.prob + (long)img * a.classes * out_plane + pix;
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (c < a.classes) dst[(long)c * out_plane] = e[c] * inv;
            }
        }
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
            for (int pt = 0; pt < NTL; ++pt) bv[ks][pt] = nx[ks][pt];
    }
}

// W1 [hidden][c_in] fp32 -> MFMA A fragments, [hidden tile][K step][lane][values]:
//   DT = 0: value            = W1[16*mt + l16][4*ks + g]
//   DT > 0: values e = 0..7  = W1[16*mt + l16][8*(4*ks + g) + e]   (16-bit)
template <int DT>
__global__ void pack_head_w1_kernel(const float *w1, void *out, int hidden, int c_in, int ht, int ksteps)
{
    const int per = DT == 0 ? 1 : 8;
    const long total = (long)ht * ksteps * 64 * per;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        long r = q;
        const int e = (int)(r % per); r /= per;
        const int lane = (int)(r % 64); r /= 64;
        const int ks = (int)(r % ksteps); r /= ksteps;
        const int mt = (int)r;
        const int m = mt * 16 + (lane & 15), g = lane >> 4;
        const int c = DT == 0 ? ks * 4 + g : (ks * 4 + g) * 8 + e;
        const float v = (m < hidden && c < c_in) ? w1[(long)m * c_in + c] : 0.f;
        if constexpr (DT == 0) static_cast<float *>(out)[q] = v;
        else if constexpr (DT == 1) static_cast<unsigned short *>(out)[q] = __builtin_bit_cast(unsigned short, static_cast<__bf16>(v));
        else static_cast<unsigned short *>(out)[q] = __builtin_bit_cast(unsigned short, static_cast<_Float16>(v));
    }
}

int head_hidden_tiles(int hidden)
{
    const int t = (hidden + 15) / 16;
    return t <= 4 ? 4 : t <= 8 ? 8 : t <= 13 ? 13 : 16;
}

int head_ksteps(int dtype, int c_in) { return dtype == 0 ? (c_in + 3) / 4 : ((c_in + 7) / 8 + 3) / 4; }

bool head_supported(int dtype, int c_in, int hidden, int classes)
{
    if (hidden < 1 || hidden > 256 || classes < 1 || classes > HEAD_MAX_CLASSES || c_in < 1 || c_in > 512) return false;
    const size_t frag = dtype == 0 ? 256 : 1024;
    const int ht = head_hidden_tiles(hidden);
    return ht * head_ksteps(dtype, c_in) * frag + (size_t)(ht * 16 * (HEAD_MAX_CLASSES + 1) + HEAD_MAX_CLASSES) * 4 <= 150 * 1024;
}

long head_w1_packed_bytes(int dtype, int c_in, int hidden)
{
    return (long)head_hidden_tiles(hidden) * head_ksteps(dtype, c_in) * (dtype == 0 ? 256 : 1024);
}

hipError_t launch_pack_head_w1(const float *w1, void *out, int dtype, int hidden, int c_in, hipStream_t stream)
{
    const int ht = head_hidden_tiles(hidden), ks = head_ksteps(dtype, c_in);
    if (dtype == 0) hipLaunchKernelGGL(pack_head_w1_kernel<0>, dim3(64), dim3(256), 0, stream, w1, out, hidden, c_in, ht, ks);
    else if (dtype == 1) hipLaunchKernelGGL(pack_head_w1_kernel<1>, dim3(64), dim3(256), 0, stream, w1, out, hidden, c_in, ht, ks);
    else hipLaunchKernelGGL(pack_head_w1_kernel<2>, dim3(64), dim3(256), 0, stream, w1, out, hidden, c_in, ht, ks);
    return hipGetLastError();
}

template <int DT, int HT, int CL>
static hipError_t launch_head_t(const HeadArgs &a, hipStream_t stream)
{
    constexpr int NTP = HT <= 4 ? 4 : (HT <= 8 ? 2 : (CL <= 2 ? 2 : 1));   // bounded by the register file
    const size_t smem = (size_t)HT * a.ksteps * (DT == 0 ? 256 : 1024) + (size_t)(HT * 16 * (CL + 1) + CL) * 4;
    static bool attr_set = false;
    if (smem > 48 * 1024 && !attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&head_fused_kernel<DT, HT, NTP, CL>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const long total = (long)a.n * a.H * a.W;
    const long groups = (total + 16 * NTP - 1) / (16 * NTP);
    long blocks = (groups + 3) / 4;
    if (blocks > 1024) blocks = 1024;     // persistent-style grid: waves stride over the pixel groups
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL((head_fused_kernel<DT, HT, NTP, CL>), dim3((int)blocks), dim3(HEAD_THREADS), smem, stream, a);
    return hipGetLastError();
}

template <int DT, int CL>
static hipError_t launch_head_cl(const HeadArgs &a, hipStream_t stream)
{
    switch (head_hidden_tiles(a.hidden)) {
    case 4: return launch_head_t<DT, 4, CL>(a, stream);
    case 8: return launch_head_t<DT, 8, CL>(a, stream);
    case 13: return launch_head_t<DT, 13, CL>(a, stream);
    default: return launch_head_t<DT, 16, CL>(a, stream);
    }
}

template <int DT, int HT, int KSTEPS, int PEND>
static hipError_t launch_head_h_p(const HeadArgs &a, hipStream_t stream)
{
    constexpr int HP = (HT + 1) / 2;
    const size_t smem = (size_t)(HT * KSTEPS + HP) * 1024 + (size_t)(HT * 16 + 4) * 4;
    static bool attr_set = false;
    if (smem > 48 * 1024 && !attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&head_fused_h_kernel<DT, HT, KSTEPS, PEND>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const long total = (long)a.n * a.H * (a.W + PEND);
    if (total >= 0x7fffffffL - 64) return hipErrorInvalidValue;
    const long groups = (total + 63) / 64;
    long blocks = (groups + 3) / 4;
    if (blocks > 512) blocks = 512;       // two workgroups per CU, persistent over the pixel groups
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL((head_fused_h_kernel<DT, HT, KSTEPS, PEND>), dim3((int)blocks), dim3(HEAD_THREADS), smem, stream, a);
    return hipGetLastError();
}

// the pending pool distances of SK nets are the kernel strides of their convolutions: powers of two up to 16
template <int DT, int HT, int KSTEPS>
static hipError_t launch_head_h_t(const HeadArgs &a, hipStream_t stream)
{
    switch (a.hd) {
    case 0: return launch_head_h_p<DT, HT, KSTEPS, 0>(a, stream);
    case 1: return launch_head_h_p<DT, HT, KSTEPS, 1>(a, stream);
    case 2: return launch_head_h_p<DT, HT, KSTEPS, 2>(a, stream);
    case 4: return launch_head_h_p<DT, HT, KSTEPS, 4>(a, stream);
    case 8: return launch_head_h_p<DT, HT, KSTEPS, 8>(a, stream);
    case 16: return launch_head_h_p<DT, HT, KSTEPS, 16>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

// the MFMA-only 16-bit kernel covers up to 4 classes and up to 64 input maps
template <int DT>
static bool launch_head_h(const HeadArgs &a, hipStream_t stream, hipError_t *err)
{
    if (a.classes > 4 || a.ksteps > 2) return false;
    const int ht = head_hidden_tiles(a.hidden);
    if (a.ksteps == 1) {
        if (ht == 4) *err = launch_head_h_t<DT, 4, 1>(a, stream);
        else if (ht == 8) *err = launch_head_h_t<DT, 8, 1>(a, stream);
        else if (ht == 13) *err = launch_head_h_t<DT, 13, 1>(a, stream);
        else *err = launch_head_h_t<DT, 16, 1>(a, stream);
    } else {
        if (ht == 4) *err = launch_head_h_t<DT, 4, 2>(a, stream);
        else if (ht == 8) *err = launch_head_h_t<DT, 8, 2>(a, stream);
        else if (ht == 13) *err = launch_head_h_t<DT, 13, 2>(a, stream);
        else *err = launch_head_h_t<DT, 16, 2>(a, stream);
    }
    return true;
}

template <int DT>
static hipError_t launch_head_dt(const HeadArgs &a, hipStream_t stream)
{
    if constexpr (DT != 0) {
        hipError_t err = hipSuccess;
        if (launch_head_h<DT>(a, stream, &err)) return err;
    }
    if (a.classes <= 2) return launch_head_cl<DT, 2>(a, stream);
    if (a.classes <= 4) return launch_head_cl<DT, 4>(a, stream);
    return launch_head_cl<DT, 8>(a, stream);
}

bool head_takes_pending_pool(int dtype, int c_in, int classes, int hd)
{
    // the MFMA-only 16-bit kernel, instantiated for the kernel strides of the SK nets
    return dtype != 0 && classes <= 4 && head_ksteps(dtype, c_in) <= 2 && (hd == 1 || hd == 2 || hd == 4 || hd == 8 || hd == 16);
}

hipError_t launch_head_fused(HeadArgs a, hipStream_t stream)
{
    if (!head_supported(a.dtype, a.c_in, a.hidden, a.classes)) return hipErrorInvalidValue;
    if ((long)a.n * a.H * a.W >= 0x7fffffffL - 64) return hipErrorInvalidValue;
    if (a.hd < 0 || (a.hd > 0 && !head_takes_pending_pool(a.dtype, a.c_in, a.classes, a.hd))) return hipErrorInvalidValue;
    a.ksteps = head_ksteps(a.dtype, a.c_in);
    if (a.dtype == 0) return launch_head_dt<0>(a, stream);
    if (a.dtype == 1) return launch_head_dt<1>(a, stream);
    return launch_head_dt<2>(a, stream);
}

}  // namespace sk
