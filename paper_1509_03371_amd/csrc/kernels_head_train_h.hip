// Backward pass of the classification head in one kernel (gfx950, 16-bit storage):
//
//   h = ReLU(W1 x + b1)   z = W2 h + b2   loss = mean over labelled pixels of -log softmax(z)[label]
//
// (the 1x1 convolutions a9 / a10 of the SK-Net and the softmax loss of Section 4.3, with the label masking of
// Section 4.2).  Run layer by layer, the backward pass of these three moves the hidden maps five times between the
// GPU and its memory (200 maps per pixel against 48 of the input): written by the forward pass, read by the second
// convolution, by its weight gradient and as the ReLU mask, and their gradient written and read twice more.
// Here a workgroup takes 64 pixels at a time and keeps everything but x and dx on the chip:
//   1. per wave, 16 pixels: h (recomputed from x, MFMA 16x16x32 with the W1 fragments in LDS), z, the softmax, the
//      loss term, dz = (p - onehot) / P, dh = (W2^T dz) * [h > 0] on the accumulator layout of h, and
//      dx = W1^T dh by a second MFMA whose K index runs over the hidden maps in the order the accumulators hold
//      them (as the forward head does for z) -- stored to memory in the octet layout;
//   2. h, dh, x and dz of the 64 pixels go to LDS in the octet layout (16-bit, rounded as the layer-by-layer path
//      rounds them when it stores them);
//   3. the weight gradients contract over pixels: dW1 = dh x^T, dW2 = dz h^T, db1 = dh 1, db2 = dz 1, MFMA operands
//      read from those tiles with the transposing LDS read (ds_read_b64_tr_b16: lane 4r + q of a group of 16 names
//      maps 4q..4q+3 of pixel r and receives pixels 0..3 of map 4q + e); wave w owns the hidden-map tiles
//      w, w + 4, ... of dW1 and dW2 and keeps them in accumulators for the whole launch.
// Each workgroup writes its sums once; head_train_reduce_kernel adds the workgroups' copies in a fixed order,
// scatters them to the two layers' dW / db and finishes the loss.
#include "sk_kernels.h"

namespace sk {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
typedef unsigned int uint2v __attribute__((ext_vector_type(2)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 halfx2 __attribute__((ext_vector_type(2)));

namespace {

constexpr int HB_THREADS = 256, HB_PIX = 64;

template <int DT> __device__ __forceinline__ floatx4 mfma32(uint4v a, uint4v b, floatx4 c)
{
    if constexpr (DT == 1) return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(halfx8, a), __builtin_bit_cast(halfx8, b), c, 0, 0, 0);
}

template <int DT> __device__ __forceinline__ unsigned pack16x2(float lo, float hi)
{
    const floatx2 r = {lo, hi};
    if constexpr (DT == 1) return __builtin_bit_cast(unsigned, __builtin_convertvector(r, bf16x2));
    else return __builtin_bit_cast(unsigned, __builtin_convertvector(r, halfx2));
}

template <int DT> __device__ __forceinline__ unsigned short to16(float f)
{
    if constexpr (DT == 1) return __builtin_bit_cast(unsigned short, static_cast<__bf16>(f));
    else return __builtin_bit_cast(unsigned short, static_cast<_Float16>(f));
}

// one operand fragment from an LDS tile in the octet layout: this lane's 8 pixels of its map, two transposing reads
__device__ __forceinline__ uint4v read_frag(const char *lds_base, unsigned off_lo, unsigned off_hi)
{
    typedef short4v __attribute__((address_space(3))) *lds_s4;
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(lds_base + off_lo));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(lds_base + off_hi));
    const uint2v l2 = __builtin_bit_cast(uint2v, lo), h2 = __builtin_bit_cast(uint2v, hi);
    return uint4v{l2[0], l2[1], h2[0], h2[1]};
}

// floats of one workgroup's sums: dW1 accumulators [HT][NT1][64][4], dW2 accumulators [HT][64][4], db1 [HT*16], db2 [16],
// the loss terms [1] (padded to a multiple of 4)
__host__ __device__ constexpr int copy_floats_of(int HT, int NT1) { return HT * NT1 * 256 + HT * 256 + HT * 16 + 16 + 4; }

template <int DT, int HT, int KSTEPS, int NT1>
__global__ __launch_bounds__(HB_THREADS) void head_train_bwd_h_kernel(HeadTrainArgs a)
{
    extern __shared__ uint4v smem16[];
    constexpr int HP = (HT + 1) / 2;                             // pairs of hidden tiles = K steps of the products over hidden maps
    constexpr int PH = HT * 32 + 16;                             // bytes of a pixel's row in the h / dh tiles (16 of padding)
    constexpr int PX = KSTEPS * 64 + 16;                         // ... in the x tile
    constexpr int SLOTS = (HT + 3) / 4;                          // hidden tiles per wave
    uint4v *w1 = smem16;                                         // [HT][KSTEPS][64]   A fragments of h = W1 x
    uint4v *w2f = w1 + HT * KSTEPS * 64;                         // [HP][64]           A fragments of z = W2 h
    uint4v *w1t = w2f + HP * 64;                                 // [NT1][HP][64]      A fragments of dx = W1^T dh
    float *w2c = reinterpret_cast<float *>(w1t + NT1 * HP * 64); // [4][HT*16]         W2 rows, fp32
    float *b1 = w2c + 4 * HT * 16;                               // [HT*16]
    float *b2 = b1 + HT * 16;                                    // [4]
    float *red = b2 + 4;                                         // [4 + 4]            block sums
    char *hs = reinterpret_cast<char *>(red + 8);                // [64][PH]
    char *dhs = hs + HB_PIX * PH;                                // [64][PH]
    char *xs = dhs + HB_PIX * PH;                                // [64][PX]
    char *dzs = xs + HB_PIX * PX;                                // [64][16]  classes 0..3 in the first 8 bytes, zeros behind
    char *zero16 = dzs + HB_PIX * 16;                            // 16 bytes of zeros: the gradient's map quads 2 and 3

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- weights into LDS --------------------------------------------------------------------------------------
    for (int q = tid; q < HT * KSTEPS * 64; q += HB_THREADS) w1[q] = static_cast<const uint4v *>(a.w1p)[q];
    for (int q = tid; q < HP * 64; q += HB_THREADS) {
        const int pr = q >> 6, ln = q & 63, cls = ln & 15, gg = ln >> 4;
        unsigned short v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int h = 16 * (2 * pr + (e >> 2)) + 4 * gg + (e & 3);
            v[e] = to16<DT>((cls < a.classes && h < a.hidden) ? a.w2[cls * a.hidden + h] : 0.f);
        }
        w2f[q] = uint4v{v[0] | ((unsigned)v[1] << 16), v[2] | ((unsigned)v[3] << 16), v[4] | ((unsigned)v[5] << 16), v[6] | ((unsigned)v[7] << 16)};
    }
    for (int q = tid; q < NT1 * HP * 64; q += HB_THREADS) {
        // row m = input map 16 nt + (lane & 15); K value 8 gg + e = hidden map 16 (2 pr + e / 4) + 4 gg + e % 4
        const int ln = q & 63, pr = (q >> 6) % HP, nt = (q >> 6) / HP, c = 16 * nt + (ln & 15), gg = ln >> 4;
        unsigned short v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int h = 16 * (2 * pr + (e >> 2)) + 4 * gg + (e & 3);
            v[e] = to16<DT>((c < a.c_in && h < a.hidden) ? a.w1[(long)h * a.c_in + c] : 0.f);
        }
        w1t[q] = uint4v{v[0] | ((unsigned)v[1] << 16), v[2] | ((unsigned)v[3] << 16), v[4] | ((unsigned)v[5] << 16), v[6] | ((unsigned)v[7] << 16)};
    }
    for (int q = tid; q < 4 * HT * 16; q += HB_THREADS) {
        const int cls = q / (HT * 16), h = q - cls * (HT * 16);
        w2c[q] = (cls < a.classes && h < a.hidden) ? a.w2[cls * a.hidden + h] : 0.f;
    }
    for (int q = tid; q < HT * 16; q += HB_THREADS) b1[q] = q < a.hidden ? a.b1[q] : 0.f;
    if (tid < 4) b2[tid] = tid < a.classes ? a.b2[tid] : 0.f;
    for (int q = tid; q < HB_PIX * 4 + 4; q += HB_THREADS) reinterpret_cast<unsigned *>(dzs)[q] = 0u;    // dzs and zero16
    // labelled pixels P (exact: integers), the same sum in every thread
    {
        long local = 0;
        for (int q = tid; q < a.ncounts; q += HB_THREADS) local += a.counts[q];
        for (int off = 32; off > 0; off >>= 1) local += __shfl_down(local, off, 64);
        long *cs = reinterpret_cast<long *>(red);                // 4 longs = the 8 floats
        if (lane == 0) cs[wave] = local;
    }
    __syncthreads();
    float invP;
    {
        const long *cs = reinterpret_cast<const long *>(red);
        const long kept = cs[0] + cs[1] + cs[2] + cs[3];
        invP = 1.f / (float)(kept > 0 ? kept : 1);
    }
    __syncthreads();

    const int plane = a.plane;
    const long total = (long)a.n * plane;
    const int c8 = (a.c_in + 7) / 8;
    const uint4v *xin = static_cast<const uint4v *>(a.x);
    const long nblocks = (total + HB_PIX - 1) / HB_PIX;

    // this lane's offsets into the tiles for the transposing reads (lane 4r + q of a 16-lane group: pixel r, map quad q)
    const int rr = l16 >> 2, q4 = l16 & 3;
    unsigned off_h[SLOTS], off_x[NT1], off_dz;
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        int t = wave + 4 * s;
        t = t < HT ? t : HT - 1;
        off_h[s] = (unsigned)((8 * g + rr) * PH + (2 * t + (q4 >> 1)) * 16 + (q4 & 1) * 8);
    }
#pragma unroll
    for (int nt = 0; nt < NT1; ++nt) off_x[nt] = (unsigned)((8 * g + rr) * PX + (2 * nt + (q4 >> 1)) * 16 + (q4 & 1) * 8);
    off_dz = (unsigned)(q4 < 2 ? (dzs - hs) + (8 * g + rr) * 16 + q4 * 8 : (zero16 - hs));      // relative to hs
    const unsigned dz_step = q4 < 2 ? 16u : 0u;                 // bytes per pixel (the zeros do not move)

    floatx4 acc1[SLOTS][NT1], acc2[SLOTS], accb1[SLOTS], accb2 = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        acc2[s] = floatx4{0.f, 0.f, 0.f, 0.f};
        accb1[s] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int nt = 0; nt < NT1; ++nt) acc1[s][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
    const unsigned one2 = DT == 1 ? 0x3F803F80u : 0x3C003C00u;  // two ones in the storage type
    const uint4v ones = uint4v{one2, one2, one2, one2};
    float loss_local = 0.f;

    auto load_x = [&](long blk, uint4v (&bv)[KSTEPS]) {
        long p = blk * HB_PIX + 16 * wave + l16;
        p = p < total ? p : total - 1;
        const long img = p / plane, pix = p - img * plane;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const int o = ks * 4 + g;
            const uint4v v = xin[(img * c8 + (o < c8 ? o : c8 - 1)) * plane + pix];
            bv[ks] = o < c8 ? v : uint4v{0u, 0u, 0u, 0u};
        }
    };

    uint4v bv[KSTEPS], nx[KSTEPS];
    if ((long)blockIdx.x < nblocks) load_x(blockIdx.x, bv);
    for (long blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
        const long nblk = blk + gridDim.x;
        load_x(nblk < nblocks ? nblk : blk, nx);                // in flight during this block
        const long p = blk * HB_PIX + 16 * wave + l16;          // this lane's pixel
        const bool inside = p < total;
        const long pc = inside ? p : total - 1;
        const long img = pc / plane, pix = pc - img * plane;
        const int lab = a.labels[pc];
        const int px = 16 * wave + l16;                          // its row in the tiles

        // ---- 1. the wave's 16 pixels ---------------------------------------------------------------------------
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) *reinterpret_cast<uint4v *>(xs + px * PX + (4 * ks + g) * 16) = bv[ks];
        floatx4 hacc[HT];
#pragma unroll
        for (int t = 0; t < HT; ++t) hacc[t] = *reinterpret_cast<const floatx4 *>(b1 + t * 16 + 4 * g);
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
            for (int t = 0; t < HT; ++t) hacc[t] = mfma32<DT>(w1[(t * KSTEPS + ks) * 64 + lane], bv[ks], hacc[t]);
        // ReLU, rounding to the storage type (what the layer-by-layer path stores), z
        unsigned hb[HT][2];
#pragma unroll
        for (int t = 0; t < HT; ++t) {
            hb[t][0] = pack16x2<DT>(fmaxf(hacc[t][0], 0.f), fmaxf(hacc[t][1], 0.f));
            hb[t][1] = pack16x2<DT>(fmaxf(hacc[t][2], 0.f), fmaxf(hacc[t][3], 0.f));
            *reinterpret_cast<uint2v *>(hs + px * PH + (2 * t + (g >> 1)) * 16 + (g & 1) * 8) = uint2v{hb[t][0], hb[t][1]};
        }
        floatx4 z = g == 0 ? *reinterpret_cast<const floatx4 *>(b2) : floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int pr = 0; pr < HP; ++pr) {
            const bool two = 2 * pr + 1 < HT;
            const uint4v hv = uint4v{hb[2 * pr][0], hb[2 * pr][1], two ? hb[2 * pr + 1 < HT ? 2 * pr + 1 : 0][0] : 0u,
                                     two ? hb[2 * pr + 1 < HT ? 2 * pr + 1 : 0][1] : 0u};
            z = mfma32<DT>(w2f[pr * 64 + lane], hv, z);
        }
        // softmax, loss term and dz in the lanes of group 0 (classes 0..3 of pixel l16), then to the pixel's other lanes
        float dz[4] = {0.f, 0.f, 0.f, 0.f};
        if (g == 0 && inside && lab >= 0 && lab < a.classes) {
            float m = z[0];
#pragma unroll
            for (int c = 1; c < 4; ++c)
                if (c < a.classes) m = fmaxf(m, z[c]);
            float e[4], sum = 0.f, zl = 0.f;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                e[c] = c < a.classes ? expf(z[c] - m) : 0.f;
                sum += e[c];
                zl = c == lab ? z[c] : zl;
            }
            loss_local -= zl - m - logf(sum);
            const float inv = 1.f / sum;
#pragma unroll
            for (int c = 0; c < 4; ++c) dz[c] = c < a.classes ? (e[c] * inv - (c == lab ? 1.f : 0.f)) * invP : 0.f;
        }
        if (g == 0) *reinterpret_cast<uint2v *>(dzs + px * 16) = uint2v{pack16x2<DT>(dz[0], dz[1]), pack16x2<DT>(dz[2], dz[3])};
#pragma unroll
        for (int c = 0; c < 4; ++c) dz[c] = __shfl(dz[c], l16, 64);
        // dh = (W2^T dz) where h > 0, rounded to the storage type; dx = W1^T dh
        unsigned dhb[HT][2];
#pragma unroll
        for (int t = 0; t < HT; ++t) {
            floatx4 v = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (c >= a.classes) break;                      // uniform
                const floatx4 w = *reinterpret_cast<const floatx4 *>(w2c + c * (HT * 16) + t * 16 + 4 * g);
                v += w * dz[c];
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] = hacc[t][r] > 0.f ? v[r] : 0.f;
            dhb[t][0] = pack16x2<DT>(v[0], v[1]);
            dhb[t][1] = pack16x2<DT>(v[2], v[3]);
            *reinterpret_cast<uint2v *>(dhs + px * PH + (2 * t + (g >> 1)) * 16 + (g & 1) * 8) = uint2v{dhb[t][0], dhb[t][1]};
        }
        if (a.dx != nullptr) {
            floatx4 dxa[NT1];
#pragma unroll
            for (int nt = 0; nt < NT1; ++nt) dxa[nt] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int pr = 0; pr < HP; ++pr) {
                const bool two = 2 * pr + 1 < HT;
                const uint4v dv = uint4v{dhb[2 * pr][0], dhb[2 * pr][1], two ? dhb[2 * pr + 1 < HT ? 2 * pr + 1 : 0][0] : 0u,
                                         two ? dhb[2 * pr + 1 < HT ? 2 * pr + 1 : 0][1] : 0u};
#pragma unroll
                for (int nt = 0; nt < NT1; ++nt) dxa[nt] = mfma32<DT>(w1t[(nt * HP + pr) * 64 + lane], dv, dxa[nt]);
            }
            // lane (g, l16) holds input maps 16 nt + 4g .. + 3 of its pixel: half an octet
            char *dxp = static_cast<char *>(a.dx);
#pragma unroll
            for (int nt = 0; nt < NT1; ++nt) {
                const int o8 = 2 * nt + (g >> 1);
                if (inside && o8 < c8)
                    *reinterpret_cast<uint2v *>(dxp + ((img * c8 + o8) * plane + pix) * 16 + (g & 1) * 8) =
                        uint2v{pack16x2<DT>(dxa[nt][0], dxa[nt][1]), pack16x2<DT>(dxa[nt][2], dxa[nt][3])};
            }
        }
        __syncthreads();                                        // the tiles of all 64 pixels are in LDS

        // ---- 2. weight gradients: contraction over the 64 pixels (two K steps of 32) ------------------------------
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            uint4v bx[NT1];
#pragma unroll
            for (int nt = 0; nt < NT1; ++nt) bx[nt] = read_frag(xs, off_x[nt] + ks * 32 * PX, off_x[nt] + (ks * 32 + 4) * PX);
            const uint4v adz = read_frag(hs, off_dz + ks * 32 * dz_step, off_dz + (ks * 32 + 4) * dz_step);
#pragma unroll
            for (int s = 0; s < SLOTS; ++s) {
                if (wave + 4 * s >= HT) break;                  // uniform
                const uint4v adh = read_frag(dhs, off_h[s] + ks * 32 * PH, off_h[s] + (ks * 32 + 4) * PH);
                const uint4v bh = read_frag(hs, off_h[s] + ks * 32 * PH, off_h[s] + (ks * 32 + 4) * PH);
#pragma unroll
                for (int nt = 0; nt < NT1; ++nt) acc1[s][nt] = mfma32<DT>(adh, bx[nt], acc1[s][nt]);
                accb1[s] = mfma32<DT>(adh, ones, accb1[s]);
                acc2[s] = mfma32<DT>(adz, bh, acc2[s]);
            }
            if (wave == 0) accb2 = mfma32<DT>(adz, ones, accb2);
        }
        __syncthreads();                                        // ... and read: the next block may overwrite them
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) bv[ks] = nx[ks];
    }

    // ---- this workgroup's sums -----------------------------------------------------------------------------------
    float *copy = a.scratch + (long)blockIdx.x * copy_floats_of(HT, NT1);
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        const int t = wave + 4 * s;
        if (t >= HT) break;
#pragma unroll
        for (int nt = 0; nt < NT1; ++nt) *reinterpret_cast<floatx4 *>(copy + ((t * NT1 + nt) * 64 + lane) * 4) = acc1[s][nt];
        *reinterpret_cast<floatx4 *>(copy + HT * NT1 * 256 + (t * 64 + lane) * 4) = acc2[s];
        if (l16 == 0) *reinterpret_cast<floatx4 *>(copy + HT * NT1 * 256 + HT * 256 + t * 16 + 4 * g) = accb1[s];   // every column holds the same sums
    }
    if (wave == 0 && l16 == 0) *reinterpret_cast<floatx4 *>(copy + HT * NT1 * 256 + HT * 256 + HT * 16 + 4 * g) = accb2;
    for (int off = 32; off > 0; off >>= 1) loss_local += __shfl_down(loss_local, off, 64);
    if (lane == 0) red[wave] = loss_local;
    __syncthreads();
    if (tid == 0) copy[HT * NT1 * 256 + HT * 256 + HT * 16 + 16] = (red[0] + red[1]) + (red[2] + red[3]);
}

// Sums the workgroups' copies element by element (fixed order) and scatters: dW1[h][c], dW2[class][h], db1, db2, loss.
__global__ void __launch_bounds__(256) head_train_reduce_kernel(HeadTrainArgs a, int copies, int HT, int NT1, int copy_floats)
{
    __shared__ float sh[4][64];
    __shared__ long cnt[4];
    const int e64 = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int e = (int)blockIdx.x * 64 + e64;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    if (e < copy_floats) {
        const float *src = a.scratch + e;
        int cp = w;
        for (; cp + 12 < copies; cp += 16) {
            s0 += src[(long)(cp + 0) * copy_floats];
            s1 += src[(long)(cp + 4) * copy_floats];
            s2 += src[(long)(cp + 8) * copy_floats];
            s3 += src[(long)(cp + 12) * copy_floats];
        }
        for (; cp < copies; cp += 4) s0 += src[(long)cp * copy_floats];
    }
    sh[w][e64] = (s0 + s1) + (s2 + s3);
    {
        long local = 0;
        for (int q = threadIdx.x; q < a.ncounts; q += blockDim.x) local += a.counts[q];
        for (int off = 32; off > 0; off >>= 1) local += __shfl_down(local, off, 64);
        if (e64 == 0) cnt[w] = local;
    }
    __syncthreads();
    if (w != 0 || e >= copy_floats) return;
    const float v = (sh[0][e64] + sh[1][e64]) + (sh[2][e64] + sh[3][e64]);
    const int n1 = HT * NT1 * 256, n2 = n1 + HT * 256, n3 = n2 + HT * 16, n4 = n3 + 16;
    if (e < n1) {               // ((t * NT1 + nt) * 64 + lane) * 4 + r: hidden map 16 t + 4 g + r, input map 16 nt + l16
        const int r = e & 3, ln = (e >> 2) & 63, tn = e >> 8, nt = tn % NT1, t = tn / NT1;
        const int h = 16 * t + 4 * (ln >> 4) + r, c = 16 * nt + (ln & 15);
        if (h < a.hidden && c < a.c_in) a.dw1[(long)h * a.c_in + c] = v;
    } else if (e < n2) {        // (t * 64 + lane) * 4 + r: class 4 g + r, hidden map 16 t + l16
        const int q = e - n1, r = q & 3, ln = (q >> 2) & 63, t = q >> 8;
        const int cls = 4 * (ln >> 4) + r, h = 16 * t + (ln & 15);
        if (cls < a.classes && h < a.hidden) a.dw2[(long)cls * a.hidden + h] = v;
    } else if (e < n3) {
        const int h = e - n2;
        if (h < a.hidden && a.db1) a.db1[h] = v;
    } else if (e < n4) {
        const int cls = e - n3;
        if (cls < a.classes && a.db2) a.db2[cls] = v;
    } else if (e == n4) {
        const long kept = cnt[0] + cnt[1] + cnt[2] + cnt[3];
        *a.loss = v / (float)(kept > 0 ? kept : 1);
    }
}

size_t smem_bytes(int HT, int KSTEPS, int NT1)
{
    const int HP = (HT + 1) / 2;
    return (size_t)(HT * KSTEPS * 64 + HP * 64 + NT1 * HP * 64) * 16 + (size_t)(4 * HT * 16 + HT * 16 + 4 + 8) * 4 +
           (size_t)HB_PIX * (2 * (HT * 32 + 16) + (KSTEPS * 64 + 16) + 16) + 16;
}

template <int DT, int HT, int KSTEPS, int NT1>
hipError_t launch_t(const HeadTrainArgs &a, int blocks, hipStream_t stream)
{
    const size_t smem = smem_bytes(HT, KSTEPS, NT1);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&head_train_bwd_h_kernel<DT, HT, KSTEPS, NT1>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((head_train_bwd_h_kernel<DT, HT, KSTEPS, NT1>), dim3(blocks), dim3(HB_THREADS), smem, stream, a);
    return hipGetLastError();
}

template <int DT, int HT>
hipError_t launch_ht(const HeadTrainArgs &a, int nt1, int blocks, hipStream_t stream)
{
    switch (nt1) {
    case 1: return launch_t<DT, HT, 1, 1>(a, blocks, stream);
    case 2: return launch_t<DT, HT, 1, 2>(a, blocks, stream);
    case 3: return launch_t<DT, HT, 2, 3>(a, blocks, stream);
    default: return hipErrorInvalidValue;
    }
}

int tiles_of(int hidden)
{
    const int t = (hidden + 15) / 16;
    return t <= 4 ? 4 : t <= 8 ? 8 : 13;
}

}  // namespace

// Which heads this kernel takes: 16-bit storage, at most 48 input maps, 208 hidden maps and 4 classes
bool head_train_supported(int dtype, int c_in, int hidden, int classes)
{
    return (dtype == 1 || dtype == 2) && c_in >= 1 && c_in <= 48 && hidden >= 1 && hidden <= 208 && classes >= 1 && classes <= 4 &&
           head_supported(dtype, c_in, hidden, classes);
}

// floats of scratch: one copy of the sums for each of up to 512 workgroups
size_t head_train_scratch_floats(int c_in, int hidden)
{
    return (size_t)512 * copy_floats_of(tiles_of(hidden), (c_in + 15) / 16);
}

// labels: [n][plane]; counts: ncounts partial counts of the labelled pixels (launch_label_count); scratch: scratch_floats floats
hipError_t launch_head_train_bwd(HeadTrainArgs a, size_t scratch_floats, hipStream_t stream)
{
    if (!head_train_supported(a.dtype, a.c_in, a.hidden, a.classes) || a.n < 1 || a.plane < 1) return hipErrorInvalidValue;
    const int HT = tiles_of(a.hidden), NT1 = (a.c_in + 15) / 16, cf = copy_floats_of(HT, NT1);
    if ((a.c_in + 7) / 8 > (NT1 == 3 ? 8 : 4)) return hipErrorInvalidValue;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    const long nblocks = ((long)a.n * a.plane + HB_PIX - 1) / HB_PIX;
    long blocks = cus;
    if (blocks > nblocks) blocks = nblocks;
    if (blocks > (long)(scratch_floats / cf)) blocks = (long)(scratch_floats / cf);
    if (blocks < 1) return hipErrorInvalidValue;
    hipError_t e = hipErrorInvalidValue;
    if (a.dtype == 1) e = HT == 4 ? launch_ht<1, 4>(a, NT1, (int)blocks, stream) : HT == 8 ? launch_ht<1, 8>(a, NT1, (int)blocks, stream) : launch_ht<1, 13>(a, NT1, (int)blocks, stream);
    else e = HT == 4 ? launch_ht<2, 4>(a, NT1, (int)blocks, stream) : HT == 8 ? launch_ht<2, 8>(a, NT1, (int)blocks, stream) : launch_ht<2, 13>(a, NT1, (int)blocks, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(head_train_reduce_kernel, dim3((cf + 63) / 64), dim3(256), 0, stream, a, (int)blocks, HT, NT1, cf);
    return hipGetLastError();
}

}  // namespace sk
