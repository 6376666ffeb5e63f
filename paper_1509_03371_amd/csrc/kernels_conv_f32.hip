// Implicit-GEMM SK (dilated) convolution for fp32 activations on gfx950, MFMA 16x16x4 fp32.
//
// GEMM view (paper, Section 5.5): M = f_out, N = output pixels, K = f_in*k*k.  Unlike the
// paper's im2col + SGEMM there is no column buffer: a workgroup stages the dilated input tile it
// needs in LDS and forms the K index (c, i, j) by address arithmetic.
//
// Tiling.  A workgroup (4 waves) owns R = 4*RW output rows that lie d apart (one row phase of the
// kernel stride d) and 64 consecutive columns.  Because the rows are d apart, the k kernel rows of
// all R output rows fall on only R + k - 1 input rows, whatever d is, so the staged tile is
// (R + k - 1) x (64 + (k-1)*d) samples per input map instead of (R + (k-1)*d) rows.  Rows are
// separate lines in memory anyway, so taking every d-th row costs no coalescing.
// Input maps are consumed four at a time (K chunk = 4*k*k); the matching slice of the packed
// weights is staged beside the tile.
//
// MFMA operand roles: A = weights (16 output maps x 4 K values), B = input (4 K values x 16
// pixels), D = 16 maps x 16 pixels.  Lane l supplies A[m = l%16][kk = l/16] and
// B[kk = l/16][pixel = l%16] and receives D[m = 4*(l/16) + r][pixel = l%16], r = 0..3, so each
// store instruction writes 64-byte runs of consecutive pixels of one map.
#include <type_traits>

#include "sk_kernels.h"

namespace sk {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int CONV_TX = 64;   // output columns per workgroup
constexpr int CONV_CC = 4;    // input maps per K chunk

// Epilogue shared by the kernels below: bias, ReLU, optional ReLU-derivative mask, predicated store.
// acc[rw][xt][nt][r] belongs to output map o_first + 16*nt + r, row oy_first + rw*d, column
// ox_first + 16*xt.  The vector memory counter is one in-order queue for loads and stores, so a
// load awaited between stores makes that wait cover every store before it.  The bias is therefore
// fetched in one batch and awaited once; the store loop without a mask then contains no load at
// all, and the masked variant fetches the masks of a whole pixel tile before its first store.
template <int NT, int RW, int XN = 4>
__device__ __forceinline__ void store_outputs(const ConvF32Args &a, floatx4 (&acc)[RW][4][NT], int b, int o_first,
                                              int oy_first, int d, int ox_first)
{
    float bia[NT][4];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) bia[nt][r4] = 0.f;
    if (a.bias) {                                       // uniform branch; the vector holds n_pad entries
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int o = o_first + nt * 16 + r4;
                bia[nt][r4] = a.bias[o < a.n_pad ? o : a.n_pad - 1];
            }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                 // vmcnt(0): the bias is in registers from here on
    __builtin_amdgcn_sched_barrier(0);
    const long oplane = (long)a.OH * a.OW;
    // mode 0: plain store; 1: ReLU-derivative mask; 2: the value already in y is added before bias and ReLU
    auto store_tiles = [&](auto mode) {
        constexpr int MODE = decltype(mode)::value;
#pragma unroll
        for (int rw = 0; rw < RW; ++rw) {
            const int oy = oy_first + rw * d;
            if (oy >= a.Ho) continue;
            const long rowbase = (((long)b * a.out_maps + a.o_off + o_first) * a.OH + (long)oy * a.oy_mul + a.oy_off) * a.OW + a.ox_off;
#pragma unroll
            for (int xt = 0; xt < XN; ++xt) {
                const int ox = ox_first + xt * 16;
                if (ox >= a.Wo) continue;
                const long pbase = rowbase + (long)ox * a.ox_mul;
                float mk[NT][4];
                if constexpr (MODE != 0) {
                    const float *side = MODE == 1 ? a.mask : a.y;
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                        for (int r4 = 0; r4 < 4; ++r4) {
                            // maps beyond c_out are never stored; their mask address is clamped to
                            // map 0 of the same pixel so that the load stays inside the tensor
                            const int oo = nt * 16 + r4;
                            mk[nt][r4] = side[pbase + (o_first + oo < a.c_out ? oo : -o_first) * oplane];
                        }
                }
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        const int oo = nt * 16 + r4;
                        if (o_first + oo >= a.c_out) continue;
                        float v = acc[rw][xt][nt][r4] + bia[nt][r4];
                        if constexpr (MODE == 2) v += mk[nt][r4];
                        if (a.relu) v = v > 0.f ? v : 0.f;
                        if constexpr (MODE == 1)
                            if (!(mk[nt][r4] > 0.f)) v = 0.f;
                        a.y[pbase + oo * oplane] = v;
                    }
            }
        }
    };
    // the four taps of an up-convolution stacked as GEMM maps: each 16-map tile belongs to one tap, which
    // moves its maps back by tap*tap_maps and its pixels to the tap's place in the 2x2 block (no mask here)
    auto store_taps = [&]() {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int o0 = o_first + nt * 16;
            const int tap = o0 / a.tap_maps, om = o0 - tap * a.tap_maps;
#pragma unroll
            for (int rw = 0; rw < RW; ++rw) {
                const int oy = oy_first + rw * d;
                if (oy >= a.Ho) continue;
                const long rowbase = (((long)b * a.out_maps + a.o_off + om) * a.OH + (long)oy * a.oy_mul + (tap >> 1)) * a.OW + (tap & 1);
#pragma unroll
                for (int xt = 0; xt < XN; ++xt) {
                    const int ox = ox_first + xt * 16;
                    if (ox >= a.Wo) continue;
                    const long pbase = rowbase + (long)ox * a.ox_mul;
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        if (o0 + r4 >= a.c_out) continue;
                        float v = acc[rw][xt][nt][r4] + bia[nt][r4];
                        if (a.relu) v = v > 0.f ? v : 0.f;
                        a.y[pbase + r4 * oplane] = v;
                    }
                }
            }
        }
    };
    if (a.tap_maps > 0) store_taps();
    else if (a.mask) store_tiles(std::integral_constant<int, 1>{});
    else if (a.accumulate) store_tiles(std::integral_constant<int, 2>{});
    else store_tiles(std::integral_constant<int, 0>{});
}

template <int NT, int RW>
__global__ __launch_bounds__(256) void conv_f32_kernel(ConvF32Args a, int tiles_hi, int tiles_lo,
                                                       int rem, int nblocks)
{
    extern __shared__ float smem[];
    constexpr int R = 4 * RW, WN = NT * 16;
    const int k = a.k, d = a.d, kk2 = k * k;
    const int RR = R + k - 1, PW = CONV_TX + (k - 1) * d, PITCH = PW;
    const int KC = CONV_CC * kk2;
    float *xs = smem;
    float *ws = xs + CONV_CC * RR * PITCH;
    int *koff = reinterpret_cast<int *>(ws + KC * WN);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l16 = lane & 15, g = lane >> 4;

    // blockIdx.y enumerates (row phase py, row tile ty): phases below `rem` have tiles_hi tiles
    int py, ty;
    {
        const int by = blockIdx.y;
        if (by < rem * tiles_hi) {
            py = by / tiles_hi;
            ty = by - py * tiles_hi;
        } else {
            const int b2 = by - rem * tiles_hi;
            py = rem + b2 / tiles_lo;
            ty = b2 % tiles_lo;
        }
    }
    const int b = blockIdx.z / nblocks, nb = blockIdx.z - b * nblocks;
    const int x0 = blockIdx.x * CONV_TX;

    for (int q = tid; q < KC; q += 256) {
        const int c = q / kk2, r = q - c * kk2;
        const int i = r / k, j = r - i * k;
        koff[q] = (c * RR + i) * PITCH + j * d;
    }

    floatx4 acc[RW][4][NT];
#pragma unroll
    for (int rw = 0; rw < RW; ++rw)
#pragma unroll
        for (int xt = 0; xt < 4; ++xt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[rw][xt][nt] = floatx4{0.f, 0.f, 0.f, 0.f};

    const long plane = (long)a.H * a.W;
    const float *xb = a.x + (long)b * (a.x_bstride ? a.x_bstride : (long)a.c_in * plane);
    const int c_pad = (a.c_in + CONV_CC - 1) / CONV_CC * CONV_CC;

    for (int c0 = 0; c0 < c_pad; c0 += CONV_CC) {
        __syncthreads();
        // stage the input tile: tile row t of map c holds input row py + d*(ty*R + t) - in_off
        for (int rowid = wave; rowid < CONV_CC * RR; rowid += 4) {
            const int cl = rowid / RR, t = rowid - cl * RR;
            const int c = c0 + cl;
            const int gy = py + d * (ty * R + t) - a.in_off;
            const bool rowok = (c < a.c_in) && gy >= 0 && gy < a.H;
            const float *src = xb + (long)c * plane + (long)gy * a.W;
            float *dst = xs + rowid * PITCH;
            for (int xc = lane; xc < PW; xc += 64) {
                const int gx = x0 + xc - a.in_off;
                float v = 0.f;
                if (rowok && gx >= 0 && gx < a.W) v = src[gx];
                dst[xc] = v;
            }
        }
        // stage the weight slice: K rows [c0*k*k, +KC), map columns [nb*WN, +WN)
        for (int q = tid; q < KC * WN; q += 256) {
            const int r = q / WN, cn = q - r * WN;
            const int col = nb * WN + cn;
            ws[q] = (col < a.n_pad) ? a.wp[(long)(c0 * kk2 + r) * a.n_pad + col] : 0.f;
        }
        __syncthreads();

        for (int kk = 0; kk < KC; kk += 4) {
            const int ko = koff[kk + g];
            float av[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) av[nt] = ws[(kk + g) * WN + nt * 16 + l16];
#pragma unroll
            for (int rw = 0; rw < RW; ++rw) {
                const float *xrow = xs + ko + (wave * RW + rw) * PITCH + l16;
#pragma unroll
                for (int xt = 0; xt < 4; ++xt) {
                    const float bv = xrow[xt * 16];
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        acc[rw][xt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[nt], bv, acc[rw][xt][nt], 0, 0, 0);
                }
            }
        }
    }

    store_outputs<NT, RW>(a, acc, b, nb * WN + 4 * g, py + d * (ty * R + wave * RW), d, x0 + l16);
}

template <int NT, int RW>
static hipError_t launch_conv_f32_t(const ConvF32Args &a, hipStream_t stream)
{
    constexpr int R = 4 * RW, WN = NT * 16;
    const int k = a.k, d = a.d;
    if (a.grp_maps != 0) return hipErrorInvalidValue;       // grouped input maps: only the kernels below
    const int RR = R + k - 1, PW = CONV_TX + (k - 1) * d;
    const int KC = CONV_CC * k * k;
    const size_t smem = sizeof(float) * ((size_t)CONV_CC * RR * PW + (size_t)KC * WN) + sizeof(int) * KC;
    if (smem > 150 * 1024) return hipErrorInvalidValue;
    static bool attr_set = false;
    if (smem > 48 * 1024 && !attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_f32_kernel<NT, RW>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    // row phases: phase py has ceil((Ho - py)/d) rows
    const int q = a.Ho / d, rem = a.Ho % d;
    const int tiles_hi = (q + 1 + R - 1) / R, tiles_lo = (q + R - 1) / R;
    const int gy = rem * tiles_hi + (d - rem) * tiles_lo;
    const int nblocks = (a.n_pad / 16 + NT - 1) / NT;
    dim3 grid((a.Wo + CONV_TX - 1) / CONV_TX, gy, a.n * nblocks);
    if (grid.x == 0 || gy <= 0 || grid.z == 0 || gy > 65535 || grid.z > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL((conv_f32_kernel<NT, RW>), grid, dim3(256), smem, stream, a, tiles_hi,
                       tiles_lo > 0 ? tiles_lo : 1, rem, nblocks);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Specialisation for a compile-time kernel size KS with register prefetch: while the MFMA loop
// works on K chunk c, the global loads of chunk c+1 (input rows and weight slab) are already in
// flight; they are written to LDS after the loop.  Wave w stages input maps c0 + w, c0 + w + 4, ...
// of the chunk (CC/4 maps, RR rows each, NCG groups of 64 columns), so every count is a compile-time
// constant and the prefetched values stay in registers.
// XNT = 16-column groups of a tile that are multiplied and stored.  A launch covers the gx column tiles from
// bx0 on: the last column tile of a map whose width is no multiple of 64 can run as a launch of its own with
// XNT = 1 or 2 (a test inside the K loop breaks its schedule, and a second K loop inside one kernel costs the
// registers of a workgroup per CU: both measured).
template <int NT, int RW, int KS, int CC, int NCG, bool PADZ, int XNT = 4>
__global__ __launch_bounds__(256) void conv_f32_pf_kernel(ConvF32Args a, int tiles_hi, int tiles_lo,
                                                          int rem, int nblocks, int gx, int gy, int total_tiles, int bx0)
{
    extern __shared__ float smem[];
    constexpr int R = 4 * RW, WN = NT * 16, RR = R + KS - 1, KK2 = KS * KS, KC = CC * KK2, CPW = CC / 4;
    constexpr int WV4 = (KC * WN / 4 + 255) / 256;   // float4 weight loads per thread and chunk
    constexpr int PITCH = 64 * NCG;                  // floats per staged row; holds 64 + (KS-1)*d columns
    const int d = a.d;
    float *xs = smem;
    float *ws = xs + CC * RR * PITCH;

    // While other waves of a SIMD stream MFMAs, every other instruction a wave issues waits tens of
    // cycles for its turn, so the staging code below is kept to as few instructions as possible:
    // wave-uniform quantities (map, row, slab bases) are made scalar, whatever is the same for every
    // K chunk (per-lane column offsets, per-thread weight and LDS offsets) is computed once, and
    // LDS offsets that depend only on the K index are compile-time constants.
    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // LDS offset of K index (c, i, j) inside the staged tile for the K values lane group g supplies
    // in step s of a chunk: klane + kconst(s) when the k*k taps of a map fill whole steps, else a
    // per-lane table in registers.
    // KTAB (k > 4 with k*k a multiple of 4): the taps of a map still fill whole steps, but the four
    // taps of a step fall on different kernel rows and columns from step to step; the per-lane
    // offsets of one map's k*k/4 steps are kept in registers and the map adds a constant.
    constexpr bool KTAB = KS > 4 && KK2 % 4 == 0;
    constexpr bool KSPLIT = !KTAB && (KK2 % 4 == 0 || KK2 == 1);
    constexpr int SPM = KK2 / 4;                     // steps per input map (KTAB)
    int klane = 0;
    int kreg[(KSPLIT || KTAB) ? 1 : KC / 4];
    int ktab[KTAB ? SPM : 1];
    if constexpr (KK2 == 1) klane = g * RR * PITCH;
    else if constexpr (KTAB) {
#pragma unroll
        for (int sidx = 0; sidx < SPM; ++sidx) {
            const int q = 4 * sidx + g;
            const int i = q / KS, j = q - i * KS;
            ktab[sidx] = i * PITCH + j * d;
        }
    } else if constexpr (KSPLIT) klane = (g / KS) * PITCH + (g % KS) * d;
    else {
#pragma unroll
        for (int sidx = 0; sidx < KC / 4; ++sidx) {
            const int q = 4 * sidx + g;
            const int c = q / KK2, r = q - c * KK2;
            const int i = r / KS, j = r - i * KS;
            kreg[sidx] = (c * RR + i) * PITCH + j * d;
        }
    }
    auto kconst = [](int sidx) {
        if constexpr (KK2 == 1) return 4 * sidx * RR * PITCH;
        else return ((4 * sidx / KK2) * RR + (4 * sidx % KK2) / KS) * PITCH;
    };

    const int kthread = wave * RW * PITCH + l16;

    // Persistent workgroups: the grid holds as many workgroups as fit on the GPU at once and each
    // walks over several tiles; a tail of tiles then runs on workgroups that are spread over all CUs
    // instead of as a second, mostly empty wave of fresh workgroups.
    // Workgroup w runs on XCD w % 8 (round-robin dispatch), and each XCD has an L2 of its own, so
    // every XCD takes one contiguous eighth of the tile list: tiles that share input rows then share
    // an L2 instead of each XCD fetching every row.
    const int xcds = (gridDim.x & 7) == 0 ? 8 : 1;
    const int xcd = blockIdx.x % xcds, per_xcd = (total_tiles + xcds - 1) / xcds;
    for (int q = blockIdx.x / xcds; q < per_xcd; q += gridDim.x / xcds) {
    const int tile = xcd * per_xcd + q;
    if (tile >= total_tiles) break;
    const int bx = tile % gx, byz = tile / gx;
    const int by = byz % gy, bz = byz / gy;
    int py, ty;
    if (by < rem * tiles_hi) {
        py = by / tiles_hi;
        ty = by - py * tiles_hi;
    } else {
        const int b2 = by - rem * tiles_hi;
        py = rem + b2 / tiles_lo;
        ty = b2 % tiles_lo;
    }
    const int b = bz / nblocks, nb = bz - b * nblocks;
    const int x0 = (bx0 + bx) * CONV_TX;

    floatx4 acc[RW][4][NT];
#pragma unroll
    for (int rw = 0; rw < RW; ++rw)
#pragma unroll
        for (int xt = 0; xt < 4; ++xt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[rw][xt][nt] = floatx4{0.f, 0.f, 0.f, 0.f};

    const long plane = (long)a.H * a.W;
    const float *xb = a.x + (long)b * (a.x_bstride ? a.x_bstride : (long)a.c_in * plane);
    const int nchunks = (a.c_in + CC - 1) / CC;
    const int gy0 = py + d * (ty * R) - a.in_off;       // input row of tile row 0
    const int gx0 = x0 - a.in_off + lane;                // input column of this lane, column group 0

    float xr[CPW][RR][NCG];
    floatx4 wr[WV4];

    // Loads are unconditional (addresses clamped into the tensor) so that they can stay in flight
    // across the MFMA loop.  With zero padding (PADZ: the transposed convolution of the backward
    // pass) what lies outside the image is replaced by zero when the registers are written to LDS.
    // Without it (in_off = 0) a clamped address can only feed outputs that are never stored, and a
    // clamped map index meets zero weights; activations are finite by contract.
    unsigned coff[NCG];        // byte offset of this lane's column inside a row
    bool colok[NCG];
#pragma unroll
    for (int cg = 0; cg < NCG; ++cg) {
        const int gx = gx0 + 64 * cg;
        colok[cg] = gx >= 0 && gx < a.W;
        coff[cg] = 4u * (unsigned)(gx < 0 ? 0 : (gx >= a.W ? a.W - 1 : gx));
    }
    int roff[RR];              // element offset of staged row t inside a map (wave-uniform)
    bool rowok[RR];
#pragma unroll
    for (int t = 0; t < RR; ++t) {
        const int gy = gy0 + t * d;
        rowok[t] = gy >= 0 && gy < a.H;
        roff[t] = (gy < 0 ? 0 : (gy >= a.H ? a.H - 1 : gy)) * a.W;
    }
    unsigned woff[WV4];        // byte offset of this thread's float4 inside a chunk's weight slab
#pragma unroll
    for (int u = 0; u < WV4; ++u) {
        int q = tid + 256 * u;               // float4 index inside the [KC][WN] slab
        q = q < KC * WN / 4 ? q : KC * WN / 4 - 1;
        const int r = q / (WN / 4), cn = (q - r * (WN / 4)) * 4;
        int col = nb * WN + cn;
        col = col < a.n_pad ? col : a.n_pad - 4;         // such columns belong to maps that are never stored
        woff[u] = 4u * (unsigned)(r * a.n_pad + col);
    }
    const int xs_thread = wave * RR * PITCH + lane;
    // input maps in groups of grp_maps (a multiple of CC) with grp_skip more floats between groups: chunks are
    // prefetched in order, so the skip that applies is kept as a running sum instead of a division per chunk
    const int grp_chunks = a.grp_maps > 0 ? a.grp_maps / CC : 0x7fffffff;
    int pf_left = grp_chunks;
    long pf_skip = 0;
    auto prefetch = [&](int chunk) {
#pragma unroll
        for (int cw = 0; cw < CPW; ++cw) {
            int c = chunk * CC + wave + 4 * cw;
            c = c < a.c_in ? c : a.c_in - 1;
            const float *src = xb + pf_skip + (long)c * plane;
#pragma unroll
            for (int t = 0; t < RR; ++t) {
                const char *row = reinterpret_cast<const char *>(src + roff[t]);
#pragma unroll
                for (int cg = 0; cg < NCG; ++cg) xr[cw][t][cg] = *reinterpret_cast<const float *>(row + coff[cg]);
            }
        }
        const char *slab = reinterpret_cast<const char *>(a.wp + (long)chunk * KC * a.n_pad);
#pragma unroll
        for (int u = 0; u < WV4; ++u) wr[u] = *reinterpret_cast<const floatx4 *>(slab + woff[u]);
        if (--pf_left == 0) {
            pf_left = grp_chunks;
            pf_skip += a.grp_skip;
        }
    };
    auto commit = [&](int chunk) {
#pragma unroll
        for (int cw = 0; cw < CPW; ++cw) {
            const bool cok = chunk * CC + wave + 4 * cw < a.c_in;
#pragma unroll
            for (int t = 0; t < RR; ++t)
#pragma unroll
                for (int cg = 0; cg < NCG; ++cg) {
                    float v = xr[cw][t][cg];
                    if constexpr (PADZ) v = (cok && rowok[t] && colok[cg]) ? v : 0.f;
                    xs[xs_thread + (4 * cw * RR + t) * PITCH + 64 * cg] = v;
                }
        }
#pragma unroll
        for (int u = 0; u < WV4; ++u) {
            const int q = tid + 256 * u;
            if (KC * WN / 4 % 256 == 0 || q < KC * WN / 4) *reinterpret_cast<floatx4 *>(ws + 4 * q) = wr[u];
        }
    };

    prefetch(0);
    for (int chunk = 0; chunk < nchunks; ++chunk) {
        __syncthreads();
        commit(chunk);
        __syncthreads();
        if (chunk + 1 < nchunks) prefetch(chunk + 1);
        // K loop with the operand fragments of step s+1 fetched from LDS while the MFMAs of step s run.
        // XN = 16-column groups of the tile that hold output columns: a tile at the right border of the
        // map (or a map narrower than 33 columns: the deep U-Net levels) multiplies only its first two.
        auto kloop = [&](auto xn) {
            constexpr int XN = decltype(xn)::value;
            float av[2][NT], bv[2][RW][XN];
            auto fetch = [&](int sidx, int buf) {
                int ko = klane + kthread + kconst(sidx);
                if constexpr (KTAB) ko = ktab[sidx % SPM] + kthread + (sidx / SPM) * RR * PITCH;
                else if constexpr (!KSPLIT) ko = kreg[sidx] + kthread;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) av[buf][nt] = ws[(4 * sidx + g) * WN + nt * 16 + l16];
#pragma unroll
                for (int rw = 0; rw < RW; ++rw)
#pragma unroll
                    for (int xt = 0; xt < XN; ++xt) bv[buf][rw][xt] = xs[ko + rw * PITCH + xt * 16];
            };
            fetch(0, 0);
#pragma unroll
            for (int sidx = 0; sidx < KC / 4; ++sidx) {
                const int cur = sidx & 1;
                if (sidx + 1 < KC / 4) fetch(sidx + 1, cur ^ 1);
                // the scheduler otherwise sinks each LDS read to just before its first use and the wave
                // waits out the LDS latency several times per step
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int rw = 0; rw < RW; ++rw)
#pragma unroll
                    for (int xt = 0; xt < XN; ++xt)
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt)
                            acc[rw][xt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[cur][nt], bv[cur][rw][xt], acc[rw][xt][nt], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        // (only the small-map instantiation carries both loops: a second copy costs the large-map kernels
        // registers -- 153 -> 210, a workgroup less per CU)
        if constexpr (KS == 3 && CC == 16) {
            if (a.Wo - x0 <= 32) kloop(std::integral_constant<int, 2>{});
            else kloop(std::integral_constant<int, 4>{});
        } else {
            kloop(std::integral_constant<int, XNT>{});
        }
    }

    store_outputs<NT, RW, XNT>(a, acc, b, nb * WN + 4 * g, py + d * (ty * R + wave * RW), d, x0 + l16);
    }
}

// one launch over the gxl column tiles from bx0 on
template <int NT, int RW, int KS, int CC, int NCG, bool PADZ, int XNT>
static hipError_t launch_conv_f32_pf_part(const ConvF32Args &a, size_t smem, int tiles_hi, int tiles_lo, int rem, int nblocks, int gxl,
                                          int gy, int bx0, hipStream_t stream)
{
    static bool attr_set = false;
    if (smem > 48 * 1024 && !attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_f32_pf_kernel<NT, RW, KS, CC, NCG, PADZ, XNT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const long total = (long)gxl * gy * a.n * nblocks;
    if (gxl <= 0 || gy <= 0 || total <= 0 || total > 0x7fffffffL) return hipErrorInvalidValue;
    static int slots = 0;                  // workgroups of this kernel that are resident at once
    if (slots == 0) {
        int dev = 0, cus = 0, per_cu = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e == hipSuccess)
            e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, conv_f32_pf_kernel<NT, RW, KS, CC, NCG, PADZ, XNT>, 256, smem);
        if (e != hipSuccess) return e;
        slots = cus * (per_cu > 0 ? per_cu : 1);
    }
    const int blocks = (int)(total < slots ? total : slots);
    hipLaunchKernelGGL((conv_f32_pf_kernel<NT, RW, KS, CC, NCG, PADZ, XNT>), dim3(blocks), dim3(256), smem, stream, a, tiles_hi,
                       tiles_lo > 0 ? tiles_lo : 1, rem, nblocks, gxl, gy, (int)total, bx0);
    return hipGetLastError();
}

template <int NT, int RW, int KS, int CC, int NCG, bool PADZ>
static hipError_t launch_conv_f32_pf_z(const ConvF32Args &a, hipStream_t stream)
{
    constexpr int R = 4 * RW, WN = NT * 16, RR = R + KS - 1, KC = CC * KS * KS, PITCH = 64 * NCG;
    if (CONV_TX + (KS - 1) * a.d > PITCH) return hipErrorInvalidValue;
    if (a.grp_maps != 0 && (a.grp_maps < 0 || a.grp_maps % CC != 0 || a.c_in % a.grp_maps != 0 || a.grp_skip < 0)) return hipErrorInvalidValue;
    if ((long)a.H * a.W >= (1L << 29)) return hipErrorInvalidValue;     // 32-bit byte offsets inside a map
    if ((long)KC * a.n_pad >= (1L << 29)) return hipErrorInvalidValue;  // and inside a weight slab
    const size_t smem = sizeof(float) * ((size_t)CC * RR * PITCH + (size_t)KC * WN);
    if (smem > 150 * 1024) return hipErrorInvalidValue;
    const int q = a.Ho / a.d, rem = a.Ho % a.d;
    const int tiles_hi = (q + 1 + R - 1) / R, tiles_lo = (q + R - 1) / R;
    const int gy = rem * tiles_hi + (a.d - rem) * tiles_lo;
    const int nblocks = (a.n_pad / 16 + NT - 1) / NT;
    const int gx = (a.Wo + CONV_TX - 1) / CONV_TX;
    // The last column tile of a map whose width is no multiple of 64 holds output columns in only some of its
    // four 16-column groups.  Where that column alone has enough tiles to fill the GPU several times (batches of
    // slices of a 3-D volume, many-map layers), it runs as a launch of its own that multiplies one or two groups.
    if constexpr ((KS == 3 && CC == 4) || KS == 8) {
        const int groups = (a.Wo - (gx - 1) * CONV_TX + 15) / 16;
        const long column = (long)gy * a.n * nblocks;
        if (gx >= 2 && groups <= 2 && column >= 512) {
            hipError_t e = launch_conv_f32_pf_part<NT, RW, KS, CC, NCG, PADZ, 4>(a, smem, tiles_hi, tiles_lo, rem, nblocks, gx - 1, gy, 0, stream);
            if (e != hipSuccess) return e;
            if (groups == 1) return launch_conv_f32_pf_part<NT, RW, KS, CC, NCG, PADZ, 1>(a, smem, tiles_hi, tiles_lo, rem, nblocks, 1, gy, gx - 1, stream);
            return launch_conv_f32_pf_part<NT, RW, KS, CC, NCG, PADZ, 2>(a, smem, tiles_hi, tiles_lo, rem, nblocks, 1, gy, gx - 1, stream);
        }
    }
    return launch_conv_f32_pf_part<NT, RW, KS, CC, NCG, PADZ, 4>(a, smem, tiles_hi, tiles_lo, rem, nblocks, gx, gy, 0, stream);
}

template <int NT, int RW, int KS, int CC, int NCG>
static hipError_t launch_conv_f32_pf_t(const ConvF32Args &a, hipStream_t stream)
{
    if (a.in_off != 0) return launch_conv_f32_pf_z<NT, RW, KS, CC, NCG, true>(a, stream);
    return launch_conv_f32_pf_z<NT, RW, KS, CC, NCG, false>(a, stream);
}

// Workgroup tiles of a launch with NT map tiles per workgroup and 4*RW rows per tile.  A layer with
// fewer tiles than about three per CU leaves CUs idle; the dispatch below then trades operand reuse
// for parallelism (fewer maps per workgroup, fewer rows per tile).
constexpr long CONV_FEW_TILES = 768;
static long conv_f32_tiles(const ConvF32Args &a, int nt, int rw)
{
    const long gx = (a.Wo + CONV_TX - 1) / CONV_TX;
    const long gy = (long)a.d * ((a.Ho / a.d + 4 * rw) / (4 * rw));       // row phases x row tiles, rounded up
    const long nblocks = (a.n_pad / 16 + nt - 1) / nt;
    return gx * gy * a.n * nblocks;
}

template <int NT>
static hipError_t launch_conv_f32_nt(const ConvF32Args &a, hipStream_t stream)
{
    const int halo = (a.k - 1) * a.d;
    if (a.k == 1) return launch_conv_f32_pf_t<NT, 2, 1, 16, 1>(a, stream);
    if (a.k == 3 && halo <= 64) {
        // small maps (the deep U-Net levels): 4-row tiles double the number of workgroups
        // ... and sixteen input maps per K chunk: these layers have hundreds of maps, and a chunk of four is
        // only 36 MFMAs per wave between two barriers (measured on the U-Net: 4.89 -> 4.69 ms)
        if (conv_f32_tiles(a, NT, 2) < CONV_FEW_TILES) return launch_conv_f32_pf_t<NT, 1, 3, 16, 2>(a, stream);
        return launch_conv_f32_pf_t<NT, 2, 3, 4, 2>(a, stream);
    }
    if (a.k == 4 && halo <= 64) {
        // 4-row tiles: twice as many workgroups as with 8 rows, which balances the 256 CUs better
        // at 512^2 (measured: 0.24 ms instead of 0.33 ms per 48->48 layer)
        return launch_conv_f32_pf_t<NT, 1, 4, 4, 2>(a, stream);
    }
    // the large kernels of the USK-Net (6x6 at d = 1, 8x8 at d = 8) and of the paper's SK-Net (10x10 at
    // d = 8, a 73-pixel window: three column groups, forward only); one chunk of four maps holds
    // 4*k*k K values and its weight slab fills most of the LDS, so one workgroup per CU
    if (a.k == 6 && halo <= 64) return launch_conv_f32_pf_t<NT, 2, 6, 4, 2>(a, stream);        // forward and data gradient (USK-Net training)
    if (a.k == 8 && halo <= 64) return launch_conv_f32_pf_t<NT, 1, 8, 4, 2>(a, stream);
    if (a.k == 10 && halo <= 128 && a.in_off == 0) return launch_conv_f32_pf_z<NT, 1, 10, 4, 3, false>(a, stream);
    return launch_conv_f32_t<NT, 2>(a, stream);
}

// ------------------------------------------------------------------------------------------------
// One input map (the first layer of the benchmark nets): K = k*k is a single MFMA step or two, and
// the layer is bound by writing its output, so it runs on the vector ALU instead.  A thread owns PX
// output pixels (64 apart in the flattened [Ho*Wo] plane, so every load and store of a wave covers
// 64 consecutive pixels), keeps their k*k taps in registers and walks over the output maps four at a
// time; the weights sit in LDS and are read with wave-uniform addresses, four per instruction.
template <int KS, int PX>
__global__ __launch_bounds__(256) void conv_c1_f32_kernel(const float *__restrict__ x, const float *__restrict__ wp,
                                                          const float *__restrict__ bias, float *__restrict__ y, int H, int W,
                                                          int Ho, int Wo, int d, int c_out, int n_pad, int out_maps, int o_off, int relu)
{
    constexpr int KK = KS * KS;
    extern __shared__ float smem[];                 // [KK][n_pad] weights, then [n_pad] bias
    float *wl = smem, *bl = smem + KK * n_pad;
    for (int q = threadIdx.x; q < KK * n_pad; q += 256) wl[q] = wp[q];
    for (int q = threadIdx.x; q < n_pad; q += 256) bl[q] = bias ? bias[q] : 0.f;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, b = blockIdx.y;
    const long P = (long)Ho * Wo;
    const long base = ((long)blockIdx.x * 4 + wave) * 64 * PX + lane;
    const float *xin = x + (long)b * H * W;
    float tap[KK][PX];
#pragma unroll
    for (int p = 0; p < PX; ++p) {
        long q = base + 64 * p;
        q = q < P ? q : P - 1;
        const int oy = (int)(q / Wo), ox = (int)(q - (long)oy * Wo);
#pragma unroll
        for (int i = 0; i < KS; ++i)
#pragma unroll
            for (int j = 0; j < KS; ++j) tap[i * KS + j][p] = xin[(long)(oy + i * d) * W + ox + j * d];
    }
    __syncthreads();
    float *yb = y + ((long)b * out_maps + o_off) * P;
    unsigned qoff[PX];
    bool qok[PX];
#pragma unroll
    for (int p = 0; p < PX; ++p) {
        qok[p] = base + 64 * p < P;
        qoff[p] = qok[p] ? 4u * (unsigned)(base + 64 * p) : 0u;
    }
    // four output maps per trip: 4*PX accumulators next to the k*k*PX taps
#pragma unroll 1
    for (int o4 = 0; o4 < n_pad; o4 += 4) {
        if (o4 >= c_out) break;                                  // uniform
        floatx4 acc[PX];
        const floatx4 bv = *reinterpret_cast<const floatx4 *>(bl + o4);
#pragma unroll
        for (int p = 0; p < PX; ++p) acc[p] = bv;
#pragma unroll
        for (int t = 0; t < KK; ++t) {
            const floatx4 w = *reinterpret_cast<const floatx4 *>(wl + t * n_pad + o4);
#pragma unroll
            for (int p = 0; p < PX; ++p)
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[p][e] = fmaf(w[e], tap[t][p], acc[p][e]);
        }
        // scalar base of the map plus a 32-bit byte offset per lane (4*P < 2^32, checked by the launcher)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (o4 + e >= c_out) break;                          // uniform
            char *ymap = reinterpret_cast<char *>(yb + (long)(o4 + e) * P);
#pragma unroll
            for (int p = 0; p < PX; ++p) {
                const float v = relu ? fmaxf(acc[p][e], 0.f) : acc[p][e];
                if (qok[p]) *reinterpret_cast<float *>(ymap + qoff[p]) = v;
            }
        }
    }
}

template <int KS>
static hipError_t launch_conv_c1_f32(const ConvF32Args &a, hipStream_t stream)
{
    constexpr int PX = 4;
    const long P = (long)a.Ho * a.Wo;
    const long blocks = (P + 256 * PX - 1) / (256 * PX);
    if (blocks > 0x7fffffffL || a.n > 65535 || P >= (1L << 29)) return hipErrorInvalidValue;
    const size_t smem = sizeof(float) * ((size_t)KS * KS + 1) * a.n_pad;
    if (smem > 48 * 1024) return hipErrorInvalidValue;          // callers check c_out first
    hipLaunchKernelGGL((conv_c1_f32_kernel<KS, PX>), dim3((unsigned)blocks, a.n), dim3(256), smem, stream, a.x, a.wp, a.bias, a.y, a.H, a.W,
                       a.Ho, a.Wo, a.d, a.c_out, a.n_pad, a.out_maps, a.o_off, a.relu);
    return hipGetLastError();
}

// grp_maps is accepted for the kernel sizes with a prefetching specialisation when it is a multiple of the
// largest K chunk (16 maps)
bool conv_f32_groups_supported(int k, int d, int grp_maps)
{
    const int halo = (k - 1) * d;
    return grp_maps > 0 && grp_maps % 16 == 0 && (k == 1 || ((k == 3 || k == 4 || k == 6 || k == 8) && halo <= 64));
}

hipError_t launch_conv_f32(const ConvF32Args &a, hipStream_t stream)
{
    if (a.n_pad % 16 != 0 || a.c_out > a.n_pad || a.k < 1 || a.d < 1 || a.Ho < 1 || a.Wo < 1)
        return hipErrorInvalidValue;
    if (a.tap_maps != 0 && (a.tap_maps < 16 || a.tap_maps % 16 != 0 || a.c_out != 4 * a.tap_maps || a.mask || a.oy_mul != 2 || a.ox_mul != 2))
        return hipErrorInvalidValue;
    if (a.accumulate && (a.mask || a.tap_maps != 0)) return hipErrorInvalidValue;
    if (a.x_bstride < 0) return hipErrorInvalidValue;
    // a single input map, plain forward placement (contiguous NCHW output, no mask)
    if (a.c_in == 1 && a.in_off == 0 && !a.mask && !a.accumulate && a.x_bstride == 0 && a.grp_maps == 0 && a.OH == a.Ho && a.OW == a.Wo && a.oy_mul == 1 && a.ox_mul == 1 &&
        a.oy_off == 0 && a.ox_off == 0 && a.Ho == a.H - (a.k - 1) * a.d && a.Wo == a.W - (a.k - 1) * a.d && a.n_pad <= 512) {
        if (a.k == 3) return launch_conv_c1_f32<3>(a, stream);
        if (a.k == 4) return launch_conv_c1_f32<4>(a, stream);
    }
    const int tiles = a.n_pad / 16;
    if (tiles == 1) return launch_conv_f32_nt<1>(a, stream);
    if (tiles == 2) return launch_conv_f32_nt<2>(a, stream);
    const int pad3 = (tiles + 2) / 3 * 3, pad4 = (tiles + 3) / 4 * 4;
    const int nt_wide = pad3 < pad4 ? 3 : 4;
    // many maps on a small image: as few maps per workgroup as it takes to fill the GPU
    if (conv_f32_tiles(a, nt_wide, 1) < CONV_FEW_TILES) {
        if (conv_f32_tiles(a, 2, 1) >= CONV_FEW_TILES) return launch_conv_f32_nt<2>(a, stream);
        return launch_conv_f32_nt<1>(a, stream);
    }
    if (nt_wide == 3) return launch_conv_f32_nt<3>(a, stream);
    return launch_conv_f32_nt<4>(a, stream);
}

// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void pack_weights_f32_body(const float *w, float *wp, int c_out, int c_in, int k,
                                                      int flip_transpose, int rows, int n_pad)
{
    const long total = (long)rows * n_pad;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const int col = (int)(q % n_pad), row = (int)(q / n_pad);
        const int j = row % k, i = (row / k) % k, m = row / (k * k);   // m = input map of this GEMM
        float v = 0.f;
        if (!flip_transpose) {
            if (m < c_in && col < c_out) v = w[(((long)col * c_in + m) * k + i) * k + j];
        } else {
            if (m < c_out && col < c_in) v = w[(((long)m * c_in + col) * k + (k - 1 - i)) * k + (k - 1 - j)];
        }
        wp[q] = v;
    }
}

__global__ void pack_weights_f32_kernel(const float *w, float *wp, int c_out, int c_in, int k,
                                        int flip_transpose, int rows, int n_pad)
{
    pack_weights_f32_body(w, wp, c_out, c_in, k, flip_transpose, rows, n_pad);
}

// Packings of a 3-D kernel W3[c_out][C][k][k][k] (depth, row, column taps) for the 2-D convolution that treats
// depth taps as input maps; al runs over the len taps of the launch:
// flip_transpose = 0 (forward, taps a0 + al):       Wp[((al*C + c)*k + i)*k + j][o]     = W3[o][c][a0 + al][i][j]
// flip_transpose = 1 (data gradient: every axis flipped, map roles swapped; taps k-1-(a0 + al)):
//                                                   Wp[((al*c_out + o)*k + i)*k + j][c] = W3[o][c][k-1-a0-al][k-1-i][k-1-j]
// Rows and columns beyond the real extents are zero.
__global__ void pack_weights3d_f32_kernel(const float *w3, float *wp, int c_out, int C, int k, int a0, int len, int flip_transpose,
                                          int rows, int n_pad)
{
    const long total = (long)rows * n_pad;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        const int col = (int)(q % n_pad), row = (int)(q / n_pad);
        const int j = row % k, i = (row / k) % k, m = row / (k * k);
        float v = 0.f;
        if (!flip_transpose) {
            const int al = m / C, c = m - al * C;
            if (al < len && col < c_out) v = w3[((((long)col * C + c) * k + a0 + al) * k + i) * k + j];
        } else {
            const int al = m / c_out, o = m - al * c_out;
            if (al < len && col < C) v = w3[((((long)o * C + col) * k + (k - 1 - a0 - al)) * k + (k - 1 - i)) * k + (k - 1 - j)];
        }
        wp[q] = v;
    }
}

hipError_t launch_pack_weights3d_f32(const float *w3, float *wp, int c_out, int C, int k, int a0, int len, int flip_transpose, int rows,
                                     int n_pad, hipStream_t stream)
{
    const long total = (long)rows * n_pad;
    const int blocks = (int)((total + 255) / 256 < 1024 ? (total + 255) / 256 : 1024);
    hipLaunchKernelGGL(pack_weights3d_f32_kernel, dim3(blocks), dim3(256), 0, stream, w3, wp, c_out, C, k, a0, len, flip_transpose, rows,
                       n_pad);
    return hipGetLastError();
}

struct PackF32Jobs { PackF32Job job[BATCH_MAX]; };
__global__ void pack_weights_f32_batch_kernel(PackF32Jobs b)
{
    const PackF32Job &j = b.job[blockIdx.y];
    pack_weights_f32_body(j.w, j.wp, j.c_out, j.c_in, j.k, j.flip_transpose, j.rows, j.n_pad);
}

hipError_t launch_pack_weights_f32_batch(const PackF32Job *jobs, int n, hipStream_t stream)
{
    if (n < 1 || n > BATCH_MAX) return hipErrorInvalidValue;
    PackF32Jobs b;
    long most = 1;
    for (int t = 0; t < n; ++t) {
        b.job[t] = jobs[t];
        const long total = (long)jobs[t].rows * jobs[t].n_pad;
        most = total > most ? total : most;
    }
    const int blocks = (int)((most + 255) / 256 < 256 ? (most + 255) / 256 : 256);
    hipLaunchKernelGGL(pack_weights_f32_batch_kernel, dim3(blocks, n), dim3(256), 0, stream, b);
    return hipGetLastError();
}

hipError_t launch_pack_weights_f32(const float *w_oihw, float *wp, int c_out, int c_in, int k,
                                   int flip_transpose, int rows, int n_pad, hipStream_t stream)
{
    const long total = (long)rows * n_pad;
    const int blocks = (int)((total + 255) / 256 < 1024 ? (total + 255) / 256 : 1024);
    hipLaunchKernelGGL(pack_weights_f32_kernel, dim3(blocks), dim3(256), 0, stream, w_oihw, wp, c_out,
                       c_in, k, flip_transpose, rows, n_pad);
    return hipGetLastError();
}

}  // namespace sk
