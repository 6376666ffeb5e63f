// Weight and bias gradient of a 4x4 SK convolution from 16-bit octet-layout activations (gfx950), second form:
// rows streamed through an LDS ring, operands transposed by the LDS read itself.
//
//   dW[o][c][i][j] = sum_{b,y,x} dY[b,o,y,x] * X[b,c,y+i*d,x+j*d]        db[o] = sum dY[b,o,y,x]
//
// (the paper's forward GEMM, Section 5.5, transposed: M = f_out, N = f_in*k*k, reduction over all output pixels).
//
// The contraction runs over pixels, so an MFMA lane must supply 8 consecutive pixels of ONE map, while the octet
// layout keeps 8 maps of one pixel together.  gfx950 has an LDS read that transposes on the way out
// (ds_read_b64_tr_b16): in every group of 16 lanes, lane 4r + q names 4 consecutive 16-bit values (here: maps
// 4q..4q+3 of pixel r), and lane 4q + e receives element e of lanes q, 4 + q, 8 + q, 12 + q (here: map 4q + e at
// pixels 0..3).  Two such reads are one MFMA 16x16x32 operand fragment (16 maps x 32 pixels, lane group g
// pixels 8g..8g+7), whatever the alignment of the pixel offset -- so rows are staged exactly as they lie in
// memory, by global_load_lds, with no register staging and no scatter, and a tap column j is an offset of
// j*d pixels into the staged row.
//
// Work unit: a "walk" down one strip of 64 output columns along the rows of one phase of the kernel stride
// (rows py, py + d, py + 2d, ...).  Step s of a walk brings in input row rho = r0 + s and output-gradient row
// rho of that phase; the MFMAs of the step pair input row rho with the gradient rows rho, rho - 1, rho - 2,
// rho - 3 (tap rows i = 0..3), whose fragments stay in registers for the four steps they are needed.  So every
// input row is staged once per strip (not once per tap row), and the 4 x 3 gradient fragments are read once.
// A walk ends with three steps whose gradient rows are zeros, which also leaves the register window clean for
// the next walk.  Wave w of the eight takes tap column j = w % 4 and the 32-pixel half w / 4 of the strip:
// per step 3 input fragments (16 maps each) x 4 tap rows x 3 map tiles = 36 MFMAs for 18 LDS reads.
//
// The eight waves issue the loads themselves (a row pair is 15 loads of 1 KB at d = 8, at most two per wave and step),
// LA steps ahead into a ring of LA + 2 slots; steps are taken in pairs: a wave waits for its own loads of the pair
// (s_waitcnt vmcnt with the exact number of younger loads) and meets the others at one LDS-only barrier per pair.
//
// Each workgroup keeps a private dW in its accumulators (the two pixel halves are added through LDS at the
// end) and writes it in accumulator order; wgrad_rows_reduce_kernel sums the copies in a fixed order and
// scatters the 36864 sums to OIHW.
#include <algorithm>

#include "sk_kernels.h"

namespace sk {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
typedef unsigned int uint2v __attribute__((ext_vector_type(2)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8v __attribute__((ext_vector_type(8)));
typedef _Float16 halfx8v __attribute__((ext_vector_type(8)));

namespace {

constexpr int WR_TX = 64;        // output columns of a strip
constexpr int WR_DP = 68;        // LDS pitch (pixels) between the octets of a gradient row: octet o + 1 lands 16 banks further
constexpr int WR_GROUP = 4;      // steps between two barriers (2 or 4)
constexpr int WR_LA = 6;         // steps loaded ahead when a group starts (>= WR_GROUP)
constexpr int WR_SLOTS = WR_LA + WR_GROUP;
constexpr int WR_WAVES = 8;
constexpr int WR_MAXMT = 3, WR_MAXCT = 3;

struct WgradRowsArgs {
    const void *x, *dy, *zeros;
    float *scratch, *bias_part;
    int n, c_in, c_out, c8i, c8o, H, W, Ho, Wo, d;
    int slot_bytes;               // bytes of a ring slot
    int xstrips, nseg, rs, total_walks;
    int copy_floats;              // floats of one private copy
};

template <int DT> __device__ __forceinline__ floatx4 mfma32(uint4v a, uint4v b, floatx4 c);
template <> __device__ __forceinline__ floatx4 mfma32<1>(uint4v a, uint4v b, floatx4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8v, a), __builtin_bit_cast(bf16x8v, b), c, 0, 0, 0);
}
template <> __device__ __forceinline__ floatx4 mfma32<2>(uint4v a, uint4v b, floatx4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(halfx8v, a), __builtin_bit_cast(halfx8v, b), c, 0, 0, 0);
}

__device__ __forceinline__ void sync_lds() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

#define SK_VMW(n) case n: __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14)); break;
__device__ __forceinline__ void wait_vmcnt(int n)
{
    switch (n) {
        SK_VMW(0) SK_VMW(1) SK_VMW(2) SK_VMW(3) SK_VMW(4) SK_VMW(5) SK_VMW(6) SK_VMW(7)
        SK_VMW(8) SK_VMW(9) SK_VMW(10) SK_VMW(11) SK_VMW(12) SK_VMW(13) SK_VMW(14) SK_VMW(15)
        SK_VMW(16) SK_VMW(17) SK_VMW(18) SK_VMW(19) SK_VMW(20) SK_VMW(21) SK_VMW(22) SK_VMW(23)
        SK_VMW(24) SK_VMW(25) SK_VMW(26) SK_VMW(27) SK_VMW(28) SK_VMW(29) SK_VMW(30) SK_VMW(31)
    default: __builtin_amdgcn_s_waitcnt(0x0F70 | 15 | (3 << 14)); break;      // 63: as good as no wait
    }
}
#undef SK_VMW

// one operand fragment: 16 maps x 32 pixels, this lane's 8 pixels of its map (two transposing reads, 4 pixels each)
__device__ __forceinline__ uint4v read_frag(const char *lds_base, unsigned off_lo, unsigned off_hi)
{
    typedef short4v __attribute__((address_space(3))) *lds_s4;
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(lds_base + off_lo));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(lds_base + off_hi));
    const uint2v l2 = __builtin_bit_cast(uint2v, lo), h2 = __builtin_bit_cast(uint2v, hi);
    return uint4v{l2[0], l2[1], h2[0], h2[1]};
}

struct Walk {
    int b, x0, py, r0, rows;      // rows: gradient rows of this walk (it has rows + 3 steps), 0 = empty
};

template <int DT, int MT, int NCT>
__global__ __launch_bounds__(64 * WR_WAVES) void wgrad_rows_h_kernel(WgradRowsArgs a)
{
    extern __shared__ uint4v smem16[];
    char *lds = reinterpret_cast<char *>(smem16);
    const int tid = threadIdx.x, lane = tid & 63, g = lane >> 4, jl = lane & 15;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tapj = wave & 3, xh = wave >> 2;
    const int d = a.d;
    // A slot of the ring: the first 64 pixels of the input row of every octet (pitch WR_DP), the gradient row of
    // every octet (pitch WR_DP), then the 3d further pixels of the input row of every octet, packed (so that one
    // 64-lane load fills the tails of several octets; a tail alone would be a load with 3d active lanes)
    const int tw = 3 * d;                                      // pixels of a tail
    const int dy_base = a.c8i * WR_DP * 16, tail_base = (a.c8i + a.c8o) * WR_DP * 16;
    const int slot_bytes = a.slot_bytes;

    // this lane's read offsets inside a slot (lane 4r + q of a 16-lane group names pixel r, map quad q)
    const int rr = jl >> 2, q = jl & 3;
    const int pix = xh * 32 + 8 * g + rr;
    unsigned a_off[MT], b_off[NCT][2];
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        int o8 = 2 * m + (q >> 1);
        o8 = o8 < a.c8o ? o8 : a.c8o - 1;
        a_off[m] = (unsigned)(dy_base + (o8 * WR_DP + pix) * 16 + (q & 1) * 8);
    }
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        int o8 = 2 * ct + (q >> 1);
        o8 = o8 < a.c8i ? o8 : a.c8i - 1;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int P = pix + tapj * d + 4 * h;               // pixel of the staged input row
            b_off[ct][h] = (unsigned)((P < WR_TX ? (o8 * WR_DP + P) * 16 : tail_base + (o8 * tw + P - WR_TX) * 16) + (q & 1) * 8);
        }
    }

    // this workgroup's walks: a contiguous range of the list (segments of one strip and phase are neighbours)
    const int w_begin = (int)((long)a.total_walks * blockIdx.x / gridDim.x), w_end = (int)((long)a.total_walks * (blockIdx.x + 1) / gridDim.x);
    auto decode = [&](int t) {
        Walk w;
        const int seg = t % a.nseg;
        int rest = t / a.nseg;
        w.py = rest % d;
        rest /= d;
        w.x0 = (rest % a.xstrips) * WR_TX;
        w.b = rest / a.xstrips;
        const int rows_p = a.Ho > w.py ? (a.Ho - w.py + d - 1) / d : 0;
        w.r0 = seg * a.rs;
        int rows = rows_p - w.r0;
        rows = rows < 0 ? 0 : (rows > a.rs ? a.rs : rows);
        w.rows = rows;
        return w;
    };
    int total_steps = 0;
    for (int t = w_begin; t < w_end; ++t) {
        const Walk w = decode(t);
        total_steps += w.rows > 0 ? w.rows + 3 : 0;
    }

    // Loads of a step, 1 KB each: one per input octet (first 64 pixels), one per gradient octet, and the packed
    // tails; load number id goes to wave id % 8 (at most two per wave: 6 + 6 + 3 for 48 -> 48 maps at d = 8).  What a
    // wave's loads are never changes, so their kind, octet and LDS offset are fixed here.
    const int ntail = (a.c8i * tw + 63) / 64;
    const int nloads = a.c8i + a.c8o + ntail;
    const int my_loads = (nloads - wave + WR_WAVES - 1) / WR_WAVES;      // <= 2 (checked by the launcher)
    const char *xg = static_cast<const char *>(a.x), *dyg = static_cast<const char *>(a.dy), *zg = static_cast<const char *>(a.zeros);
    const long xplane = (long)a.H * a.W * 16, yplane = (long)a.Ho * a.Wo * 16;
    int kind[2], oct[2], ldst[2], tpx[2];                       // kind 0 input, 1 gradient, 2 tails; tpx: this lane's tail pixel
    long toff[2];                                                // tails: this lane's octet plane
    bool tact[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int id = wave + WR_WAVES * u;
        kind[u] = id < a.c8i ? 0 : (id < a.c8i + a.c8o ? 1 : 2);
        oct[u] = kind[u] == 0 ? id : id - a.c8i;
        ldst[u] = kind[u] == 0 ? oct[u] * WR_DP * 16 : (kind[u] == 1 ? dy_base + oct[u] * WR_DP * 16 : tail_base + (id - a.c8i - a.c8o) * 1024);
        const int L = (id - a.c8i - a.c8o) * 64 + lane;         // tails: packed pixel index
        const int o8 = kind[u] == 2 ? L / tw : 0;
        tact[u] = kind[u] == 2 && o8 < a.c8i;
        tpx[u] = WR_TX + L - o8 * tw;
        toff[u] = (long)(tact[u] ? o8 : 0) * xplane;
    }

    // The issue cursor: the walk whose rows are being loaded, the step inside it, and this lane's source address of
    // each of the wave's loads, which moves on by d rows per step; a new walk (every rows + 3 steps) sets them afresh.
    int it = w_begin, is = 0, irows = 0;
    const char *src[2] = {zg, zg};
    const long xstep = (long)d * a.W * 16, ystep = (long)d * a.Wo * 16;
    const char *zsrc = zg + lane * 16;
    bool yok[2] = {false, false};                               // gradient loads: this lane's column lies inside the gradient
    auto start_walk = [&]() {
        Walk w;
        w.rows = 0;
        while (it < w_end) {
            w = decode(it);
            if (w.rows > 0) break;
            ++it;
        }
        irows = w.rows;
        is = 0;
        if (irows == 0) return;
        const int gy = w.py + w.r0 * d;
        const char *yrow = dyg + ((long)w.b * a.c8o * a.Ho + gy) * (long)a.Wo * 16;
        const char *xrow = xg + ((long)w.b * a.c8i * a.H + gy) * (long)a.W * 16;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (kind[u] == 1) {
                const int gx = w.x0 + lane;
                yok[u] = gx < a.Wo;
                src[u] = yrow + oct[u] * yplane + (yok[u] ? gx : 0) * 16;
            } else {
                int gx = w.x0 + (kind[u] == 0 ? lane : tpx[u]);
                gx = gx < a.W ? gx : a.W - 1;
                src[u] = xrow + (kind[u] == 0 ? oct[u] * xplane : toff[u]) + gx * 16;
            }
        }
    };
    auto issue = [&](int slot) {
        char *dst = lds + slot * slot_bytes;
        const bool grad_row = is < irows;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (u >= my_loads) break;                           // uniform
            const char *p = src[u];
            if (kind[u] == 1) {
                p = (grad_row && yok[u]) ? p : zsrc;
                src[u] += ystep;
            } else {
                src[u] += xstep;
            }
            if (kind[u] != 2 || tact[u])
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)p,
                                                 (__attribute__((address_space(3))) void *)(dst + ldst[u]), 16, 0, 0);
        }
        if (++is == irows + 3) {
            ++it;
            start_walk();
        }
    };

    floatx4 acc[NCT][4][MT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int m = 0; m < MT; ++m) acc[ct][i][m] = floatx4{0.f, 0.f, 0.f, 0.f};
    floatx4 bacc = floatx4{0.f, 0.f, 0.f, 0.f};
    const unsigned one2 = DT == 1 ? 0x3F803F80u : 0x3C003C00u;  // two ones in the storage type
    const uint4v ones = uint4v{one2, one2, one2, one2};
    const bool sum_dy = a.bias_part != nullptr && tapj < MT;    // wave-uniform: tap column j sums map tile j

    uint4v awin[4][MT];                                          // gradient fragments of the last four rows
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int m = 0; m < MT; ++m) awin[u][m] = uint4v{0u, 0u, 0u, 0u};

    start_walk();
    int issued = 0;
    for (; issued < WR_LA && issued < total_steps; ++issued) issue(issued);
    int islot = issued % WR_SLOTS, cslot = 0;

    // Steps go in pairs: one wait and one barrier per two rows (the matrix unit idles while a SIMD's two waves sit at
    // a barrier and fetch their first fragments, so fewer, longer stretches between barriers are worth two ring slots).
    for (int step = 0; step < total_steps; step += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (step + u >= total_steps) break;                 // uniform
            if (u % WR_GROUP == 0) {
                // this wave's loads of the group have landed ...
                const int cur = step + u, group = total_steps - cur < WR_GROUP ? total_steps - cur : WR_GROUP;
                if (issued - cur == WR_LA) {
                    if (my_loads == 2) wait_vmcnt(2 * (WR_LA - WR_GROUP));
                    else if (my_loads == 1) wait_vmcnt(WR_LA - WR_GROUP);
                } else {
                    wait_vmcnt((issued - cur - group) * my_loads);
                }
                sync_lds();                                     // ... and everybody's; the slots of the group before are free
#pragma unroll
                for (int e = 0; e < WR_GROUP; ++e)
                    if (issued < total_steps) {
                        issue(islot);
                        ++issued;
                        islot = islot == WR_SLOTS - 1 ? 0 : islot + 1;
                    }
            }
            const char *slot = lds + cslot * slot_bytes;
            cslot = cslot == WR_SLOTS - 1 ? 0 : cslot + 1;
#pragma unroll
            for (int m = 0; m < MT; ++m) awin[u][m] = read_frag(slot, a_off[m], a_off[m] + 64);
            uint4v bf[NCT];
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) bf[ct] = read_frag(slot, b_off[ct][0], b_off[ct][1]);
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int m = 0; m < MT; ++m) acc[ct][i][m] = mfma32<DT>(awin[(u - i) & 3][m], bf[ct], acc[ct][i][m]);
            if (sum_dy) {
                uint4v aw = awin[u][0];
#pragma unroll
                for (int m = 1; m < MT; ++m) aw = tapj == m ? awin[u][m] : aw;
                bacc = mfma32<DT>(aw, ones, bacc);
            }
        }
    }

    // the two pixel halves: waves 4..7 hand their sums to waves 0..3 through LDS (one input-map tile at a time),
    // which add and write the private copy in accumulator order: [tap column][ct][tap row][map tile][lane][4]
    float *red = reinterpret_cast<float *>(lds);
    float *copy = a.scratch + (long)blockIdx.x * a.copy_floats;
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        __syncthreads();
        if (xh == 1) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int m = 0; m < MT; ++m)
                    *reinterpret_cast<floatx4 *>(red + (((tapj * 4 + i) * MT + m) * 64 + lane) * 4) = acc[ct][i][m];
        }
        __syncthreads();
        if (xh == 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int m = 0; m < MT; ++m) {
                    const floatx4 o = *reinterpret_cast<const floatx4 *>(red + (((tapj * 4 + i) * MT + m) * 64 + lane) * 4);
                    *reinterpret_cast<floatx4 *>(copy + ((((tapj * NCT + ct) * 4 + i) * MT + m) * 64 + lane) * 4) = acc[ct][i][m] + o;
                }
        }
    }
    if (a.bias_part != nullptr) {
        __syncthreads();
        if (xh == 1 && sum_dy) *reinterpret_cast<floatx4 *>(red + (tapj * 64 + lane) * 4) = bacc;
        __syncthreads();
        if (xh == 0 && sum_dy && jl == 0) {                     // every column of bacc holds the same sums
            const floatx4 o = *reinterpret_cast<const floatx4 *>(red + (tapj * 64 + lane) * 4);
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) a.bias_part[(long)blockIdx.x * (MT * 16) + tapj * 16 + 4 * g + r4] = bacc[r4] + o[r4];
        }
    }
}

// dW[o][c][i][j] = sum over the private copies (fixed order), db[o] = sum over the workgroups' bias partials.
// One thread per accumulator element: the copies are read as they were written, the 4-byte results are scattered.
__global__ void __launch_bounds__(256) wgrad_rows_reduce_kernel(const float *__restrict__ scratch, float *__restrict__ dw, int copies, int copy_floats,
                                                                int c_out, int c_in, int MT, int NCT, int dw_blocks,
                                                                const float *__restrict__ bias_part, float *__restrict__ db)
{
    __shared__ float sh[4][64];
    const int e64 = threadIdx.x & 63, w = threadIdx.x >> 6;
    if ((int)blockIdx.x >= dw_blocks) {
        const int o = ((int)blockIdx.x - dw_blocks) * 64 + e64;
        float v = 0.f;
        if (o < c_out)
            for (int cp = w; cp < copies; cp += 4) v += bias_part[(long)cp * (MT * 16) + o];
        sh[w][e64] = v;
        __syncthreads();
        if (w == 0 && o < c_out) db[o] = (sh[0][e64] + sh[1][e64]) + (sh[2][e64] + sh[3][e64]);
        return;
    }
    const int e = (int)blockIdx.x * 64 + e64;                   // element of a copy
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    if (e < copy_floats) {
        const float *src = scratch + e;
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
    __syncthreads();
    if (w == 0 && e < copy_floats) {
        // e = ((((j * NCT + ct) * 4 + i) * MT + m) * 64 + lane) * 4 + r4, lane = 16 g + l16: map o = 16 m + 4 g + r4, input map c = 16 ct + l16
        const int r4 = e & 3, ln = (e >> 2) & 63;
        int rest = e >> 8;
        const int m = rest % MT;
        rest /= MT;
        const int i = rest & 3;
        rest >>= 2;
        const int ct = rest % NCT, j = rest / NCT;
        const int o = 16 * m + 4 * (ln >> 4) + r4, c = 16 * ct + (ln & 15);
        if (o < c_out && c < c_in) dw[((long)o * c_in + c) * 16 + i * 4 + j] = (sh[0][e64] + sh[1][e64]) + (sh[2][e64] + sh[3][e64]);
    }
}

template <int DT, int MT, int NCT>
hipError_t launch_t(const WgradRowsArgs &a, size_t smem, int blocks, hipStream_t stream)
{
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&wgrad_rows_h_kernel<DT, MT, NCT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((wgrad_rows_h_kernel<DT, MT, NCT>), dim3(blocks), dim3(64 * WR_WAVES), smem, stream, a);
    return hipGetLastError();
}

template <int DT>
hipError_t launch_dt(const WgradRowsArgs &a, int MT, int NCT, size_t smem, int blocks, hipStream_t stream)
{
#define SK_WR_CASE(mt, nct) if (MT == mt && NCT == nct) return launch_t<DT, mt, nct>(a, smem, blocks, stream);
    SK_WR_CASE(1, 1) SK_WR_CASE(2, 1) SK_WR_CASE(3, 1)
    SK_WR_CASE(1, 2) SK_WR_CASE(2, 2) SK_WR_CASE(3, 2)
    SK_WR_CASE(1, 3) SK_WR_CASE(2, 3) SK_WR_CASE(3, 3)
#undef SK_WR_CASE
    return hipErrorInvalidValue;
}

}  // namespace

// Which gradients take this form: 16-bit storage, 4x4 kernel, at most 48 maps on either side, a staged row of at
// most 128 pixels, and a scratch buffer that holds at least one copy.
static size_t slot_bytes_of(int c8i, int c8o, int d)
{
    const int ntail = (c8i * 3 * d + 63) / 64;                  // whole 1 KB loads of packed tails
    return (size_t)((c8i + c8o) * WR_DP + ntail * 64) * 16;
}

bool wgrad_rows_h_supported(int c_in, int c_out, int k, int d)
{
    if (!(k == 4 && d >= 1 && 3 * d <= 64 && c_in >= 1 && c_in <= 16 * WR_MAXCT && c_out >= 1 && c_out <= 16 * WR_MAXMT)) return false;
    const int c8i = (c_in + 7) / 8, c8o = (c_out + 7) / 8;
    if (c8i + c8o + (c8i * 3 * d + 63) / 64 > 2 * WR_WAVES) return false;       // two loads per wave and step
    return slot_bytes_of(c8i, c8o, d) * WR_SLOTS <= 160 * 1024;
}

// one private copy and its bias partials for each of up to 512 workgroups
size_t wgrad_rows_h_scratch_floats(int c_in, int c_out)
{
    const size_t MT = (c_out + 15) / 16, NCT = (c_in + 15) / 16;
    return 512 * (16 * NCT * MT * 256 + MT * 16);
}

// scratch: scratch_floats floats (private copies, then the bias partials).  zeros: at least 1 KB of zeros.
hipError_t launch_wgrad_rows_h(const void *x, const void *dy, const void *zeros, float *dw, float *db, float *scratch, size_t scratch_floats,
                               int dtype, int n, int c_in, int H, int W, int c_out, int d, hipStream_t stream)
{
    if (!wgrad_rows_h_supported(c_in, c_out, 4, d) || !zeros || (dtype != 1 && dtype != 2)) return hipErrorInvalidValue;
    WgradRowsArgs a;
    a.x = x; a.dy = dy; a.zeros = zeros; a.scratch = scratch;
    a.n = n; a.c_in = c_in; a.c_out = c_out; a.c8i = (c_in + 7) / 8; a.c8o = (c_out + 7) / 8;
    a.H = H; a.W = W; a.Ho = H - 3 * d; a.Wo = W - 3 * d; a.d = d;
    if (a.Ho < 1 || a.Wo < 1 || n < 1) return hipErrorInvalidValue;
    const int MT = (c_out + 15) / 16, NCT = (c_in + 15) / 16;
    a.slot_bytes = (int)slot_bytes_of(a.c8i, a.c8o, d);
    a.copy_floats = 16 * NCT * MT * 256;
    const size_t bias_floats = (size_t)MT * 16;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    long blocks = cus;
    const long fit = (long)(scratch_floats / ((size_t)a.copy_floats + bias_floats));
    if (fit < 1) return hipErrorInvalidValue;
    if (blocks > fit) blocks = fit;
    // rows per walk: about one workgroup's share of all rows, so that the three extra steps of a walk stay a small part
    a.xstrips = (a.Wo + WR_TX - 1) / WR_TX;
    const long total_rows = (long)n * a.xstrips * a.Ho;
    long rs = (total_rows + blocks - 1) / blocks;
    rs = rs < 8 ? 8 : (rs > 128 ? 128 : rs);
    const int rows_p = (a.Ho + d - 1) / d;                      // rows of the longest phase
    a.nseg = (int)((rows_p + rs - 1) / rs);
    a.rs = (rows_p + a.nseg - 1) / a.nseg;                      // equal segments
    const long walks = (long)n * a.xstrips * d * a.nseg;
    if (walks > 0x7fffffffL) return hipErrorInvalidValue;
    a.total_walks = (int)walks;
    if (blocks > walks) blocks = walks;
    a.bias_part = db ? scratch + (size_t)blocks * a.copy_floats : nullptr;
    size_t smem = (size_t)a.slot_bytes * WR_SLOTS;
    const size_t red = (size_t)16 * MT * 64 * 16 + 4096;        // the hand-over of one input-map tile, the bias sums
    if (smem < red) smem = red;
    if (smem > 160 * 1024) return hipErrorInvalidValue;
    hipError_t e = dtype == 1 ? launch_dt<1>(a, MT, NCT, smem, (int)blocks, stream) : launch_dt<2>(a, MT, NCT, smem, (int)blocks, stream);
    if (e != hipSuccess) return e;
    const int dw_blocks = (a.copy_floats + 63) / 64, db_blocks = db ? (c_out + 63) / 64 : 0;
    hipLaunchKernelGGL(wgrad_rows_reduce_kernel, dim3(dw_blocks + db_blocks), dim3(256), 0, stream, scratch, dw, (int)blocks, a.copy_floats, c_out,
                       c_in, MT, NCT, dw_blocks, a.bias_part, db);
    return hipGetLastError();
}

}  // namespace sk
