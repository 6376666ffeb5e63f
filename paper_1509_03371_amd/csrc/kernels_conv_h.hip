// Implicit-GEMM SK (dilated) convolution for 16-bit activations (bf16 or fp16, fp32 accumulate) on
// gfx950, MFMA 16x16x32.
//
// Storage ("octet layout"): a tensor with C maps is [n][ceil(C/8)][H][W][8] 16-bit elements, so
// the 8 consecutive K values that one MFMA lane supplies are one aligned 16-byte load, and
// consecutive pixels are consecutive 16-byte units (coalesced in HBM, conflict-free in LDS).
// Maps beyond C inside the last octet are zero.
//
// GEMM view (paper, Section 5.5): M = f_out, N = output pixels, K = f_in*k*k; no column buffer.
// MFMA roles: A = weights (16 output maps x 32 K), B = input (32 K x 16 pixels); lane (g = l/16,
// l16 = l%16) supplies K values 8g..8g+7 and receives D[map 4g+r][pixel l16], r = 0..3: four
// consecutive maps of one pixel, i.e. half an octet, so lanes g = 2q and 2q+1 together write one
// 16-byte unit and 16 lanes write 256 contiguous bytes.
//
// How the 32 K values of one MFMA are chosen ("column step"):
//   MAP4 (k >= 4): the four lane groups take four consecutive kernel columns j = 4*cs + g of one input octet
//                  (ceil(k/4) column steps; columns j >= k carry zero weights and read the staged tile
//                  (k - 1) < j columns further right, which is why the tile is staged that wide).
//   otherwise   : the four lane groups take four input octets at one kernel column j.
// Either way a B fragment is tied to one INPUT row r of the staged tile and is reused for every
// kernel row i (output row y = r - i) and every output-map tile: the rows of a tile lie d apart
// (one row phase of the kernel stride), so tile row r + i is the input row of output row r, tap i.
// Per column step a wave reads R + k - 1 B fragments and k*MT A fragments from LDS for R*k*MT MFMAs.
//
// A workgroup is 8 waves and owns R output rows (d apart) x 128 columns (wave w: columns 16w..);
// the grid is persistent (one workgroup per CU), walks tiles in an XCD-aware order and keeps a
// two-stage LDS pipeline running across tile boundaries: while chunk q is multiplied, chunk q+1
// (next octets, or the first octets of the next tile) is in flight from HBM/L2 into registers.
#include "sk_kernels.h"

namespace sk {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
typedef unsigned int uint2v __attribute__((ext_vector_type(2)));

constexpr int CH_TX = 128;     // output columns per workgroup
constexpr int CH_WAVES = 8;
constexpr int CH_THREADS = 64 * CH_WAVES;
constexpr int CH_VU = 3;       // 64-unit column groups staged per row: tile width <= 192 units

template <int DT> struct H;    // DT = 1 bf16, 2 fp16
template <> struct H<1> {
    static __device__ __forceinline__ floatx4 mfma(uint4v a, uint4v b, floatx4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ unsigned short cvt(float f)
    {
        return __builtin_bit_cast(unsigned short, static_cast<__bf16>(f));
    }
    static __device__ __forceinline__ float up(unsigned short u) { return __uint_as_float((unsigned)u << 16); }
};
template <> struct H<2> {
    static __device__ __forceinline__ floatx4 mfma(uint4v a, uint4v b, floatx4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(halfx8, a), __builtin_bit_cast(halfx8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ unsigned short cvt(float f)
    {
        return __builtin_bit_cast(unsigned short, static_cast<_Float16>(f));
    }
    static __device__ __forceinline__ float up(unsigned short u) { return (float)__builtin_bit_cast(_Float16, u); }
};

// element-wise maximum of two pairs / two octets of unsigned 16-bit values (the order of non-negative bf16 and
// fp16 numbers is the unsigned order of their bit patterns)
__device__ __forceinline__ unsigned pk_max_u16(unsigned x, unsigned y)
{
    unsigned r;
    asm("v_pk_max_u16 %0, %1, %2" : "=v"(r) : "v"(x), "v"(y));
    return r;
}
__device__ __forceinline__ uint4v max_u16x8(uint4v x, uint4v y)
{
    return uint4v{pk_max_u16(x[0], y[0]), pk_max_u16(x[1], y[1]), pk_max_u16(x[2], y[2]), pk_max_u16(x[3], y[3])};
}

// positive (> 0) test on a 16-bit float bit pattern (both formats: sign bit clear, magnitude non-zero)
__device__ __forceinline__ bool pos16(unsigned v) { return (v & 0x8000u) == 0 && (v & 0x7fffu) != 0; }

// Workgroup barrier for LDS traffic only: wait for this wave's own LDS operations, then s_barrier.
// (__syncthreads() also drains every outstanding global load and store of the wave, which would
// serialise the chunk pipelines below with HBM latency.)
__device__ __forceinline__ void block_sync_lds() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// s_waitcnt vmcnt(n) with n chosen at run time (the instruction takes an immediate): n in 0..63
#define SK_VMW(n) case n: __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14)); break;
__device__ __forceinline__ void wait_vmcnt_at_most(int n)
{
    switch (n) {
        SK_VMW(0) SK_VMW(1) SK_VMW(2) SK_VMW(3) SK_VMW(4) SK_VMW(5) SK_VMW(6) SK_VMW(7)
        SK_VMW(8) SK_VMW(9) SK_VMW(10) SK_VMW(11) SK_VMW(12) SK_VMW(13) SK_VMW(14) SK_VMW(15)
        SK_VMW(16) SK_VMW(17) SK_VMW(18) SK_VMW(19) SK_VMW(20) SK_VMW(21) SK_VMW(22) SK_VMW(23)
        SK_VMW(24) SK_VMW(25) SK_VMW(26) SK_VMW(27) SK_VMW(28) SK_VMW(29) SK_VMW(30) SK_VMW(31)
        SK_VMW(32) SK_VMW(33) SK_VMW(34) SK_VMW(35) SK_VMW(36) SK_VMW(37) SK_VMW(38) SK_VMW(39)
        SK_VMW(40) SK_VMW(41) SK_VMW(42) SK_VMW(43) SK_VMW(44) SK_VMW(45) SK_VMW(46) SK_VMW(47)
        SK_VMW(48) SK_VMW(49) SK_VMW(50) SK_VMW(51) SK_VMW(52) SK_VMW(53) SK_VMW(54) SK_VMW(55)
        SK_VMW(56) SK_VMW(57) SK_VMW(58) SK_VMW(59) SK_VMW(60) SK_VMW(61) SK_VMW(62)
    default: __builtin_amdgcn_s_waitcnt(0x0F70 | 15 | (3 << 14)); break;
    }
}
#undef SK_VMW

struct TilePos {
    int b, mg, py, ty, x0;
};

// XW: waves across a tile's columns (16 each); the other 8 / XW wave rows take R output rows each, so a tile is
// 16*XW columns x R*8/XW rows of one residue class: 128 x 4, 64 x 8 or 32 x 16 output pixels.  Squarer tiles stage less
// halo per output and waste less of a narrow or ragged map (a 28-wide map fills 22 % of a 128-column tile).
template <int DT, int KS, int MT, bool MAP4, int R, bool HAS_MASK, int VU = CH_VU, int XW = 8>
__global__ __launch_bounds__(CH_THREADS) void conv_h_kernel(ConvHArgs a)
{
    extern __shared__ uint4v lds[];
    constexpr int YW = CH_WAVES / XW, RT = R * YW, TX = 16 * XW;   // wave rows, output rows and columns of a tile
    constexpr int RR = RT + KS - 1;
    constexpr int OC = MAP4 ? 1 : 4;            // input octets per chunk
    constexpr int CS = MAP4 ? (KS + 3) / 4 : KS; // column steps per chunk
    constexpr int TAPW = MAP4 ? 4 * CS : KS;    // kernel columns the tile is staged for
    constexpr int ROWS = OC * RR;               // staged tile rows per chunk
    constexpr int RU = (ROWS + CH_WAVES - 1) / CH_WAVES;
    constexpr int WUNITS = CS * KS * MT * 64;   // 16-byte units of the weight slab of one chunk
    constexpr int WU = (WUNITS + CH_THREADS - 1) / CH_THREADS;

    const int d = a.d;
    const int PW = TX + (TAPW - 1) * d;         // tile width in 16-byte units
    const int tile_units = ROWS * PW;
    const int stage_units = tile_units + WUNITS;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l16 = lane & 15, g = lane >> 4;
    // this wave's 16 columns and R rows inside the tile (constants of the flat shape spelled out for the compiler)
    const int wcol = XW == CH_WAVES ? wave : wave % XW, wrow = XW == CH_WAVES ? 0 : wave / XW;

    // XCD-aware persistent schedule: workgroup ids go round-robin over the 8 XCDs, so XCD x takes
    // the x-th contiguous eighth of the tile list (neighbouring tiles share halo in that XCD's L2)
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, nslots = gridDim.x >> 3;
    const int t_begin = (int)((long)a.total_tiles * xcd / 8), t_end = (int)((long)a.total_tiles * (xcd + 1) / 8);

    auto decode = [&](int t) {
        TilePos p;
        const int xt = t % a.xtiles;
        int rest = t / a.xtiles;
        const int yt = rest % a.ytiles_total;
        rest /= a.ytiles_total;
        p.mg = rest % a.mgroups;
        p.b = rest / a.mgroups;
        if (yt < a.rem * a.tiles_hi) {
            p.py = yt / a.tiles_hi;
            p.ty = yt - p.py * a.tiles_hi;
        } else {
            const int y2 = yt - a.rem * a.tiles_hi;
            p.py = a.rem + y2 / a.tiles_lo;
            p.ty = y2 % a.tiles_lo;
        }
        p.x0 = xt * TX;
        return p;
    };

    // chunk-invariant column bookkeeping of this lane
    const long plane = (long)a.H * a.W;
    // octet plane of input octet o of image b (slices of a volume as images: overlapping images, octets in groups)
    const int xb8 = a.xb8 > 0 ? a.xb8 : a.c8_in;
    auto in_plane = [&](int b, int o) -> long { return (long)b * xb8 + o + (a.grp8 > 0 ? (o / a.grp8) * a.skip8 : 0); };
    uint4v xr[RU][VU];
    uint4v wr[WU];

    auto prefetch = [&](const TilePos &p, int ch) {
        const int gy0 = p.py + d * (p.ty * RT) - a.in_off;
        const int gx0 = p.x0 - a.in_off;
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            int rid = wave + CH_WAVES * u;
            rid = rid < ROWS ? rid : ROWS - 1;
            const int oc = rid / RR, r = rid - oc * RR;
            int o = ch * OC + oc;
            o = o < a.c8_in ? o : a.c8_in - 1;
            int gy = gy0 + r * d;
            gy = gy < 0 ? 0 : (gy >= a.H ? a.H - 1 : gy);
            const uint4v *row = reinterpret_cast<const uint4v *>(a.x) + in_plane(p.b, o) * plane + (long)gy * a.W;
#pragma unroll
            for (int v = 0; v < VU; ++v) {
                int gx = gx0 + lane + 64 * v;
                gx = gx < 0 ? 0 : (gx >= a.W ? a.W - 1 : gx);
                xr[u][v] = row[gx];
            }
        }
        const uint4v *wsrc = reinterpret_cast<const uint4v *>(a.wp) + ((long)p.mg * a.nchunks + ch) * WUNITS;
#pragma unroll
        for (int u = 0; u < WU; ++u) {
            int q = tid + CH_THREADS * u;
            q = q < WUNITS ? q : WUNITS - 1;
            wr[u] = wsrc[q];
        }
    };
    auto commit = [&](const TilePos &p, int ch, int buf) {
        uint4v *dst = lds + buf * stage_units;
        const int gy0 = p.py + d * (p.ty * RT) - a.in_off;
        const int gx0 = p.x0 - a.in_off;
        const uint4v zero = uint4v{0u, 0u, 0u, 0u};
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            const int rid = wave + CH_WAVES * u;
            if (rid < ROWS) {
                const int oc = rid / RR, r = rid - oc * RR;
                const int gy = gy0 + r * d;
                const bool rowok = (ch * OC + oc < a.c8_in) && gy >= 0 && gy < a.H;
#pragma unroll
                for (int v = 0; v < VU; ++v) {
                    const int xc = lane + 64 * v, gx = gx0 + xc;
                    if (xc < PW) dst[rid * PW + xc] = (rowok && gx >= 0 && gx < a.W) ? xr[u][v] : zero;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < WU; ++u) {
            const int q = tid + CH_THREADS * u;
            if (q < WUNITS) dst[tile_units + q] = wr[u];
        }
    };

    floatx4 acc[R][MT];
#pragma unroll
    for (int y = 0; y < R; ++y)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[y][mt] = floatx4{0.f, 0.f, 0.f, 0.f};

    auto compute = [&](int buf) {
        const uint4v *tile = lds + buf * stage_units;
        const uint4v *wl = tile + tile_units;
#pragma unroll
        for (int cs = 0; cs < CS; ++cs) {
            uint4v afr[KS][MT];
#pragma unroll
            for (int i = 0; i < KS; ++i)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) afr[i][mt] = wl[((cs * KS + i) * MT + mt) * 64 + lane];
            const int off = (MAP4 ? (4 * cs + g) * d : g * RR * PW + cs * d) + wrow * R * PW + wcol * 16 + l16;
            uint4v bcur = tile[off];
#pragma unroll
            for (int r = 0; r < R + KS - 1; ++r) {              // the input rows under this wave's R output rows
                uint4v bnext = bcur;
                if (r + 1 < R + KS - 1) bnext = tile[off + (r + 1) * PW];
#pragma unroll
                for (int i = 0; i < KS; ++i) {
                    const int y = r - i;
                    if (y >= 0 && y < R) {
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) acc[y][mt] = H<DT>::mfma(afr[i][mt], bcur, acc[y][mt]);
                    }
                }
                bcur = bnext;
            }
        }
    };

    // bias of every output map, staged in LDS once (zeros when the layer has none)
    float *bias_lds = reinterpret_cast<float *>(lds + 2 * stage_units);
    for (int q = tid; q < a.mgroups * MT * 16; q += CH_THREADS) bias_lds[q] = (a.bias && q < a.m_tiles * 16) ? a.bias[q] : 0.f;

    // Epilogue of one tile.  Everything it reads comes first (bias from LDS, the optional ReLU mask
    // in one batch of global loads) and the stores follow without any load in between: on this ISA a
    // wait for a load also waits for every store issued before it, which would serialise the stores.
    auto epilogue = [&](const TilePos &p) {
        const int ox = p.x0 + wcol * 16 + l16;
        const bool colok = ox < a.Wo;
        const int oxc = colok ? ox : 0;
        float bia[MT][4];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) bia[mt][r4] = bias_lds[(p.mg * MT + mt) * 16 + 4 * g + r4];
        // byte offsets inside one image of the destination stay below 2^31 (checked by the launcher)
        const int row_bytes = a.OW * (a.out_f32 ? 4 : 16);
        const int plane_bytes = a.OH * row_bytes;
        char *ybase;      // this lane's column in map (or octet) 0, row 0 of image b
        if (a.out_f32)
            ybase = reinterpret_cast<char *>(a.y) + (long)p.b * a.c_out * plane_bytes + (long)(oxc * a.ox_mul + a.ox_off) * 4;
        else
            ybase = reinterpret_cast<char *>(a.y) + ((long)p.b * a.c8_out_total + a.o8_off) * plane_bytes +
                    (long)(oxc * a.ox_mul + a.ox_off) * 16 + (g & 1) * 8;
        uint2v mk[HAS_MASK ? R : 1][HAS_MASK ? MT : 1];
        if constexpr (HAS_MASK) {
            const char *mbase = reinterpret_cast<const char *>(a.mask) + (ybase - reinterpret_cast<char *>(a.y));
#pragma unroll
            for (int y = 0; y < R; ++y) {
                int oy = p.py + d * (p.ty * RT + wrow * R + y);
                oy = oy < a.Ho ? oy : a.Ho - 1;
                const int yoff = (oy * a.oy_mul + a.oy_off) * row_bytes;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    int o8 = (p.mg * MT + mt) * 2 + (g >> 1);
                    o8 = o8 < a.c8_out ? o8 : a.c8_out - 1;
                    mk[y][mt] = *reinterpret_cast<const uint2v *>(mbase + o8 * plane_bytes + yoff);
                }
            }
        }
#pragma unroll
        for (int y = 0; y < R; ++y) {
            const int oy = p.py + d * (p.ty * RT + wrow * R + y);
            const int yoff = (oy * a.oy_mul + a.oy_off) * row_bytes;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int mtile = p.mg * MT + mt;
                floatx4 v = acc[y][mt];
                acc[y][mt] = floatx4{0.f, 0.f, 0.f, 0.f};
                if (oy >= a.Ho || mtile >= a.m_tiles) continue;      // uniform
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    v[r4] += bia[mt][r4];
                    if (a.relu) v[r4] = fmaxf(v[r4], 0.f);
                }
                if (a.out_f32) {
                    const int o = mtile * 16 + 4 * g;
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4)
                        if (colok && o + r4 < a.c_out) *reinterpret_cast<float *>(ybase + (o + r4) * plane_bytes + yoff) = v[r4];
                } else {
                    const int o8 = mtile * 2 + (g >> 1);
                    // stacked up-convolution taps: the tile's tap moves its octets back and its pixel inside the 2x2 block
                    int tapadj = 0;
                    if (a.tap_maps > 0) {
                        const int tap = mtile * 16 / a.tap_maps;
                        tapadj = (tap >> 1) * row_bytes + (tap & 1) * 16 - tap * (a.tap_maps / 8) * plane_bytes;
                    }
                    unsigned short h[4];
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) h[r4] = H<DT>::cvt(v[r4]);
                    uint2v packed = uint2v{(unsigned)h[0] | ((unsigned)h[1] << 16), (unsigned)h[2] | ((unsigned)h[3] << 16)};
                    if constexpr (HAS_MASK) {
                        const uint2v m = mk[y][mt];
                        unsigned lo = packed[0], hi = packed[1];
                        if (!pos16(m[0] & 0xffffu)) lo &= 0xffff0000u;
                        if (!pos16(m[0] >> 16)) lo &= 0x0000ffffu;
                        if (!pos16(m[1] & 0xffffu)) hi &= 0xffff0000u;
                        if (!pos16(m[1] >> 16)) hi &= 0x0000ffffu;
                        packed = uint2v{lo, hi};
                    }
                    if (colok && o8 < a.c8_out) *reinterpret_cast<uint2v *>(ybase + o8 * plane_bytes + yoff + tapadj) = packed;
                }
            }
        }
    };

    int t = t_begin + slot;
    if (t >= t_end) return;
    // The chunk pipeline is written without data-dependent branches around the loads and the LDS
    // writes (the last chunk is peeled off), so that the compiler's wait-count bookkeeping stays
    // exact and the prefetched loads really remain in flight across the MFMA block.
    const int my_tiles = (t_end - t + nslots - 1) / nslots;
    const int total_chunks = my_tiles * a.nchunks;
    TilePos cur = decode(t), nxt = cur;
    int ch = 0, buf = 0;
    prefetch(cur, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);
    commit(cur, 0, 0);
    block_sync_lds();
    for (int q = 0; q + 1 < total_chunks; ++q) {
        int nch = ch + 1;
        if (nch == a.nchunks) {
            nch = 0;
            t += nslots;
            nxt = decode(t);
        }
        prefetch(nxt, nch);
        // a wave whose 16 columns lie right of the image (narrow maps: most waves of a 128-column tile) multiplies nothing
        if (__builtin_amdgcn_readfirstlane((int)(cur.x0 + (XW == CH_WAVES ? (tid >> 6) : (tid >> 6) % XW) * 16 < a.Wo))) compute(buf);
        // Explicit vmcnt(0): every prefetched register is consumed below, some only by part of the
        // lanes; without it the compiler would carry "load pending" states around the loop and wait
        // (also for the stores of the epilogue) before it reuses those registers.  The stores of the
        // previous tile are older than these loads and long finished, and the epilogue's own stores
        // come after the commit, so nothing here waits for a store in flight.
        __builtin_amdgcn_sched_barrier(0);   // keep the wait behind the MFMA block
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __builtin_amdgcn_sched_barrier(0);
        commit(nxt, nch, buf ^ 1);
        if (nch == 0) epilogue(cur);
        block_sync_lds();
        ch = nch;
        cur = nxt;
        buf ^= 1;
    }
    if (__builtin_amdgcn_readfirstlane((int)(cur.x0 + (XW == CH_WAVES ? (tid >> 6) : (tid >> 6) % XW) * 16 < a.Wo))) compute(buf);
    epilogue(cur);
}

// ------------------------------------------------------------------------------------------------
// Ring variant: the same tiling and MFMA schedule, but the input tile and the weight slab of a
// chunk go from HBM/L2 straight into LDS (global_load_lds_dwordx4: lane l's 16 bytes land at
// base + 16*l, inactive lanes write nothing), into a ring of S stages.  No staging registers and no
// LDS-write instructions; the loads of the next S-1 chunks are in flight while one chunk is
// multiplied, which is what covers the HBM latency (one chunk of look-ahead does not).
// What lies outside the image is read from a small zero buffer instead.
// NP > 0 adds NP producer waves to the eight that multiply: the producers issue every load (and
// wait for it), the others never touch the memory queue except for their tile's stores.  A load
// or store instruction can sit in that queue for hundreds of cycles when HBM is the limit, and a
// wave that waits there issues no MFMA; with the loads on waves of their own the multiplying waves
// lose that time only for their stores.
// VPOOL (with producer waves only): the layer's ReLU output is max-pooled over the kernel-stride neighbour
// BELOW before it is stored (the vertical half of the SK pool k = 2 at this layer's d; rows of a tile lie d
// apart, so that neighbour is the wave's own next accumulator row).  Tiles are then walked down the columns
// of the tile grid in contiguous runs, and the last row of a tile is carried in registers to the next one.
// a.hd > 0 (producer waves only): the input was written by such a launch with kernel stride hd; the producer
// waves finish its pool on the way in, tile[x] = max(in[x], in[x + hd]), in registers between the global loads and
// the LDS write.
template <int DT, int KS, int MT, bool MAP4, int R, bool HAS_MASK, int S, bool RESW, int NP, bool VPOOL = false>
__global__ __launch_bounds__(CH_THREADS + 64 * NP) void conv_h_ring_kernel(ConvHArgs a)
{
    static_assert(!VPOOL || (NP > 0 && !HAS_MASK && (R % 2 == 0)), "vertical pooling runs in the producer-wave variant");
    constexpr int NTHREADS = CH_THREADS + 64 * NP;
    constexpr int LW = NP > 0 ? NP : CH_WAVES;                 // waves that share a chunk's loads
    extern __shared__ uint4v lds[];
    constexpr int RR = R + KS - 1;
    constexpr int OC = MAP4 ? 1 : 4;
    constexpr int CS = MAP4 ? 1 : KS;
    static_assert(!MAP4 || KS == 4 || KS == 3, "the ring kernel maps the four lane groups to four kernel columns (a 3x3 kernel leaves the fourth zero)");
    constexpr int ROWS = OC * RR;
    constexpr int RU = (ROWS + LW - 1) / LW;
    constexpr int WUNITS = CS * KS * MT * 64;
    constexpr int WBLK = WUNITS / 64;                          // 1 KB fragments in the weight slab
    constexpr int WL = (WBLK + LW - 1) / LW;
    constexpr int VUE = KS == 1 ? 2 : 3;                       // 64-unit column groups per staged row

    const int d = a.d;
    const int hd = NP > 0 ? a.hd : 0;                          // the input's pending horizontal pool distance
    // rows from one row tile to the next: R, or (VPOOL on a launch with few tiles per workgroup) R - 1, so that every
    // tile holds the row below its last pooled row itself and nothing is carried from tile to tile
    const int ypitch = VPOOL ? a.ypitch : R;
    const int PWL = CH_TX + (MAP4 ? 3 : KS - 1) * d;           // tile width the multiplication reads
    const int PW = PWL;                                        // staged row pitch
    const int tile_units = ROWS * PW;
    // RESW: the weights of every chunk stay in LDS for the whole kernel (one map group only) and the
    // ring stages hold input tiles only; otherwise each stage also carries its chunk's weight slab
    const int stage_units = tile_units + (RESW ? 0 : WUNITS);
    const int wres_units = RESW ? a.nchunks * WUNITS : 0;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), l16 = lane & 15, g = lane >> 4;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, nslots = gridDim.x >> 3;
    const int t_begin = (int)((long)a.total_tiles * xcd / 8), t_end = (int)((long)a.total_tiles * (xcd + 1) / 8);

    // (row phase, row tile) of every y-tile index, looked up instead of divided out per tile
    const uint4v *wres = lds + S * stage_units;
    float *bias_lds = reinterpret_cast<float *>(lds + S * stage_units + wres_units);
    int *ypos = reinterpret_cast<int *>(bias_lds + a.mgroups * MT * 16);
    if constexpr (RESW) {
        uint4v *wdst = lds + S * stage_units;
        const uint4v *wsrc_all = reinterpret_cast<const uint4v *>(a.wp);
        for (int q = tid; q < wres_units; q += NTHREADS) wdst[q] = wsrc_all[q];
    }
    for (int q = tid; q < a.mgroups * MT * 16; q += NTHREADS) bias_lds[q] = (a.bias && q < a.m_tiles * 16) ? a.bias[q] : 0.f;
    for (int yt = tid; yt < a.ytiles_total; yt += NTHREADS) {
        int py, ty;
        if (yt < a.rem * a.tiles_hi) {
            py = yt / a.tiles_hi;
            ty = yt - py * a.tiles_hi;
        } else {
            const int y2 = yt - a.rem * a.tiles_hi;
            py = a.rem + y2 / a.tiles_lo;
            ty = y2 % a.tiles_lo;
        }
        ypos[yt] = (py << 16) | ty;
    }

    // A tile cursor: index t split into (x tile, y tile, image*mgroups + mgroup); advancing by the
    // persistent stride nslots is three adds with carries (the split of nslots comes from the host)
    struct Cursor {
        int xt, yt, mb;
    };
    auto cursor_at = [&](int t) {
        Cursor c;
        if constexpr (VPOOL) {                       // y tiles fastest: consecutive tiles go down one column of tiles
            c.yt = t % a.ytiles_total;
            const int rest = t / a.ytiles_total;
            c.xt = rest % a.xtiles;
            c.mb = rest / a.xtiles;
        } else {
            c.xt = t % a.xtiles;
            const int rest = t / a.xtiles;
            c.yt = rest % a.ytiles_total;
            c.mb = rest / a.ytiles_total;
        }
        return c;
    };
    const int step_x = nslots % a.xtiles, step_y = (nslots / a.xtiles) % a.ytiles_total,
              step_mb = nslots / a.xtiles / a.ytiles_total;
    auto advance = [&](Cursor &c) {
        if constexpr (VPOOL) {                       // the next tile of a contiguous run
            int carry = ++c.yt >= a.ytiles_total;
            c.yt -= carry ? a.ytiles_total : 0;
            c.xt += carry;
            carry = c.xt >= a.xtiles;
            c.xt -= carry ? a.xtiles : 0;
            c.mb += carry;
            return;
        }
        c.xt += step_x;
        int carry = c.xt >= a.xtiles;
        c.xt -= carry ? a.xtiles : 0;
        c.yt += step_y + carry;
        carry = c.yt >= a.ytiles_total;
        c.yt -= carry ? a.ytiles_total : 0;
        c.mb += step_mb + carry;
    };
    auto position = [&](const Cursor &c) {
        TilePos p;
        const int yp = ypos[c.yt];
        p.py = yp >> 16;
        p.ty = yp & 0xffff;
        p.x0 = c.xt * CH_TX;
        if (a.mgroups == 1) {
            p.mg = 0;
            p.b = c.mb;
        } else {
            p.b = c.mb / a.mgroups;
            p.mg = c.mb - p.b * a.mgroups;
        }
        return p;
    };

    // loads this wave issues per chunk: its tile rows (wave, wave + 8, ...) times the column groups,
    // plus its 1 KB blocks of the weight slab
    // lw: this wave's index among the waves that issue loads (all eight, or the NP producers)
    const int lw = NP > 0 ? wave - CH_WAVES : wave;
    const int L = lw < 0 ? 0 : ((ROWS - lw + LW - 1) / LW) * VUE + (RESW ? 0 : (WBLK - lw + LW - 1) / LW);
    // Waves 4..7 share their SIMDs with waves 0..3.  The first four issue a chunk's loads before
    // they multiply, the last four after: while one wave of a SIMD sits in the memory pipeline's
    // queue, the other one keeps the matrix unit busy.
    const bool late_issue = wave >= CH_WAVES / 2;
    const int Wmem = a.W + hd;                                 // columns of an input row in memory
    const long plane_bytes_in = (long)a.H * Wmem * 16;
    const char *zeros = reinterpret_cast<const char *>(a.zeros);
    // octet plane of input octet o of image b (slices of a volume as images: overlapping images, octets in groups)
    const int xb8 = a.xb8 > 0 ? a.xb8 : a.c8_in;
    auto in_plane = [&](int b, int o) -> long { return (long)b * xb8 + o + (a.grp8 > 0 ? (o / a.grp8) * a.skip8 : 0); };

    // Loads of chunk `ch` of the tile at `p` into ring stage `st`.  Exactly L load instructions for
    // this wave, whatever the position (the pipeline counts them): a row or a 64-column group that lies
    // outside the image as a whole is read from the zero page; a group that straddles the image
    // border is loaded for the lanes inside and the lanes outside write their zeros themselves.
    // Inside the image the address is a scalar row base plus a per-lane 32-bit column offset.
    auto issue = [&](const TilePos &p, int ch, int st) {
        uint4v *dst = lds + st * stage_units;
        const int gy0 = p.py + d * (p.ty * ypitch) - a.in_off;
        const int gx0 = p.x0 - a.in_off + lane;
        unsigned coff[VUE];
        bool cok[VUE];
#pragma unroll
        for (int v = 0; v < VUE; ++v) {
            const int gx = gx0 + 64 * v;
            cok[v] = gx >= 0 && gx < Wmem;
            coff[v] = (unsigned)(cok[v] ? gx : 0) * 16u;
        }
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            const int rid = lw + LW * u;
            if (rid >= ROWS) break;                              // uniform: this wave has no further row
            const int oc = rid / RR, r = rid - oc * RR;
            const int o = ch * OC + oc;
            const int gy = gy0 + r * d;
            const bool rowok = o < a.c8_in && gy >= 0 && gy < a.H;
            const char *rowbase = reinterpret_cast<const char *>(a.x) + in_plane(p.b, rowok ? o : 0) * plane_bytes_in +
                                  (long)(rowok ? gy : 0) * Wmem * 16;
#pragma unroll
            for (int v = 0; v < VUE; ++v) {
                const int xc = lane + 64 * v;
                uint4v *slot_dst = dst + rid * PW + 64 * v;
                const bool inside = cok[v] && xc < PW;
                const bool any_inside = __builtin_amdgcn_ballot_w64(inside) != 0;
                if (rowok && any_inside) {
                    if (inside)
                        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(rowbase + coff[v]),
                                                         (__attribute__((address_space(3))) void *)slot_dst, 16, 0, 0);
                    else if (xc < PW)
                        slot_dst[lane] = uint4v{0u, 0u, 0u, 0u};
                } else if (xc < PW) {
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(zeros + lane * 16),
                                                     (__attribute__((address_space(3))) void *)slot_dst, 16, 0, 0);
                }
            }
        }
        const char *wsrc = reinterpret_cast<const char *>(a.wp) + ((long)p.mg * a.nchunks + ch) * (WUNITS * 16);
#pragma unroll
        for (int u = 0; u < (RESW ? 0 : WL); ++u) {
            const int blk = lw + LW * u;
            if (blk >= WBLK) break;                              // uniform
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(wsrc + (unsigned)(blk * 1024 + lane * 16)),
                                             (__attribute__((address_space(3))) void *)(dst + tile_units + blk * 64), 16, 0, 0);
        }
    };

    floatx4 acc[R][MT];
#pragma unroll
    for (int y = 0; y < R; ++y)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[y][mt] = floatx4{0.f, 0.f, 0.f, 0.f};

    auto compute = [&](int buf, int chunk) {
        const uint4v *tile = lds + buf * stage_units;
        const uint4v *wl = RESW ? wres + chunk * WUNITS : tile + tile_units;
#pragma unroll
        for (int cs = 0; cs < CS; ++cs) {
            // Tap row i is first needed by input row r = i, so its A fragments are fetched one input
            // row ahead instead of all at the top: right after the barrier all waves would otherwise
            // queue KS*MT + 1 LDS reads each before anybody's first MFMA.
            uint4v afr[KS][MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) afr[0][mt] = wl[((cs * KS + 0) * MT + mt) * 64 + lane];
            const int off = (MAP4 ? g * d : g * RR * PW + cs * d) + wave * 16 + l16;
            uint4v bcur = tile[off];
#pragma unroll
            for (int r = 0; r < RR; ++r) {
                uint4v bnext = bcur;
                if (r + 1 < RR) bnext = tile[off + (r + 1) * PW];
                if (r + 1 < KS) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) afr[r + 1][mt] = wl[((cs * KS + r + 1) * MT + mt) * 64 + lane];
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < KS; ++i) {
                    const int y = r - i;
                    if (y >= 0 && y < R) {
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) acc[y][mt] = H<DT>::mfma(afr[i][mt], bcur, acc[y][mt]);
                    }
                }
                bcur = bnext;
            }
        }
    };



    // Epilogue of one tile: bias, ReLU, optional ReLU mask of the layer below, conversion, store.
    // Everything it reads comes first (bias from LDS, the mask in one batch) and the stores follow
    // without a load in between.  Rows / map tiles outside the output are skipped by uniform
    // branches, columns outside by the lane mask; the number of memory instructions actually issued
    // is returned, because the pipeline below counts outstanding operations.
    auto epilogue = [&](const TilePos &p) -> int {
        const int ox = p.x0 + wave * 16 + l16;
        const bool colok = ox < a.Wo;
        if (__builtin_amdgcn_ballot_w64(colok) == 0) {          // this wave's 16 columns lie outside
#pragma unroll
            for (int y = 0; y < R; ++y)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) acc[y][mt] = floatx4{0.f, 0.f, 0.f, 0.f};
            return 0;
        }
        int ops = 0;
        float bia[MT][4];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) bia[mt][r4] = bias_lds[(p.mg * MT + mt) * 16 + 4 * g + r4];
        // byte offsets inside one image of the destination stay below 2^31 (checked by the launcher)
        const int row_bytes = a.OW * (a.out_f32 ? 4 : 16);
        const int plane_bytes = a.OH * row_bytes;
        const int oxc = colok ? ox : 0;
        // scalar base of image b (and of the first octet / map), per-lane 32-bit offsets of the column
        // and of each map tile
        char *img_base = reinterpret_cast<char *>(a.y) + (a.out_f32 ? (long)p.b * a.c_out : (long)p.b * a.c8_out_total + a.o8_off) * plane_bytes;
        const char *mask_base = reinterpret_cast<const char *>(a.mask) + (img_base - reinterpret_cast<char *>(a.y));
        unsigned voff[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int mtile = p.mg * MT + mt;
            if (a.out_f32) voff[mt] = (unsigned)((mtile * 16 + 4 * g) * plane_bytes + (oxc * a.ox_mul + a.ox_off) * 4);
            else {
                int off = (mtile * 2 + (g >> 1)) * plane_bytes + (oxc * a.ox_mul + a.ox_off) * 16 + (g & 1) * 8;
                if (a.tap_maps > 0) {        // stacked up-convolution taps (see ConvHArgs)
                    const int tap = mtile * 16 / a.tap_maps;
                    off += (tap >> 1) * row_bytes + (tap & 1) * 16 - tap * (a.tap_maps / 8) * plane_bytes;
                }
                voff[mt] = (unsigned)off;
            }
        }
        uint2v mk[HAS_MASK ? R : 1][HAS_MASK ? MT : 1];
        if constexpr (HAS_MASK) {
#pragma unroll
            for (int y = 0; y < R; ++y) {
                const int oy = p.py + d * (p.ty * ypitch + y);
                if (oy >= a.Ho) continue;
                const char *rowp = mask_base + (long)(oy * a.oy_mul + a.oy_off) * row_bytes;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    if (p.mg * MT + mt >= a.m_tiles) continue;
                    const bool ok = colok && (p.mg * MT + mt) * 2 + (g >> 1) < a.c8_out;
                    mk[y][mt] = uint2v{0u, 0u};
                    if (ok) mk[y][mt] = *reinterpret_cast<const uint2v *>(rowp + voff[mt]);
                    ++ops;
                }
            }
        }
#pragma unroll
        for (int y = 0; y < R; ++y) {
            const int oy = p.py + d * (p.ty * ypitch + y);
            char *rowp = img_base + (long)(oy * a.oy_mul + a.oy_off) * row_bytes;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int mtile = p.mg * MT + mt;
                floatx4 v = acc[y][mt];
                acc[y][mt] = floatx4{0.f, 0.f, 0.f, 0.f};
                if (oy >= a.Ho || mtile >= a.m_tiles) continue;      // uniform
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    v[r4] += bia[mt][r4];
                    if (a.relu) v[r4] = fmaxf(v[r4], 0.f);
                }
                if (a.out_f32) {
                    const int o = mtile * 16 + 4 * g;
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        // lane group 0 of a valid column always owns a real map, so every one of these is issued
                        if (colok && o + r4 < a.c_out) *reinterpret_cast<float *>(rowp + voff[mt] + (unsigned)(r4 * plane_bytes)) = v[r4];
                        ops += (mtile * 16 + r4 < a.c_out) ? 1 : 0;
                    }
                } else {
                    unsigned short h[4];
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) h[r4] = H<DT>::cvt(v[r4]);
                    uint2v packed = uint2v{(unsigned)h[0] | ((unsigned)h[1] << 16), (unsigned)h[2] | ((unsigned)h[3] << 16)};
                    if constexpr (HAS_MASK) {
                        const uint2v m = mk[y][mt];
                        unsigned lo = packed[0], hi = packed[1];
                        if (!pos16(m[0] & 0xffffu)) lo &= 0xffff0000u;
                        if (!pos16(m[0] >> 16)) lo &= 0x0000ffffu;
                        if (!pos16(m[1] & 0xffffu)) hi &= 0xffff0000u;
                        if (!pos16(m[1] >> 16)) hi &= 0x0000ffffu;
                        packed = uint2v{lo, hi};
                    }
                    if (colok && mtile * 2 + (g >> 1) < a.c8_out) *reinterpret_cast<uint2v *>(rowp + voff[mt]) = packed;
                    ++ops;
                }
            }
        }
        return ops;
    };

    // Epilogue with 16-byte stores (16-bit output, no mask).  The memory pipeline takes about as long
    // for a store instruction of 8 bytes per lane as for one of 16, so rows are stored in pairs:
    // lanes of the even lane groups hold the low half of an octet and their neighbours 16 lanes up
    // the high half; after one v_permlane16_swap per register the even groups own the whole octet
    // of row y and the odd groups that of row y + 1, and one instruction stores both rows.
    auto epilogue16 = [&](const TilePos &p) {
        const int ox = p.x0 + wave * 16 + l16;
        const bool colok = ox < a.Wo;
        if (__builtin_amdgcn_ballot_w64(colok) == 0) {          // this wave's 16 columns lie outside
#pragma unroll
            for (int y = 0; y < R; ++y)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) acc[y][mt] = floatx4{0.f, 0.f, 0.f, 0.f};
            return;
        }
        const int row_bytes = a.OW * 16, plane_bytes = a.OH * row_bytes;   // < 2^31 (checked by the launcher)
        const int oxc = colok ? ox : 0;
        char *img_base = reinterpret_cast<char *>(a.y) + ((long)p.b * a.c8_out_total + a.o8_off) * plane_bytes;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int mtile = p.mg * MT + mt;
            float bia[4];
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) bia[r4] = bias_lds[mtile * 16 + 4 * g + r4];
            const bool octet_ok = colok && mtile < a.m_tiles && mtile * 2 + (g >> 1) < a.c8_out;
            const unsigned voff = (unsigned)((mtile * 2 + (g >> 1)) * plane_bytes + (oxc * a.ox_mul + a.ox_off) * 16);
#pragma unroll
            for (int y = 0; y < R; y += 2) {
                unsigned lo[2], hi[2];          // this lane's half octet of rows y and y + 1
#pragma unroll
                for (int yy = 0; yy < 2; ++yy) {
                    floatx4 v = acc[y + yy][mt];
                    acc[y + yy][mt] = floatx4{0.f, 0.f, 0.f, 0.f};
                    unsigned short h[4];
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        v[r4] += bia[r4];
                        if (a.relu) v[r4] = fmaxf(v[r4], 0.f);
                        h[r4] = H<DT>::cvt(v[r4]);
                    }
                    lo[yy] = (unsigned)h[0] | ((unsigned)h[1] << 16);
                    hi[yy] = (unsigned)h[2] | ((unsigned)h[3] << 16);
                }
                // odd groups of the first operand <-> even groups of the second
                const auto s0 = __builtin_amdgcn_permlane16_swap(lo[0], lo[1], false, false);
                const auto s1 = __builtin_amdgcn_permlane16_swap(hi[0], hi[1], false, false);
                // even group: {own row y half, neighbour's row y half}; odd group: {neighbour's row y+1 half, own}
                const uint4v octet = uint4v{s0[0], s1[0], s0[1], s1[1]};
                const int oy = p.py + d * (p.ty * ypitch + y + (g & 1));
                if (octet_ok && oy < a.Ho)
                    *reinterpret_cast<uint4v *>(img_base + (long)(oy * a.oy_mul + a.oy_off) * row_bytes + voff) = octet;
            }
        }
    };

    // Epilogue with the vertical half of the SK pool (VPOOL): bias, ReLU, conversion as in epilogue16, then pooled
    // row j - 1 of the tile = max(conv row j - 1, conv row j), j = 0..R-1, where conv row -1 is the last row of the
    // tile above, carried in `carry` (have_carry: there is such a tile and this wave multiplied it).  Pooled rows
    // are stored in pairs like the rows of epilogue16.  store = false (the extra tile in front of a run that
    // starts inside a column of tiles) only leaves its last row behind.  The ReLU is a signed-integer max on the
    // fp32 bit pattern (negative values and -0 become +0), after which the packed unsigned 16-bit max is the
    // numerical max.
    unsigned carry[VPOOL ? MT : 1][2] = {};
    auto epilogue_vpool = [&](const TilePos &p, bool have_carry, bool store) {
        auto pkmax = [](unsigned x, unsigned y) { return pk_max_u16(x, y); };
        const int ox = p.x0 + wave * 16 + l16;
        const bool colok = ox < a.Wo;
        const int row_bytes = a.OW * 16, plane_bytes = a.OH * row_bytes;   // < 2^31 (checked by the launcher)
        const int oxc = colok ? ox : 0;
        char *img_base = reinterpret_cast<char *>(a.y) + ((long)p.b * a.c8_out_total + a.o8_off) * plane_bytes;
        const int Hp = a.Ho - d;                                           // pooled rows
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int mtile = p.mg * MT + mt;
            float bia[4];
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) bia[r4] = bias_lds[mtile * 16 + 4 * g + r4];
            const bool octet_ok = store && colok && mtile < a.m_tiles && mtile * 2 + (g >> 1) < a.c8_out;
            const unsigned voff = (unsigned)((mtile * 2 + (g >> 1)) * plane_bytes + oxc * 16);
            unsigned prev_lo = carry[mt][0], prev_hi = carry[mt][1];
#pragma unroll
            for (int y = 0; y < R; y += 2) {
                unsigned lo[2], hi[2];          // this lane's half octet of pooled rows y - 1 and y
#pragma unroll
                for (int yy = 0; yy < 2; ++yy) {
                    floatx4 v = acc[y + yy][mt];
                    unsigned short h[4];
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        const int bits = __float_as_int(v[r4] + bia[r4]);
                        h[r4] = H<DT>::cvt(__int_as_float(bits > 0 ? bits : 0));
                    }
                    const unsigned cl = (unsigned)h[0] | ((unsigned)h[1] << 16), chh = (unsigned)h[2] | ((unsigned)h[3] << 16);
                    lo[yy] = pkmax(prev_lo, cl);
                    hi[yy] = pkmax(prev_hi, chh);
                    prev_lo = cl;
                    prev_hi = chh;
                }
                const auto s0 = __builtin_amdgcn_permlane16_swap(lo[0], lo[1], false, false);
                const auto s1 = __builtin_amdgcn_permlane16_swap(hi[0], hi[1], false, false);
                const uint4v octet = uint4v{s0[0], s1[0], s0[1], s1[1]};
                // even lane groups own pooled row y - 1, odd ones pooled row y (tile-local; -1 is the carried row's)
                const int j = y - 1 + (g & 1);
                const int oy = p.py + d * (p.ty * ypitch + j);
                if (octet_ok && (j >= 0 || have_carry) && oy < Hp)
                    *reinterpret_cast<uint4v *>(img_base + (long)oy * row_bytes + voff) = octet;
            }
            carry[mt][0] = prev_lo;
            carry[mt][1] = prev_hi;
        }
    };

    // This workgroup's tiles: every nslots-th tile of its XCD's eighth of the list, or (VPOOL) a contiguous run of
    // that eighth -- with the tile above its first one in front when the run starts inside a column of tiles.
    int t = t_begin + slot;
    int my_tiles = 0;
    bool lead_in = false;
    if constexpr (VPOOL) {
        const long len = t_end - t_begin;
        const int r0 = t_begin + (int)(len * slot / nslots), r1 = t_begin + (int)(len * (slot + 1) / nslots);
        if (r0 >= r1) return;
        const int yt0 = r0 % a.ytiles_total;             // its row tile inside its row phase (as in the ypos table)
        const int ty0 = yt0 < a.rem * a.tiles_hi ? yt0 % a.tiles_hi : (yt0 - a.rem * a.tiles_hi) % a.tiles_lo;
        lead_in = ty0 > 0 && ypitch == R;
        t = r0 - (lead_in ? 1 : 0);
        my_tiles = r1 - t;
    } else {
        if (t >= t_end) return;
        my_tiles = (t_end - t + nslots - 1) / nslots;
    }
    const int total_chunks = my_tiles * a.nchunks;
    block_sync_lds();                                   // ypos / bias tables are in place

    // issue cursor (runs S-1 chunks ahead of the compute cursor)
    Cursor icur = cursor_at(t), ccur = icur;
    TilePos ipos = position(icur);
    int ich = 0, issued = 0, itiles = 0;
    // the next chunk in this workgroup's order: its tile position and its chunk number inside the tile
    auto take_next = [&](TilePos &p, int &ch) {
        p = ipos;
        ch = ich;
        ++issued;
        if (++ich == a.nchunks) {
            ich = 0;
            if (++itiles < my_tiles) {
                advance(icur);
                ipos = position(icur);
            }
        }
    };
    auto issue_next = [&]() {
        TilePos p;
        int ch;
        const int st = issued % S;
        take_next(p, ch);
        issue(p, ch, st);
    };
    // (a pending pool of the input is finished in registers on the way into LDS: see the producer branch below)
    if (!(NP > 0 && hd > 0)) {
#pragma unroll
        for (int j = 0; j < S - 1; ++j)
            if (j < total_chunks && lw >= 0) issue_next();
    }

    if constexpr (NP > 0) {
        // Every wave meets the same barrier once per chunk.  A producer arrives when its loads of
        // chunk q have landed and then refills the stage that was multiplied in the previous
        // iteration; a multiplying wave arrives when it is done with chunk q - 1.
        if (wave >= CH_WAVES && hd > 0) {
            // The input lacks the horizontal half of its pool: unit x of the tile is max(X[x], X[x + hd]).  The producer
            // waves load both operands into registers (two chunks in flight, in two register sets), take the maximum
            // and write the result into the ring stage -- one LDS write per unit, where loading the raw row straight
            // into LDS and pooling it in place cost the direct write, two reads and a write.  Chunk c is loaded
            // after barrier c - 3, written after barrier c - 1 (its stage was multiplied before barrier c - 2) and
            // multiplied after barrier c.  The values are ReLU outputs (>= +0): the unsigned 16-bit order of the
            // bit patterns is their numerical order.
            const int my_rows = (ROWS - lw + LW - 1) / LW;         // tile rows this wave stages
            const int Lr = 2 * my_rows * VUE;                      // its loads per chunk
            uint4v rA[RU][VUE][2], rB[RU][VUE][2];
            TilePos pA = ipos, pB = ipos;
            int cA = 0, cB = 0;
            auto gload = [&](uint4v (&r)[RU][VUE][2], const TilePos &p, int ch) {
                const int gy0 = p.py + d * (p.ty * ypitch), gx0 = p.x0 + lane;
#pragma unroll
                for (int u = 0; u < RU; ++u) {
                    const int rid = lw + LW * u;
                    if (rid >= ROWS) break;                          // uniform: this wave has no further row
                    const int oc = rid / RR, rr = rid - oc * RR;
                    int o = ch * OC + oc, gy = gy0 + rr * d;
                    o = o < a.c8_in ? o : a.c8_in - 1;
                    gy = gy < a.H ? gy : a.H - 1;
                    const uint4v *row = reinterpret_cast<const uint4v *>(reinterpret_cast<const char *>(a.x) + in_plane(p.b, o) * plane_bytes_in +
                                                                         (long)gy * Wmem * 16);
#pragma unroll
                    for (int v = 0; v < VUE; ++v) {
                        int gx = gx0 + 64 * v;
                        gx = gx < a.W ? gx : a.W - 1;                // clamped: what lies outside is replaced by zero when it is stored
                        r[u][v][0] = row[gx];
                        r[u][v][1] = row[gx + hd];
                    }
                }
            };
            auto gstore = [&](uint4v (&r)[RU][VUE][2], const TilePos &p, int ch, int st) {
                uint4v *dst = lds + st * stage_units;
                const int gy0 = p.py + d * (p.ty * ypitch), gx0 = p.x0 + lane;
#pragma unroll
                for (int u = 0; u < RU; ++u) {
                    const int rid = lw + LW * u;
                    if (rid >= ROWS) break;
                    const int oc = rid / RR, rr = rid - oc * RR;
                    const bool rowok = ch * OC + oc < a.c8_in && gy0 + rr * d < a.H;
#pragma unroll
                    for (int v = 0; v < VUE; ++v) {
                        const int xc = lane + 64 * v;
                        uint4v m = max_u16x8(r[u][v][0], r[u][v][1]);
                        if (!(rowok && gx0 + 64 * v < a.W)) m = uint4v{0u, 0u, 0u, 0u};
                        if (xc < PWL) dst[rid * PW + xc] = m;
                    }
                }
            };
            // chunk c (c >= 1), right after barrier c - 1: from its register set into its stage, then chunk c + 2 into the set
            auto step = [&](uint4v (&r)[RU][VUE][2], TilePos &p, int &ch, int c) {
                if (c >= total_chunks) return;
                __builtin_amdgcn_sched_barrier(0);
                wait_vmcnt_at_most(c + 1 < total_chunks ? Lr : 0);   // the loads of chunk c + 1 are younger and may be in flight
                __builtin_amdgcn_sched_barrier(0);
                gstore(r, p, ch, c % S);
                if (c + 2 < total_chunks) {
                    take_next(p, ch);
                    gload(r, p, ch);
                }
            };
            take_next(pA, cA);
            gload(rA, pA, cA);                                       // chunk 0
            if (total_chunks > 1) {
                take_next(pB, cB);
                gload(rB, pB, cB);                                   // chunk 1
            }
            __builtin_amdgcn_sched_barrier(0);
            wait_vmcnt_at_most(total_chunks > 1 ? Lr : 0);
            __builtin_amdgcn_sched_barrier(0);
            gstore(rA, pA, cA, 0);
            if (total_chunks > 2) {
                take_next(pA, cA);
                gload(rA, pA, cA);                                   // chunk 2
            }
            for (int q = 0; q < total_chunks; q += 2) {
                block_sync_lds();                                    // barrier q: chunk q is in LDS
                step(rB, pB, cB, q + 1);
                if (q + 1 < total_chunks) {
                    block_sync_lds();                                // barrier q + 1
                    step(rA, pA, cA, q + 2);
                }
            }
            return;
        }
        if (wave >= CH_WAVES) {
            for (int q = 0; q < total_chunks; ++q) {
                int allow = (issued - q - 1) * L;          // loads of younger chunks may still be in flight
                allow = allow < 63 ? allow : 63;
                __builtin_amdgcn_sched_barrier(0);
                wait_vmcnt_at_most(allow);
                __builtin_amdgcn_sched_barrier(0);
                block_sync_lds();
                if (issued < total_chunks) issue_next();
            }
            return;
        }
        // One tile per trip, so that the accumulators live inside the trip only: a wave whose 16
        // columns lie right of the image (the ragged last x tile) then skips the tile's MFMAs and
        // stores as a whole and only keeps the barriers, and its SIMD is left to the other wave.
        TilePos cur = position(ccur);
        int st = 0;
        for (int ctile = 0; ctile < my_tiles; ++ctile) {
            const bool idle = __builtin_amdgcn_readfirstlane((int)(cur.x0 + wave * 16 >= a.Wo)) != 0;
            if (idle) {
                for (int ch = 0; ch < a.nchunks; ++ch) {
                    block_sync_lds();
                    st = st + 1 == S ? 0 : st + 1;
                }
            } else {
#pragma unroll
                for (int y = 0; y < R; ++y)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) acc[y][mt] = floatx4{0.f, 0.f, 0.f, 0.f};
                for (int ch = 0; ch < a.nchunks; ++ch) {
                    block_sync_lds();
                    compute(st, ch);
                    st = st + 1 == S ? 0 : st + 1;
                }
                if constexpr (VPOOL) epilogue_vpool(cur, ypitch == R && cur.ty > 0 && ctile > 0, !(lead_in && ctile == 0));
                else if (HAS_MASK || a.out_f32 || (R & 1)) epilogue(cur);
                else epilogue16(cur);
            }
            if (ctile + 1 < my_tiles) {
                advance(ccur);
                cur = position(ccur);
            }
        }
        return;
    }
    TilePos cur = position(ccur);
    int ch = 0, ctiles = 0;
    int ep_ops[S - 1];            // memory operations of the epilogues of the last S-1 iterations
#pragma unroll
    for (int j = 0; j < S - 1; ++j) ep_ops[j] = 0;
    for (int q = 0; q < total_chunks; ++q) {
        // Chunk q must have landed.  The counter retires operations in issue order, so it may still
        // show whatever was issued after chunk q's loads: the loads of the (up to S-2) younger chunks
        // and the epilogue operations of the last S-1 iterations.  Allowing fewer is safe (it only
        // waits longer), allowing more is not.
        int allow = (issued - q - 1) * L;
#pragma unroll
        for (int j = 0; j < S - 1; ++j)
            if (j < S - 2 || !late_issue) allow += ep_ops[j];   // a late issuer's oldest epilogue precedes chunk q's loads
        allow = allow < 63 ? allow : 63;
        __builtin_amdgcn_sched_barrier(0);
        wait_vmcnt_at_most(allow);
        __builtin_amdgcn_sched_barrier(0);
        block_sync_lds();
        // stage (q-1)%S was read by everybody before this barrier: refill it, before or after the
        // multiplication depending on the wave
        if (!late_issue && issued < total_chunks) issue_next();
        compute(q % S, ch);
#pragma unroll
        for (int j = S - 2; j > 0; --j) ep_ops[j] = ep_ops[j - 1];
        ep_ops[0] = 0;
        if (ch == a.nchunks - 1) {
            ep_ops[0] = epilogue(cur);
            ch = 0;
            if (++ctiles < my_tiles) {
                advance(ccur);
                cur = position(ccur);
            }
        } else {
            ++ch;
        }
        if (late_issue && issued < total_chunks) issue_next();
    }
}

template <int DT, int KS, int MT, bool MAP4, int R, bool HAS_MASK, int VU = CH_VU, int XW = 8>
static hipError_t launch_conv_h_m(ConvHArgs a, hipStream_t stream)
{
    constexpr int RT = R * (CH_WAVES / XW), TX = 16 * XW;       // output rows and columns of a tile
    constexpr int RR = RT + KS - 1, OC = MAP4 ? 1 : 4, CS = MAP4 ? (KS + 3) / 4 : KS, TAPW = MAP4 ? 4 * CS : KS;
    const int PW = TX + (TAPW - 1) * a.d;
    if (PW > 64 * VU) return hipErrorInvalidValue;
    if (a.vpool || a.hd) return hipErrorInvalidValue;
    const size_t stage = (size_t)OC * RR * PW + (size_t)CS * KS * MT * 64;
    const int m_tiles_all = ((a.c_out + 15) / 16 + MT - 1) / MT * MT;
    const size_t smem = 2 * stage * 16 + (size_t)m_tiles_all * 16 * sizeof(float);
    if (smem > 160 * 1024) return hipErrorInvalidValue;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_h_kernel<DT, KS, MT, MAP4, R, HAS_MASK, VU, XW>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    a.m_tiles = (a.c_out + 15) / 16;
    a.mgroups = (a.m_tiles + MT - 1) / MT;
    a.nchunks = (a.c8_in + OC - 1) / OC;
    a.xtiles = (a.Wo + TX - 1) / TX;
    const int q = a.Ho / a.d;
    a.rem = a.Ho % a.d;
    a.tiles_hi = (q + 1 + RT - 1) / RT;
    a.tiles_lo = (q + RT - 1) / RT;
    a.ytiles_total = a.rem * a.tiles_hi + (a.d - a.rem) * a.tiles_lo;
    if (a.tiles_lo < 1) a.tiles_lo = 1;
    const long total = (long)a.xtiles * a.ytiles_total * a.mgroups * a.n;
    if (total < 1 || total > 0x7fffffffL) return hipErrorInvalidValue;
    // the epilogue addresses one image of the destination with 32-bit byte offsets
    if ((long)(a.out_f32 ? a.c_out * 4L : a.c8_out_total * 16L) * a.OH * a.OW >= 0x7fffffffL) return hipErrorInvalidValue;
    a.total_tiles = (int)total;
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 8)
            cus = 256;
    }
    int blocks = cus / 8 * 8;               // one workgroup per CU, a multiple of the 8 XCDs
    if (total < blocks) blocks = (int)((total + 7) / 8 * 8);
    hipLaunchKernelGGL((conv_h_kernel<DT, KS, MT, MAP4, R, HAS_MASK, VU, XW>), dim3(blocks), dim3(CH_THREADS), smem, stream, a);
    return hipGetLastError();
}

static int device_cus();

// Tiles of tx columns x rt rows (per residue class of the rows) that cover the output of a launch
static long conv_h_tile_count(const ConvHArgs &a, int mt, int tx, int rt)
{
    const int q = a.Ho / a.d, rem = a.Ho % a.d;
    const long ytiles = (long)rem * ((q + 1 + rt - 1) / rt) + (long)(a.d - rem) * std::max(1, (q + rt - 1) / rt);
    return (long)((a.Wo + tx - 1) / tx) * ytiles * (((a.c_out + 15) / 16 + mt - 1) / mt) * a.n;
}

template <int DT, int KS, int MT, bool MAP4, int R, int VU = CH_VU>
static hipError_t launch_conv_h_t(const ConvHArgs &a, hipStream_t stream)
{
    if constexpr (!MAP4 && (KS == 2 || KS == 3) && VU == CH_VU) {
        // Tile shape: 128 x 4, 64 x 8 or 32 x 16 output pixels.  Every tile costs about the same (512 pixels of every
        // chunk), so the shape that covers the output in the fewest rounds of one tile per CU wins: ragged maps waste
        // less of a squarer tile, which also stages less halo -- but a 32-column tile stages 72 short rows per chunk
        // where the 128-column one stages 24 long ones (twice the memory instructions; counted as a quarter more
        // time), and maps too small to give every CU a tile keep the flat shape, which has the most tiles.  Measured on
        // the U-Net's 64 -> 64 layer at 568^2: 48.2 -> 42.9 us (64 x 8); 128 -> 128 at 280^2: 49.1 -> 44.0 us (32 x 16).
        auto fits = [&](int tx, int rt) {               // staged rows of at most 128 units, two stages within the LDS
            const int pw = tx + (KS - 1) * a.d;
            const size_t stage = (size_t)4 * (rt + KS - 1) * pw + (size_t)KS * KS * MT * 64;
            return pw <= 128 && 2 * stage * 16 + (size_t)(((a.c_out + 15) / 16 + MT - 1) / MT * MT) * 64 <= 160 * 1024;
        };
        const int cus = device_cus();
        auto rounds = [&](int tx, int rt) { return (double)((conv_h_tile_count(a, MT, tx, rt) + cus - 1) / cus); };
        const double c8 = rounds(128, R), c4 = fits(64, 2 * R) ? rounds(64, 2 * R) : 1e30, c2 = fits(32, 4 * R) ? 1.25 * rounds(32, 4 * R) : 1e30;
        if (c2 < c4 && c2 < c8) {
            if (a.mask) return launch_conv_h_m<DT, KS, MT, MAP4, R, true, 2, 2>(a, stream);
            return launch_conv_h_m<DT, KS, MT, MAP4, R, false, 2, 2>(a, stream);
        }
        if (c4 < c8) {
            if (a.mask) return launch_conv_h_m<DT, KS, MT, MAP4, R, true, 2, 4>(a, stream);
            return launch_conv_h_m<DT, KS, MT, MAP4, R, false, 2, 4>(a, stream);
        }
    }
    if (a.mask) return launch_conv_h_m<DT, KS, MT, MAP4, R, true, VU>(a, stream);
    return launch_conv_h_m<DT, KS, MT, MAP4, R, false, VU>(a, stream);
}

// kernels larger than 4x4: the register-staged kernel with the lane groups on four consecutive kernel columns, four
// output rows per tile, forward only; tiles wider than 192 units (10x10 at d = 8) stage a fourth column group per row
template <int DT, int KS, int MT>
static hipError_t launch_conv_h_big(const ConvHArgs &a, hipStream_t stream)
{
    if (a.mask) return hipErrorInvalidValue;
    constexpr int TAPW = 4 * ((KS + 3) / 4), CS = (KS + 3) / 4;
    if constexpr (KS == 6 || KS == 8 || KS == 10) {
        // 64 x 8 pixel tiles where they cover the output in fewer rounds of one tile per CU (see launch_conv_h_t): the
        // k - 1 halo rows weigh less under eight output rows than under four, and ragged maps waste less
        const int pw = 64 + (TAPW - 1) * a.d, cus = device_cus();
        const size_t stage = (size_t)(8 + KS - 1) * pw + (size_t)CS * KS * MT * 64;
        const bool fits = pw <= 192 && 2 * stage * 16 + (size_t)(((a.c_out + 15) / 16 + MT - 1) / MT * MT) * 64 <= 160 * 1024;
        if (fits && (conv_h_tile_count(a, MT, 64, 8) + cus - 1) / cus < (conv_h_tile_count(a, MT, 128, 4) + cus - 1) / cus) {
            if (pw <= 128) return launch_conv_h_m<DT, KS, MT, true, 4, false, 2, 4>(a, stream);
            return launch_conv_h_m<DT, KS, MT, true, 4, false, 3, 4>(a, stream);
        }
    }
    if (CH_TX + (TAPW - 1) * a.d > 64 * CH_VU) return launch_conv_h_m<DT, KS, MT, true, 4, false, 4>(a, stream);
    return launch_conv_h_m<DT, KS, MT, true, 4, false, CH_VU>(a, stream);
}

static int device_cus()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 8)
            cus = 256;
    }
    return cus;
}

// LDS bytes of the ring kernel: S stages (+ resident weights) + bias + y-tile table
template <int KS, int MT, bool MAP4, int R, int S, bool RESW>
static size_t ring_smem(int d, int c_out, int c8_in, int Ho, int hd = 0)
{
    constexpr int RR = R + KS - 1, OC = MAP4 ? 1 : 4, CS = MAP4 ? 1 : KS;
    const int PW = CH_TX + (MAP4 ? 3 : KS - 1) * d;            // (a pending pool of the input is finished before the tile is staged)
    (void)hd;
    const size_t tile = (size_t)OC * RR * PW, slab = (size_t)CS * KS * MT * 64;
    const int nchunks = (c8_in + OC - 1) / OC;
    const int m_tiles_all = ((c_out + 15) / 16 + MT - 1) / MT * MT;
    const size_t units = RESW ? S * tile + nchunks * slab : S * (tile + slab);
    return units * 16 + (size_t)m_tiles_all * 64 + (size_t)(Ho / R + 2 * d + 2) * 4;
}

template <int DT, int KS, int MT, bool MAP4, int R, bool HAS_MASK, int S, bool RESW, int NP = 0, bool VPOOL = false>
static hipError_t launch_conv_h_ring_m(ConvHArgs a, hipStream_t stream)
{
    constexpr int OC = MAP4 ? 1 : 4;
    if (NP == 0 && a.hd != 0) return hipErrorInvalidValue;         // the pending pool is finished by producer waves
    if (a.hd != 0 && (a.in_off != 0 || a.hd < 1 || CH_TX + (KS - 1) * a.d + a.hd > 64 * (KS == 1 ? 2 : 3))) return hipErrorInvalidValue;
    if (VPOOL && (!a.relu || a.out_f32 || a.tap_maps != 0 || a.oy_mul != 1 || a.ox_mul != 1 || a.oy_off != 0 || a.ox_off != 0 ||
                  a.OH != a.Ho - a.d || a.OW != a.Wo || a.Ho <= a.d))
        return hipErrorInvalidValue;
    const size_t smem = ring_smem<KS, MT, MAP4, R, S, RESW>(a.d, a.c_out, a.c8_in, a.Ho, a.hd);
    if (smem > 160 * 1024) return hipErrorInvalidValue;            // callers check the size first
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_h_ring_kernel<DT, KS, MT, MAP4, R, HAS_MASK, S, RESW, NP, VPOOL>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    if (!a.zeros) return hipErrorInvalidValue;                     // the caller's page of zeros (allocated with its plan)
    a.m_tiles = (a.c_out + 15) / 16;
    a.mgroups = (a.m_tiles + MT - 1) / MT;
    a.nchunks = (a.c8_in + OC - 1) / OC;
    a.xtiles = (a.Wo + CH_TX - 1) / CH_TX;
    const int q = a.Ho / a.d;
    a.rem = a.Ho % a.d;
    a.ypitch = R;
    a.tiles_hi = (q + 1 + R - 1) / R;
    a.tiles_lo = (q + R - 1) / R;
    if (VPOOL) {
        // carried rows pay one extra tile per workgroup (the tile above its run): worth it from about eight tiles per
        // workgroup; below that, tiles that overlap by one row (R - 1 pooled rows each) cost less
        const long per_wg = (long)a.xtiles * (a.rem * a.tiles_hi + (a.d - a.rem) * a.tiles_lo) * a.n / (device_cus() / 8 * 8);
        if (per_wg < 8) {
            a.ypitch = R - 1;
            a.tiles_hi = q >= 1 ? (q + R - 2) / (R - 1) : 1;         // q + 1 rows: q pooled rows
            a.tiles_lo = q >= 2 ? (q - 1 + R - 2) / (R - 1) : 1;     // q rows: q - 1 pooled rows
        }
    }
    a.ytiles_total = a.rem * a.tiles_hi + (a.d - a.rem) * a.tiles_lo;
    if (a.tiles_lo < 1) a.tiles_lo = 1;
    if (RESW && a.mgroups != 1) return hipErrorInvalidValue;
    const long total = (long)a.xtiles * a.ytiles_total * a.mgroups * a.n;
    if (total < 1 || total > 0x7fffffffL) return hipErrorInvalidValue;
    if ((long)(a.out_f32 ? a.c_out * 4L : a.c8_out_total * 16L) * a.OH * a.OW >= 0x7fffffffL) return hipErrorInvalidValue;
    a.total_tiles = (int)total;
    int blocks = device_cus() / 8 * 8;
    if (total < blocks) blocks = (int)((total + 7) / 8 * 8);
    hipLaunchKernelGGL((conv_h_ring_kernel<DT, KS, MT, MAP4, R, HAS_MASK, S, RESW, NP, VPOOL>), dim3(blocks), dim3(CH_THREADS + 64 * NP), smem, stream, a);
    return hipGetLastError();
}

template <int DT, int KS, int MT, bool MAP4, int R, int S, bool RESW>
static hipError_t launch_conv_h_ring_mask(const ConvHArgs &a, hipStream_t stream)
{
    if (a.mask) return launch_conv_h_ring_m<DT, KS, MT, MAP4, R, true, S, RESW>(a, stream);
    return launch_conv_h_ring_m<DT, KS, MT, MAP4, R, false, S, RESW>(a, stream);
}

// Preference: weights resident in LDS with a 3-stage ring of input tiles (one map group, all chunk
// slabs fit), else a 4-stage ring that streams the weight slab with each chunk, else the
// register-staged two-stage kernel.
template <int DT, int KS, int MT, bool MAP4, int R>
static hipError_t launch_conv_h_ring_or_staged(const ConvHArgs &a, hipStream_t stream)
{
    const bool one_group = ((a.c_out + 15) / 16 + MT - 1) / MT == 1;
    if (one_group && ring_smem<KS, MT, MAP4, R, 3, true>(a.d, a.c_out, a.c8_in, a.Ho, a.hd) <= 160 * 1024) {
        // the forward 4x4 convolution of the benchmark nets: loads on four waves of their own (three waves per SIMD)
        if constexpr (KS == 4 && MAP4 && R == 8)
            if (!a.mask) {
                if (a.vpool) return launch_conv_h_ring_m<DT, KS, MT, MAP4, R, false, 3, true, 4, true>(a, stream);
                return launch_conv_h_ring_m<DT, KS, MT, MAP4, R, false, 3, true, 4>(a, stream);
            }
        if (a.vpool || a.hd) return hipErrorInvalidValue;
        return launch_conv_h_ring_mask<DT, KS, MT, MAP4, R, 3, true>(a, stream);
    }
    if (a.vpool || a.hd) return hipErrorInvalidValue;              // callers ask conv_h_pool_fusable first
    if (ring_smem<KS, MT, MAP4, R, 4, false>(a.d, a.c_out, a.c8_in, a.Ho) <= 160 * 1024)
        return launch_conv_h_ring_mask<DT, KS, MT, MAP4, R, 4, false>(a, stream);
    return launch_conv_h_t<DT, KS, MT, MAP4, R>(a, stream);
}

template <int DT, int MT>
static hipError_t launch_conv_h_mt(const ConvHArgs &a, hipStream_t stream)
{
    switch (a.k) {
    case 1: return launch_conv_h_ring_or_staged<DT, 1, MT, false, 4>(a, stream);
    case 2: return launch_conv_h_t<DT, 2, MT, false, 4>(a, stream);
    case 3:
        if constexpr (MT <= 3) return launch_conv_h_t<DT, 3, MT, false, 4>(a, stream);
        else return hipErrorInvalidValue;
    case 4:
        if constexpr (MT <= 3) return launch_conv_h_ring_or_staged<DT, 4, MT, true, 8>(a, stream);
        else return launch_conv_h_ring_or_staged<DT, 4, MT, true, 4>(a, stream);
    case 5: if constexpr (MT <= 3) return launch_conv_h_big<DT, 5, MT>(a, stream); else return hipErrorInvalidValue;
    case 6: if constexpr (MT <= 3) return launch_conv_h_big<DT, 6, MT>(a, stream); else return hipErrorInvalidValue;
    case 7: if constexpr (MT <= 3) return launch_conv_h_big<DT, 7, MT>(a, stream); else return hipErrorInvalidValue;
    case 8: if constexpr (MT <= 2) return launch_conv_h_big<DT, 8, MT>(a, stream); else return hipErrorInvalidValue;
    case 10: if constexpr (MT <= 2) return launch_conv_h_big<DT, 10, MT>(a, stream); else return hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
    }
}

// 3x3 kernels on a single input octet (the first layer of the U-Net and the USK-Net): the ring kernel with the lane
// groups on the kernel columns (the fourth column's weights are zero), so the one octet that exists fills a K step with
// three of its four columns instead of one quarter of a four-octet chunk, and eight output rows per tile.  Measured on
// the U-Net's 1 -> 64 layer at 570^2: 29.5 -> 19.9 us.  With more input maps the register-staged kernel is faster
// (64 -> 128 at 282^2: 30.7 against 45.7 us; 128 -> 128 at 280^2: 47.5 against 75.6 us).
template <int DT, int MT>
static hipError_t launch_conv_h_k3_tapcols(const ConvHArgs &a, hipStream_t stream)
{
    if (CH_TX + 3 * a.d > 64 * 3) return hipErrorInvalidValue;
    const bool one_group = ((a.c_out + 15) / 16 + MT - 1) / MT == 1;
    if (one_group && ring_smem<3, MT, true, 8, 3, true>(a.d, a.c_out, a.c8_in, a.Ho) <= 160 * 1024)
        return launch_conv_h_ring_m<DT, 3, MT, true, 8, false, 3, true>(a, stream);
    if (ring_smem<3, MT, true, 8, 4, false>(a.d, a.c_out, a.c8_in, a.Ho) <= 160 * 1024)
        return launch_conv_h_ring_m<DT, 3, MT, true, 8, false, 4, false>(a, stream);
    return hipErrorInvalidValue;
}

// Map tiles per workgroup for a forward layer, with CONV_H_TAPCOLS set where launch_conv_h_k3_tapcols is the better
// kernel: 3x3 at d = 1, one input octet and at least 128 x 128 output pixels per image
int conv_h_pick_mode(int c_out, int c_in, int k, int d, int n, int Ho, int Wo)
{
    if (k == 3 && d == 1 && c_in <= 8 && c_out >= 32 && (long)Ho * Wo >= 128L * 128) {
        const int tiles = (c_out + 15) / 16;
        return ((tiles % 3 == 0 || tiles >= 8) ? 3 : 2) | CONV_H_TAPCOLS;
    }
    return conv_h_pick_mt(c_out, k, n, Ho, Wo);
}

// output-map tiles (16 maps each) per workgroup: as few padded tiles as possible; a 3x3 kernel's
// weight slab (k*k KB per tile and chunk) only leaves LDS room for three
int conv_h_mt(int c_out, int k)
{
    const int tiles = (c_out + 15) / 16;
    // kernels beyond 4x4: the weight slab of a chunk is ceil(k/4)*k KB per map tile and shares the LDS with a tile of
    // k + 3 rows, twice (two stages)
    if (k >= 9) return 1;
    if (k >= 8) return tiles < 2 ? tiles : 2;
    if (tiles <= 2) return tiles;
    if (k >= 5) return 3;
    const int pad3 = (tiles + 2) / 3 * 3, pad4 = (tiles + 3) / 4 * 4;
    if (k == 3) return tiles == 4 ? 2 : 3;         // 64 maps: two groups of two tiles, not two groups of three with a third of them empty
    return pad3 <= pad4 ? 3 : 4;
}

// Can this forward layer run in the producer-wave kernel, which is the one that stores its output pooled
// vertically (vpool) and finishes a pending horizontal pool of its input (hd)?
bool conv_h_pool_fusable(int k, int d, int c_out, int c8_in, int Ho, int hd)
{
    if (k != 4 || c_out < 1 || c_out > 48 || d < 1 || hd < 0 || Ho < 1) return false;
    if (CH_TX + 3 * d + hd > 64 * 3) return false;
    const int mt = conv_h_mt(c_out, k);
    if (mt == 1) return ring_smem<4, 1, true, 8, 3, true>(d, c_out, c8_in, Ho, hd) <= 160 * 1024;
    if (mt == 2) return ring_smem<4, 2, true, 8, 3, true>(d, c_out, c8_in, Ho, hd) <= 160 * 1024;
    return ring_smem<4, 3, true, 8, 3, true>(d, c_out, c8_in, Ho, hd) <= 160 * 1024;
}

// widest staged tile: the 4x4 and smaller kernels three 64-unit groups per row, the larger ones (register-staged
// kernel only) four
static int conv_h_tile_width(int k, int d) { return CH_TX + ((k >= 4 ? 4 * ((k + 3) / 4) : k) - 1) * d; }

bool conv_h_supported(int k, int d)
{
    if (k >= 1 && k <= 4) return conv_h_tile_width(k, d) <= 64 * CH_VU;
    return (k == 5 || k == 6 || k == 7 || k == 8 || k == 10) && d >= 1 && conv_h_tile_width(k, d) <= 64 * 4;
}

// ... and the two-stage tile of the register-staged kernel (what every shape can fall back to) fits
// the LDS for a GEMM with gemm_m output maps: a 3x3 kernel with 48 maps or more stops at d = 6
bool conv_h_supported(int k, int d, int gemm_m)
{
    if (!conv_h_supported(k, d) || gemm_m < 1) return false;
    const int mt = conv_h_mt(gemm_m, k);
    const bool map4 = k >= 4;
    const int R = k == 4 && mt <= 3 ? 8 : 4, RR = R + k - 1, OC = map4 ? 1 : 4, CS = map4 ? (k + 3) / 4 : k;
    const long PW = conv_h_tile_width(k, d);
    const long stage = OC * RR * PW + (long)CS * k * mt * 64;
    const long m_tiles_all = ((gemm_m + 15) / 16 + mt - 1) / mt * mt;
    return 2 * stage * 16 + m_tiles_all * 64 <= 160 * 1024;
}

// ------------------------------------------------------------------------------------------------
// First layer of a net on a one-map image (k = 4: 16 taps): HBM-write-bound -- 2 bytes read and 2 * c_out written per
// pixel -- so it gets a kernel built for the stores instead of the ring kernel's tile machinery.  The 16 taps of the
// single input map ARE the K dimension of one MFMA 16x16x32 (lane groups 0 and 1 carry taps 0..7 and 8..15, groups 2 and
// 3 zeros), so 16 pixels x 16 output maps cost one MFMA.  A workgroup of four waves takes 64 columns x rb rows: the
// input tile (one 16-bit sample per pixel) goes to LDS once; a wave takes all 64 columns of rb / 4 rows.  The MFMA leaves
// a lane with four maps of one pixel; the wave passes its row through LDS so that lane L holds the whole octets of pixel
// L and every store instruction writes 1 KB of consecutive addresses per octet plane (the 8-byte halves of 16-pixel
// groups the other kernels store reach about half the rate on a layer that does nothing but store).  With VP (the
// vertical half of the SK pool that follows, kernel stride 1; ReLU required, so the 16-bit patterns order like the
// values) a wave computes one row more, keeps the previous row's packed values and stores max(Y[y], Y[y + 1]).
constexpr int C1_TX = 64;

template <int DT, int MT, bool VP>
__global__ __launch_bounds__(256) void conv_c1_h_kernel(ConvHArgs a, int xtiles, int ytiles, int pitch, int rb)
{
    extern __shared__ uint4v c1_smem[];
    const int KS = a.k, d = a.d, halo = (KS - 1) * d;
    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int xt = blockIdx.x % xtiles, rest = blockIdx.x / xtiles, yt = rest % ytiles, b = rest / ytiles;
    const int x0 = xt * C1_TX, y0 = yt * rb;
    int nrows = a.Ho - y0;                                          // convolution rows of this tile
    nrows = nrows < rb + (VP ? 1 : 0) ? nrows : rb + (VP ? 1 : 0);
    const int in_rows = nrows + halo;
    // LDS: per wave 2 * MT octet planes x 64 pixels x 16 bytes for the row exchange, then the input tile
    char *xch = reinterpret_cast<char *>(c1_smem) + wave * (2 * MT * 64 * 16);
    unsigned short *tile = reinterpret_cast<unsigned short *>(reinterpret_cast<char *>(c1_smem) + 4 * (2 * MT * 64 * 16));

    // input tile: map 0 of the octet at every pixel (addresses clamped into the image: such samples only reach
    // outputs that are not stored)
    const unsigned *xin = static_cast<const unsigned *>(a.x) + (long)b * a.H * a.W * 4;
    const float *img = a.img ? a.img + (long)b * a.img_h * a.img_w : nullptr;
    auto mirror = [&](int t, int len) {
        if (len == 1) return 0;
        const int period = a.pad_mode == 0 ? 2 * (len - 1) : 2 * len;
        t %= period;
        if (t < 0) t += period;
        return t < len ? t : (a.pad_mode == 0 ? period - t : period - 1 - t);
    };
    for (int idx = tid; idx < in_rows * pitch; idx += 256) {
        const int r = idx / pitch, c = idx - r * pitch;
        int gy = y0 + r, gx = x0 + c;
        gy = gy < a.H ? gy : a.H - 1;
        gx = gx < a.W ? gx : a.W - 1;
        if (img)                                                    // the caller's image, mirror-padded and rounded here
            tile[idx] = H<DT>::cvt(img[(long)mirror(gy - a.pad_top, a.img_h) * a.img_w + mirror(gx - a.pad_left, a.img_w)]);
        else
            tile[idx] = (unsigned short)(xin[((long)gy * a.W + gx) * 4] & 0xffffu);
    }
    // A fragments from the packed weights ([kernel row i][map tile][lane group = kernel column j][map][channel]): this
    // lane's K values are taps 8g .. 8g + 7 of map 16 mt + l16, channel 0
    const unsigned short *wp = static_cast<const unsigned short *>(a.wp);
    uint4v af[MT];
    int toff[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int t = 8 * g + e, i = t / KS, j = t - i * KS;
        toff[e] = t < KS * KS ? i * d * pitch + j * d : 0;
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        unsigned short v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int t = 8 * g + e, i = t / KS, j = t - i * KS;
            v[e] = t < KS * KS ? wp[(((long)i * MT + mt) * 64 + j * 16 + l16) * 8] : (unsigned short)0;
        }
        af[mt] = uint4v{v[0] | ((unsigned)v[1] << 16), v[2] | ((unsigned)v[3] << 16), v[4] | ((unsigned)v[5] << 16), v[6] | ((unsigned)v[7] << 16)};
    }
    float bia[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) bia[mt][r4] = a.bias ? a.bias[mt * 16 + 4 * g + r4] : 0.f;
    __syncthreads();

    const int rw = rb >> 2;                                         // rows of this wave
    const int r_first = wave * rw;
    int r_end = r_first + rw + (VP ? 1 : 0);
    r_end = r_end < nrows ? r_end : nrows;
    const int ox = x0 + lane;
    const bool colok = ox < a.Wo;
    const long plane = (long)a.OH * a.OW;
    uint4v *ybase = static_cast<uint4v *>(a.y) + ((long)b * a.c8_out_total + a.o8_off) * plane + (colok ? ox : 0);
    const bool taps_here = 8 * g < KS * KS;
    uint2v prev[4][MT];
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) prev[ct][mt] = uint2v{0u, 0u};
    for (int r = r_first; r < r_end; ++r) {
        uint4v bf[4];
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) {
            const unsigned short *src = tile + r * pitch + 16 * ct + l16;
            unsigned short v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = taps_here ? src[toff[e]] : (unsigned short)0;
            bf[ct] = uint4v{v[0] | ((unsigned)v[1] << 16), v[2] | ((unsigned)v[3] << 16), v[4] | ((unsigned)v[5] << 16), v[6] | ((unsigned)v[7] << 16)};
        }
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const floatx4 acc = H<DT>::mfma(af[mt], bf[ct], floatx4{0.f, 0.f, 0.f, 0.f});
                float val[4];
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    val[r4] = acc[r4] + bia[mt][r4];
                    if (a.relu) val[r4] = fmaxf(val[r4], 0.f);
                }
                uint2v pk = uint2v{(unsigned)H<DT>::cvt(val[0]) | ((unsigned)H<DT>::cvt(val[1]) << 16),
                                   (unsigned)H<DT>::cvt(val[2]) | ((unsigned)H<DT>::cvt(val[3]) << 16)};
                uint2v out = pk;
                if constexpr (VP) {
                    out = uint2v{pk_max_u16(prev[ct][mt][0], pk[0]), pk_max_u16(prev[ct][mt][1], pk[1])};
                    prev[ct][mt] = pk;
                }
                // this lane's four maps of pixel 16 ct + l16: half (g & 1) of octet 2 mt + (g >> 1)
                *reinterpret_cast<uint2v *>(xch + ((2 * mt + (g >> 1)) * 64 + 16 * ct + l16) * 16 + (g & 1) * 8) = out;
            }
        if (!VP || r > r_first) {                                   // (uniform)
            const int oy = VP ? y0 + r - 1 : y0 + r;
            uint4v oct[2 * MT];
#pragma unroll
            for (int o = 0; o < 2 * MT; ++o) oct[o] = *reinterpret_cast<const uint4v *>(xch + (o * 64 + lane) * 16);
#pragma unroll
            for (int o = 0; o < 2 * MT; ++o)
                if (colok && o < a.c8_out) ybase[(long)o * plane + (long)oy * a.OW] = oct[o];
        }
    }
}

// can (and should) this launch run on conv_c1_h_kernel?
static bool conv_c1_h_applies(const ConvHArgs &a, int mt_packed)
{
    const int m_tiles = (a.c_out + 15) / 16;
    return a.single_map && a.c8_in == 1 && a.k == 4 && a.d >= 1 && 3 * a.d <= 32 && !a.mask && a.in_off == 0 && a.hd == 0 && !a.out_f32 &&
           a.tap_maps == 0 && a.oy_mul == 1 && a.ox_mul == 1 && a.oy_off == 0 && a.ox_off == 0 && !a.xb8 && !a.grp8 && m_tiles <= 3 &&
           mt_packed == m_tiles && (!a.vpool || (a.d == 1 && a.relu && a.OH == a.Ho - 1 && a.OW == a.Wo)) &&
           (a.vpool || (a.OH == a.Ho && a.OW == a.Wo));
}

template <int DT, int MT>
static hipError_t launch_conv_c1_h(const ConvHArgs &a, hipStream_t stream)
{
    const int xtiles = (a.Wo + C1_TX - 1) / C1_TX;
    const int out_rows = a.vpool ? a.Ho - 1 : a.Ho;
    if (out_rows < 1) return hipErrorInvalidValue;
    // rows per workgroup: 32, or fewer where that leaves the GPU short of workgroups (a 512^2 image)
    int rb = 32;
    while (rb > 8 && (long)xtiles * ((out_rows + rb - 1) / rb) * a.n < 8L * device_cus()) rb >>= 1;
    const int ytiles = (out_rows + rb - 1) / rb;
    const int pitch = (C1_TX + 3 * a.d + 2) & ~1;
    const size_t smem = (size_t)4 * 2 * MT * 64 * 16 + sizeof(unsigned short) * (size_t)(rb + 1 + 3 * a.d) * pitch;
    const long blocks = (long)xtiles * ytiles * a.n;
    if (blocks < 1 || blocks > 0x7fffffffL || smem > 48 * 1024) return hipErrorInvalidValue;
    if (a.vpool) hipLaunchKernelGGL((conv_c1_h_kernel<DT, MT, true>), dim3((unsigned)blocks), dim3(256), smem, stream, a, xtiles, ytiles, pitch, rb);
    else hipLaunchKernelGGL((conv_c1_h_kernel<DT, MT, false>), dim3((unsigned)blocks), dim3(256), smem, stream, a, xtiles, ytiles, pitch, rb);
    return hipGetLastError();
}

bool conv_h_reads_image(const ConvHArgs &a)
{
    if (a.img || (a.dtype != 1 && a.dtype != 2) || !conv_h_supported(a.k, a.d)) return false;
    return conv_c1_h_applies(a, a.mt > 0 ? a.mt : conv_h_mt(a.c_out, a.k));
}

hipError_t launch_conv_h(const ConvHArgs &a, hipStream_t stream)
{
    if (!conv_h_supported(a.k, a.d) || a.Ho < 1 || a.Wo < 1 || a.c8_in < 1 || a.c_out < 1) return hipErrorInvalidValue;
    if (a.xb8 < 0 || a.grp8 < 0 || a.skip8 < 0 || (a.grp8 > 0 && a.c8_in % a.grp8 != 0) || (a.grp8 == 0 && a.skip8 != 0)) return hipErrorInvalidValue;
    if ((a.xb8 || a.grp8) && (a.vpool || a.hd)) return hipErrorInvalidValue;      // slices as images: no pool work inside the launch
    if ((a.vpool || a.hd) && (a.mt > 0 && a.mt != conv_h_mt(a.c_out, a.k))) return hipErrorInvalidValue;
    if ((a.vpool || a.hd) && !conv_h_pool_fusable(a.k, a.d, a.c_out, a.c8_in, a.Ho, a.hd)) return hipErrorInvalidValue;
    if (a.tap_maps != 0 && (a.tap_maps < 16 || a.tap_maps % 16 != 0 || a.c_out != 4 * a.tap_maps || a.mask || a.out_f32 || a.oy_mul != 2 ||
                            a.ox_mul != 2 || a.k != 1))
        return hipErrorInvalidValue;
    // 3x3 layers whose weights were packed with the kernel columns on the lane groups (conv_h_pick_mode)
    if (a.mt > 0 && (a.mt & CONV_H_TAPCOLS)) {
        if (a.k != 3 || a.mask || a.in_off || a.vpool || a.hd || a.tap_maps || a.xb8 || a.grp8) return hipErrorInvalidValue;
        ConvHArgs b = a;
        b.mt = a.mt & ~CONV_H_TAPCOLS;
        if (a.dtype == 1) return b.mt == 2 ? launch_conv_h_k3_tapcols<1, 2>(b, stream) : (b.mt == 3 ? launch_conv_h_k3_tapcols<1, 3>(b, stream) : hipErrorInvalidValue);
        if (a.dtype == 2) return b.mt == 2 ? launch_conv_h_k3_tapcols<2, 2>(b, stream) : (b.mt == 3 ? launch_conv_h_k3_tapcols<2, 3>(b, stream) : hipErrorInvalidValue);
        return hipErrorInvalidValue;
    }
    // the packed weights were laid out for this many map tiles per group (0 = the default choice)
    const int mt = a.mt > 0 ? a.mt : conv_h_mt(a.c_out, a.k);
    if (a.img && (!conv_c1_h_applies(a, mt) || a.img_h < 1 || a.img_w < 1 || a.pad_top < 0 || a.pad_left < 0 || (a.pad_mode != 0 && a.pad_mode != 1)))
        return hipErrorInvalidValue;                                // only that kernel reads the image
    if (conv_c1_h_applies(a, mt)) {
        if (a.dtype == 1) return mt == 1 ? launch_conv_c1_h<1, 1>(a, stream) : (mt == 2 ? launch_conv_c1_h<1, 2>(a, stream) : launch_conv_c1_h<1, 3>(a, stream));
        if (a.dtype == 2) return mt == 1 ? launch_conv_c1_h<2, 1>(a, stream) : (mt == 2 ? launch_conv_c1_h<2, 2>(a, stream) : launch_conv_c1_h<2, 3>(a, stream));
    }
    if (mt > 4 || (a.k == 3 && mt > 3)) return hipErrorInvalidValue;
    if (a.k > 4 && !conv_h_supported(a.k, a.d, a.c_out)) return hipErrorInvalidValue;
    if (a.dtype == 1) {
        switch (mt) {
        case 1: return launch_conv_h_mt<1, 1>(a, stream);
        case 2: return launch_conv_h_mt<1, 2>(a, stream);
        case 3: return launch_conv_h_mt<1, 3>(a, stream);
        default: return launch_conv_h_mt<1, 4>(a, stream);
        }
    }
    if (a.dtype == 2) {
        switch (mt) {
        case 1: return launch_conv_h_mt<2, 1>(a, stream);
        case 2: return launch_conv_h_mt<2, 2>(a, stream);
        case 3: return launch_conv_h_mt<2, 3>(a, stream);
        default: return launch_conv_h_mt<2, 4>(a, stream);
        }
    }
    return hipErrorInvalidValue;
}

// ------------------------------------------------------------------------------------------------
// Weight packing for conv_h_kernel.  The packed array is a sequence of 1 KB MFMA A fragments,
//   [mgroup][chunk][column step cs][kernel row i][m-tile mt][lane group g][l16][e = 0..7]
// with element = W[o][c][i][j] (forward) where o = (mgroup*MT + mt)*16 + l16 and
//   MAP4 (k >= 4): c = chunk*8 + e,           j = 4*cs + g (zero for j >= k)
//   otherwise   : c = (chunk*4 + g)*8 + e,    j = cs
// flip_transpose = 1 builds the data-gradient operator instead: the roles of input and output maps
// are swapped and both taps are mirrored (element = W[c][o][k-1-i][k-1-j]).
// Entries whose o or c lie beyond the real extents are zero.
template <int DT>
__device__ __forceinline__ void pack_weights_h_body(const float *w, unsigned short *wp, int c_out, int c_in, int k, int flip_transpose,
                                                    int mt_per_group, int map4, int gemm_m, int gemm_c8, long total)
{
    const int OC = map4 ? 1 : 4, CS = map4 ? (k + 3) / 4 : k;
    const int nchunks = (gemm_c8 + OC - 1) / OC;
    for (long q = blockIdx.x * (long)blockDim.x + threadIdx.x; q < total; q += (long)gridDim.x * blockDim.x) {
        long r = q;
        const int e = (int)(r % 8); r /= 8;
        const int l16 = (int)(r % 16); r /= 16;
        const int g = (int)(r % 4); r /= 4;
        const int mt = (int)(r % mt_per_group); r /= mt_per_group;
        const int i = (int)(r % k); r /= k;
        const int cs = (int)(r % CS); r /= CS;
        const int ch = (int)(r % nchunks); r /= nchunks;
        const int mg = (int)r;
        const int m = (mg * mt_per_group + mt) * 16 + l16;          // GEMM output map
        const int c = map4 ? ch * 8 + e : (ch * 4 + g) * 8 + e;     // GEMM input map
        const int j = map4 ? 4 * cs + g : cs;
        float v = 0.f;
        if (m < gemm_m && c < gemm_c8 * 8 && j < k) {
            if (!flip_transpose) {
                if (m < c_out && c < c_in) v = w[(((long)m * c_in + c) * k + i) * k + j];
            } else {
                if (c < c_out && m < c_in) v = w[(((long)c * c_in + m) * k + (k - 1 - i)) * k + (k - 1 - j)];
            }
        }
        wp[q] = H<DT>::cvt(v);
    }
}

template <int DT>
__global__ void pack_weights_h_kernel(const float *w, unsigned short *wp, int c_out, int c_in, int k, int flip_transpose,
                                      int mt_per_group, int map4, int gemm_m, int gemm_c8, long total)
{
    pack_weights_h_body<DT>(w, wp, c_out, c_in, k, flip_transpose, mt_per_group, map4, gemm_m, gemm_c8, total);
}

struct PackHJobDev { const float *w; unsigned short *wp; int c_out, c_in, k, flip_transpose, mt, map4, gemm_m, gemm_c8; long total; };
// Batched packing through LDS.  One workgroup builds the fragments of one (map tile, chunk): it reads the slab of
// W they come from -- 16 maps x (8 or 32) input maps x k*k taps, runs of whole rows of W, consecutive threads on
// consecutive floats -- into LDS (zero where the maps end), and writes each 16-byte unit (eight input maps of one
// row of a fragment) with one store.  Workgroups are dealt out over the jobs in proportion to their tile counts
// (start[t] = first workgroup of job t).
struct PackHJobs { PackHJobDev job[BATCH_MAX]; int start[BATCH_MAX + 1]; int n; };

template <int DT>
__global__ void __launch_bounds__(256) pack_weights_h_batch_kernel(PackHJobs b)
{
    extern __shared__ float pack_slab[];
    int t = 0;
    while (t + 1 < b.n && (int)blockIdx.x >= b.start[t + 1]) ++t;
    const PackHJobDev &jb = b.job[t];
    const int k = jb.k, k2 = k * k, MT = jb.mt, map4 = jb.map4, flip = jb.flip_transpose;
    const int OC = map4 ? 1 : 4, CS = map4 ? (k + 3) / 4 : k, nchunks = (jb.gemm_c8 + OC - 1) / OC, Cc = 8 * OC;
    const int lb = (int)blockIdx.x - b.start[t], mtile = lb / nchunks, ch = lb - mtile * nchunks;
    const int m0 = mtile * 16, c0 = ch * Cc;                  // first GEMM output map / GEMM input map of the slab
    // forward: slab[ml][cl*k2 + tap] = W[m0+ml][c0+cl][tap]; data-gradient operator: slab[cl][ml*k2 + tap] =
    // W[c0+cl][m0+ml][tap] -- in both cases the order the floats have in W; rows one float apart from a multiple of
    // the bank count
    const int run = (flip ? 16 : Cc) * k2, rows = flip ? Cc : 16, row_lim = jb.c_out, col0 = flip ? m0 : c0;
    const int row0 = flip ? c0 : m0;
    for (int s = threadIdx.x; s < rows * run; s += 256) {
        const int r = s / run, rem = s - r * run, cc = rem / k2;
        float v = 0.f;
        if (row0 + r < row_lim && col0 + cc < jb.c_in) v = jb.w[((long)(row0 + r) * jb.c_in + col0) * k2 + rem];
        pack_slab[r * (run + 1) + rem] = v;
    }
    __syncthreads();
    const int units = CS * k * 64;
    const long frag0 = (((long)(mtile / MT) * nchunks + ch) * CS * k) * MT + mtile % MT;
    for (int u = threadIdx.x; u < units; u += 256) {
        const int l16 = u & 15, g = (u >> 4) & 3, ci = u >> 6, cs = ci / k, i = ci - cs * k;
        const int j = map4 ? 4 * cs + g : cs;
        unsigned short h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int cl = map4 ? e : g * 8 + e;
            float v = 0.f;
            if (j < k) v = flip ? pack_slab[cl * (run + 1) + l16 * k2 + (k - 1 - i) * k + (k - 1 - j)] : pack_slab[l16 * (run + 1) + cl * k2 + i * k + j];
            h[e] = H<DT>::cvt(v);
        }
        uint4v out = {(unsigned)h[0] | ((unsigned)h[1] << 16), (unsigned)h[2] | ((unsigned)h[3] << 16),
                      (unsigned)h[4] | ((unsigned)h[5] << 16), (unsigned)h[6] | ((unsigned)h[7] << 16)};
        *reinterpret_cast<uint4v *>(jb.wp + (frag0 + (long)ci * MT) * 512 + (g * 16 + l16) * 8) = out;
    }
}

// size in 16-bit elements of the packing of a GEMM with gemm_m output maps and gemm_c8 input octets
// Map tiles per workgroup for a forward layer with this output size.  Many maps on a small image (the
// deep U-Net levels): with one persistent workgroup per CU a layer wants at least about 160 tiles, and
// fewer map tiles per workgroup give more of them (each then re-reads the input, so not more than needed).  The weights must be packed for the same value.
int conv_h_pick_mt(int c_out, int k, int n, int Ho, int Wo)
{
    int mt = conv_h_mt(c_out, k);
    const long sp = (long)((Wo + CH_TX - 1) / CH_TX) * ((Ho + 3) / 4) * n;   // tiles of 4 rows at least
    const int m_tiles = (c_out + 15) / 16;
    while (mt > 1 && sp * ((m_tiles + mt - 1) / mt) < 160) --mt;   // measured on the U-Net: 96..160 best, 256 worse
    return mt;
}

long packed_h_elems(int gemm_m, int gemm_c8, int k, int mt)
{
    const bool tapcols = mt > 0 && (mt & CONV_H_TAPCOLS) != 0;
    if (mt > 0) mt &= ~CONV_H_TAPCOLS;
    if (mt <= 0) mt = conv_h_mt(gemm_m, k);
    const int m_tiles = (gemm_m + 15) / 16, mgroups = (m_tiles + mt - 1) / mt;
    const bool map4 = k >= 4 || tapcols;
    const int OC = map4 ? 1 : 4, CS = map4 ? (k + 3) / 4 : k;
    const int nchunks = (gemm_c8 + OC - 1) / OC;
    return (long)mgroups * nchunks * CS * k * mt * 512;
}

hipError_t launch_pack_weights_h(const float *w_oihw, void *wp, int dtype, int c_out, int c_in, int k,
                                 int flip_transpose, int mt, hipStream_t stream)
{
    const int gemm_m = flip_transpose ? c_in : c_out;
    const int gemm_c8 = ((flip_transpose ? c_out : c_in) + 7) / 8;
    const int map4 = (k >= 4 || (mt > 0 && (mt & CONV_H_TAPCOLS))) ? 1 : 0;
    const long total = packed_h_elems(gemm_m, gemm_c8, k, mt);
    if (mt > 0) mt &= ~CONV_H_TAPCOLS;
    if (mt <= 0) mt = conv_h_mt(gemm_m, k);
    const int blocks = (int)((total + 255) / 256 < 2048 ? (total + 255) / 256 : 2048);
    if (dtype == 1)
        hipLaunchKernelGGL(pack_weights_h_kernel<1>, dim3(blocks), dim3(256), 0, stream, w_oihw,
                           static_cast<unsigned short *>(wp), c_out, c_in, k, flip_transpose, mt, map4, gemm_m, gemm_c8, total);
    else
        hipLaunchKernelGGL(pack_weights_h_kernel<2>, dim3(blocks), dim3(256), 0, stream, w_oihw,
                           static_cast<unsigned short *>(wp), c_out, c_in, k, flip_transpose, mt, map4, gemm_m, gemm_c8, total);
    return hipGetLastError();
}

hipError_t launch_pack_weights_h_batch(const PackHJob *jobs, int n, int dtype, hipStream_t stream)
{
    if (n < 1 || n > BATCH_MAX || (dtype != 1 && dtype != 2)) return hipErrorInvalidValue;
    PackHJobs b;
    long blocks = 0;
    size_t smem = 0;
    for (int t = 0; t < n; ++t) {
        const PackHJob &j = jobs[t];
        PackHJobDev &o = b.job[t];
        o.w = j.w; o.wp = static_cast<unsigned short *>(j.wp);
        o.c_out = j.c_out; o.c_in = j.c_in; o.k = j.k; o.flip_transpose = j.flip_transpose;
        o.gemm_m = j.flip_transpose ? j.c_in : j.c_out;
        o.gemm_c8 = ((j.flip_transpose ? j.c_out : j.c_in) + 7) / 8;
        o.map4 = (j.k >= 4 || (j.mt > 0 && (j.mt & CONV_H_TAPCOLS))) ? 1 : 0;
        o.total = packed_h_elems(o.gemm_m, o.gemm_c8, j.k, j.mt);
        o.mt = j.mt > 0 ? (j.mt & ~CONV_H_TAPCOLS) : 0;
        if (o.mt <= 0) o.mt = conv_h_mt(o.gemm_m, j.k);
        const int OC = o.map4 ? 1 : 4, CS = o.map4 ? (j.k + 3) / 4 : j.k, nchunks = (o.gemm_c8 + OC - 1) / OC;
        const long tiles = o.total / ((long)CS * j.k * 512);                 // (map tiles of all groups) x chunks
        if (tiles % nchunks != 0) return hipErrorInvalidValue;
        smem = std::max(smem, sizeof(float) * (16 * 8 * OC * j.k * j.k + 32));
        b.start[t] = (int)blocks;
        blocks += tiles;
        if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    }
    for (int t = n; t <= BATCH_MAX; ++t) b.start[t] = (int)blocks;
    b.n = n;
    if (blocks == 0) return hipSuccess;
    if (smem > 64 * 1024) {
        // kernels too large for the slab: one plain launch per job
        for (int t = 0; t < n; ++t) {
            const hipError_t e = launch_pack_weights_h(jobs[t].w, jobs[t].wp, dtype, jobs[t].c_out, jobs[t].c_in, jobs[t].k, jobs[t].flip_transpose,
                                                       jobs[t].mt, stream);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    if (dtype == 1) hipLaunchKernelGGL(pack_weights_h_batch_kernel<1>, dim3((unsigned)blocks), dim3(256), smem, stream, b);
    else hipLaunchKernelGGL(pack_weights_h_batch_kernel<2>, dim3((unsigned)blocks), dim3(256), smem, stream, b);
    return hipGetLastError();
}

}  // namespace sk
