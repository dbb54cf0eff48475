// One residual block per launch for the layer-by-layer ResNet path (model-size variants of Sections 4.1 / 4.2):
//   x' = x + conv_b(ReLU(conv_a(ReLU(x))))        3x3 SAME, C -> C, bf16 MFMA operands, fp32 x and accumulators.
// Run as two separate convolutions a block moves the fp32 residual stream through HBM twice and the bf16 maps R
// and U four times; here a workgroup takes a TH x TW tile of one image, stages ReLU(x) of the tile plus a two-pixel
// halo in LDS, computes U = ReLU(conv_a) on the tile plus a one-pixel halo into LDS (zero where that lies
// outside the image: conv_b's SAME padding), then conv_b on the tile, adds x and writes x' (and / or its bf16
// copy): HBM sees x once in and once out.  The halo of U is recomputed by neighbouring tiles ((TH + 2)(TW + 2) /
// (TH TW) of conv_a's work).
//
// Both convolutions are implicit GEMMs over planar LDS maps [C/8][rows][pitch][8 bf16] with the weight packing
// of conv3x3_lds_kernel (A fragments [feature tile][chunk][lane][8], k = tap * C + ci, fetched from global
// memory three chunks ahead).  A region's pixels are cut row-major into tiles of 16 (or, `flat`, the region is
// walked as wide as its map and a tile is 16 consecutive cells); wavefront w takes feature tiles FTW * (w % NFG) ...
// and every NPG-th pixel tile from w / NFG, at most TPW of them.
//
// What set the time, in the order it was found (1024 images, 32 channels on 36 x 48): the weight fragments one
// chunk ahead (each chunk waited out a trip to L2: 260 -> 230 us with three ahead), the staging loop's loads
// one round at a time (280 -> 260), and tiles whose maps fill LDS so that one workgroup per compute unit
// loads, multiplies and stores in turn (230 -> 175 with tiles for two), a test per pixel tile inside a chunk of the
// convolution loop (rb_conv_n), and a division per (pixel tile, feature tile) in the epilogues (tile_coords: 172 ->
// 156; the vector ALU, not the matrix pipe, was the busiest unit of these kernels).  At 64 and 128 channels the kernel is
// bound by operand delivery: with two feature tiles per wavefront the weight fragments fill the vector L1's
// bandwidth (16 wavefronts x 2 KiB per chunk) and the map fragments most of LDS's.
#pragma once
#include "bf16_common.h"

namespace seedinf {

struct ResBlockArgs {
    const float* x_in;                 // [B, H, W, C] fp32 residual stream
    const bf16x8* wpa; const bf16x8* wpb;
    const float* bias_a; const float* bias_b;
    float* x_out;                      // fp32 x' [B, H, W, C], or nullptr; must not alias x_in (tiles read each other's halos)
    __bf16* y;                         // bf16 copy of x', or nullptr
    int y_relu;                        // rectify y
    int ldy;                           // 0: y is NHWC; > 0: y is the feature matrix [B, ldy], (h, w, c) order
    int B, H, W, TH, TW, tiles_y, tiles_x, kchunks;
    int flat;                          // walk the regions as wide as their maps (see resblock_fused_kernel)
};

constexpr int RB_THREADS = 512, RB_TPW = 6;
constexpr size_t RB_LDS_MAX = 128 * 1024;

template <int C>
struct ResBlockCfg {
    static_assert(C % 16 == 0 && C <= 128, "channels: a multiple of 16 up to 128");
    static constexpr int NCG = C / 8, NFT = C / 16;
    static constexpr int FTW = NFT % 2 == 0 ? 2 : 1;        // feature tiles a wavefront multiplies with one fragment
    static constexpr int NFG = NFT / FTW;                   // feature groups
    static_assert(8 % NFG == 0, "feature groups must divide the eight wavefronts");
    static constexpr int NPG = 8 / NFG;                     // wavefronts (pixel groups) per feature group
    static constexpr int MAX_PIX = 16 * RB_TPW * NPG;       // pixels of conv_a's region a workgroup can take
    // cells of a map plane, in whole 256 bytes; walked flat, the last tile's taps reach two cells past the map
    __host__ __device__ static constexpr int plane(int rows, int pitch, bool flat) { return (rows * pitch + (flat ? 2 : 0) + 15) / 16 * 16; }
    static size_t lds_bytes(int TH, int TW, bool flat) { return (size_t)NCG * (plane(TH + 4, TW + 4, flat) + plane(TH + 2, TW + 2, flat)) * 16; }
    // tile extents for an H x W map: the cheapest cut whose conv_a region fits a workgroup and whose maps fit LDS
    static bool choose(int H, int W, bool flat, int& TH, int& TW)
    {
        const int ea = flat ? 4 : 2, eb = flat ? 2 : 0;           // columns walked beyond the tile: conv_a's region, conv_b's
        long best = -1;
        for (int ny = 1; ny <= H; ++ny) {
            const int th = (H + ny - 1) / ny;
            for (int nx = 1; nx <= W; ++nx) {
                const int tw = (W + nx - 1) / nx;
                if ((th + 2) * (tw + ea) > MAX_PIX || lds_bytes(th, tw, flat) > RB_LDS_MAX) continue;
                // cost: the pixels both convolutions compute over all tiles (halo recomputation); half as much
                // again when the maps leave no room for a second workgroup on the compute unit, whose MFMAs
                // would run under this one's loads and stores
                long cost = (long)ny * nx * ((th + 2) * (tw + ea) + th * (tw + eb));
                if (lds_bytes(th, tw, flat) > 80 * 1024) cost += cost / 2;
                if (best < 0 || cost < best) { best = cost; TH = th; TW = tw; }
            }
        }
        return best >= 0;
    }
};

// Region coordinates (row, column) of the lane's pixel in the pixel tiles first, first + stride, ... of a
// region RW pixels wide (a tile is 16 consecutive pixels of the row-major region, the lane's is pixel n of it): one
// division for the first tile, then steps whose sizes are uniform.  A division per tile and feature tile was half
// of the vector instructions of these kernels' epilogues, and those - not the MFMAs - fill most of their time.
template <int NTILE>
__device__ __forceinline__ void tile_coords(int first, int stride, int n, int RW, int (&r)[NTILE], int (&c)[NTILE])
{
    const int q0 = first * 16 + n;
    r[0] = q0 / RW;
    c[0] = q0 - r[0] * RW;
    const int step = stride * 16, dr = step / RW, dc = step - dr * RW;
#pragma unroll
    for (int i = 1; i < NTILE; ++i) {
        const bool wrap = c[i - 1] + dc >= RW;
        c[i] = c[i - 1] + dc - (wrap ? RW : 0);
        r[i] = r[i - 1] + dr + (wrap ? 1 : 0);
    }
}

// One implicit-GEMM pass, CIN -> COUT channels: region of RW-wide pixels (npix of them) over the planar map `src`
// (plane cells PL, pitch PITCH; a region pixel (r, c) has its tap (0, 0) at cell r * PITCH + c).  acc[i][j]: pixel
// tile pg + NPG * i, feature tile ft0 + j.
//
// rb_conv_n is the loop for a wavefront that owns exactly NT pixel tiles: with the count a constant a chunk is one
// straight run - NT map fragments requested, then NT * FTW MFMAs, each waiting only for its own fragment - where
// a test per tile ("does this wavefront have an i-th tile?") cuts the chunk into NT blocks of load, wait, multiply,
// and every fragment's LDS latency is paid in full.
template <int CIN, int COUT, int TPW, int NT>
__device__ __forceinline__ void rb_conv_n(const char* src, int PL, int PITCH, const int (&base)[TPW], const bf16x8* __restrict__ wl,
                                          int kchunks, int g, floatx4 (&acc)[TPW][ResBlockCfg<COUT>::FTW])
{
    using K = ResBlockCfg<COUT>;
    constexpr int C = CIN;
    // weight fragments run AHEAD chunks ahead of their use: they come from L2 (the first wavefront to ask) or the
    // vector L1, and one chunk of MFMAs is shorter than either trip
    constexpr int AHEAD = COUT == 16 ? 1 : 3;                  // measured at 16 channels (54 x 72): 150 us with 1, 178 with 3, 186 with all 5
    bf16x8 a[AHEAD][K::FTW];
#pragma unroll
    for (int d = 0; d < AHEAD; ++d)
#pragma unroll
        for (int j = 0; j < K::FTW; ++j) a[d][j] = wl[((size_t)j * kchunks + min(d, kchunks - 1)) * 64];
    for (int kc0 = 0; kc0 < kchunks; kc0 += AHEAD) {
#pragma unroll
        for (int d = 0; d < AHEAD; ++d) {
            const int kc = kc0 + d;
            if (kc >= kchunks) break;                           // uniform
            bf16x8 cur[K::FTW];
#pragma unroll
            for (int j = 0; j < K::FTW; ++j) cur[j] = a[d][j];
            const int kn = min(kc + AHEAD, kchunks - 1);
#pragma unroll
            for (int j = 0; j < K::FTW; ++j) a[d][j] = wl[((size_t)j * kchunks + kn) * 64];
            // the lane's 8 consecutive k of this chunk: one tap, one channel group (k past 9 C has zero weights: any cell)
            const int k0 = kc * 32 + g * 8;
            const int tap = min(k0 / C, 8), cg = (k0 % C) >> 3;
            const char* s = src + ((size_t)cg * PL + (tap / 3) * PITCH + tap % 3) * 16;
            bf16x8 bfr[NT];
#pragma unroll
            for (int i = 0; i < NT; ++i) bfr[i] = *(const bf16x8*)(s + base[i] * 16);
#pragma unroll
            for (int i = 0; i < NT; ++i)
#pragma unroll
                for (int j = 0; j < K::FTW; ++j) acc[i][j] = mfma16(cur[j], bfr[i], acc[i][j]);
        }
    }
}

template <int CIN, int COUT, int TPW = RB_TPW>
__device__ __forceinline__ void rb_conv(const char* src, int PL, int PITCH, int RW, int npix, const bf16x8* __restrict__ wp,
                                        int kchunks, int ft0, int pg, int lane, floatx4 (&acc)[TPW][ResBlockCfg<COUT>::FTW])
{
    using K = ResBlockCfg<COUT>;
    const int g = lane >> 4, n = lane & 15;
    const int ntiles = (npix + 15) / 16;
    int base[TPW], pr[TPW], pc[TPW];
    tile_coords<TPW>(pg, K::NPG, n, RW, pr, pc);
    const int last = ((npix - 1) / RW) * PITCH + (npix - 1) % RW;          // uniform: pixels past the region read its last one
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        base[i] = (pg + K::NPG * i) * 16 + n < npix ? pr[i] * PITCH + pc[i] : last;
#pragma unroll
        for (int j = 0; j < K::FTW; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
    const bf16x8* wl = wp + (size_t)ft0 * kchunks * 64 + lane;
    const int nt = min(max((ntiles - pg + K::NPG - 1) / K::NPG, 0), TPW);      // this wavefront's tiles (uniform)
    static_assert(TPW <= 8, "tile counts up to eight");
    switch (nt) {
    case 1: rb_conv_n<CIN, COUT, TPW, 1>(src, PL, PITCH, base, wl, kchunks, g, acc); break;
    case 2: rb_conv_n<CIN, COUT, TPW, 2>(src, PL, PITCH, base, wl, kchunks, g, acc); break;
    case 3: rb_conv_n<CIN, COUT, TPW, TPW >= 3 ? 3 : TPW>(src, PL, PITCH, base, wl, kchunks, g, acc); break;
    case 4: rb_conv_n<CIN, COUT, TPW, TPW >= 4 ? 4 : TPW>(src, PL, PITCH, base, wl, kchunks, g, acc); break;
    case 5: rb_conv_n<CIN, COUT, TPW, TPW >= 5 ? 5 : TPW>(src, PL, PITCH, base, wl, kchunks, g, acc); break;
    case 6: rb_conv_n<CIN, COUT, TPW, TPW >= 6 ? 6 : TPW>(src, PL, PITCH, base, wl, kchunks, g, acc); break;
    case 7: rb_conv_n<CIN, COUT, TPW, TPW >= 7 ? 7 : TPW>(src, PL, PITCH, base, wl, kchunks, g, acc); break;
    case 8: rb_conv_n<CIN, COUT, TPW, TPW >= 8 ? 8 : TPW>(src, PL, PITCH, base, wl, kchunks, g, acc); break;
    default: break;
    }
}

template <int C>
__global__ __launch_bounds__(RB_THREADS, 4) void resblock_fused_kernel(ResBlockArgs p)
{
    using K = ResBlockCfg<C>;
    extern __shared__ __attribute__((aligned(16))) char rb_lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, n = lane & 15;
    const int tiles = p.tiles_y * p.tiles_x;
    const int b = blockIdx.x / tiles, t = blockIdx.x % tiles;
    const int y0 = (t / p.tiles_x) * p.TH, x0 = (t % p.tiles_x) * p.TW;
    const int RP = p.TW + 4, RPL = K::plane(p.TH + 4, RP, p.flat != 0);          // ReLU(x): tile + 2
    const int UP = p.TW + 2, UPL = K::plane(p.TH + 2, UP, p.flat != 0);          // U: tile + 1
    char* Rm = rb_lds;
    char* Um = rb_lds + (size_t)K::NCG * RPL * 16;
    const float* ximg = p.x_in + (size_t)b * p.H * p.W * C;

    // ---- R = ReLU(x) as bf16, zeros outside the image ----
    // four items' loads are issued before the first is converted: one after the other, the rounds of this loop
    // each wait out a trip to memory and the staging, not the bandwidth, sets the kernel's time
    const int rcells = (p.TH + 4) * RP;
    constexpr int UNR = 4;
    static_assert(RB_THREADS % K::NCG == 0, "a thread keeps its channel group");
    constexpr int CSTEP = RB_THREADS / K::NCG;
    const int cg = tid % K::NCG;                                           // a pixel's channel groups are adjacent in memory
    RowWalk rw(tid / K::NCG, CSTEP, RP);
    for (int cell0 = tid / K::NCG; cell0 < rcells; cell0 += UNR * CSTEP) {
        floatx4 lo[UNR], hi[UNR];
        int at[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int cell = cell0 + u * CSTEP;
            const int r = rw.r, c = rw.c;
            rw.next();
            const int gy = y0 - 2 + r, gx = x0 - 2 + c;
            at[u] = cell < rcells ? (cg * RPL + cell) * 16 : -1;
            lo[u] = hi[u] = floatx4{0.f, 0.f, 0.f, 0.f};
            if (at[u] >= 0 && gy >= 0 && gy < p.H && gx >= 0 && gx < p.W) {
                const float* s = ximg + ((size_t)gy * p.W + gx) * C + cg * 8;
                lo[u] = *(const floatx4*)s;
                hi[u] = *(const floatx4*)(s + 4);
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            if (at[u] < 0) continue;
            const bf16x8 raw = to_bf16x8(lo[u], hi[u]);
            const bf16x4 l = relu_bf16x4(__builtin_shufflevector(raw, raw, 0, 1, 2, 3));
            const bf16x4 h = relu_bf16x4(__builtin_shufflevector(raw, raw, 4, 5, 6, 7));
            *(bf16x8*)(Rm + at[u]) = __builtin_shufflevector(l, h, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    }
    __syncthreads();

    const int fg = wave % K::NFG, pg = wave / K::NFG;
    const int ft0 = fg * K::FTW;
    floatx4 acc[RB_TPW][K::FTW];

    // ---- U = ReLU(conv_a(R) + bias) on the tile + 1, zero outside the image ----
    {
        // `flat`: the region is walked as wide as the map (RP columns, the last two of each row computed and
        // dropped): a tile is then 16 consecutive cells - 256 distinct bank bytes, the full LDS rate - where 16
        // row-major pixels of an 18-wide region wrap rows two cells apart and read at 57 %.  It pays where the map
        // fragments bound the kernel (64 channels on 36 x 48: 552 -> 502 us at 1024 images) and costs its extra
        // columns elsewhere (128 channels: 305 -> 320; 16 channels: 149 -> 160), so the host decides.
        const int UW = p.flat ? RP : p.TW + 2, npix = (p.TH + 2) * UW;
        rb_conv<C, C>(Rm, RPL, RP, UW, npix, p.wpa, p.kchunks, ft0, pg, lane, acc);
        int er[RB_TPW], ec[RB_TPW];
        tile_coords<RB_TPW>(pg, K::NPG, n, UW, er, ec);
        floatx4 bva[K::FTW];
#pragma unroll
        for (int j = 0; j < K::FTW; ++j) bva[j] = *(const floatx4*)(p.bias_a + (ft0 + j) * 16 + g * 4);
#pragma unroll
        for (int i = 0; i < RB_TPW; ++i) {
            const int q = (pg + K::NPG * i) * 16 + n;
            const int r = er[i], c = ec[i];
            if (q >= npix || c >= p.TW + 2) continue;
            const int gy = y0 - 1 + r, gx = x0 - 1 + c;
            const bool inside = gy >= 0 && gy < p.H && gx >= 0 && gx < p.W;
            char* cell = Um + (r * UP + c) * 16 + (g & 1) * 8;
#pragma unroll
            for (int j = 0; j < K::FTW; ++j) {
                const int f = (ft0 + j) * 16 + g * 4;
                bf16x4 o = {};
                if (inside) o = relu_bf16x4(to_bf16x4(acc[i][j] + bva[j]));
                *(bf16x4*)(cell + (f >> 3) * UPL * 16) = o;
            }
        }
    }
    __syncthreads();

    // ---- x' = x + conv_b(U) + bias on the tile ----
    {
        const int BW = p.flat ? UP : p.TW, npix = p.TH * BW;
        rb_conv<C, C>(Um, UPL, UP, BW, npix, p.wpb, p.kchunks, ft0, pg, lane, acc);
        const int hw = p.H * p.W;
        int er[RB_TPW], ec[RB_TPW];
        tile_coords<RB_TPW>(pg, K::NPG, n, BW, er, ec);
        floatx4 bvb[K::FTW];
#pragma unroll
        for (int j = 0; j < K::FTW; ++j) bvb[j] = *(const floatx4*)(p.bias_b + (ft0 + j) * 16 + g * 4);
#pragma unroll
        for (int i = 0; i < RB_TPW; ++i) {
            const int q = (pg + K::NPG * i) * 16 + n;
            const int gy = y0 + er[i], gx = x0 + ec[i];
            if (q >= npix || ec[i] >= p.TW || gy >= p.H || gx >= p.W) continue;
            const int pl = gy * p.W + gx;
            const size_t pix = (size_t)b * hw + pl;
            const size_t ybase = p.ldy > 0 ? (size_t)b * p.ldy + (size_t)pl * C : pix * C;
#pragma unroll
            for (int j = 0; j < K::FTW; ++j) {
                const int f = (ft0 + j) * 16 + g * 4;
                floatx4 v = acc[i][j] + bvb[j];
                v += *(const floatx4*)(p.x_in + pix * C + f);
                if (p.x_out) *(floatx4*)(p.x_out + pix * C + f) = v;
                if (p.y) {
                    const bf16x4 o = to_bf16x4(v);
                    *(bf16x4*)(p.y + ybase + f) = p.y_relu ? relu_bf16x4(o) : o;
                }
            }
        }
    }
}

}  // namespace seedinf
