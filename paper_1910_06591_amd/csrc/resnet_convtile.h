// One 3x3 SAME convolution C -> C of a residual block per launch, for the widths at which the whole block in one
// launch (resblock_fused_kernel) is bound by operand delivery: with only the input map in LDS a workgroup's tile
// holds twice the pixels, a wavefront multiplies each weight fragment with up to eight pixel tiles instead of four,
// and the weight traffic through the vector L1 halves.  The price is U's round trip through HBM as bf16.
//   IN_F32: the input is the fp32 residual stream x, rectified and rounded to bf16 while it is staged (conv_a);
//           else a bf16 NHWC map that is already rectified (conv_b reading U).
//   Output: v = conv + bias (+ resid); x_out = v as fp32 and / or y = v (rectified if y_relu) as bf16, NHWC or
//           feature rows, as in resblock_fused_kernel.
#pragma once
#include "resnet_blockfused.h"

namespace seedinf {

struct ConvTileArgs {
    const void* in;                    // [B, H, W, C]: fp32 (IN_F32) or bf16
    const bf16x8* wp;                  // [C / 16][chunks][64 lanes][8], k = tap * C + ci
    const float* bias;
    const float* resid;                // [B, H, W, C] fp32 added to the output, or nullptr
    float* x_out;                      // fp32 output, or nullptr; must not alias `in`
    __bf16* y;                         // bf16 output, or nullptr; must not alias `in`
    int y_relu, ldy;
    int B, H, W, TH, TW, tiles_y, tiles_x, kchunks;
};

constexpr int CT_TPW = 8;
constexpr size_t CT_LDS_MAX = 80 * 1024;                    // two workgroups per compute unit

template <int C>
struct ConvTileCfg {
    using K = ResBlockCfg<C>;
    static constexpr int NCG = C / 8;
    static constexpr int MAX_PIX = 16 * CT_TPW * K::NPG;
    __host__ __device__ static constexpr int plane(int TH, int TW) { return ((TH + 2) * (TW + 2) + 15) / 16 * 16; }
    static size_t lds_bytes(int TH, int TW) { return (size_t)NCG * plane(TH, TW) * 16; }
    // the cut with the fewest patch pixels (halo re-reads) whose tile fits a workgroup and LDS
    static bool choose(int H, int W, int& TH, int& TW)
    {
        long best = -1;
        for (int ny = 1; ny <= H; ++ny) {
            const int th = (H + ny - 1) / ny;
            for (int nx = 1; nx <= W; ++nx) {
                const int tw = (W + nx - 1) / nx;
                if (th * tw > MAX_PIX || lds_bytes(th, tw) > CT_LDS_MAX) continue;
                const long cost = (long)ny * nx * ((th + 2) * (tw + 2) + 64);
                if (best < 0 || cost < best) { best = cost; TH = th; TW = tw; }
            }
        }
        return best >= 0;
    }
};

template <int C, bool IN_F32>
__global__ __launch_bounds__(RB_THREADS, 4) void conv_tile_kernel(ConvTileArgs p)
{
    using CT = ConvTileCfg<C>;
    using K = ResBlockCfg<C>;
    extern __shared__ __attribute__((aligned(16))) char ct_lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, n = lane & 15;
    const int tiles = p.tiles_y * p.tiles_x;
    const int b = blockIdx.x / tiles, t = blockIdx.x % tiles;
    const int y0 = (t / p.tiles_x) * p.TH, x0 = (t % p.tiles_x) * p.TW;
    const int PP = p.TW + 2, PL = CT::plane(p.TH, p.TW);
    const size_t img = (size_t)b * p.H * p.W * C;

    // ---- input patch: cell (r, c) = image pixel (y0 - 1 + r, x0 - 1 + c), zeros outside the image; loads in batches ----
    constexpr int UNR = 4;
    const int cells = (p.TH + 2) * PP;
    static_assert(RB_THREADS % CT::NCG == 0, "a thread keeps its channel group");
    constexpr int CSTEP = RB_THREADS / CT::NCG;
    const int cg = tid % CT::NCG;                                          // a pixel's channel groups are adjacent in memory
    RowWalk rw(tid / CT::NCG, CSTEP, PP);
    for (int cell0 = tid / CT::NCG; cell0 < cells; cell0 += UNR * CSTEP) {
        floatx4 lo[UNR], hi[UNR];
        bf16x8 v[UNR];
        int at[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int cell = cell0 + u * CSTEP;
            const int r = rw.r, c = rw.c;
            rw.next();
            const int gy = y0 - 1 + r, gx = x0 - 1 + c;
            at[u] = cell < cells ? (cg * PL + cell) * 16 : -1;
            const bool inside = at[u] >= 0 && gy >= 0 && gy < p.H && gx >= 0 && gx < p.W;
            const size_t off = img + ((size_t)gy * p.W + gx) * C + cg * 8;
            if constexpr (IN_F32) {
                lo[u] = hi[u] = floatx4{0.f, 0.f, 0.f, 0.f};
                if (inside) {
                    lo[u] = *(const floatx4*)((const float*)p.in + off);
                    hi[u] = *(const floatx4*)((const float*)p.in + off + 4);
                }
            } else {
                v[u] = bf16x8{};
                if (inside) v[u] = *(const bf16x8*)((const __bf16*)p.in + off);
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            if (at[u] < 0) continue;
            if constexpr (IN_F32) {
                const bf16x8 raw = to_bf16x8(lo[u], hi[u]);
                const bf16x4 l = relu_bf16x4(__builtin_shufflevector(raw, raw, 0, 1, 2, 3));
                const bf16x4 h = relu_bf16x4(__builtin_shufflevector(raw, raw, 4, 5, 6, 7));
                v[u] = __builtin_shufflevector(l, h, 0, 1, 2, 3, 4, 5, 6, 7);
            }
            *(bf16x8*)(ct_lds + at[u]) = v[u];
        }
    }
    __syncthreads();

    const int fg = wave % K::NFG, pg = wave / K::NFG;
    const int ft0 = fg * K::FTW;
    floatx4 acc[CT_TPW][K::FTW];
    const int npix = p.TH * p.TW;
    rb_conv<C, C, CT_TPW>(ct_lds, PL, PP, p.TW, npix, p.wp, p.kchunks, ft0, pg, lane, acc);
    const int hw = p.H * p.W;
    int er[CT_TPW], ec[CT_TPW];
    tile_coords<CT_TPW>(pg, K::NPG, n, p.TW, er, ec);
    floatx4 bvs[K::FTW];
#pragma unroll
    for (int j = 0; j < K::FTW; ++j) bvs[j] = *(const floatx4*)(p.bias + (ft0 + j) * 16 + g * 4);
#pragma unroll
    for (int i = 0; i < CT_TPW; ++i) {
        const int q = (pg + K::NPG * i) * 16 + n;
        const int gy = y0 + er[i], gx = x0 + ec[i];
        if (q >= npix || gy >= p.H || gx >= p.W) continue;
        const int pl = gy * p.W + gx;
        const size_t pix = (size_t)b * hw + pl;
        const size_t ybase = p.ldy > 0 ? (size_t)b * p.ldy + (size_t)pl * C : pix * C;
#pragma unroll
        for (int j = 0; j < K::FTW; ++j) {
            const int f = (ft0 + j) * 16 + g * 4;
            floatx4 v = acc[i][j] + bvs[j];
            if (p.resid) v += *(const floatx4*)(p.resid + pix * C + f);
            if (p.x_out) *(floatx4*)(p.x_out + pix * C + f) = v;
            if (p.y) {
                const bf16x4 o = to_bf16x4(v);
                *(bf16x4*)(p.y + ybase + f) = p.y_relu ? relu_bf16x4(o) : o;
            }
        }
    }
}

}  // namespace seedinf
