// conv0 of a later section of the layer-by-layer ResNet path with its pooling, in one launch: bf16 NHWC input
// (the previous section's un-rectified output) -> 3x3 SAME convolution CIN -> COUT -> 3x3 / stride-2 max-pool with
// TF-style SAME padding -> the section's fp32 residual stream x (and, on request, R = ReLU(x) as bf16).  As two
// launches the full-resolution bf16 map goes out to HBM and comes back 2.25 times; here it lives in LDS.
//
// A workgroup takes a PTH x PTW tile of pooled pixels of one image: the input patch under the (2 PTH + 1) x
// (2 PTW + 1) convolution pixels those windows cover is staged as planar bf16 [CIN/8][rows][pitch][8] (zero
// outside the image), the convolution runs over it as in the fused residual block (rb_conv), its tile goes to LDS
// as bf16 [pixel][COUT] (outside the image a value below every activation, so the maximum ignores it) and is pooled from
// there.
#pragma once
#include "resnet_blockfused.h"

namespace seedinf {

struct ConvPoolArgs {
    const __bf16* in;                  // [B, H, W, CIN]
    const bf16x8* wp;                  // [COUT / 16][chunks][64 lanes][8], k = tap * CIN + ci
    const float* bias;
    float* x;                          // [B, PH, PW, COUT] fp32
    __bf16* r;                         // [B, PH, PW, COUT] ReLU(x) as bf16, or nullptr
    int B, H, W, PH, PW, pad_h, pad_w;
    int PTH, PTW, tiles_y, tiles_x, kchunks;
};

constexpr size_t CP_LDS_MAX = 80 * 1024;                    // two workgroups per compute unit

template <int CIN, int COUT>
struct ConvPoolCfg {
    using K = ResBlockCfg<COUT>;
    static constexpr int NCG = CIN / 8;
    // bytes between the convolution tile's pixels in LDS (16 more than the COUT values: see first_pool_kernel)
    static constexpr int CSTRIDE = COUT * 2 + (COUT >= 64 ? 16 : 0);
    __host__ __device__ static constexpr int patch_plane(int PTH, int PTW) { return ((2 * PTH + 3) * (2 * PTW + 3) + 15) / 16 * 16; }
    static size_t lds_bytes(int PTH, int PTW)
    {
        return (size_t)NCG * patch_plane(PTH, PTW) * 16 + (size_t)(2 * PTH + 1) * (2 * PTW + 1) * CSTRIDE;
    }
    // the fewest convolution pixels over all tiles whose region fits a workgroup and whose maps fit
    static bool choose(int PH, int PW, int& PTH, int& PTW)
    {
        long best = -1;
        for (int ny = 1; ny <= PH; ++ny)
            for (int nx = 1; nx <= PW; ++nx) {
                const int th = (PH + ny - 1) / ny, tw = (PW + nx - 1) / nx;
                if ((2 * th + 1) * (2 * tw + 1) > K::MAX_PIX || lds_bytes(th, tw) > CP_LDS_MAX) continue;
                const long cost = (long)ny * nx * ((2 * th + 1) * (2 * tw + 1) + 64);
                if (best < 0 || cost < best) { best = cost; PTH = th; PTW = tw; }
                break;
            }
        return best >= 0;
    }
};

template <int CIN, int COUT>
__global__ __launch_bounds__(RB_THREADS, 4) void conv_pool_kernel(ConvPoolArgs p)
{
    using CP = ConvPoolCfg<CIN, COUT>;
    using K = ResBlockCfg<COUT>;
    extern __shared__ __attribute__((aligned(16))) char cp_lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, n = lane & 15;
    const int tiles = p.tiles_y * p.tiles_x;
    const int b = blockIdx.x / tiles, t = blockIdx.x % tiles;
    const int ph0 = (t / p.tiles_x) * p.PTH, pw0 = (t % p.tiles_x) * p.PTW;
    const int cy0 = 2 * ph0 - p.pad_h, cx0 = 2 * pw0 - p.pad_w;           // image coordinates of convolution pixel (0, 0)
    const int CRH = 2 * p.PTH + 1, CRW = 2 * p.PTW + 1;
    const int PP = CRW + 2, PRH = CRH + 2, PL = CP::patch_plane(p.PTH, p.PTW);
    char* patch = cp_lds;
    char* cmap = cp_lds + (size_t)CP::NCG * PL * 16;

    // ---- input patch: cell (r, c) = image pixel (cy0 - 1 + r, cx0 - 1 + c), loads in batches of four ----
    const __bf16* img = p.in + (size_t)b * p.H * p.W * CIN;
    constexpr int UNR = 4;
    const int cells = PRH * PP;
    static_assert(RB_THREADS % CP::NCG == 0, "a thread keeps its channel group");
    constexpr int CSTEP = RB_THREADS / CP::NCG;
    const int cgi = tid % CP::NCG;                                         // a pixel's channel groups are adjacent in memory
    RowWalk rw(tid / CP::NCG, CSTEP, PP);
    for (int cell0 = tid / CP::NCG; cell0 < cells; cell0 += UNR * CSTEP) {
        bf16x8 v[UNR];
        int at[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int cell = cell0 + u * CSTEP;
            const int cg = cgi;
            const int r = rw.r, c = rw.c;
            rw.next();
            const int y = cy0 - 1 + r, x = cx0 - 1 + c;
            at[u] = cell < cells ? (cg * PL + cell) * 16 : -1;
            v[u] = bf16x8{};
            if (at[u] >= 0 && y >= 0 && y < p.H && x >= 0 && x < p.W) v[u] = *(const bf16x8*)(img + ((size_t)y * p.W + x) * CIN + cg * 8);
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u)
            if (at[u] >= 0) *(bf16x8*)(patch + at[u]) = v[u];
    }
    __syncthreads();

    // ---- convolution tile -> cmap ----
    {
        const int fg = wave % K::NFG, pg = wave / K::NFG;
        const int ft0 = fg * K::FTW;
        floatx4 acc[RB_TPW][K::FTW];
        const int npix = CRH * CRW;
        rb_conv<CIN, COUT>(patch, PL, PP, CRW, npix, p.wp, p.kchunks, ft0, pg, lane, acc);
        int er[RB_TPW], ec[RB_TPW];
        tile_coords<RB_TPW>(pg, K::NPG, n, CRW, er, ec);
        floatx4 bvs[K::FTW];
#pragma unroll
        for (int j = 0; j < K::FTW; ++j) bvs[j] = *(const floatx4*)(p.bias + (ft0 + j) * 16 + g * 4);
#pragma unroll
        for (int i = 0; i < RB_TPW; ++i) {
            const int q = (pg + K::NPG * i) * 16 + n;
            if (q >= npix) continue;
            const int y = cy0 + er[i], x = cx0 + ec[i];
            const bool outside = y < 0 || y >= p.H || x < 0 || x >= p.W;
            char* cell = cmap + q * CP::CSTRIDE + g * 8;
#pragma unroll
            for (int j = 0; j < K::FTW; ++j) {
                uint2 o = __builtin_bit_cast(uint2, to_bf16x4(acc[i][j] + bvs[j]));
                if (outside) o = uint2{BF16X2_LOWEST, BF16X2_LOWEST};
                *(uint2*)(cell + (ft0 + j) * 32) = o;
            }
        }
    }
    __syncthreads();

    // ---- 3x3 / 2 maximum: pooled pixel (ph, pw) covers region rows 2 ph .. 2 ph + 2, columns 2 pw .. 2 pw + 2 ----
    constexpr int NCGO = COUT / 8;
    static_assert(RB_THREADS % NCGO == 0, "a thread keeps its channel group");
    const int cg = tid % NCGO;
    RowWalk pwk(tid / NCGO, RB_THREADS / NCGO, p.PTW);
    for (int pp = tid / NCGO; pp < p.PTH * p.PTW; pp += RB_THREADS / NCGO) {
        const int ph = pwk.r, pw = pwk.c;
        pwk.next();
        if (ph0 + ph >= p.PH || pw0 + pw >= p.PW) continue;
        const char* win = cmap + (size_t)(2 * ph * CRW + 2 * pw) * CP::CSTRIDE + cg * 16;
        uint4 m = *(const uint4*)win;
#pragma unroll
        for (int dy = 0; dy < 3; ++dy)
#pragma unroll
            for (int dx = 0; dx < 3; ++dx)
                if (dy + dx > 0) m = bf16x8_max(m, *(const uint4*)(win + (size_t)(dy * CRW + dx) * CP::CSTRIDE));
        const size_t o = (((size_t)b * p.PH + ph0 + ph) * p.PW + pw0 + pw) * COUT + cg * 8;
        *(floatx4*)(p.x + o) = floatx4{bf16_lo_f32(m.x), bf16_hi_f32(m.x), bf16_lo_f32(m.y), bf16_hi_f32(m.y)};
        *(floatx4*)(p.x + o + 4) = floatx4{bf16_lo_f32(m.z), bf16_hi_f32(m.z), bf16_lo_f32(m.w), bf16_hi_f32(m.w)};
        if (p.r) {
            const bf16x8 mv = __builtin_bit_cast(bf16x8, m);
            const bf16x4 rl = relu_bf16x4(__builtin_shufflevector(mv, mv, 0, 1, 2, 3)), rh = relu_bf16x4(__builtin_shufflevector(mv, mv, 4, 5, 6, 7));
            *(bf16x8*)(p.r + o) = __builtin_shufflevector(rl, rh, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    }
}

}  // namespace seedinf
