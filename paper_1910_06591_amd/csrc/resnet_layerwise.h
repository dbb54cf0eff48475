// Layer-by-layer bf16 ResNet torso for the shapes the fused kernel does not
// cover (wider filters, larger frames, other channel counts: the model-size
// variants of Section 4.1 / 4.2).  Same network as resnet_fused.h: per section
// conv3x3 SAME -> max-pool 3x3/2 SAME -> two pre-activation residual blocks.
//
// Every 3x3 convolution is one launch of an implicit GEMM on bf16 MFMA:
// n = pixel (over the whole batch), m = output channel, k = tap * Cin + ci.
// With Cin a multiple of 8 a lane's B fragment (8 consecutive k) is 8
// contiguous channels of one tap of one pixel: one 16-byte load from the NHWC
// map, or zeros when the tap falls outside the image (SAME padding).  A small
// per-layer table gives each (chunk, lane group) its tap and element offset.
// The first layer reads the uint8 frame (any channel count, element-wise
// gather when Cin is not a multiple of 8) and scales the accumulator by 1/255.
// Activations live in HBM between layers: conv inputs as bf16 (rectified where
// the next layer wants them rectified), the residual stream x as fp32, so the
// rounding budget is the fused kernel's.
#pragma once
#include "bf16_common.h"

namespace seedinf {

struct LwConvArgs {
    const void* in;          // NHWC input: uint8 (first layer) or bf16
    const bf16x8* wp;        // A fragments [ftile][kchunk][lane][8], k = tap * Cin + ci, zero past 9 * Cin
    const float* bias;       // [Cout]
    const int2* ktab;        // [kchunks * 4]: x = element offset (dy * W + dx) * Cin + c0, y = (dy + 1) | (dx + 1) << 8, or y < 0: no such k
    const float* x_in;       // fp32 NHWC residual added to the output, or nullptr
    float* x_out;            // fp32 NHWC output (the residual stream), or nullptr; may alias x_in
    __bf16* y;               // bf16 output, or nullptr
    int y_relu;              // rectify y
    int ldy;                 // 0: y is NHWC [B, H, W, Cout]; > 0: y is the feature matrix [B, ldy], (h, w, c) order
    int B, H, W, Cin, Cout, kchunks;
    float scale;             // 1/255 for the uint8 layer, else 1
};

template <int FT, int RT, bool U8IN>
__global__ __launch_bounds__(256) void conv3x3_lw_kernel(LwConvArgs p)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int g = lane >> 4, n = lane & 15;
    const int ft0 = blockIdx.y * FT;
    const long npix = (long)p.B * p.H * p.W;
    const long p0 = ((long)blockIdx.x * 4 + wave) * (RT * 16);
    if (p0 >= npix) return;                               // uniform per wavefront

    long base[RT];
    int py[RT], px[RT];
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        const long pix = min(p0 + r * 16 + n, npix - 1);
        px[r] = (int)(pix % p.W);
        py[r] = (int)((pix / p.W) % p.H);
        base[r] = pix * p.Cin;
    }
    floatx4 acc[RT][FT];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int j = 0; j < FT; ++j) acc[r][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    const bool vec = !U8IN || (p.Cin & 7) == 0;           // 8 consecutive k = 8 contiguous channels of one tap
    for (int kc = 0; kc < p.kchunks; ++kc) {
        bf16x8 a[FT], b[RT];
#pragma unroll
        for (int j = 0; j < FT; ++j) a[j] = p.wp[((size_t)(ft0 + j) * p.kchunks + kc) * 64 + lane];
        if (vec) {
            const int2 t = p.ktab[kc * 4 + g];
            const int dy = (t.y & 0xff) - 1, dx = ((t.y >> 8) & 0xff) - 1;
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                const int yy = py[r] + dy, xx = px[r] + dx;
                const bool ok = t.y >= 0 && yy >= 0 && yy < p.H && xx >= 0 && xx < p.W;
                const long off = ok ? base[r] + t.x : base[r];        // any valid address when masked
                if constexpr (U8IN) {
                    const uint2 v = *(const uint2*)((const uint8_t*)p.in + off);
                    b[r] = u8x8_to_bf16x8(ok ? v.x : 0u, ok ? v.y : 0u);
                } else {
                    const bf16x8 v = *(const bf16x8*)((const __bf16*)p.in + off);
                    const bf16x8 z = {};
                    b[r] = ok ? v : z;
                }
            }
        } else {
            // uint8 frame with a channel count that is not a multiple of 8: gather the 8 values one by one
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int k = kc * 32 + g * 8 + e;
                    const int tap = k / p.Cin, ci = k - tap * p.Cin;
                    const int yy = py[r] + tap / 3 - 1, xx = px[r] + tap % 3 - 1;
                    const bool ok = tap < 9 && yy >= 0 && yy < p.H && xx >= 0 && xx < p.W;
                    const long off = ok ? base[r] + ((long)(tap / 3 - 1) * p.W + (tap % 3 - 1)) * p.Cin + ci : base[r];
                    v[e] = ok ? (float)((const uint8_t*)p.in)[off] : 0.f;
                }
                b[r] = to_bf16x8(floatx4{v[0], v[1], v[2], v[3]}, floatx4{v[4], v[5], v[6], v[7]});
            }
        }
#pragma unroll
        for (int r = 0; r < RT; ++r)
#pragma unroll
            for (int j = 0; j < FT; ++j) acc[r][j] = mfma16(a[j], b[r], acc[r][j]);
    }

    const int hw = p.H * p.W;
#pragma unroll
    for (int j = 0; j < FT; ++j) {
        const int f = (ft0 + j) * 16 + g * 4;
        const floatx4 bv = *(const floatx4*)(p.bias + f);
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            const long pix = p0 + r * 16 + n;
            if (pix >= npix) continue;
            floatx4 v = acc[r][j] * p.scale + bv;
            if (p.x_in) v += *(const floatx4*)(p.x_in + pix * p.Cout + f);
            if (p.x_out) *(floatx4*)(p.x_out + pix * p.Cout + f) = v;
            if (p.y) {
                const bf16x4 o = to_bf16x4(v);
                const long at = p.ldy > 0 ? (pix / hw) * p.ldy + (pix % hw) * p.Cout + f : pix * p.Cout + f;
                *(bf16x4*)(p.y + at) = p.y_relu ? relu_bf16x4(o) : o;
            }
        }
    }
}

// LDS-tiled variant for bf16 inputs whose channel count is a multiple of 32.  A block takes 128 consecutive
// pixels of one image (row-major, so narrow maps lose nothing to ragged tiles) and NF feature tiles; the input
// rows those pixels touch, one row above and below and a zero column left and right, are staged once in LDS as
// channel-group planes [Cin/8][rows][W+2][8 bf16] (plane stride a multiple of 256 B), so every input value is
// read from global memory once per block instead of nine times and a B fragment is one 16-byte LDS read.
// Wavefront w of the 8 multiplies feature tile w % NF with the pixel tiles w / NF, w / NF + 8 / NF, ...; chunk kc
// = (tap, 32 channels) matches the packed weight order k = tap * Cin + ci.
constexpr int LT_THREADS = 512, LT_PIX = 128;
constexpr size_t LT_LDS_MAX = 128 * 1024;                   // dynamic LDS the kernel may ask for

// rows of the staged patch: the rows 128 consecutive pixels can touch, plus one above and one below
inline int lt_patch_rows(int W) { return (LT_PIX + W - 2) / W + 1 + 2; }
inline int lt_plane_cells(int W) { return (lt_patch_rows(W) * (W + 2) + 15) / 16 * 16; }
inline size_t lt_lds_bytes(int W, int Cin) { return (size_t)(Cin / 8) * lt_plane_cells(W) * 16; }

template <int NF>
__global__ __launch_bounds__(LT_THREADS) void conv3x3_lds_kernel(LwConvArgs p, int plane_cells)
{
    static_assert(NF == 1 || NF == 2 || NF == 4, "feature tiles per block");
    constexpr int NPG = 8 / NF;                            // pixel groups (wavefronts per feature tile)
    constexpr int TPW = (LT_PIX / 16) / NPG;               // pixel tiles per wavefront
    extern __shared__ __attribute__((aligned(16))) char lt_lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, n = lane & 15;
    const int hw = p.H * p.W;
    const int nblk = (hw + LT_PIX - 1) / LT_PIX;
    const int b = blockIdx.x / nblk;
    const int p0 = (blockIdx.x % nblk) * LT_PIX;
    const int p1 = min(p0 + LT_PIX, hw);
    const int y0 = p0 / p.W, y1 = (p1 - 1) / p.W;
    const int prow = y1 - y0 + 3;                          // patch rows: image rows y0-1 .. y1+1
    const int PW2 = p.W + 2;
    const int ncg = p.Cin >> 3;

    // stage the patch (zeros outside the image)
    const __bf16* img = (const __bf16*)p.in + (size_t)b * hw * p.Cin;
    const int cells = prow * PW2;
    for (int idx = threadIdx.x; idx < cells * ncg; idx += LT_THREADS) {
        const int cell = idx / ncg, cg = idx - cell * ncg;             // channel groups of one pixel are adjacent in memory
        const int r = cell / PW2, c = cell - r * PW2;
        const int y = y0 - 1 + r, x = c - 1;
        bf16x8 v = {};
        if (y >= 0 && y < p.H && x >= 0 && x < p.W) v = *(const bf16x8*)(img + ((size_t)y * p.W + x) * p.Cin + cg * 8);
        *(bf16x8*)(lt_lds + ((size_t)cg * plane_cells + cell) * 16) = v;
    }
    __syncthreads();

    const int ft = blockIdx.y * NF + wave % NF;
    const int pg = wave / NF;
    int base[TPW];                                         // patch cell of the lane's pixel, tap (0, 0)
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        const int pix = min(p0 + (pg + NPG * i) * 16 + n, p1 - 1);
        const int y = pix / p.W, x = pix - y * p.W;
        base[i] = (y - y0) * PW2 + x;
    }
    floatx4 acc[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    const int cq_n = p.Cin >> 5;
    const bf16x8* wl = p.wp + (size_t)ft * p.kchunks * 64 + lane;
    const char* lane_plane = lt_lds + (size_t)g * plane_cells * 16;
    bf16x8 a = wl[0];
    int kc = 0;
    for (int tap = 0; tap < 9; ++tap) {
        const int toff = (tap / 3) * PW2 + tap % 3;
        for (int cq = 0; cq < cq_n; ++cq, ++kc) {
            const bf16x8 a_next = wl[(size_t)min(kc + 1, p.kchunks - 1) * 64];
            const char* src = lane_plane + ((size_t)cq * 4 * plane_cells + toff) * 16;
#pragma unroll
            for (int i = 0; i < TPW; ++i) acc[i] = mfma16(a, *(const bf16x8*)(src + base[i] * 16), acc[i]);
            a = a_next;
        }
    }

    const int f = ft * 16 + g * 4;
    const floatx4 bv = *(const floatx4*)(p.bias + f);
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        const int pl = p0 + (pg + NPG * i) * 16 + n;
        if (pl >= p1) continue;
        const long pix = (long)b * hw + pl;
        floatx4 v = acc[i] + bv;
        if (p.x_in) v += *(const floatx4*)(p.x_in + pix * p.Cout + f);
        if (p.x_out) *(floatx4*)(p.x_out + pix * p.Cout + f) = v;
        if (p.y) {
            const bf16x4 o = to_bf16x4(v);
            const long at = p.ldy > 0 ? (long)b * p.ldy + (long)pl * p.Cout + f : pix * p.Cout + f;
            *(bf16x4*)(p.y + at) = p.y_relu ? relu_bf16x4(o) : o;
        }
    }
}

// 3x3 / stride-2 max-pool with TF-style SAME padding on a bf16 NHWC map: writes the pooled values as the fp32
// residual stream x and, if r is given, their rectified bf16 copy R (the input of a block that runs as two
// launches).  One thread per 4 channels.
__global__ __launch_bounds__(256) void pool3x3s2_lw_kernel(const __bf16* __restrict__ in, float* __restrict__ x,
                                                           __bf16* __restrict__ r, int B, int H, int W, int C, int PH, int PW,
                                                           int pad_h, int pad_w)
{
    const long total = (long)B * PH * PW * (C / 4);
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int c4 = (int)(idx % (C / 4));
    long t = idx / (C / 4);
    const int pw = (int)(t % PW);
    t /= PW;
    const int ph = (int)(t % PH);
    const long b = t / PH;
    floatx4 m = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    for (int dy = 0; dy < 3; ++dy) {
        const int yy = 2 * ph - pad_h + dy;
        if (yy < 0 || yy >= H) continue;
        for (int dx = 0; dx < 3; ++dx) {
            const int xx = 2 * pw - pad_w + dx;
            if (xx < 0 || xx >= W) continue;
            m = max4(m, to_floatx4(*(const bf16x4*)(in + ((b * H + yy) * W + xx) * C + c4 * 4)));
        }
    }
    const long o = ((b * PH + ph) * PW + pw) * C + c4 * 4;
    *(floatx4*)(x + o) = m;
    if (r) *(bf16x4*)(r + o) = relu_bf16x4(to_bf16x4(m));
}

}  // namespace seedinf
