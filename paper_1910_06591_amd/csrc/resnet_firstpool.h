// First layer of the layer-by-layer ResNet path in one launch: uint8 frame -> 3x3 SAME convolution (the 1/255
// input scaling folded into the epilogue) -> 3x3 / stride-2 max-pool with TF-style SAME padding -> the fp32
// residual stream x of the first section (and, on request, R = ReLU(x) as bf16).  Run as a convolution and a pooling
// kernel the full-resolution map (four times the pooled one) goes out to HBM as bf16 and comes back 2.25 times;
// here it lives in LDS only.
//
// A workgroup takes a PTH x PTW tile of pooled pixels of one image: it stages the frame patch under the
// (2 PTH + 1) x (2 PTW + 1) convolution pixels those windows cover as bf16 cells of 4 channels (exact integers,
// zero outside the frame, zero in the padding channels), multiplies, writes the convolution tile to LDS as
// bf16 [pixel][C0] (outside the frame a value below every activation, so the maximum ignores it) and pools from there.
//
// K layout, frames of up to 4 planes (CELL = 4; weights packed to match, `first_pool_k`): with 4-channel cells two
// horizontally adjacent taps are 16 contiguous bytes, so a kernel row is padded to four columns (the fourth with
// zero weights) and lane group g of chunk kc reads kernel row 2 kc + (g >> 1), columns 2 (g & 1) and 2 (g & 1) + 1;
// chunk 1's groups 2 and 3 are padding.  Two MFMAs per tile for 27 or 36 useful k - the layer is a hundredth of
// the network's arithmetic.  Frames of 8 or 16 planes (CELL = planes): the layer-by-layer kernels' packing, k = tap
// * planes + plane, a lane group's 8 values are 16 aligned bytes of one cell.
#pragma once
#include "bf16_common.h"

namespace seedinf {

struct FirstPoolArgs {
    const uint8_t* obs;                // [B, H, W, Cin]
    const bf16x8* wp;                  // [C0 / 16][chunks][64 lanes][8]
    const float* bias;
    float scale;
    float* x;                          // [B, PH, PW, C0] fp32
    __bf16* r;                         // [B, PH, PW, C0] ReLU(x) as bf16, or nullptr
    int B, H, W, Cin, PH, PW, pad_h, pad_w;
    int PTH, PTW, tiles_y, tiles_x;
};

constexpr int FP_THREADS = 512;

// value(f, k) for pack_a: k = chunk * 32 + group * 8 + e -> (kernel row, kernel column, channel), see above
inline void first_pool_k(int k, int& dy, int& dx, int& ci)
{
    const int kc = k >> 5, g = (k >> 3) & 3, e = k & 7;
    dy = 2 * kc + (g >> 1);
    dx = 2 * (g & 1) + (e >> 2);
    ci = e & 3;
}

template <int C0, int CELL>
struct FirstPoolCfg {
    static_assert(C0 == 16 || C0 == 32 || C0 == 64, "first-layer widths with a fused kernel");
    static_assert(CELL == 4 || CELL == 8 || CELL == 16, "planes per frame cell");
    static constexpr int NFT = C0 / 16;
    static constexpr int KCH = CELL == 4 ? 2 : (9 * CELL + 31) / 32;
    // LDS per workgroup: four workgroups per compute unit up to 32 channels (the kernel is a chain of latencies:
    // patch, convolution, pooling, store), two at 64, where a tile's fixed costs weigh more than the overlap
    // (measured at 1024 images: x4 variant 2.61 -> 2.51 ms with 80 KB; x2 and the 144 x 108 map 1 - 2 % slower)
    static constexpr size_t LDS_MAX = (C0 >= 64 ? 80 : 40) * 1024;
    // bytes between the convolution tile's pixels in LDS: 16 more than the C0 values, so that the 16 pixels of an
    // accumulator tile's 8-byte stores spread over the banks (at a power-of-two stride they fall on two to eight)
    static constexpr int CSTRIDE = C0 * 2 + (C0 >= 64 ? 16 : 0);   // (narrower tiles: the padding costs more tile area than the conflicts cost time)
    __host__ __device__ static constexpr int patch_pitch(int PTW) { return 2 * PTW + 1 + 3; }     // + halo 2 + the zero-weight column
    __host__ __device__ static constexpr int patch_bytes(int PTH, int PTW) { return ((2 * PTH + 3) * patch_pitch(PTW) * CELL * 2 + 15) / 16 * 16; }
    static size_t lds_bytes(int PTH, int PTW) { return (size_t)patch_bytes(PTH, PTW) + (size_t)(2 * PTH + 1) * (2 * PTW + 1) * CSTRIDE; }
    // the fewest tiles whose maps fit
    static bool choose(int PH, int PW, int& PTH, int& PTW)
    {
        long best = -1;
        for (int ny = 1; ny <= PH; ++ny)
            for (int nx = 1; nx <= PW; ++nx) {
                const int th = (PH + ny - 1) / ny, tw = (PW + nx - 1) / nx;
                if (lds_bytes(th, tw) > LDS_MAX) continue;
                const long cost = (long)ny * nx * ((2 * th + 1) * (2 * tw + 1) + 64);     // convolution pixels + a fixed price per tile
                if (best < 0 || cost < best) { best = cost; PTH = th; PTW = tw; }
                break;
            }
        return best >= 0;
    }
};

template <int C0, int CELL>
__global__ __launch_bounds__(FP_THREADS) void first_pool_kernel(FirstPoolArgs p)
{
    using K = FirstPoolCfg<C0, CELL>;
    constexpr int NFT = K::NFT, KCH = K::KCH;
    extern __shared__ __attribute__((aligned(16))) char fp_lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, n = lane & 15;
    const int tiles = p.tiles_y * p.tiles_x;
    const int b = blockIdx.x / tiles, t = blockIdx.x % tiles;
    const int ph0 = (t / p.tiles_x) * p.PTH, pw0 = (t % p.tiles_x) * p.PTW;
    const int cy0 = 2 * ph0 - p.pad_h, cx0 = 2 * pw0 - p.pad_w;           // frame coordinates of convolution pixel (0, 0)
    const int CRH = 2 * p.PTH + 1, CRW = 2 * p.PTW + 1;
    const int PP = K::patch_pitch(p.PTW), PRH = CRH + 2;
    char* patch = fp_lds;
    char* cmap = fp_lds + K::patch_bytes(p.PTH, p.PTW);

    // weights: all feature tiles, all chunks
    bf16x8 a[NFT][KCH];
#pragma unroll
    for (int j = 0; j < NFT; ++j)
#pragma unroll
        for (int kc = 0; kc < KCH; ++kc) a[j][kc] = p.wp[(j * KCH + kc) * 64 + lane];

    // ---- frame patch: cell (r, c) = frame pixel (cy0 - 1 + r, cx0 - 1 + c), CELL bf16 ----
    const uint8_t* img = p.obs + (size_t)b * p.H * p.W * p.Cin;
    // (the loads of three rounds are issued before the first is converted: one round at a time, each waits out a
    // trip to memory)
    constexpr int UNR = 3;
    if constexpr (CELL == 4) {
        RowWalk rw(tid, FP_THREADS, PP);
        for (int cell0 = tid; cell0 < PRH * PP; cell0 += UNR * FP_THREADS) {
            uint32_t raw[UNR][4];
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int cell = cell0 + u * FP_THREADS;
                const int r = rw.r, c = rw.c;
                rw.next();
                const int y = cy0 - 1 + r, x = cx0 - 1 + c;
                raw[u][0] = raw[u][1] = raw[u][2] = raw[u][3] = 0;
                if (cell < PRH * PP && y >= 0 && y < p.H && x >= 0 && x < p.W) {
                    const uint8_t* s = img + ((size_t)y * p.W + x) * p.Cin;
                    raw[u][0] = s[0];
                    if (p.Cin > 1) raw[u][1] = s[1];
                    if (p.Cin > 2) raw[u][2] = s[2];
                    if (p.Cin > 3) raw[u][3] = s[3];
                }
            }
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int cell = cell0 + u * FP_THREADS;
                if (cell >= PRH * PP) continue;
                const floatx4 v = {(float)raw[u][0], (float)raw[u][1], (float)raw[u][2], (float)raw[u][3]};
                *(bf16x4*)(patch + cell * 8) = to_bf16x4(v);
            }
        }
    } else {
        constexpr int HALVES = CELL / 8;                       // 8 planes = 8 aligned bytes of the frame -> 16 bytes of the cell
        const int h = tid % HALVES;
        RowWalk rw(tid / HALVES, FP_THREADS / HALVES, PP);
        for (int idx0 = tid; idx0 < PRH * PP * HALVES; idx0 += UNR * FP_THREADS) {
            uint2 raw[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int idx = idx0 + u * FP_THREADS;
                const int r = rw.r, c = rw.c;
                rw.next();
                const int y = cy0 - 1 + r, x = cx0 - 1 + c;
                raw[u] = uint2{0u, 0u};
                if (idx < PRH * PP * HALVES && y >= 0 && y < p.H && x >= 0 && x < p.W)
                    raw[u] = *(const uint2*)(img + ((size_t)y * p.W + x) * CELL + h * 8);
            }
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int idx = idx0 + u * FP_THREADS;
                if (idx >= PRH * PP * HALVES) continue;
                *(bf16x8*)(patch + (size_t)idx * 16) = u8x8_to_bf16x8(raw[u].x, raw[u].y);
            }
        }
    }
    __syncthreads();

    // ---- convolution tile -> cmap, one 16-pixel tile (row-major over the region) at a time ----
    {
        const int npix = CRH * CRW, ntiles = (npix + 15) / 16;
        // byte offset of the lane group's fragment from the pixel's tap (0, 0) cell, per chunk
        int off[KCH];
        if constexpr (CELL == 4) {
            // kernel row 2 kc + (g >> 1) (clamped onto row 2 for the padding groups), columns 2 (g & 1), + 1
            off[0] = ((g >> 1) * PP + 2 * (g & 1)) * 8;
            off[1] = (2 * PP + 2 * (g & 1)) * 8;
        } else {
#pragma unroll
            for (int kc = 0; kc < KCH; ++kc) {
                const int k0 = kc * 32 + g * 8;
                const int tap = min(k0 / CELL, 8);                 // k past 9 planes has zero weights: any cell
                off[kc] = ((tap / 3) * PP + tap % 3) * CELL * 2 + (k0 % CELL) * 2;
            }
        }
        floatx4 bv[NFT];
#pragma unroll
        for (int j = 0; j < NFT; ++j) bv[j] = *(const floatx4*)(p.bias + j * 16 + g * 4);
        // the lane's pixel walks the region FP_THREADS / 4 pixels per round: one division here, none in the loop
        constexpr int QSTEP = FP_THREADS / 4;
        const int dr = QSTEP / CRW, dc = QSTEP - dr * CRW;
        int r = (wave * 16 + n) / CRW, c = wave * 16 + n - r * CRW;
        for (int tile = wave; tile < ntiles; tile += FP_THREADS / 64, r += dr, c += dc) {
            if (c >= CRW) { c -= CRW; ++r; }
            const bool tail = tile * 16 + n >= npix;                   // past the region: the last pixel again, not stored
            const int q = tail ? npix - 1 : tile * 16 + n;
            const int rr = tail ? CRH - 1 : r, cc = tail ? CRW - 1 : c;
            const char* s = patch + (size_t)(rr * PP + cc) * CELL * 2;
            bf16x8 bfrag[KCH];
#pragma unroll
            for (int kc = 0; kc < KCH; ++kc) {
                if constexpr (CELL == 4) {                              // 8-byte cells: the 16 bytes are 8-byte aligned only
                    const bf16x4 l = *(const bf16x4*)(s + off[kc]), h = *(const bf16x4*)(s + off[kc] + 8);
                    bfrag[kc] = __builtin_shufflevector(l, h, 0, 1, 2, 3, 4, 5, 6, 7);
                } else {
                    bfrag[kc] = *(const bf16x8*)(s + off[kc]);
                }
            }
            const int y = cy0 + rr, x = cx0 + cc;
            const bool inside = y >= 0 && y < p.H && x >= 0 && x < p.W;
#pragma unroll
            for (int j = 0; j < NFT; ++j) {
                floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kc = 0; kc < KCH; ++kc) acc = mfma16(a[j][kc], bfrag[kc], acc);
                uint2 o = __builtin_bit_cast(uint2, to_bf16x4(acc * p.scale + bv[j]));
                if (!inside) o = uint2{BF16X2_LOWEST, BF16X2_LOWEST};
                if (!tail) *(uint2*)(cmap + (size_t)q * K::CSTRIDE + (j * 16 + g * 4) * 2) = o;
            }
        }
    }
    __syncthreads();

    // ---- 3x3 / 2 maximum: pooled pixel (ph, pw) covers region rows 2 ph .. 2 ph + 2, columns 2 pw .. 2 pw + 2 ----
    constexpr int NCG = C0 / 8;
    static_assert(FP_THREADS % NCG == 0, "a thread keeps its channel group");
    const int cg = tid % NCG;
    RowWalk pwk(tid / NCG, FP_THREADS / NCG, p.PTW);
    for (int pp = tid / NCG; pp < p.PTH * p.PTW; pp += FP_THREADS / NCG) {
        const int ph = pwk.r, pw = pwk.c;
        pwk.next();
        if (ph0 + ph >= p.PH || pw0 + pw >= p.PW) continue;
        const char* win = cmap + (size_t)(2 * ph * CRW + 2 * pw) * K::CSTRIDE + cg * 16;
        uint4 m = *(const uint4*)win;
#pragma unroll
        for (int dy = 0; dy < 3; ++dy)
#pragma unroll
            for (int dx = 0; dx < 3; ++dx)
                if (dy + dx > 0) m = bf16x8_max(m, *(const uint4*)(win + (size_t)(dy * CRW + dx) * K::CSTRIDE));
        const size_t o = (((size_t)b * p.PH + ph0 + ph) * p.PW + pw0 + pw) * C0 + cg * 8;
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
