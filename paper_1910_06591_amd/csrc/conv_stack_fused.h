// Fused bf16 torso of the recurrent Atari agent (Appendix A.3.1): 84x84xCIN uint8 frame -> conv 8x8/4 (32) ->
// conv 4x4/2 (64) -> conv 3x3/1 (64), "valid" padding, ReLU after each, flattened (h, w, c).  CIN = 4 (four
// stacked frames) or 1 (no frame stacking, the configuration of Section 4.3's fastest Atari run).
//
// One persistent workgroup of 8 wavefronts per compute unit takes one image at a time through all three
// layers with every activation in LDS, and keeps ALL convolution weights (152 KiB of bf16) in registers for its
// whole life, spread over the wavefronts:
//   conv1 (K = 64 CIN, 2 feature tiles): every wavefront holds all 16 (CIN = 4) or 4 (CIN = 1) weight fragments
//          and takes every eighth pixel tile of the 20 x 20 map;
//   conv2 (K = 512, 4 feature tiles) and conv3 (K = 576, 4 feature tiles): wavefront w holds feature tile
//          w % 4 and half w / 4 of K (8 and 9 fragments), multiplies every pixel tile of the 9 x 9 / 7 x 7 map
//          by them, and the two halves swap partial sums through LDS (each finishes half of the tiles).
// So an image costs no weight traffic at all; what moves is the frame (global -> LDS, asynchronous, issued one
// image ahead) and the 3136 output features.
//
// LDS layouts.  Every activation fragment (16 pixels x 8 channels of one tap) is read as 16 consecutive 16-byte
// cells, which is what keeps the reads free of bank conflicts; the strided and shifted windows of the
// convolutions are absorbed by storing shifted copies, written by the producing layer's epilogue:
//   frame  the raw uint8 frame, twice (the next image lands while this one is computed).  A conv1 fragment
//          (CIN = 4: kernel row kh, pixels 4 ow + 2 g, + 1; CIN = 1: kernel row 4 c + g, pixels 4 ow .. + 7) is 8
//          consecutive bytes, converted to bf16 in registers.
//   act1   bf16 [copy 2][plane 4 (8 channels)][x parity 2][y parity 2][yh 10][9 cells]: conv2 (stride 2) reads
//          x = 2 ow + kw, y = 2 oh + kh -> parities kw & 1, kh & 1; copy kw >> 1 holds column xh = ow' + copy at
//          ow', so tap (kh, kw) of output pixel p = 9 oh + ow is cell (kh >> 1) * 9 + p of its sub-plane
//   act2   bf16 [copy 3][plane 8][y 9][7 cells]: conv3 (stride 1); copy kw holds column x + kw at x, so tap
//          (kh, kw) of output pixel p = 7 oh + ow is cell kh * 7 + p
//   Sub-planes are padded to multiples of 256 bytes (the two lane groups of a half-wavefront read different
//   planes, and this LDS serves them at full rate only when they are a multiple of 256 bytes apart).
// Weight fragments come from the conv stack's packed A operands ([ftile][chunk][lane], k = (kh, kw, ci)): a
// chunk of 32 k is one kernel row of conv1 (four rows with CIN = 1), one tap of conv2 and half a tap of conv3.
#pragma once
#include "bf16_common.h"

namespace seedinf {

struct R2d2TorsoArgs {
    const uint8_t* obs;          // [B, 84, 84, CIN]
    const bf16x8* w1; const bf16x8* w2; const bf16x8* w3;     // packed A fragments of the three layers
    const float* b1; const float* b2; const float* b3;        // fp32 biases [32], [64], [64]
    __bf16* feat; int ldf;       // [B, ldf] rectified features
    int B;
};

#define R2D2_TILE_FENCE __builtin_amdgcn_sched_barrier(0)

namespace r2d2 {
constexpr int H = 84, W = 84;
constexpr int O1 = 20, O2 = 9, O3 = 7;
constexpr int NP1 = O1 * O1, NP2 = O2 * O2, NP3 = O3 * O3;      // 400, 81, 49 output pixels
constexpr int NT1 = NP1 / 16, NT2 = (NP2 + 15) / 16, NT3 = (NP3 + 15) / 16;   // 25, 6, 4 pixel tiles
constexpr int RAW_BYTES = 28 * 1024;                          // one raw frame (CIN = 4: 28224 bytes, 28 loads of 1 KiB)
constexpr int RAW_OFF = 0;                                    // two of them
constexpr int A1_SUB = 96 * 16;                               // act1 sub-plane: 90 cells, padded
constexpr int ACT1_OFF = RAW_OFF + 2 * RAW_BYTES, ACT1_BYTES = 2 * 4 * 4 * A1_SUB;       // 49152
constexpr int A2_SUB = 64 * 16;                               // act2 sub-plane: 63 cells, padded
constexpr int ACT2_OFF = ACT1_OFF + ACT1_BYTES, ACT2_BYTES = 3 * 8 * A2_SUB;             // 24576
constexpr int EX_OFF = ACT2_OFF + ACT2_BYTES, EX_BYTES = 8 * 3 * 1024;                   // partial sums handed over
constexpr int LDS_BYTES = EX_OFF + EX_BYTES;
static_assert(NT1 * 16 == NP1 && LDS_BYTES <= 160 * 1024, "R2D2 torso LDS plan");
constexpr int THREADS = 512;
}  // namespace r2d2

template <int CIN>
__global__ __launch_bounds__(r2d2::THREADS) void r2d2_torso_bf16_kernel(R2d2TorsoArgs p)
{
    using namespace r2d2;
    static_assert(CIN == 4 || CIN == 1, "stacked or single frames");
    constexpr int FRAME_U8 = H * W * CIN, NLOAD = (FRAME_U8 + 1023) / 1024;
    constexpr int NW1 = CIN == 4 ? 16 : 4;                     // conv1 weight fragments: [ftile 2][chunk 8 or 2]
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g0 = lane >> 4, n0 = lane & 15;
    const int f23 = wave & 3, half = wave >> 2;               // conv2 / conv3: feature tile and K half

    // ---- resident weights and biases ----
    bf16x8 w1[NW1], w2[8], w3[9];
#pragma unroll
    for (int i = 0; i < NW1; ++i) w1[i] = p.w1[i * 64 + lane];
#pragma unroll
    for (int i = 0; i < 8; ++i) w2[i] = p.w2[((size_t)f23 * 16 + half * 8 + i) * 64 + lane];
#pragma unroll
    for (int i = 0; i < 9; ++i) w3[i] = p.w3[((size_t)f23 * 18 + half * 9 + i) * 64 + lane];
    // (the biases are re-read from global memory where they are used: the weights leave no registers to spare)

    // asynchronous copy of image b's raw frame into raw buffer `buf`, 28 loads of 1 KiB; the last load's lanes
    // past the frame's end re-read its last 16 bytes (the bytes they deliver are never used).
    // Issuing such a load occupies the wavefront for a few hundred cycles, so the seven wavefronts that have
    // three conv1 tiles (wavefront 0 has four) issue them, after their tiles, while they would wait for it anyway.
    auto fetch_frame = [&](int b, int buf) {
        if (wave == 0) return;
        const uint8_t* src = p.obs + (size_t)b * FRAME_U8;
#pragma unroll
        for (int j = 0; j < (NLOAD + 6) / 7; ++j) {
            const int c = wave - 1 + 7 * j;                    // uniform
            if (c < NLOAD) {
                const int off = min(c * 1024 + lane * 16, FRAME_U8 - 16);
                g2lds16(src + off, lds0 + RAW_OFF + buf * RAW_BYTES + c * 1024);
            }
        }
    };

    int b = blockIdx.x, buf = 0;
    if (b < p.B) fetch_frame(b, 0);
    for (; b < p.B; b += gridDim.x, buf ^= 1) {
        // opaque per-iteration copies of the lane coordinates: address arithmetic derived from them stays inside the
        // loop instead of being hoisted into registers the weights need
        int g = g0, n = n0;
        asm volatile("" : "+v"(g), "+v"(n));
        stage_wait();
        __syncthreads();                                       // the raw frame has landed; the previous image is finished

        // ---- conv1: 8x8 stride 4, 4 -> 32 channels, ReLU; acc holds 255 x the true sum ----
        const floatx4 bias1[2] = {*(const floatx4*)(p.b1 + g * 4), *(const floatx4*)(p.b1 + 16 + g * 4)};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int t = wave + 8 * i;                        // uniform
            if (t >= NT1) break;
            const int pix = t * 16 + n;
            const int oh = pix / O1, ow = pix - oh * O1;
            floatx4 a0 = {0.f, 0.f, 0.f, 0.f}, a1 = a0;
            if constexpr (CIN == 4) {
                const char* fb = lds + RAW_OFF + buf * RAW_BYTES + ((4 * oh) * W + 4 * ow + 2 * g) * 4;
#pragma unroll
                for (int kh = 0; kh < 8; ++kh) {
                    const uint2 v = *(const uint2*)(fb + kh * (W * 4));
                    const bf16x8 bf = u8x8_to_bf16x8(v.x, v.y);
                    a0 = mfma16(w1[kh], bf, a0);
                    a1 = mfma16(w1[8 + kh], bf, a1);
                }
            } else {
                // chunk c: kernel rows 4 c .. 4 c + 3, one per lane group; 8 bytes at a 4-byte aligned address
                const char* fb = lds + RAW_OFF + buf * RAW_BYTES + (4 * oh + g) * W + 4 * ow;
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const uint32_t lo = *(const uint32_t*)(fb + c * (4 * W)), hi = *(const uint32_t*)(fb + c * (4 * W) + 4);
                    const bf16x8 bf = u8x8_to_bf16x8(lo, hi);
                    a0 = mfma16(w1[c], bf, a0);
                    a1 = mfma16(w1[2 + c], bf, a1);
                }
            }
            // channels f * 16 + 4 g .. + 3 of pixel (oh, ow): plane 2 f + (g >> 1), 8-byte half g & 1, sub-plane
            // (x parity, y parity), row oh >> 1; copy 0 takes column xh = ow >> 1 if it is < 9, copy 1 stores xh >= 1 at xh - 1
            const bf16x4 o0 = relu_bf16x4(to_bf16x4(a0 * (1.0f / 255.0f) + bias1[0]));
            const bf16x4 o1 = relu_bf16x4(to_bf16x4(a1 * (1.0f / 255.0f) + bias1[1]));
            const int xh = ow >> 1;
            char* d = lds + ACT1_OFF + ((g >> 1) * 4 + (ow & 1) * 2 + (oh & 1)) * A1_SUB + ((oh >> 1) * 9 + xh) * 16 + (g & 1) * 8;
            if (xh < 9) { *(bf16x4*)d = o0; *(bf16x4*)(d + 2 * 4 * A1_SUB) = o1; }
            if (xh >= 1) { *(bf16x4*)(d + 16 * A1_SUB - 16) = o0; *(bf16x4*)(d + (16 + 8) * A1_SUB - 16) = o1; }
            R2D2_TILE_FENCE;                                 // one tile's fragments in registers at a time
        }
        // the other raw buffer was last read by the previous image's conv1, two barriers ago
        if (b + (int)gridDim.x < p.B) fetch_frame(b + gridDim.x, buf ^ 1);
        __syncthreads();

        // ---- conv2: 4x4 stride 2, 32 -> 64 channels; this wavefront: feature tile f23, taps half*8 .. +7 ----
        {
            const floatx4 bias2 = *(const floatx4*)(p.b2 + f23 * 16 + g * 4);
            floatx4 acc[NT2];
            // the fragments of tile t + 1 are requested before tile t is multiplied
            bf16x8 bq[2][8];
            auto fetch2 = [&](int t, bf16x8 (&b)[8]) {
                const int pix = min(t * 16 + n, NP2 - 1);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int kh = half * 2 + (i >> 2), kw = i & 3;                              // uniform
                    const int sub = ((kw >> 1) * 4 + g) * 4 + (kw & 1) * 2 + (kh & 1);
                    b[i] = *(const bf16x8*)(lds + ACT1_OFF + sub * A1_SUB + ((kh >> 1) * 9 + pix) * 16);
                }
            };
            fetch2(0, bq[0]);
#pragma unroll
            for (int t = 0; t < NT2; ++t) {
                if (t + 1 < NT2) fetch2(t + 1, bq[(t + 1) & 1]);
                R2D2_TILE_FENCE;
                acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[t] = mfma16(w2[i], bq[t & 1][i], acc[t]);
                R2D2_TILE_FENCE;
            }
            // swap halves: K half 0 finishes tiles 0..2, K half 1 tiles 3..5
            floatx4* ex = (floatx4*)(lds + EX_OFF);
            auto finish = [&](auto keep0) {
                constexpr int K0 = decltype(keep0)::value, S0 = 3 - K0;
#pragma unroll
                for (int t = 0; t < 3; ++t) ex[(wave * 3 + t) * 64 + lane] = acc[S0 + t];
                __syncthreads();
#pragma unroll
                for (int t = 0; t < 3; ++t) {
                    const int pix = (K0 + t) * 16 + n;
                    const floatx4 v = acc[K0 + t] + ex[(((wave + 4) & 7) * 3 + t) * 64 + lane] + bias2;
                    if (pix < NP2) {
                        // plane 2 f + (g >> 1); copy c holds column ow at ow - c (if that is one of its 7 columns)
                        const int oh = pix / O2, ow = pix - oh * O2;
                        const bf16x4 o = relu_bf16x4(to_bf16x4(v));
                        char* d = lds + ACT2_OFF + (2 * f23 + (g >> 1)) * A2_SUB + (oh * 7 + ow) * 16 + (g & 1) * 8;
                        if (ow < 7) *(bf16x4*)d = o;
                        if (ow >= 1 && ow < 8) *(bf16x4*)(d + 8 * A2_SUB - 16) = o;
                        if (ow >= 2) *(bf16x4*)(d + 16 * A2_SUB - 32) = o;
                    }
                }
            };
            if (half == 0) finish(std::integral_constant<int, 0>{});
            else finish(std::integral_constant<int, 3>{});
        }
        __syncthreads();

        // ---- conv3: 3x3 stride 1, 64 -> 64 channels; this wavefront: feature tile f23, chunks half*9 .. +8 ----
        {
            const floatx4 bias3 = *(const floatx4*)(p.b3 + f23 * 16 + g * 4);
            floatx4 acc[NT3];
            bf16x8 bq[2][9];
            auto fetch3 = [&](int t, bf16x8 (&b)[9]) {
                const int pix = min(t * 16 + n, NP3 - 1);
#pragma unroll
                for (int i = 0; i < 9; ++i) {
                    const int kc = half * 9 + i, tap = kc >> 1, kh = tap / 3, kw = tap - 3 * kh;     // uniform
                    b[i] = *(const bf16x8*)(lds + ACT2_OFF + ((kw * 8 + (kc & 1) * 4 + g) * A2_SUB) + (kh * 7 + pix) * 16);
                }
            };
            fetch3(0, bq[0]);
#pragma unroll
            for (int t = 0; t < NT3; ++t) {
                if (t + 1 < NT3) fetch3(t + 1, bq[(t + 1) & 1]);
                R2D2_TILE_FENCE;
                acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int i = 0; i < 9; ++i) acc[t] = mfma16(w3[i], bq[t & 1][i], acc[t]);
                R2D2_TILE_FENCE;
            }
            floatx4* ex = (floatx4*)(lds + EX_OFF);
            __bf16* frow = p.feat + (size_t)b * p.ldf;
            auto finish = [&](auto keep0) {
                constexpr int K0 = decltype(keep0)::value, S0 = 2 - K0;
#pragma unroll
                for (int t = 0; t < 2; ++t) ex[(wave * 3 + t) * 64 + lane] = acc[S0 + t];
                __syncthreads();
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const int pix = (K0 + t) * 16 + n;
                    const floatx4 v = acc[K0 + t] + ex[(((wave + 4) & 7) * 3 + t) * 64 + lane] + bias3;
                    if (pix < NP3) *(bf16x4*)(frow + pix * 64 + f23 * 16 + g * 4) = relu_bf16x4(to_bf16x4(v));
                }
            };
            if (half == 0) finish(std::integral_constant<int, 0>{});
            else finish(std::integral_constant<int, 2>{});
        }
        // (the next image's first barrier separates these reads of `ex` and `act2` from their next writes)
    }
    stage_wait();
}

}  // namespace seedinf
