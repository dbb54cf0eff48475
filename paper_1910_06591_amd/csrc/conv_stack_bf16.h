// bf16 MFMA implicit-GEMM convolution for the "valid"-padded strided conv
// stack (Appendix A.3.1: kernels 8x8/4, 4x4/2, 3x3/1 with ReLU).
//
// GEMM view: n = output pixel (over the whole batch), m = output channel,
// k = (kh, kw, ci) with ci fastest.  A lane's B fragment is 8 consecutive k:
// because kw*Cin runs are contiguous in an NHWC row and k*Cin is a multiple of
// 8, those 8 values are 8 contiguous elements of the input image, so each lane
// gathers its fragment with one 8- or 16-byte load and nothing is staged.
// The first layer reads the uint8 frame directly: bytes convert to bf16
// exactly, and the 1/255 scale is applied to the fp32 accumulator.
// Per-chunk element offsets (kh*W*Cin + kw*Cin + ci for each of the 4 lane
// groups) come from a small table built on the host.
#pragma once
#include "bf16_common.h"

namespace seedinf {

struct ConvStackArgs {
    const void* x;           // NHWC input: uint8 (first layer) or bf16
    const bf16x8* wp;        // packed A fragments [ftile][kchunk][lane]
    const float* bias;       // [Cout]
    const int* koff;         // [kchunks*4] element offsets of each lane group's fragment
    __bf16* y;               // NHWC bf16 output, ReLU applied
    int B, H, W, Cin, OH, OW, Cout, stride, kchunks;
    float scale;             // 1/255 for the uint8 layer, else 1
};

template <int FT, int RT, bool U8IN>
__global__ __launch_bounds__(256) void conv_stack_bf16_kernel(ConvStackArgs p)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int g = lane >> 4, n = lane & 15;
    const int ft0 = blockIdx.y * FT;
    const long npix = (long)p.B * p.OH * p.OW;
    const long p0 = ((long)blockIdx.x * 4 + wave) * (RT * 16);
    if (p0 >= npix) return;

    long base[RT];
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        long pix = min(p0 + r * 16 + n, npix - 1);
        int ow = (int)(pix % p.OW);
        long t = pix / p.OW;
        int oh = (int)(t % p.OH);
        long b = t / p.OH;
        base[r] = ((b * p.H + (long)oh * p.stride) * p.W + (long)ow * p.stride) * p.Cin;
    }
    floatx4 acc[RT][FT];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int j = 0; j < FT; ++j) acc[r][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    for (int kc = 0; kc < p.kchunks; ++kc) {
        const int ko = p.koff[kc * 4 + g];
        bf16x8 a[FT], b[RT];
#pragma unroll
        for (int j = 0; j < FT; ++j) a[j] = p.wp[((size_t)(ft0 + j) * p.kchunks + kc) * 64 + lane];
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            if constexpr (U8IN) {
                const uint2 v = *(const uint2*)((const uint8_t*)p.x + base[r] + ko);
                b[r] = u8x8_to_bf16x8(v.x, v.y);
            } else {
                b[r] = *(const bf16x8*)((const __bf16*)p.x + base[r] + ko);
            }
        }
#pragma unroll
        for (int r = 0; r < RT; ++r)
#pragma unroll
            for (int j = 0; j < FT; ++j) acc[r][j] = mfma16(a[j], b[r], acc[r][j]);
    }
#pragma unroll
    for (int j = 0; j < FT; ++j) {
        const int f = (ft0 + j) * 16 + g * 4;
        const floatx4 bv = *(const floatx4*)(p.bias + f);
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            const long pix = p0 + r * 16 + n;
            if (pix >= npix) continue;
            floatx4 v = relu4(acc[r][j] * p.scale + bv);
            *(bf16x4*)(p.y + pix * p.Cout + f) = to_bf16x4(v);
        }
    }
}

}  // namespace seedinf
