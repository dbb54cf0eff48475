// Fused deep-ResNet torso (the model Sections 4.1 / 4.2 name) on bf16 MFMA.
//
// One workgroup (8 wavefronts) walks ONE image through every section with all
// activations resident in LDS; a persistent grid strides over the batch.  HBM
// sees only the uint8 frame coming in and the rectified feature vector going
// out, so the torso runs against the matrix-core roofline, not the HBM one.
//
// Per section (conv 3x3 SAME -> max-pool 3x3/2 SAME -> 2 residual blocks):
//   * conv0 runs in strips of pooled rows: the strip's conv rows are written
//     as bf16 to a staging area, then each pooled pixel's owner takes the 3x3
//     maximum (window cells outside the image are replaced by an in-window,
//     in-image cell, which leaves the maximum unchanged).
//   * The residual stream x never leaves registers and stays fp32: pooled
//     pixel tile t (16 pixels) belongs to wavefront t % 8 for the whole
//     section, in the MFMA accumulator layout, so "x + conv_b(...)" is just the
//     MFMA's C operand.  LDS holds only the two rectified bf16 conv inputs
//     R = ReLU(x) and U = ReLU(conv_a(R)), each with a zero halo ring so SAME
//     padding needs no bounds tests in the K loop.
//   * LDS maps are channel-group planar, [C/8][rows+2][cols+2][8 bf16]: a B
//     fragment (8 consecutive input channels of one tap of one pixel) is one
//     16-byte ds_read and the 16 lanes of a lane group read 256 contiguous
//     bytes.
//   * Conv weights live in registers as A fragments (at most 18 per layer).
// The 3-channel first layer keeps its strip as [row][col][4] (one zero lane):
// K = 3 rows x (2 fragments of 2 pixels x 4 channels) = 48, two MFMAs per tile.
// uint8 inputs enter as exact bf16 integers; 1/255 scales the accumulator.
#pragma once
#include "bf16_common.h"

namespace seedinf {

constexpr int RN_WAVES = 8;
constexpr int RN_THREADS = RN_WAVES * 64;

enum { IN_LDS = 0, IN_U8_C3 = 1, IN_U8_PLANAR = 2 };

// Compile-time description of one section.  SR = pooled rows per conv0 strip.
template <int H_, int W_, int CIN_, int C_, int INKIND_, int SR_>
struct SecCfg {
    static constexpr int H = H_, W = W_, CIN = CIN_, C = C_, INKIND = INKIND_, SR = SR_;
    static constexpr int PH = (H + 1) / 2, PW = (W + 1) / 2;
    static constexpr int PADH = (((PH - 1) * 2 + 3 - H) > 0 ? ((PH - 1) * 2 + 3 - H) : 0) / 2;
    static constexpr int PADW = (((PW - 1) * 2 + 3 - W) > 0 ? ((PW - 1) * 2 + 3 - W) : 0) / 2;
    static constexpr int FT = C / 16;
    static constexpr int KC0 = INKIND == IN_U8_C3 ? 2 : (9 * CIN + 31) / 32;
    static constexpr int KCB = (9 * C + 31) / 32;
    static constexpr int NPIX = PH * PW;
    static constexpr int NTILES = (NPIX + 15) / 16;
    static constexpr int NT = (NTILES + RN_WAVES - 1) / RN_WAVES;
    static constexpr int NSTRIPS = (PH + SR - 1) / SR;
    static constexpr int SROWS = 2 * SR + 1;                 // conv rows staged per strip (at most)
    static constexpr int IROWS = SROWS + 2;                  // input rows a strip needs (with halo rows)
    // LDS bytes
    static constexpr int ACT_BYTES = (C / 8) * (PH + 2) * (PW + 2) * 16;      // R or U of this section
    static constexpr int STAGE_BYTES = SROWS * W * C * 2;
    static constexpr int IN_BYTES = INKIND == IN_LDS ? (CIN / 8) * (H + 2) * (W + 2) * 16
                                  : INKIND == IN_U8_C3 ? IROWS * (W + 2) * 8 + 16      // + the cell a kw = 3 fragment half may touch
                                                       : (CIN / 8) * IROWS * (W + 2) * 16;
    static constexpr int BUF0_BYTES = ACT_BYTES > IN_BYTES ? ACT_BYTES : IN_BYTES;
    static constexpr int BUF1_BYTES = ACT_BYTES > STAGE_BYTES ? ACT_BYTES : STAGE_BYTES;
    static_assert(C % 16 == 0, "section channels must be a multiple of 16");
    static_assert(INKIND == IN_U8_C3 ? CIN == 3 : CIN % 8 == 0, "input channels: 3 (uint8) or a multiple of 8");
    static_assert(INKIND != IN_U8_C3 || (W * 3) % 4 == 0, "3-channel rows must be whole dwords");
};

struct SecWeights {
    const bf16x8* w0;        // conv0 A fragments [FT][KC0][64]
    const bf16x8* wb[4];     // block1.a, block1.b, block2.a, block2.b: [FT][KCB][64]
    const float* b0;         // fp32 biases
    const float* bb[4];
};

struct TorsoArgs {
    const uint8_t* obs;      // [B, H, W, Cin]
    SecWeights sec[4];
    __bf16* feat;            // [B, ldf] rectified features, (h, w, c) order
    int ldf;
    int B;
};

template <int N>
__device__ __forceinline__ void load_frags(bf16x8 (&w)[N], const bf16x8* __restrict__ src, int lane)
{
#pragma unroll
    for (int i = 0; i < N; ++i) w[i] = src[i * 64 + lane];
}

// offsets (in 16-byte cells) of each K chunk's fragment relative to the pixel's
// tap (0,0) cell in plane 0, for a planar map with `plane` cells per plane and
// `pitch` cells per row.  Taps past the 9th point at the 9th (their weights are 0).
template <int CIN, int KC>
__device__ __forceinline__ void planar_koff(int (&koff)[KC], int g, int plane, int pitch)
{
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
        int k0 = kc * 32 + g * 8;
        int tap = k0 / CIN;
        int cg = (k0 % CIN) / 8;
        if (tap > 8) { tap = 8; cg = 0; }
        koff[kc] = cg * plane + (tap / 3) * pitch + (tap % 3);
    }
}

// 3x3 SAME conv C -> C on the section's pooled map, this wavefront's tiles.
// src/dst: planar maps with halo.  OUT: 0 = store ReLU(v) to dst, 1 = store v
// to dst, 2 = store ReLU(v) to the global feature row.
template <class S, bool ADD_X, int OUT>
__device__ __forceinline__ void block_conv(const char* src, char* dst, const bf16x8* __restrict__ wsrc,
                                           const float* __restrict__ bias, floatx4 (&x)[S::NT][S::FT],
                                           __bf16* __restrict__ feat_row, int lane, int wave)
{
    constexpr int PITCH = S::PW + 2, PLANE = (S::PH + 2) * PITCH;
    const int g = lane >> 4, n = lane & 15;
    bf16x8 w[S::FT * S::KCB];
    load_frags(w, wsrc, lane);
    int koff[S::KCB];
    planar_koff<S::C, S::KCB>(koff, g, PLANE, PITCH);
    floatx4 bv[S::FT];
#pragma unroll
    for (int j = 0; j < S::FT; ++j) bv[j] = *(const floatx4*)(bias + j * 16 + g * 4);

#pragma unroll
    for (int i = 0; i < S::NT; ++i) {
        const int t = wave + RN_WAVES * i;
        if (t >= S::NTILES) break;
        const int p = t * 16 + n;
        const int pc = p < S::NPIX ? p : S::NPIX - 1;
        const int y = pc / S::PW, xx = pc % S::PW;
        const int base = y * PITCH + xx;
        floatx4 acc[S::FT];
#pragma unroll
        for (int j = 0; j < S::FT; ++j) acc[j] = ADD_X ? x[i][j] + bv[j] : bv[j];
#pragma unroll
        for (int kc = 0; kc < S::KCB; ++kc) {
            const bf16x8 b = *(const bf16x8*)(src + (base + koff[kc]) * 16);
#pragma unroll
            for (int j = 0; j < S::FT; ++j) acc[j] = mfma16(w[j * S::KCB + kc], b, acc[j]);
        }
#pragma unroll
        for (int j = 0; j < S::FT; ++j) {
            if (ADD_X) x[i][j] = acc[j];
            if (p < S::NPIX) {
                const floatx4 v = OUT == 1 ? acc[j] : relu4(acc[j]);
                if (OUT == 2) {
                    *(bf16x4*)(feat_row + (size_t)p * S::C + j * 16 + g * 4) = to_bf16x4(v);
                } else {
                    const int cgo = 2 * j + (g >> 1);
                    *(bf16x4*)(dst + (cgo * PLANE + (y + 1) * PITCH + xx + 1) * 16 + (g & 1) * 8) = to_bf16x4(v);
                }
            }
        }
    }
}

// zero the halo ring of a planar map of CG planes, interior IH x IW
template <int CG, int IH, int IW>
__device__ __forceinline__ void zero_halo(char* buf, int tid)
{
    constexpr int PITCH = IW + 2, ROWS = IH + 2;
    constexpr int RING = 2 * PITCH + 2 * IH;          // cells in one plane's ring
    const bf16x8 z = {};
    for (int i = tid; i < CG * RING; i += RN_THREADS) {
        const int cg = i / RING, r = i % RING;
        int y, xx;
        if (r < PITCH) { y = 0; xx = r; }
        else if (r < 2 * PITCH) { y = ROWS - 1; xx = r - PITCH; }
        else { const int q = r - 2 * PITCH; y = 1 + (q >> 1); xx = (q & 1) ? PITCH - 1 : 0; }
        *(bf16x8*)(buf + ((cg * ROWS + y) * PITCH + xx) * 16) = z;
    }
}

// One section for one image.  On entry (INKIND == IN_LDS) buf0 holds the
// previous section's un-rectified output as a planar map with halo; on exit
// (not LAST) buf0 holds this section's.  LAST writes ReLU(x) to feat_row.
template <class S, bool LAST>
__device__ __forceinline__ void run_section(char* buf0, char* buf1, const SecWeights& sw,
                                            const uint8_t* __restrict__ obs_img, __bf16* __restrict__ feat_row,
                                            int tid)
{
    const int lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, n = lane & 15;
    floatx4 x[S::NT][S::FT];
#pragma unroll
    for (int i = 0; i < S::NT; ++i)
#pragma unroll
        for (int j = 0; j < S::FT; ++j) x[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    // ---------------- conv0 + max-pool, strip by strip ----------------
    {
        bf16x8 w0[S::FT * S::KC0];
        load_frags(w0, sw.w0, lane);
        floatx4 bv[S::FT];
#pragma unroll
        for (int j = 0; j < S::FT; ++j) bv[j] = *(const floatx4*)(sw.b0 + j * 16 + g * 4);
        constexpr float SCALE = S::INKIND == IN_LDS ? 1.0f : 1.0f / 255.0f;
        // input map geometry seen by conv0
        constexpr int IPITCH = S::W + 2;
        constexpr int IPLANE = (S::INKIND == IN_LDS ? S::H + 2 : S::IROWS) * IPITCH;
        int koff[S::KC0];
        if constexpr (S::INKIND == IN_U8_C3) {
            // slot s = kc*4 + g -> (kh = s/2, half = s%2); 8-byte cells
#pragma unroll
            for (int kc = 0; kc < 2; ++kc) {
                int s = kc * 4 + g;
                if (s > 5) s = 0;
                koff[kc] = (s >> 1) * IPITCH + (s & 1) * 2;
            }
        } else {
            planar_koff<S::CIN, S::KC0>(koff, g, IPLANE, IPITCH);
        }

        for (int strip = 0; strip < S::NSTRIPS; ++strip) {
            const int pr0 = strip * S::SR;
            const int pr1 = min(pr0 + S::SR, S::PH);                       // pooled rows [pr0, pr1)
            const int r0 = max(2 * pr0 - S::PADH, 0);
            const int r1 = min(2 * (pr1 - 1) - S::PADH + 2, S::H - 1);     // conv rows [r0, r1]
            const int nrows = r1 - r0 + 1;

            if constexpr (S::INKIND != IN_LDS) {
                // stage input rows r0-1 .. r1+1 of the uint8 frame into buf0 as bf16
                const int nin = nrows + 2;
                if constexpr (S::INKIND == IN_U8_C3) {
                    constexpr int GPR = S::W / 4;                          // 4-pixel groups per row
                    for (int i = tid; i < nin * GPR; i += RN_THREADS) {
                        const int ry = i / GPR, gx = i % GPR;
                        const int iy = r0 - 1 + ry;
                        uint32_t d0 = 0, d1 = 0, d2 = 0;
                        if (iy >= 0 && iy < S::H) {
                            const uint32_t* s = (const uint32_t*)(obs_img + (size_t)iy * S::W * 3) + gx * 3;
                            d0 = s[0]; d1 = s[1]; d2 = s[2];
                        }
                        // 12 bytes = 4 pixels x 3 channels
                        const uint32_t by[12] = {d0 & 0xff, (d0 >> 8) & 0xff, (d0 >> 16) & 0xff, d0 >> 24,
                                                 d1 & 0xff, (d1 >> 8) & 0xff, (d1 >> 16) & 0xff, d1 >> 24,
                                                 d2 & 0xff, (d2 >> 8) & 0xff, (d2 >> 16) & 0xff, d2 >> 24};
                        char* d = buf0 + (ry * IPITCH + gx * 4 + 1) * 8;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            bf16x4 c;
                            c[0] = (__bf16)(float)by[q * 3]; c[1] = (__bf16)(float)by[q * 3 + 1];
                            c[2] = (__bf16)(float)by[q * 3 + 2]; c[3] = (__bf16)0.0f;
                            *(bf16x4*)(d + q * 8) = c;
                        }
                    }
                    const bf16x4 z = {};
                    for (int i = tid; i < nin * 2; i += RN_THREADS)
                        *(bf16x4*)(buf0 + ((i >> 1) * IPITCH + ((i & 1) ? IPITCH - 1 : 0)) * 8) = z;
                    // the (zero-weight) kw = 3 half of the last row's last fragment reads one cell past the strip
                    if (tid == 0) *(bf16x4*)(buf0 + nin * IPITCH * 8) = z;
                } else {
                    constexpr int CG = S::CIN / 8;
                    for (int i = tid; i < nin * S::W * CG; i += RN_THREADS) {
                        const int cg = i % CG, px = (i / CG) % S::W, ry = i / (CG * S::W);
                        const int iy = r0 - 1 + ry;
                        uint2 v = {0u, 0u};
                        if (iy >= 0 && iy < S::H) v = *(const uint2*)(obs_img + ((size_t)iy * S::W + px) * S::CIN + cg * 8);
                        *(bf16x8*)(buf0 + (cg * IPLANE + ry * IPITCH + px + 1) * 16) = u8x8_to_bf16x8(v.x, v.y);
                    }
                    const bf16x8 z = {};
                    for (int i = tid; i < nin * 2 * CG; i += RN_THREADS) {
                        const int cg = i % CG, q = i / CG;
                        *(bf16x8*)(buf0 + (cg * IPLANE + (q >> 1) * IPITCH + ((q & 1) ? IPITCH - 1 : 0)) * 16) = z;
                    }
                }
                __syncthreads();
            }

            // conv rows r0..r1 -> staging (buf1), planes of 4 channels: [C/4][SROWS][W] cells of 8 bytes
            const int npx = nrows * S::W;
            const int ntl = (npx + 15) >> 4;
            // row of the input map that holds conv row r0's tap row kh = 0
            const int ybase = S::INKIND == IN_LDS ? r0 : 0;
            for (int t = wave; t < ntl; t += RN_WAVES) {
                const int p = t * 16 + n;
                const int pc = p < npx ? p : npx - 1;
                const int ry = pc / S::W, xx = pc % S::W;
                const int base = (ybase + ry) * IPITCH + xx;
                floatx4 acc[S::FT];
#pragma unroll
                for (int j = 0; j < S::FT; ++j) acc[j] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kc = 0; kc < S::KC0; ++kc) {
                    bf16x8 b;
                    if constexpr (S::INKIND == IN_U8_C3) {
                        const char* s = buf0 + (base + koff[kc]) * 8;
                        const bf16x4 lo = *(const bf16x4*)s, hi = *(const bf16x4*)(s + 8);
                        b = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    } else {
                        b = *(const bf16x8*)(buf0 + (base + koff[kc]) * 16);
                    }
#pragma unroll
                    for (int j = 0; j < S::FT; ++j) acc[j] = mfma16(w0[j * S::KC0 + kc], b, acc[j]);
                }
                if (p < npx) {
#pragma unroll
                    for (int j = 0; j < S::FT; ++j) {
                        const floatx4 v = acc[j] * SCALE + bv[j];
                        *(bf16x4*)(buf1 + (((4 * j + g) * S::SROWS + ry) * S::W + xx) * 8) = to_bf16x4(v);
                    }
                }
            }
            __syncthreads();

            // pool: owners of pooled rows pr0..pr1-1 take the 3x3 maximum
#pragma unroll
            for (int i = 0; i < S::NT; ++i) {
                const int t = wave + RN_WAVES * i;
                if (t >= S::NTILES) break;
                if (t * 16 + 15 < pr0 * S::PW || t * 16 >= pr1 * S::PW) continue;     // uniform per wavefront
                const int p = t * 16 + n;
                const int py = p / S::PW, px = p % S::PW;
                if (p < S::NPIX && py >= pr0 && py < pr1) {
                    int rr[3], cc[3];
#pragma unroll
                    for (int a = 0; a < 3; ++a) {
                        rr[a] = min(max(2 * py - S::PADH + a, 0), S::H - 1) - r0;
                        cc[a] = min(max(2 * px - S::PADW + a, 0), S::W - 1);
                    }
#pragma unroll
                    for (int j = 0; j < S::FT; ++j) {
                        const char* pl = buf1 + (size_t)((4 * j + g) * S::SROWS) * S::W * 8;
                        floatx4 m = to_floatx4(*(const bf16x4*)(pl + (rr[0] * S::W + cc[0]) * 8));
#pragma unroll
                        for (int a = 0; a < 3; ++a)
#pragma unroll
                            for (int b = 0; b < 3; ++b)
                                if (a | b) m = max4(m, to_floatx4(*(const bf16x4*)(pl + (rr[a] * S::W + cc[b]) * 8)));
                        x[i][j] = m;
                    }
                }
            }
            __syncthreads();
        }
    }

    // ---------------- residual blocks ----------------
    constexpr int PITCH = S::PW + 2, PLANE = (S::PH + 2) * PITCH;
    zero_halo<S::C / 8, S::PH, S::PW>(buf0, tid);
    zero_halo<S::C / 8, S::PH, S::PW>(buf1, tid);
    // R = ReLU(x) into buf0's interior
#pragma unroll
    for (int i = 0; i < S::NT; ++i) {
        const int t = wave + RN_WAVES * i;
        if (t >= S::NTILES) break;
        const int p = t * 16 + n;
        if (p < S::NPIX) {
            const int y = p / S::PW, xx = p % S::PW;
#pragma unroll
            for (int j = 0; j < S::FT; ++j) {
                const int cgo = 2 * j + (g >> 1);
                *(bf16x4*)(buf0 + (cgo * PLANE + (y + 1) * PITCH + xx + 1) * 16 + (g & 1) * 8) = to_bf16x4(relu4(x[i][j]));
            }
        }
    }
    __syncthreads();
    block_conv<S, false, 0>(buf0, buf1, sw.wb[0], sw.bb[0], x, nullptr, lane, wave);
    __syncthreads();
    block_conv<S, true, 0>(buf1, buf0, sw.wb[1], sw.bb[1], x, nullptr, lane, wave);
    __syncthreads();
    block_conv<S, false, 0>(buf0, buf1, sw.wb[2], sw.bb[2], x, nullptr, lane, wave);
    __syncthreads();
    block_conv<S, true, LAST ? 2 : 1>(buf1, buf0, sw.wb[3], sw.bb[3], x, feat_row, lane, wave);
    __syncthreads();
}

template <class S1, class S2, class S3>
struct Net3 {
    static constexpr int B0 = S1::BUF0_BYTES > S2::BUF0_BYTES ? (S1::BUF0_BYTES > S3::BUF0_BYTES ? S1::BUF0_BYTES : S3::BUF0_BYTES)
                                                              : (S2::BUF0_BYTES > S3::BUF0_BYTES ? S2::BUF0_BYTES : S3::BUF0_BYTES);
    static constexpr int B1 = S1::BUF1_BYTES > S2::BUF1_BYTES ? (S1::BUF1_BYTES > S3::BUF1_BYTES ? S1::BUF1_BYTES : S3::BUF1_BYTES)
                                                              : (S2::BUF1_BYTES > S3::BUF1_BYTES ? S2::BUF1_BYTES : S3::BUF1_BYTES);
    static constexpr int LDS_BYTES = B0 + B1;
};

template <class S1, class S2, class S3>
__global__ __launch_bounds__(RN_THREADS) void resnet3_bf16_kernel(TorsoArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    using N = Net3<S1, S2, S3>;
    char* buf0 = lds;
    char* buf1 = lds + N::B0;
    const int tid = threadIdx.x;
    constexpr size_t FRAME = (size_t)S1::H * S1::W * S1::CIN;
    for (int img = blockIdx.x; img < a.B; img += gridDim.x) {
        const uint8_t* obs_img = a.obs + FRAME * img;
        __bf16* feat_row = a.feat + (size_t)img * a.ldf;
        run_section<S1, false>(buf0, buf1, a.sec[0], obs_img, feat_row, tid);
        run_section<S2, false>(buf0, buf1, a.sec[1], obs_img, feat_row, tid);
        run_section<S3, true>(buf0, buf1, a.sec[2], obs_img, feat_row, tid);
    }
}

template <class S1, class S2, class S3, class S4>
struct Net4 {
    using A = Net3<S1, S2, S3>;
    static constexpr int B0 = A::B0 > S4::BUF0_BYTES ? A::B0 : S4::BUF0_BYTES;
    static constexpr int B1 = A::B1 > S4::BUF1_BYTES ? A::B1 : S4::BUF1_BYTES;
    static constexpr int LDS_BYTES = B0 + B1;
};

template <class S1, class S2, class S3, class S4>
__global__ __launch_bounds__(RN_THREADS) void resnet4_bf16_kernel(TorsoArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    using N = Net4<S1, S2, S3, S4>;
    char* buf0 = lds;
    char* buf1 = lds + N::B0;
    const int tid = threadIdx.x;
    constexpr size_t FRAME = (size_t)S1::H * S1::W * S1::CIN;
    for (int img = blockIdx.x; img < a.B; img += gridDim.x) {
        const uint8_t* obs_img = a.obs + FRAME * img;
        __bf16* feat_row = a.feat + (size_t)img * a.ldf;
        run_section<S1, false>(buf0, buf1, a.sec[0], obs_img, feat_row, tid);
        run_section<S2, false>(buf0, buf1, a.sec[1], obs_img, feat_row, tid);
        run_section<S3, false>(buf0, buf1, a.sec[2], obs_img, feat_row, tid);
        run_section<S4, true>(buf0, buf1, a.sec[3], obs_img, feat_row, tid);
    }
}

}  // namespace seedinf
