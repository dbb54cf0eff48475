// Fused deep-ResNet torso (the model Sections 4.1 / 4.2 name) on bf16 MFMA.
//
// One workgroup (8 wavefronts) walks ONE image through every section with all
// activations resident in LDS; a persistent grid strides over the batch.  HBM
// sees only the uint8 frame coming in and the rectified feature vector going
// out, so the torso runs against the matrix-core roofline, not the HBM one.
//
// Per section (conv 3x3 SAME -> max-pool 3x3/2 SAME -> 2 residual blocks):
//   * conv0 + pool: a unit of work is a 16-column strip x a band of pooled
//     rows.  The wavefront walks its unit top to bottom, keeps the last conv
//     row in registers, takes the vertical 3-maximum lane-wise and the
//     horizontal 3-maximum (stride 2) with DPP row shifts, and writes the
//     pooled bf16 value.  The one neighbour column a strip lacks comes from the
//     next strip through a small edge buffer.  The full-resolution conv output
//     never exists in memory.
//   * The residual stream x stays in fp32 registers: pooled pixel tile t (16
//     pixels) belongs to wavefront t % 8 for the whole section, in the MFMA
//     accumulator layout, so "x + conv_b(...)" is the MFMA's C operand.  LDS
//     holds the two rectified bf16 conv inputs R = ReLU(x) and
//     U = ReLU(conv_a(R)), each with a zero halo ring (SAME padding without
//     bounds tests).
//   * LDS maps are channel-group planar, [C/8][rows+2][cols+2][8 bf16]: a B
//     fragment (8 consecutive input channels of one tap of one pixel) is one
//     16-byte ds_read, and the 16 lanes of a lane group read 256 contiguous
//     bytes.
//   * Weights: every wavefront needs the whole A operand of a layer, so the
//     workgroup copies each layer's packed fragments global -> LDS once, one
//     phase ahead (the loads are issued before the current layer's math and
//     committed after it), and the wavefronts fill their registers from LDS.
//   * The uint8 frame (or the next strip of it) is prefetched into registers
//     one phase ahead as well.
// The 3-channel first layer keeps its frame as [row][col][4] (one zero lane):
// K = 3 rows x (2 fragments of 2 pixels x 4 channels) = 48, two MFMAs per tile.
// uint8 inputs enter as exact bf16 integers; 1/255 scales the accumulator.
#pragma once
#include "bf16_common.h"

namespace seedinf {

// Optional developer instrumentation: per-phase cycle totals (summed over workgroups) of the
// torso kernel.  Compiled out unless SEEDINF_PHASE_TIMING is defined.
#ifdef SEEDINF_PHASE_TIMING
__device__ unsigned long long seed_phase_cycles[32];
#define PHASE_MARK(id)                                                                  \
    do {                                                                                \
        if (tid == 0) {                                                                 \
            const unsigned long long now_ = clock64();                                  \
            atomicAdd(&seed_phase_cycles[id], now_ - phase_last_);                      \
            phase_last_ = now_;                                                         \
        }                                                                               \
    } while (0)
#define PHASE_DECL unsigned long long phase_last_ = clock64()
#else
#define PHASE_MARK(id) do { } while (0)
#define PHASE_DECL do { } while (0)
#endif

constexpr int RN_WAVES = 8;
constexpr int RN_THREADS = RN_WAVES * 64;
constexpr int LDS_TOTAL = 160 * 1024;
constexpr int WSLOT_BYTES = 19 * 1024;          // largest layer: 18 fragments of 1 KiB + the bias chunk

enum { IN_LDS = 0, IN_U8_C3 = 1, IN_U8_PLANAR = 2 };

// Workgroup barrier for LDS-only communication: waits for this wavefront's LDS
// traffic, not for its outstanding global loads (the prefetches stay in flight).
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Compile-time description of one section.
//   NB = bands of pooled rows per conv0 pass, SR = pooled rows per input strip
//   (uint8 sections only; IN_LDS sections have their whole input resident).
template <int H_, int W_, int CIN_, int C_, int INKIND_, int NB_, int SR_>
struct SecCfg {
    static constexpr int H = H_, W = W_, CIN = CIN_, C = C_, INKIND = INKIND_, NB = NB_;
    static constexpr int PH = (H + 1) / 2, PW = (W + 1) / 2;
    static constexpr int PADH = (((PH - 1) * 2 + 3 - H) > 0 ? ((PH - 1) * 2 + 3 - H) : 0) / 2;
    static constexpr int SR = INKIND == IN_LDS ? PH : SR_;
    static constexpr int NSTRIPS = (PH + SR - 1) / SR;
    static constexpr int FT = C / 16;
    static constexpr int KC0 = INKIND == IN_U8_C3 ? 2 : (9 * CIN + 31) / 32;
    static constexpr int KCB = (9 * C + 31) / 32;
    static constexpr int W0_FRAGS = FT * KC0, WB_FRAGS = FT * KCB;
    // a staged weight set = the fragments + one 1 KiB chunk whose first C floats are the biases
    static constexpr int W0_SET = W0_FRAGS + 1, WB_SET = WB_FRAGS + 1;
    static constexpr int NPIX = PH * PW;
    static constexpr int NTILES = (NPIX + 15) / 16;
    static constexpr int NT = (NTILES + RN_WAVES - 1) / RN_WAVES;
    static constexpr int NCS = (W + 15) / 16;               // 16-column strips of the conv0 output
    static constexpr int NUNITS = NCS * NB;
    static constexpr int NU = (NUNITS + RN_WAVES - 1) / RN_WAVES;
    // input map of conv0 as it sits in buf0
    static constexpr int IROWS = INKIND == IN_LDS ? H + 2 : (2 * SR + 1 < H ? 2 * SR + 1 : H) + 2;
    static constexpr int IPITCH = W + 2;
    static constexpr int ICELL = INKIND == IN_U8_C3 ? 8 : 16;
    static constexpr int IPLANE = IROWS * IPITCH;
    static constexpr int IN_BYTES = (INKIND == IN_U8_C3 ? 1 : CIN / 8) * IPLANE * ICELL + 16;
    static constexpr int PITCH = PW + 2, PLANE = (PH + 2) * PITCH;
    static constexpr int ACT_BYTES = (C / 8) * PLANE * 16;
    static constexpr int EDGE_BYTES = NCS * PH * C * 2;
    // prefetch registers for the uint8 input: items of PRE_DW dwords, PRE_N per thread
    static constexpr int PRE_DW = INKIND == IN_U8_C3 ? 3 : (INKIND == IN_U8_PLANAR ? CIN / 4 : 1);
    static constexpr int PRE_ITEMS = INKIND == IN_U8_C3 ? (IROWS - 2) * (W / 4) : (INKIND == IN_U8_PLANAR ? (IROWS - 2 + 2) * W : 0);
    static constexpr int PRE_N = INKIND == IN_LDS ? 1 : (PRE_ITEMS + RN_THREADS - 1) / RN_THREADS;
    static_assert(C % 16 == 0, "section channels must be a multiple of 16");
    static_assert(W % 2 == 0, "even width (pool padding only after the last column)");
    static_assert(INKIND == IN_U8_C3 ? CIN == 3 : CIN % 8 == 0, "input channels: 3 (uint8) or a multiple of 8");
    static_assert(INKIND != IN_U8_C3 || ((W * 3) % 4 == 0 && W % 4 == 0), "3-channel rows must be whole dwords");
    static_assert(INKIND != IN_U8_PLANAR || CIN == 16, "planar uint8 input: 16 channels");
    static_assert(INKIND != IN_U8_C3 || NSTRIPS == 1, "the 3-channel frame is kept whole");
};

struct SecWeights {
    const bf16x8* w0;        // conv0 weight set: A fragments [FT][KC0][64], then the bias chunk
    const bf16x8* wb[4];     // block1.a, block1.b, block2.a, block2.b: [FT][KCB][64] + bias chunk
};

struct TorsoArgs {
    const uint8_t* obs;      // [B, H, W, Cin]
    SecWeights sec[4];
    __bf16* feat;            // [B, ldf] rectified features, (h, w, c) order
    int ldf;
    int B;
};

// ---- weight staging: global -> registers (issue) -> LDS slot (commit) -> A fragments ----
template <int NF>
struct WStage {
    static constexpr int N = (NF * 64 + RN_THREADS - 1) / RN_THREADS;
    bf16x8 r[N];
};

template <int NF>
__device__ __forceinline__ void wstage_issue(WStage<NF>& s, const bf16x8* __restrict__ src, int tid)
{
#pragma unroll
    for (int j = 0; j < WStage<NF>::N; ++j) {
        const int i = tid + j * RN_THREADS;
        if (i < NF * 64) s.r[j] = src[i];
    }
}

template <int NF>
__device__ __forceinline__ void wstage_commit(const WStage<NF>& s, char* slot, int tid)
{
#pragma unroll
    for (int j = 0; j < WStage<NF>::N; ++j) {
        const int i = tid + j * RN_THREADS;
        if (i < NF * 64) *(bf16x8*)(slot + i * 16) = s.r[j];
    }
}

template <int NF>
__device__ __forceinline__ void load_a_frags(bf16x8 (&w)[NF], const char* slot, int lane)
{
#pragma unroll
    for (int i = 0; i < NF; ++i) w[i] = *(const bf16x8*)(slot + (i * 64 + lane) * 16);
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

// ---- uint8 frame prefetch --------------------------------------------------------
template <class S>
struct Prefetch {
    uint32_t d[S::PRE_N][S::PRE_DW];
};

// conv rows [r0, r1] of the strip that covers pooled rows [pr0, pr1)
template <class S>
__device__ __forceinline__ void strip_rows(int strip, int& pr0, int& pr1, int& r0, int& r1)
{
    pr0 = strip * S::SR;
    pr1 = min(pr0 + S::SR, S::PH);
    r0 = max(2 * pr0 - S::PADH, 0);
    r1 = min(2 * (pr1 - 1) - S::PADH + 2, S::H - 1);
}

// issue the global loads for input rows r0-1 .. r1+1 of `obs_img`
template <class S>
__device__ __forceinline__ void prefetch_issue(Prefetch<S>& p, const uint8_t* __restrict__ obs_img, int strip, int tid)
{
    if constexpr (S::INKIND != IN_LDS) {
        int pr0, pr1, r0, r1;
        strip_rows<S>(strip, pr0, pr1, r0, r1);
        if constexpr (S::INKIND == IN_U8_C3) {
            constexpr int GPR = S::W / 4;
            const int nitems = (r1 - r0 + 1) * GPR;            // real rows only (whole frame: r0 = 0, r1 = H-1)
#pragma unroll
            for (int j = 0; j < S::PRE_N; ++j) {
                const int i = tid + j * RN_THREADS;
                if (i < nitems) {
                    const uint32_t* s = (const uint32_t*)(obs_img + (size_t)(r0 + i / GPR) * S::W * 3) + (i % GPR) * 3;
                    p.d[j][0] = s[0]; p.d[j][1] = s[1]; p.d[j][2] = s[2];
                }
            }
        } else {
            const int nin = r1 - r0 + 3;
#pragma unroll
            for (int j = 0; j < S::PRE_N; ++j) {
                const int i = tid + j * RN_THREADS;
                const int ry = i / S::W, px = i % S::W;
                const int iy = r0 - 1 + ry;
#pragma unroll
                for (int q = 0; q < S::PRE_DW; ++q) p.d[j][q] = 0u;
                if (ry < nin && iy >= 0 && iy < S::H) {
                    const uint4 v = *(const uint4*)(obs_img + ((size_t)iy * S::W + px) * S::CIN);
                    p.d[j][0] = v.x; p.d[j][1] = v.y; p.d[j][2] = v.z; p.d[j][3] = v.w;
                }
            }
        }
    }
}

// convert the prefetched bytes to bf16 and lay them out in buf0 (with zero halo)
template <class S>
__device__ __forceinline__ void prefetch_commit(const Prefetch<S>& p, char* buf0, int strip, int tid)
{
    if constexpr (S::INKIND != IN_LDS) {
        int pr0, pr1, r0, r1;
        strip_rows<S>(strip, pr0, pr1, r0, r1);
        const int nin = r1 - r0 + 3;                           // buffer rows: input rows r0-1 .. r1+1
        if constexpr (S::INKIND == IN_U8_C3) {
            constexpr int GPR = S::W / 4;
            const int nitems = (r1 - r0 + 1) * GPR;
#pragma unroll
            for (int j = 0; j < S::PRE_N; ++j) {
                const int i = tid + j * RN_THREADS;
                if (i < nitems) {
                    const uint32_t d0 = p.d[j][0], d1 = p.d[j][1], d2 = p.d[j][2];
                    const uint32_t by[12] = {d0 & 0xff, (d0 >> 8) & 0xff, (d0 >> 16) & 0xff, d0 >> 24,
                                             d1 & 0xff, (d1 >> 8) & 0xff, (d1 >> 16) & 0xff, d1 >> 24,
                                             d2 & 0xff, (d2 >> 8) & 0xff, (d2 >> 16) & 0xff, d2 >> 24};
                    // buffer row of image row iy is iy - (r0 - 1); whole frame: r0 = 0 -> iy + 1
                    char* d = buf0 + ((i / GPR + 1) * S::IPITCH + (i % GPR) * 4 + 1) * 8;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        bf16x4 c;
                        c[0] = (__bf16)(float)by[q * 3]; c[1] = (__bf16)(float)by[q * 3 + 1];
                        c[2] = (__bf16)(float)by[q * 3 + 2]; c[3] = (__bf16)0.0f;
                        *(bf16x4*)(d + q * 8) = c;
                    }
                }
            }
            const bf16x4 z = {};
            // halo: first and last buffer rows, first and last columns, and the cell past the end that
            // the (zero-weight) kw = 3 half of the last fragment may touch
            for (int i = tid; i < 2 * S::IPITCH; i += RN_THREADS)
                *(bf16x4*)(buf0 + ((i < S::IPITCH ? 0 : nin - 1) * S::IPITCH + (i % S::IPITCH)) * 8) = z;
            for (int i = tid; i < nin * 2; i += RN_THREADS)
                *(bf16x4*)(buf0 + ((i >> 1) * S::IPITCH + ((i & 1) ? S::IPITCH - 1 : 0)) * 8) = z;
            if (tid == 0) *(bf16x4*)(buf0 + nin * S::IPITCH * 8) = z;
        } else {
#pragma unroll
            for (int j = 0; j < S::PRE_N; ++j) {
                const int i = tid + j * RN_THREADS;
                const int ry = i / S::W, px = i % S::W;
                if (ry < nin) {
                    *(bf16x8*)(buf0 + (ry * S::IPITCH + px + 1) * 16) = u8x8_to_bf16x8(p.d[j][0], p.d[j][1]);
                    *(bf16x8*)(buf0 + (S::IPLANE + ry * S::IPITCH + px + 1) * 16) = u8x8_to_bf16x8(p.d[j][2], p.d[j][3]);
                }
            }
            const bf16x8 z = {};
            for (int i = tid; i < nin * 4; i += RN_THREADS) {
                const int cg = i & 1, q = i >> 1;
                *(bf16x8*)(buf0 + (cg * S::IPLANE + (q >> 1) * S::IPITCH + ((q & 1) ? S::IPITCH - 1 : 0)) * 16) = z;
            }
        }
    }
}

// ---- conv0 + max-pool ----------------------------------------------------------------
// h[n] = max(v[n], v[n+1], v[n+2]) within each row of 16 lanes; lanes whose neighbour lies outside the
// row keep the partial maximum (a DPP op with an invalid source lane leaves its destination untouched).
__device__ __forceinline__ float hmax3_row16(float v)
{
#ifdef SEEDINF_DPP_BUILTIN
    const int i = __builtin_bit_cast(int, v);
    const float s1 = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(i, i, 0x101, 0xf, 0xf, false));
    const float s2 = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(i, i, 0x102, 0xf, 0xf, false));
    return fmaxf(fmaxf(v, s1), s2);
#endif
    // h and v must be different registers: the second op still needs the unshifted v
    float h;
    asm volatile("v_mov_b32 %0, %1\n\ts_nop 0\n\t"
                 "v_max_f32_dpp %0, %1, %0 row_shl:1 row_mask:0xf bank_mask:0xf\n\t"
                 "v_max_f32_dpp %0, %1, %0 row_shl:2 row_mask:0xf bank_mask:0xf"
                 : "=&v"(h) : "v"(v));
    return h;
}

// B fragments of one conv0 output tile (16 consecutive columns of one conv row); `base` = cell index of
// the tile's tap (0,0) in plane 0.
template <class S>
__device__ __forceinline__ void conv0_load(bf16x8 (&b)[S::KC0], const char* in, int base, const int (&koff)[S::KC0])
{
#pragma unroll
    for (int kc = 0; kc < S::KC0; ++kc) {
        if constexpr (S::INKIND == IN_U8_C3) {
            const char* s = in + (base + koff[kc]) * 8;
            const bf16x4 lo = *(const bf16x4*)s, hi = *(const bf16x4*)(s + 8);
            b[kc] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        } else {
            b[kc] = *(const bf16x8*)(in + (base + koff[kc]) * 16);
        }
    }
}

template <class S>
__device__ __forceinline__ void conv0_mma(floatx4 (&acc)[S::FT], const bf16x8 (&b)[S::KC0], const bf16x8 (&w0)[S::W0_FRAGS])
{
#pragma unroll
    for (int j = 0; j < S::FT; ++j) acc[j] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kc = 0; kc < S::KC0; ++kc)
#pragma unroll
        for (int j = 0; j < S::FT; ++j) acc[j] = mfma16(w0[j * S::KC0 + kc], b[kc], acc[j]);
}

// conv0 + pool over pooled rows [pr0, pr1); `rbuf0` = image row held by buffer row 0 of `in`
// (so conv row r's tap row kh sits in buffer row r - 1 + kh - rbuf0).  Writes un-rectified
// pooled bf16 values into `xout` (planar map with halo, this section's pooled geometry) and
// each strip's first-column vertical maxima into `edge`.  `wslot`: conv0's staged weight set.
template <class S>
__device__ __forceinline__ void conv0_pool(const char* in, char* xout, char* edge, const bf16x8 (&w0)[S::W0_FRAGS],
                                           const char* wslot, int pr0, int pr1, int rbuf0, int lane, int wave)
{
    const int g = lane >> 4, n = lane & 15;
    constexpr float SCALE = S::INKIND == IN_LDS ? 1.0f : 1.0f / 255.0f;
    constexpr bool FULL = S::W % 16 == 0;                 // no partial column strip
    floatx4 bv[S::FT];
#pragma unroll
    for (int j = 0; j < S::FT; ++j) bv[j] = *(const floatx4*)(wslot + S::W0_FRAGS * 1024 + (j * 4 + g) * 16);
    int koff[S::KC0];
    if constexpr (S::INKIND == IN_U8_C3) {
        // K slot s = kc*4 + g -> (kernel row s/2, pixel pair s%2); 8-byte cells
#pragma unroll
        for (int kc = 0; kc < 2; ++kc) {
            int s = kc * 4 + g;
            if (s > 5) s = 0;
            koff[kc] = (s >> 1) * S::IPITCH + (s & 1) * 2;
        }
    } else {
        planar_koff<S::CIN, S::KC0>(koff, g, S::IPLANE, S::IPITCH);
    }
    const int npr = pr1 - pr0;
    const floatx4 NEG = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};

#pragma unroll 1
    for (int ui = 0; ui < S::NU; ++ui) {
        const int u = wave + RN_WAVES * ui;
        if (u >= S::NUNITS) break;
        const int cs = u % S::NCS, b = u / S::NCS;
        const int pb0 = pr0 + b * npr / S::NB, pb1 = pr0 + (b + 1) * npr / S::NB;
        if (pb0 >= pb1) continue;
        const int col = cs * 16 + n;
        const bool live = FULL || col < S::W;
        const int colc = live ? col : S::W - 1;
        // cell index of conv row r, tap (0,0): (r - 1 - rbuf0) * IPITCH + colc
        const int cbase = colc - (1 + rbuf0) * S::IPITCH;
        floatx4 top[S::FT], mid[S::FT], bot[S::FT];
        bf16x8 fa[S::KC0], fb[S::KC0];
        const int rt = 2 * pb0 - S::PADH;
        if (rt >= 0) {
            conv0_load<S>(fa, in, cbase + rt * S::IPITCH, koff);
            conv0_mma<S>(top, fa, w0);
        } else {
#pragma unroll
            for (int j = 0; j < S::FT; ++j) top[j] = NEG;
        }
        // output addresses of this unit's first pooled row; they advance by one row per iteration
        const int px = col >> 1;
        int xoff = ((pb0 + 1) * S::PITCH + px + 1) * 16 + (g >> 1) * (S::PLANE * 16) + (g & 1) * 8;
        int eoff = ((cs * S::PH + pb0) * S::C + g * 4) * 2;
#pragma unroll 1
        for (int py = pb0; py < pb1; ++py) {
            const int rm = 2 * py - S::PADH + 1;
            const bool has_bot = rm + 1 < S::H;             // uniform
            conv0_load<S>(fa, in, cbase + rm * S::IPITCH, koff);
            conv0_load<S>(fb, in, cbase + (has_bot ? rm + 1 : rm) * S::IPITCH, koff);
            conv0_mma<S>(mid, fa, w0);
            conv0_mma<S>(bot, fb, w0);
#pragma unroll
            for (int j = 0; j < S::FT; ++j) {
                floatx4 v = max4(max4(top[j], mid[j]), bot[j]) * SCALE + bv[j];
                if (!FULL && !live) v = NEG;
                if (n == 0 && cs > 0) *(bf16x4*)(edge + eoff + j * 32) = to_bf16x4(v);
                floatx4 h;
#pragma unroll
                for (int i = 0; i < 4; ++i) h[i] = hmax3_row16(v[i]);
                if (live && !(n & 1)) *(bf16x4*)(xout + xoff + j * (2 * S::PLANE * 16)) = to_bf16x4(h);
                top[j] = bot[j];
            }
            xoff += S::PITCH * 16;
            eoff += S::C * 2;
        }
    }
}

// 3x3 SAME conv C -> C on the section's pooled map, this wavefront's tiles.
// src/dst: planar maps with halo.  OUT: 0 = store ReLU(v) to dst, 1 = store v
// to dst, 2 = store ReLU(v) to the global feature row.  The B fragments of tile
// i+1 are read from LDS while tile i's MFMAs run.
template <class S, bool ADD_X, int OUT>
__device__ __forceinline__ void block_conv(const char* src, char* dst, const char* wslot,
                                           floatx4 (&x)[S::NT][S::FT], __bf16* __restrict__ feat_row, int lane, int wave)
{
    const int g = lane >> 4, n = lane & 15;
    bf16x8 w[S::WB_FRAGS];
    load_a_frags(w, wslot, lane);
    floatx4 bv[S::FT];
#pragma unroll
    for (int j = 0; j < S::FT; ++j) bv[j] = *(const floatx4*)(wslot + S::WB_FRAGS * 1024 + (j * 4 + g) * 16);
    int koff[S::KCB];
    planar_koff<S::C, S::KCB>(koff, g, S::PLANE, S::PITCH);

    auto tile_base = [&](int i, int& p, int& y, int& xx) {
        p = (wave + RN_WAVES * i) * 16 + n;
        const int pc = p < S::NPIX ? p : S::NPIX - 1;
        y = pc / S::PW; xx = pc % S::PW;
        return y * S::PITCH + xx;
    };
    bf16x8 bcur[S::KCB], bnxt[S::KCB];
    int p, y, xx;
    {
        const int base = tile_base(0, p, y, xx);
#pragma unroll
        for (int kc = 0; kc < S::KCB; ++kc) bcur[kc] = *(const bf16x8*)(src + (base + koff[kc]) * 16);
    }
#pragma unroll
    for (int i = 0; i < S::NT; ++i) {
        const int t = wave + RN_WAVES * i;
        if (t >= S::NTILES) break;
        int pn = 0, yn = 0, xn = 0;
        const bool more = i + 1 < S::NT && t + RN_WAVES < S::NTILES;     // uniform
        if (more) {
            const int base = tile_base(i + 1, pn, yn, xn);
#pragma unroll
            for (int kc = 0; kc < S::KCB; ++kc) bnxt[kc] = *(const bf16x8*)(src + (base + koff[kc]) * 16);
        }
        floatx4 acc[S::FT];
#pragma unroll
        for (int j = 0; j < S::FT; ++j) acc[j] = ADD_X ? x[i][j] + bv[j] : bv[j];
#pragma unroll
        for (int kc = 0; kc < S::KCB; ++kc)
#pragma unroll
            for (int j = 0; j < S::FT; ++j) acc[j] = mfma16(w[j * S::KCB + kc], bcur[kc], acc[j]);
#pragma unroll
        for (int j = 0; j < S::FT; ++j) {
            if (ADD_X) x[i][j] = acc[j];
            if (p < S::NPIX) {
                const floatx4 v = OUT == 1 ? acc[j] : relu4(acc[j]);
                if (OUT == 2) {
                    *(bf16x4*)(feat_row + (size_t)p * S::C + j * 16 + g * 4) = to_bf16x4(v);
                } else {
                    const int cgo = 2 * j + (g >> 1);
                    *(bf16x4*)(dst + (cgo * S::PLANE + (y + 1) * S::PITCH + xx + 1) * 16 + (g & 1) * 8) = to_bf16x4(v);
                }
            }
        }
        if (more) {
#pragma unroll
            for (int kc = 0; kc < S::KCB; ++kc) bcur[kc] = bnxt[kc];
            p = pn; y = yn; xx = xn;
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

// LDS layout shared by the sections of one network.
template <int B0_, int B1_, int EDGE_, int PERM_>
struct LdsMap {
    static constexpr int r256(int v) { return (v + 255) / 256 * 256; }
    static constexpr int BUF0 = 0;
    static constexpr int BUF1 = r256(B0_);
    static constexpr int EDGE = BUF1 + r256(B1_);
    static constexpr int WSA = EDGE + r256(EDGE_);
    static constexpr int WSB_HI = WSA + WSLOT_BYTES;
    static constexpr int PERM = LDS_TOTAL - r256(PERM_);           // first layer's weights, resident for the whole kernel
    static constexpr int WSB_HI_CAP = PERM - WSB_HI;
    static constexpr int WSB_LO = BUF1 + 36 * 1024;                // inside buf1's tail: only while buf1 holds <= 36 KiB
    static_assert(WSB_HI_CAP >= 0, "LDS layout does not fit");
    static_assert(WSB_LO + WSLOT_BYTES <= EDGE, "low weight slot must fit in buf1's tail");
};

// Where one section finds its five layers' weight sets in LDS and what it stages for the next section.
//   C0, B0..B3: byte offsets of the conv0 / block-layer slots.  STAGE_B0: conv0's phase stages B0.
//   NEXT / NEXT_SET: slot and size (KiB chunks) of the set staged during the last block (0: nothing).
template <int C0_, int B0_, int B1_, int B2_, int B3_, int NEXT_, int NEXT_SET_, bool STAGE_B0_>
struct Slots {
    static constexpr int C0 = C0_, B0 = B0_, B1 = B1_, B2 = B2_, B3 = B3_, NEXT = NEXT_, NEXT_SET = NEXT_SET_;
    static constexpr bool STAGE_B0 = STAGE_B0_;
};

// One section for one image.  On entry (INKIND == IN_LDS) buf0 holds the previous section's un-rectified
// output as a planar map with halo; on exit (not LAST) buf0 holds this section's.  LAST writes ReLU(x) to
// feat_row.  next_src: global address of the weight set SL::NEXT receives.
template <class S, class M, class SL, bool LAST, int SI, class PreT>
__device__ __forceinline__ void run_section(char* lds, const SecWeights& sw, const bf16x8* __restrict__ next_src,
                                            const uint8_t* __restrict__ obs_img, PreT& pre,
                                            __bf16* __restrict__ feat_row, int tid)
{
    // keep per-tile index arithmetic inside the image loop: hoisted out of it, it would occupy
    // (and spill) hundreds of registers for the whole kernel
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, n = lane & 15;
    char* buf0 = lds + M::BUF0;
    char* buf1 = lds + M::BUF1;
    char* edge = lds + M::EDGE;
    static_assert(S::ACT_BYTES <= 36 * 1024 || (SL::C0 != M::WSB_LO && SL::B0 != M::WSB_LO && SL::B1 != M::WSB_LO &&
                                                 SL::B2 != M::WSB_LO && SL::B3 != M::WSB_LO),
                  "low weight slot used while buf1 is fully occupied");
    static_assert(S::WB_SET * 1024 <= WSLOT_BYTES && S::W0_SET * 1024 <= WSLOT_BYTES, "weight set larger than a slot");
    floatx4 x[S::NT][S::FT];
    PHASE_DECL;

    // ---------------- conv0 + max-pool ----------------
    {
        WStage<S::WB_SET> st;
        if constexpr (SL::STAGE_B0) wstage_issue(st, sw.wb[0], tid);
        zero_halo<S::C / 8, S::PH, S::PW>(buf1, tid);
        bf16x8 w0[S::W0_FRAGS];
        if constexpr (S::INKIND == IN_LDS) {
            load_a_frags(w0, lds + SL::C0, lane);
            conv0_pool<S>(buf0, buf1, edge, w0, lds + SL::C0, 0, S::PH, -1, lane, wave);
        } else {
#pragma unroll 1
            for (int strip = 0; strip < S::NSTRIPS; ++strip) {
                prefetch_commit<S>(pre, buf0, strip, tid);
                if (strip + 1 < S::NSTRIPS) prefetch_issue<S>(pre, obs_img, strip + 1, tid);
                lds_barrier();
                PHASE_MARK(SI * 8 + 0);
                if (strip == 0) load_a_frags(w0, lds + SL::C0, lane);
                int pr0, pr1, r0, r1;
                strip_rows<S>(strip, pr0, pr1, r0, r1);
                conv0_pool<S>(buf0, buf1, edge, w0, lds + SL::C0, pr0, pr1, r0 - 1, lane, wave);
                if (strip + 1 < S::NSTRIPS) lds_barrier();
            }
        }
        if constexpr (SL::STAGE_B0) wstage_commit(st, lds + SL::B0, tid);
        lds_barrier();
        PHASE_MARK(SI * 8 + 1);
    }

    // ---------------- x <- pooled map (+ edge columns); R = ReLU(x) ----------------
    {
        WStage<S::WB_SET> st;
        wstage_issue(st, sw.wb[1], tid);
        zero_halo<S::C / 8, S::PH, S::PW>(buf0, tid);
#pragma unroll
        for (int i = 0; i < S::NT; ++i) {
            const int t = wave + RN_WAVES * i;
            if (t >= S::NTILES) break;
            const int p = t * 16 + n;
            const bool ok = p < S::NPIX;
            const int pc = ok ? p : S::NPIX - 1;
            const int y = pc / S::PW, xx = pc % S::PW;
            // the pooled value of a strip's last column lacks its right neighbour: it is the next strip's edge column
            const bool fix = (xx & 7) == 7 && xx + 1 < S::PW;
            const int cs = fix ? (xx + 1) >> 3 : 0;
            const int off = ((y + 1) * S::PITCH + xx + 1) * 16 + (g >> 1) * (S::PLANE * 16) + (g & 1) * 8;
            const int eoff = ((cs * S::PH + y) * S::C + g * 4) * 2;
            bf16x4 pv[S::FT], ev[S::FT];
#pragma unroll
            for (int j = 0; j < S::FT; ++j) {
                pv[j] = *(const bf16x4*)(buf1 + off + j * (2 * S::PLANE * 16));
                ev[j] = *(const bf16x4*)(edge + eoff + j * 32);
            }
#pragma unroll
            for (int j = 0; j < S::FT; ++j) {
                floatx4 v = to_floatx4(pv[j]);
                const floatx4 e = to_floatx4(ev[j]);
                if (fix) v = max4(v, e);
                if (!ok) v = floatx4{0.f, 0.f, 0.f, 0.f};
                x[i][j] = v;
                if (ok) *(bf16x4*)(buf0 + off + j * (2 * S::PLANE * 16)) = to_bf16x4(relu4(v));
            }
        }
        lds_barrier();
        PHASE_MARK(SI * 8 + 3);

        // ---------------- residual blocks ----------------
        block_conv<S, false, 0>(buf0, buf1, lds + SL::B0, x, nullptr, lane, wave);
        wstage_commit(st, lds + SL::B1, tid);
        lds_barrier();
        PHASE_MARK(SI * 8 + 4);
        wstage_issue(st, sw.wb[2], tid);
        block_conv<S, true, 0>(buf1, buf0, lds + SL::B1, x, nullptr, lane, wave);
        wstage_commit(st, lds + SL::B2, tid);
        lds_barrier();
        PHASE_MARK(SI * 8 + 5);
        wstage_issue(st, sw.wb[3], tid);
        block_conv<S, false, 0>(buf0, buf1, lds + SL::B2, x, nullptr, lane, wave);
        wstage_commit(st, lds + SL::B3, tid);
        lds_barrier();
        PHASE_MARK(SI * 8 + 6);
    }
    {
        WStage<(SL::NEXT_SET > 0 ? SL::NEXT_SET : 1)> st;
        if constexpr (SL::NEXT_SET > 0) wstage_issue(st, next_src, tid);
        block_conv<S, true, LAST ? 2 : 1>(buf1, buf0, lds + SL::B3, x, feat_row, lane, wave);
        if constexpr (SL::NEXT_SET > 0) wstage_commit(st, lds + SL::NEXT, tid);
        lds_barrier();
        PHASE_MARK(SI * 8 + 7);
    }
}

// Slot plan shared by both networks: the first layer's set is resident; every other set is staged one
// phase before its use, alternating between slot A and slot B (B = the high slot while buf1 is full,
// i.e. during section 1, else the low slot inside buf1's unused tail).  Section 2's conv0 is staged
// during section 1's last block, so it must sit in A; the alternation below guarantees that.
template <class M, class S, class SN, bool FIRST, bool HAS_NEXT>
struct SlotPlan {
    static constexpr int A = M::WSA;
    static constexpr int B = S::ACT_BYTES > 36 * 1024 ? M::WSB_HI : M::WSB_LO;
    static constexpr int BN = SN::ACT_BYTES > 36 * 1024 ? M::WSB_HI : M::WSB_LO;   // B as the next section sees it
    static_assert(S::ACT_BYTES <= 36 * 1024 || S::WB_SET * 1024 <= M::WSB_HI_CAP, "block weights do not fit the high slot");
    // first section: conv0 resident, blocks A B A B, next conv0 -> A
    // later sections alternate between (conv0 A, blocks B A B A, next -> B) and (conv0 B, blocks A B A B, next -> A)
    using First = Slots<M::PERM, A, B, A, B, A, HAS_NEXT ? SN::W0_SET : 0, true>;
    using EvenC0A = Slots<A, B, A, B, A, BN, HAS_NEXT ? SN::W0_SET : 0, true>;
    using OddC0B = Slots<B, A, B, A, B, A, HAS_NEXT ? SN::W0_SET : 0, true>;
};

template <class S1, class S2, class S3>
struct Net3 {
    static constexpr int mx(int a, int b) { return a > b ? a : b; }
    static constexpr int B0 = mx(mx(mx(S1::ACT_BYTES, S1::IN_BYTES), mx(S2::ACT_BYTES, S2::IN_BYTES)), mx(S3::ACT_BYTES, S3::IN_BYTES));
    static constexpr int B1 = mx(mx(S1::ACT_BYTES, S2::ACT_BYTES), S3::ACT_BYTES);
    static constexpr int EDGE = mx(mx(S1::EDGE_BYTES, S2::EDGE_BYTES), S3::EDGE_BYTES);
    using M = LdsMap<B0, B1, EDGE, S1::W0_SET * 1024>;
    using SL1 = typename SlotPlan<M, S1, S2, true, true>::First;
    using SL2 = typename SlotPlan<M, S2, S3, false, true>::EvenC0A;
    using SL3 = typename SlotPlan<M, S3, S3, false, false>::OddC0B;
    static constexpr int LDS_BYTES = LDS_TOTAL;
};

template <class S1, class S2, class S3>
__global__ __launch_bounds__(RN_THREADS) void resnet3_bf16_kernel(TorsoArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    using N = Net3<S1, S2, S3>;
    using M = typename N::M;
    const int tid = threadIdx.x;
    constexpr size_t FRAME = (size_t)S1::H * S1::W * S1::CIN;
    if ((int)blockIdx.x >= a.B) return;
    {   // the resident first-layer weight set
        WStage<S1::W0_SET> s0;
        wstage_issue(s0, a.sec[0].w0, tid);
        wstage_commit(s0, lds + M::PERM, tid);
    }
    Prefetch<S1> pre;
    prefetch_issue<S1>(pre, a.obs + FRAME * blockIdx.x, 0, tid);
    for (int img = blockIdx.x; img < a.B; img += gridDim.x) {
        const uint8_t* obs_img = a.obs + FRAME * img;
        __bf16* feat_row = a.feat + (size_t)img * a.ldf;
        run_section<S1, M, typename N::SL1, false, 0>(lds, a.sec[0], a.sec[1].w0, obs_img, pre, feat_row, tid);
        // the next frame's bytes travel while sections 2 and 3 compute
        const int nimg = img + gridDim.x;
        if (nimg < a.B) prefetch_issue<S1>(pre, a.obs + FRAME * nimg, 0, tid);
        run_section<S2, M, typename N::SL2, false, 1>(lds, a.sec[1], a.sec[2].w0, obs_img, pre, feat_row, tid);
        run_section<S3, M, typename N::SL3, true, 2>(lds, a.sec[2], nullptr, obs_img, pre, feat_row, tid);
    }
}

template <class S1, class S2, class S3, class S4>
struct Net4 {
    static constexpr int mx(int a, int b) { return a > b ? a : b; }
    static constexpr int B0 = mx(mx(mx(S1::ACT_BYTES, S1::IN_BYTES), mx(S2::ACT_BYTES, S2::IN_BYTES)),
                                 mx(mx(S3::ACT_BYTES, S3::IN_BYTES), mx(S4::ACT_BYTES, S4::IN_BYTES)));
    static constexpr int B1 = mx(mx(S1::ACT_BYTES, S2::ACT_BYTES), mx(S3::ACT_BYTES, S4::ACT_BYTES));
    static constexpr int EDGE = mx(mx(S1::EDGE_BYTES, S2::EDGE_BYTES), mx(S3::EDGE_BYTES, S4::EDGE_BYTES));
    using M = LdsMap<B0, B1, EDGE, S1::W0_SET * 1024>;
    using SL1 = typename SlotPlan<M, S1, S2, true, true>::First;
    using SL2 = typename SlotPlan<M, S2, S3, false, true>::EvenC0A;
    using SL3 = typename SlotPlan<M, S3, S4, false, true>::OddC0B;
    using SL4 = typename SlotPlan<M, S4, S4, false, false>::EvenC0A;
    static constexpr int LDS_BYTES = LDS_TOTAL;
};

template <class S1, class S2, class S3, class S4>
__global__ __launch_bounds__(RN_THREADS) void resnet4_bf16_kernel(TorsoArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    using N = Net4<S1, S2, S3, S4>;
    using M = typename N::M;
    const int tid = threadIdx.x;
    constexpr size_t FRAME = (size_t)S1::H * S1::W * S1::CIN;
    if ((int)blockIdx.x >= a.B) return;
    {
        WStage<S1::W0_SET> s0;
        wstage_issue(s0, a.sec[0].w0, tid);
        wstage_commit(s0, lds + M::PERM, tid);
    }
    Prefetch<S1> pre;
    prefetch_issue<S1>(pre, a.obs + FRAME * blockIdx.x, 0, tid);
    for (int img = blockIdx.x; img < a.B; img += gridDim.x) {
        const uint8_t* obs_img = a.obs + FRAME * img;
        __bf16* feat_row = a.feat + (size_t)img * a.ldf;
        run_section<S1, M, typename N::SL1, false, 0>(lds, a.sec[0], a.sec[1].w0, obs_img, pre, feat_row, tid);
        const int nimg = img + gridDim.x;
        if (nimg < a.B) prefetch_issue<S1>(pre, a.obs + FRAME * nimg, 0, tid);
        run_section<S2, M, typename N::SL2, false, 1>(lds, a.sec[1], a.sec[2].w0, obs_img, pre, feat_row, tid);
        run_section<S3, M, typename N::SL3, false, 2>(lds, a.sec[2], a.sec[3].w0, obs_img, pre, feat_row, tid);
        run_section<S4, M, typename N::SL4, true, 3>(lds, a.sec[3], nullptr, obs_img, pre, feat_row, tid);
    }
}

}  // namespace seedinf
