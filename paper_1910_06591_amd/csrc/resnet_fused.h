// Fused deep-ResNet torso (the model Sections 4.1 / 4.2 name) on bf16 MFMA.
//
// One workgroup (8 wavefronts) walks ONE image through every section with all
// activations resident in LDS; a persistent grid strides over the batch.  HBM
// sees only the uint8 frame coming in and the rectified feature vector going
// out, so the torso runs against the matrix-core roofline, not the HBM one.
//
// Per section (conv 3x3 SAME -> max-pool 3x3/2 SAME -> 2 residual blocks):
//   * conv0 + pool, three schemes.  The 3-channel first layer (conv0_pool3_x): a lane owns a POOLED column and
//     takes its three conv columns from three MFMA tiles one frame cell apart, so the 3x3/2 maximum is lane-wise
//     and the pooled values stay in registers as the section's residual stream.  16 -> 32 channels on the
//     36 x 48 map (conv0_pool): 16-column strips x runs of pooled rows, vertical maximum lane-wise, horizontal
//     with DPP row shifts, the neighbour column a strip lacks through a small edge buffer; the conv output
//     never exists in memory.  Small 32 -> 32 channel maps (conv_map): the conv output goes to LDS at full
//     resolution and is pooled while the residual stream is read.
//   * The residual stream x stays in fp32 registers: a pooled tile of 16 pixels belongs to one wavefront for
//     the whole section, in the MFMA accumulator layout, so "x + conv_b(...)" is the MFMA's C operand.  LDS
//     holds the two rectified bf16 conv inputs R = ReLU(x) and U = ReLU(conv_a(R)), each with a zero halo
//     ring (SAME padding without bounds tests).
//   * LDS maps are channel-group planar, [C/8][rows+2][cols+2][8 bf16]: a B fragment (8 consecutive input
//     channels of one tap of one pixel) is one 16-byte ds_read, and the 16 lanes of a lane group read 256
//     contiguous bytes.
//   * Weights: every wavefront needs the whole A operand of a layer, so the workgroup copies each layer's
//     packed fragments global -> LDS once with asynchronous direct loads, one phase ahead, and the wavefronts
//     fill their registers from LDS.
//   * The uint8 frame of the next image is prefetched into registers before the last section and converted
//     into LDS during that section's phases.
// The 3-channel first layer keeps its frame as [row][col][4] (one zero lane): a B fragment covers two frame
// rows x 4 pixels x 4 channels, two MFMAs per conv-row tile.  uint8 inputs enter as exact bf16 integers; 1/255
// scales the accumulator.
#pragma once
#include <type_traits>
#include <utility>

#include "bf16_common.h"

namespace seedinf {

constexpr int RN_WAVES = 8;
// images a workgroup takes through the last section's block phases together (3 and, with a low weight slot at
// 40 KiB, 4 were measured within 1 % of 2)
constexpr int RN_GROUP = 2;
constexpr int RN_THREADS = RN_WAVES * 64;
constexpr int LDS_TOTAL = 160 * 1024;
constexpr int WSLOT_BYTES = 19 * 1024;          // largest layer: 18 fragments of 1 KiB + the bias chunk

enum { IN_LDS = 0, IN_U8_C3 = 1, IN_U8_PLANAR = 2 };

// Keeps the instruction scheduler from moving anything across this point: the hand-written order (fragment
// requests of the next tiles, the MFMA chains, the epilogue pieces placed between them) is the software
// pipeline.  A wavefront's own vector-ALU work does issue under its running MFMAs (measured: about two vector
// instructions per MFMA ride along free; an MFMA takes ~8 issue cycles of its wavefront, 16 of the pipe), so the
// epilogue of a finished tile is spread over the chain of the next one.
#define SCHED_FENCE __builtin_amdgcn_sched_barrier(0)

// f(integral_constant<int, 0>{}) ... f(integral_constant<int, N - 1>{})
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) { (f(std::integral_constant<int, I>{}), ...); }
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) { static_for_impl(f, std::make_integer_sequence<int, N>{}); }

// A 16-byte LDS read that stays where it is written relative to the scheduling fences (a volatile access to
// the LDS address space; through a generic pointer it would become a flat load).
__device__ __forceinline__ bf16x8 lds_read_pinned(const char* p)
{
    return *(const volatile __attribute__((address_space(3))) bf16x8*)(const __attribute__((address_space(3))) char*)p;
}

// Workgroup barrier for LDS-only communication: waits for this wavefront's LDS
// traffic, not for its outstanding global loads (the prefetches stay in flight).
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Compile-time description of one section.
//   NB = bands of pooled rows per conv0 pass, SR = pooled rows per input strip
//   (uint8 sections only; IN_LDS sections have their whole input resident), NWA = wavefronts that
//   own pooled tiles: small maps use fewer, so fewer wavefronts re-read the layer's whole A operand.
//   PADX / IPADX = unused cells at the end of every row of the section's pooled maps / of its LDS input map
//   (which is the previous section's pooled map, so IPADX must be that section's PADX): a row pitch chosen so
//   that the tiles' fragment reads are free of LDS bank conflicts (see TileMap1824).
template <int H_, int W_, int CIN_, int C_, int INKIND_, int NB_, int SR_, int NWA_ = RN_WAVES, int PADX_ = 0, int IPADX_ = 0>
struct SecCfg {
    static constexpr int H = H_, W = W_, CIN = CIN_, C = C_, INKIND = INKIND_, NB = NB_, PADX = PADX_, IPADX = IPADX_;
    static constexpr int PH = (H + 1) / 2, PW = (W + 1) / 2;
    static constexpr int PADH = (((PH - 1) * 2 + 3 - H) > 0 ? ((PH - 1) * 2 + 3 - H) : 0) / 2;
    static constexpr int SR = INKIND == IN_LDS ? PH : SR_;
    static constexpr int NSTRIPS = (PH + SR - 1) / SR;
    static constexpr int FT = C / 16;
    // conv0 weight fragments per feature tile (the 3-channel layer: two per conv-row parity, see conv0_pool3)
    static constexpr int KC0 = INKIND == IN_U8_C3 ? 4 : (9 * CIN + 31) / 32;
    static constexpr int KCB = (9 * C + 31) / 32;
    static constexpr int NK0 = INKIND == IN_U8_C3 ? 2 : (CIN == 16 ? 3 : 1);   // offset registers conv0 keeps per lane
    static constexpr int NWA = NWA_;                        // wavefronts that own pooled tiles (x-read and blocks)
    // 16-channel sections on the 36x48 pooled map run their block convolutions with the sliding-window
    // scheme (block_conv_slide16): column chains of tiles, seven weight fragments per layer
    static constexpr bool SLIDE = C == 16 && PH == 36 && PW == 48 && NWA == 8 && RN_WAVES == 8;
    static constexpr int W0_FRAGS = FT * KC0, WB_FRAGS = SLIDE ? 7 : FT * KCB;
    // a staged weight set = the fragments + one 1 KiB chunk whose first C floats are the biases
    static constexpr int W0_SET = W0_FRAGS + 1, WB_SET = WB_FRAGS + 1;
    // The 3-channel first layer pools without lane shifts (conv0_pool3): it needs no edge buffer and its
    // pooled map is complete when the conv0 phase ends.
    static constexpr bool POOL3 = INKIND == IN_U8_C3;
    // With lane-wise pooling AND the sliding block scheme, a conv0 unit (16 pooled columns of one pooled row) is
    // exactly a block tile in the accumulator layout: conv0 then walks the wavefront's own tile chains, keeps
    // the pooled values as the residual stream x in registers and stores ReLU(x) directly, and the section
    // needs no x-read phase.  Its maps swap roles (R in buf1, U in buf0), so its output lands in buf1.
    static constexpr bool XFUSED = POOL3 && SLIDE;
    // Small 32 -> 32 channel sections write conv0's full-resolution output to LDS as a planar map (conv_map)
    // and pool it while the residual stream is read: on a map this narrow the strip scheme wastes half of its
    // second column strip and its per-row pooling costs more than the extra LDS round trip.
    static constexpr int CM_BYTES = (C / 8) * (((H + 2) * (W + 2 + IPADX_) + 15) / 16 * 16) * 16;
    static constexpr bool CONVMAP = INKIND == IN_LDS && CIN == 32 && C == 32 && CM_BYTES <= 36 * 1024;
    static constexpr int NPIX = PH * PW;
    static constexpr int NTILES = (NPIX + 15) / 16;
    // 32 channels on the 18 x 24 pooled map with a 28-cell pitch: conflict-free tiles in sliding chains (TileMap1824)
    static constexpr bool V2 = C == 32 && PH == 18 && PW == 24 && PADX == 2 && NWA == 8 && RN_WAVES == 8;
    static constexpr int NT = SLIDE ? 14 : (V2 ? 4 : (NTILES + NWA - 1) / NWA);
    static constexpr int NCS = (W + 15) / 16;               // 16-column strips of the conv0 output
    static constexpr int NUNITS = NCS * NB;
    static constexpr int NU = (NUNITS + RN_WAVES - 1) / RN_WAVES;
    // input map of conv0 as it sits in buf0
    static constexpr int IROWS = INKIND == IN_LDS ? H + 2 : (2 * SR + 1 < H ? 2 * SR + 1 : H) + 2;
    static constexpr int IPITCH = W + 2 + IPADX;
    static constexpr int ICELL = INKIND == IN_U8_C3 ? 8 : 16;
    // plane strides are multiples of 16 cells (256 B): a ds_read_b128 whose two lane groups of a half-wave sit
    // a non-multiple of 256 B (and more than 64 B) apart runs at about 60 % rate on this LDS
    static constexpr int IPLANE = (IROWS * IPITCH + 15) / 16 * 16;
    static constexpr int IN_BYTES = (INKIND == IN_U8_C3 ? 1 : CIN / 8) * IPLANE * ICELL + 16;
    static constexpr int PITCH = PW + 2 + PADX, PLANE = ((PH + 2) * PITCH + 15) / 16 * 16;
    static constexpr int ACT_BYTES = (C / 8) * PLANE * 16;
    static constexpr int EDGE_BYTES = POOL3 || CONVMAP ? 0 : NCS * PH * C * 2;
    // prefetch registers for the uint8 input: items of PRE_DW dwords, PRE_N per thread
    static constexpr int PRE_DW = INKIND == IN_U8_C3 ? 3 : (INKIND == IN_U8_PLANAR ? CIN / 4 : 1);
    static constexpr int PRE_ITEMS = INKIND == IN_U8_C3 ? (IROWS - 2) * (W / 4) : (INKIND == IN_U8_PLANAR ? (IROWS - 2 + 2) * W : 0);
    static constexpr int PRE_N = INKIND == IN_LDS ? 1 : (PRE_ITEMS + RN_THREADS - 1) / RN_THREADS;
    // 3-channel frame: first byte of buf0 that the items j >= 1 of a sliced conversion write (see prefetch_commit)
    static constexpr int PRE_SPLIT_BYTES = INKIND == IN_U8_C3 ? (RN_THREADS / (W / 4) + 1) * IPITCH * 8 : 0;
    static_assert(C % 16 == 0, "section channels must be a multiple of 16");
    static_assert(W % 2 == 0, "even width (pool padding only after the last column)");
    static_assert(INKIND == IN_U8_C3 ? CIN == 3 : (CIN == 16 || CIN == 32), "input channels: 3 (uint8), 16 or 32");
    static_assert(C == 16 || C == 32, "section channels: 16 or 32");
    static_assert(INKIND != IN_U8_C3 || ((W * 3) % 4 == 0 && W % 4 == 0), "3-channel rows must be whole dwords");
    static_assert(INKIND != IN_U8_PLANAR || CIN == 16, "planar uint8 input: 16 channels");
    static_assert(INKIND != IN_U8_C3 || NSTRIPS == 1, "the 3-channel frame is kept whole");
    static_assert(INKIND == IN_LDS || IPADX == 0, "only LDS input maps carry a pitch pad");
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

// ---- weight staging: global -> LDS slot (asynchronous, no registers) -> A fragments ----
// A set is NF chunks of 1 KiB; chunk c is moved by wavefront c % RN_WAVES with one asynchronous load (g2lds16):
// it stays in flight for the whole phase and stage_wait() (before the phase's closing barrier) collects it.
template <int NF>
__device__ __forceinline__ void stage_set(const bf16x8* __restrict__ src, char* slot, int lane, int wave)
{
    const uint32_t base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)slot;
#pragma unroll
    for (int j = 0; j < (NF + RN_WAVES - 1) / RN_WAVES; ++j) {
        const int c = wave + j * RN_WAVES;                       // wave-uniform
        if ((j + 1) * RN_WAVES <= NF || c < NF) g2lds16(src + c * 64 + lane, base + c * 1024);
    }
}

template <int NF>
__device__ __forceinline__ void load_a_frags(bf16x8 (&w)[NF], const char* slot, int lane)
{
#pragma unroll
    for (int i = 0; i < NF; ++i) w[i] = *(const bf16x8*)(slot + (i * 64 + lane) * 16);
}

// ---- K layout of the 3x3 convolutions over planar maps --------------------------------------
// A K chunk is 32 values = 4 lane groups x 8 channels.  The fragment a lane reads for chunk kc sits at
//   (its pixel's tap (0,0) cell) + lane base [which one: kbase(kc)] + immediate kimm(kc)
// so per output tile only the (at most three) lane bases are added in registers; the per-chunk part is a
// compile-time ds_read offset.
//   32 input channels: chunk kc = tap kc, lane group g = channel group g.
//   16 input channels: chunks 0..2 = kernel row kc, lane group g -> kernel column g>>1, channel group g&1;
//     chunk 3 = column 2 of kernel rows 0 (g < 2) and 2 (g >= 2); chunk 4 = column 2 of kernel row 1
//     (g < 2; the g >= 2 half is padding with zero weights and re-reads chunk 3's cell).
//   The host packs each layer's weights in the same order (kmap_tap / kmap_cg in the packer).
template <int CIN>
struct KMap {
    static_assert(CIN == 16 || CIN == 32, "planar convolutions take 16 or 32 input channels");
    static constexpr int KC = CIN == 16 ? 5 : 9;
    static constexpr int NBASE = CIN == 16 ? 3 : 1;
    static constexpr int kbase(int kc) { return CIN == 16 ? (kc < 3 ? 0 : kc - 2) : 0; }
    static constexpr int kimm(int kc, int pitch) { return CIN == 16 ? (kc < 3 ? kc * pitch : 0) : (kc / 3) * pitch + kc % 3; }
    // host + device: kernel tap (kh*3+kw, or -1 for padding) and channel group of slot (kc, g)
    static constexpr int tap(int kc, int g)
    {
        if (CIN == 32) return kc;
        if (kc < 3) return kc * 3 + (g >> 1);
        if (kc == 3) return (g < 2 ? 0 : 2) * 3 + 2;
        return g < 2 ? 1 * 3 + 2 : -1;
    }
    static constexpr int cg(int kc, int g) { return CIN == 32 ? g : (g & 1); }
    __device__ static __forceinline__ void lane_bases(int (&lb)[NBASE], int g, int plane, int pitch)
    {
        if constexpr (CIN == 32) {
            lb[0] = g * plane;
        } else {
            const int pl = (g & 1) * plane;
            lb[0] = pl + (g >> 1);
            lb[1] = pl + 2 + (g < 2 ? 0 : 2 * pitch);
            lb[2] = pl + 2 + (g < 2 ? pitch : 2 * pitch);
        }
    }
};

// ---- sliding-window K layout of the 16-channel block convolutions ----------------------------
// A tile is 16 consecutive columns of one pooled row; a wavefront walks a column of tiles downwards (a
// "chain") and keeps the B fragments that consecutive tiles share in registers.  Two kinds of fragment,
// both addressed by buffer row (= pooled row + halo) of the source map:
//   R(r): row r, lane group g -> kernel column g>>1 (0 or 1), channel group g&1.  The tile of pooled row y
//         multiplies R(y), R(y+1), R(y+2) with the weight fragments 0, 1, 2 (kernel rows 0, 1, 2).
//   E(k): kernel column 2 of the row pair (2k, 2k+1): lane groups 0,1 -> row 2k, groups 2,3 -> row 2k+1,
//         channel group g&1.  A tile of even row y = 2k needs rows 2k, 2k+1 | 2k+2: E(k) x fragment 3
//         (kernel rows 0 | 1) and E(k+1) x fragment 4 (kernel row 2 | zeros); a tile of odd row y = 2k+1
//         needs rows 2k+1 | 2k+2, 2k+3: E(k) x fragment 5 (zeros | kernel row 0) and E(k+1) x fragment 6
//         (kernel rows 1 | 2).  So the pair-aligned E fragments serve both parities and only the weights
//         differ: per tile one new R and half a new E fragment are read instead of five fragments.
struct SlideMap16 {
    static constexpr int NFRAG = 7;
    // kernel tap kh*3+kw (or -1: zero weights) of lane group g in weight fragment f
    static constexpr int tap(int f, int g)
    {
        if (f < 3) return f * 3 + (g >> 1);
        if (f == 3) return (g < 2 ? 0 : 1) * 3 + 2;
        if (f == 4) return g < 2 ? 2 * 3 + 2 : -1;
        if (f == 5) return g < 2 ? -1 : 0 * 3 + 2;
        return (g < 2 ? 1 : 2) * 3 + 2;
    }
    static constexpr int cg(int g) { return g & 1; }
    // Chains of the 36 x 48 pooled map (3 column strips x 36 rows = 108 tiles): every wavefront owns chain 0
    // (8 tiles) and chain 1 (4 tiles for wavefronts 0 and 1, else 6); all chains start on an even row.
    static constexpr int LEN0 = 8, LEN1 = 6;
    __device__ static __forceinline__ void chain(int wave, int c, int& strip, int& row0, int& nt)
    {
        if (c == 0) { strip = wave >> 2; row0 = (wave & 3) * 8; nt = 8; }
        else if (wave < 2) { strip = wave; row0 = 32; nt = 4; }
        else { strip = 2; row0 = (wave - 2) * 6; nt = 6; }
    }
};

// ---- tiles of the 18 x 24 maps (32 channels) ----------------------------------------------
// LDS serves a 16-byte read of 16 lanes at full rate only when their 256 bytes fall on 256 distinct bank bytes
// (measured: a tile of 16 row-major pixels that wraps from one 24-pixel row to the next, two halo cells further,
// reads at 57 % of that).  The 27 tiles of this map are therefore
//   strip A: columns 0..15 of one row (18 tiles, 256 contiguous bytes), and
//   strip B: columns 16..23 of the two rows (r, r + 10), r = 0..7: with a pitch of 28 cells the rows sit
//            10 * 28 * 16 = 17.5 * 256 bytes apart, i.e. on the other half of the banks; rows 8 and 9 form the
//            one tile left over (adjacent rows: its reads do conflict, one tile in 27),
// and consecutive tiles of a strip (r -> r + 1) form a chain: the window rows r, r+1 of tile r are the rows
// r-1+1, r+1 ... of tile r + 1, so a wavefront that walks down a chain reads three new fragments per tile
// instead of nine.  Wavefront w owns at most four consecutive tiles:
//   w0..w2: A rows 4w .. 4w+3;  w3: A 12..14;  w4: A 15..17;  w5: B r = 0..2;  w6: B r = 3..5;
//   w7: B r = 6, 7 and the left-over tile (a new chain).
// On a SIMD (wavefronts w and w + 4) that makes 7, 7, 7 and 6 tiles.
struct TileMap1824 {
    static constexpr int NT = 4;
    __device__ static __forceinline__ int ntiles(int wave) { return wave < 3 ? 4 : 3; }
    // pixel (y, xx) that lane n holds in slot i of `wave` (a missing slot repeats the last one)
    __device__ static __forceinline__ void pixel(int wave, int i, int n, int& y, int& xx, bool& ok)
    {
        const int nt = ntiles(wave);
        ok = i < nt;
        const int ii = ok ? i : nt - 1;
        if (wave < 5) {
            y = (wave < 3 ? wave * 4 : 12 + (wave - 3) * 3) + ii;
            xx = n;
        } else {
            const int r = (wave - 5) * 3 + ii;               // 0..7: the pair (r, r + 10); 8: rows 8 and 9
            y = r < 8 ? (n < 8 ? r : r + 10) : (n < 8 ? 8 : 9);
            xx = 16 + (n & 7);
        }
    }
    // slot i starts a new chain (its window shares nothing with slot i - 1)
    __device__ static __forceinline__ bool fresh(int wave, int i) { return i == 0 || (wave == 7 && i == 2); }
};

// ---- uint8 frame prefetch --------------------------------------------------------
template <class S>
struct Prefetch {
    using Sec = S;
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
            for (int j = 0; j < S::PRE_N; ++j) {             // unconditional (clamped) loads: under a branch the later wait would cover ALL outstanding loads
                const int i = min(tid + j * RN_THREADS, nitems - 1);
                const uint32_t* s = (const uint32_t*)(obs_img + (size_t)(r0 + i / GPR) * S::W * 3) + (i % GPR) * 3;
                p.d[j][0] = s[0]; p.d[j][1] = s[1]; p.d[j][2] = s[2];
            }
        } else {
            // unconditional loads from a clamped row: a select on the loaded value here would wait for the memory
            // round trip at once; rows outside the frame are zeroed when the registers are converted
#pragma unroll
            for (int j = 0; j < S::PRE_N; ++j) {
                const int i = tid + j * RN_THREADS;
                const int ry = i / S::W, px = i % S::W;
                const int iy = min(max(r0 - 1 + ry, 0), S::H - 1);
                const uint4 v = *(const uint4*)(obs_img + ((size_t)iy * S::W + px) * S::CIN);
                p.d[j][0] = v.x; p.d[j][1] = v.y; p.d[j][2] = v.z; p.d[j][3] = v.w;
            }
        }
    }
}

// convert the prefetched bytes to bf16 and lay them out in buf0 (with zero halo).
// PART < 0: everything.  The whole 3-channel frame can also be converted in slices: PART = j > 0 converts
// only every thread's j-th item, PART = 0 the first items and the halo.  With LIMIT > 0 the slices j > 0 leave
// out the cells below byte LIMIT of the buffer (live maps sit there); slice 0 converts those too.
template <class S, int PART = -1, int LIMIT = 0>
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
                if (PART > 0 && j != PART) continue;
                if (PART == 0 && LIMIT == 0 && j != 0) continue;
                const int i = tid + j * RN_THREADS;
                const int cell = (i / GPR + 1) * S::IPITCH + (i % GPR) * 4 + 1;
                const bool low = LIMIT > 0 && j > 0 && cell * 8 < LIMIT;       // this item's cells start below LIMIT
                if (i < nitems && (PART < 0 || j == 0 || (PART == 0) == low)) {
                    const uint32_t d0 = p.d[j][0], d1 = p.d[j][1], d2 = p.d[j][2];
                    const uint32_t by[12] = {d0 & 0xff, (d0 >> 8) & 0xff, (d0 >> 16) & 0xff, d0 >> 24,
                                             d1 & 0xff, (d1 >> 8) & 0xff, (d1 >> 16) & 0xff, d1 >> 24,
                                             d2 & 0xff, (d2 >> 8) & 0xff, (d2 >> 16) & 0xff, d2 >> 24};
                    // buffer row of image row iy is iy - (r0 - 1); whole frame: r0 = 0 -> iy + 1
                    char* d = buf0 + cell * 8;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const floatx4 c = {(float)by[q * 3], (float)by[q * 3 + 1], (float)by[q * 3 + 2], 0.0f};
                        *(bf16x4*)(d + q * 8) = to_bf16x4(c);
                    }
                }
            }
            if (PART > 0) return;
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
                    const int iy = r0 - 1 + ry;
                    const bool inside = iy >= 0 && iy < S::H;                   // the rows above and below the frame: zeros
                    const bf16x8 z = {};
                    *(bf16x8*)(buf0 + (ry * S::IPITCH + px + 1) * 16) = inside ? u8x8_to_bf16x8(p.d[j][0], p.d[j][1]) : z;
                    *(bf16x8*)(buf0 + (S::IPLANE + ry * S::IPITCH + px + 1) * 16) = inside ? u8x8_to_bf16x8(p.d[j][2], p.d[j][3]) : z;
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

template <bool FIRST, class A, class B>
__device__ __forceinline__ auto& pick_ref(A& a, B& b)
{
    if constexpr (FIRST) return a;
    else return b;
}

// ---- conv0 + max-pool ----------------------------------------------------------------
// h[n] = max(v[n], v[n+1], v[n+2]) within each row of 16 lanes, for the four channels a lane holds.
// A DPP op whose source lane lies outside the row leaves its destination untouched, so lane 14 ends
// with max(v[14], v[15]) (completed later from the next strip's edge column) and lane 15 with
// garbage; only even lanes are pooled outputs.
__device__ __forceinline__ floatx4 hmax3_row16(floatx4 v)
{
    float h0, h1, h2, h3;
    asm volatile("s_nop 1\n\t"
                 "v_max_f32_dpp %0, %4, %4 row_shl:1 row_mask:0xf bank_mask:0xf\n\t"
                 "v_max_f32_dpp %1, %5, %5 row_shl:1 row_mask:0xf bank_mask:0xf\n\t"
                 "v_max_f32_dpp %2, %6, %6 row_shl:1 row_mask:0xf bank_mask:0xf\n\t"
                 "v_max_f32_dpp %3, %7, %7 row_shl:1 row_mask:0xf bank_mask:0xf\n\t"
                 "v_max_f32_dpp %0, %4, %0 row_shl:2 row_mask:0xf bank_mask:0xf\n\t"
                 "v_max_f32_dpp %1, %5, %1 row_shl:2 row_mask:0xf bank_mask:0xf\n\t"
                 "v_max_f32_dpp %2, %6, %2 row_shl:2 row_mask:0xf bank_mask:0xf\n\t"
                 "v_max_f32_dpp %3, %7, %3 row_shl:2 row_mask:0xf bank_mask:0xf"
                 : "=&v"(h0), "=&v"(h1), "=&v"(h2), "=&v"(h3)
                 : "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]));
    return floatx4{h0, h1, h2, h3};
}

// B fragments of one conv0 output tile (16 consecutive columns of one conv row); `base` = cell index of
// the tile's tap (0,0) in plane 0.
template <class S>
__device__ __forceinline__ void conv0_load(bf16x8 (&b)[S::KC0], const char* in, int base, const int (&koff)[S::NK0])
{
    if constexpr (S::INKIND == IN_U8_C3) {
#pragma unroll
        for (int kc = 0; kc < S::KC0; ++kc) {
            const char* s = in + (base + koff[kc]) * 8;
            const bf16x4 lo = *(const bf16x4*)s, hi = *(const bf16x4*)(s + 8);
            b[kc] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    } else {
        using K = KMap<S::CIN>;
        const char* pa[K::NBASE];
#pragma unroll
        for (int q = 0; q < K::NBASE; ++q) pa[q] = in + (base + koff[q]) * 16;
#pragma unroll
        for (int kc = 0; kc < S::KC0; ++kc) b[kc] = *(const bf16x8*)(pa[K::kbase(kc)] + K::kimm(kc, S::IPITCH) * 16);
    }
}

// The same for planar inputs from per-lane base pointers that already include the tile's cell: the chunk and
// row offsets are ds_read immediates.
template <class S, int ROWOFF>
__device__ __forceinline__ void conv0_load_p(bf16x8 (&b)[S::KC0], const char* const (&pa)[KMap<S::CIN>::NBASE])
{
    using K = KMap<S::CIN>;
#pragma unroll
    for (int kc = 0; kc < S::KC0; ++kc) b[kc] = *(const bf16x8*)(pa[K::kbase(kc)] + (K::kimm(kc, S::IPITCH) + ROWOFF * S::IPITCH) * 16);
}

// acc = init + W * b: `init` carries the bias (divided by the input scale), so the epilogue has no bias add
template <class S>
__device__ __forceinline__ void conv0_mma(floatx4 (&acc)[S::FT], const bf16x8 (&b)[S::KC0], const bf16x8 (&w0)[S::W0_FRAGS],
                                          const floatx4 (&init)[S::FT])
{
#pragma unroll
    for (int j = 0; j < S::FT; ++j) acc[j] = init[j];
#pragma unroll
    for (int kc = 0; kc < S::KC0; ++kc)
#pragma unroll
        for (int j = 0; j < S::FT; ++j) acc[j] = mfma16(w0[j * S::KC0 + kc], b[kc], acc[j]);
}

// conv0 + pool over pooled rows [pr0, pr1); `rbuf0` = image row held by buffer row 0 of `in`
// (so conv row r's tap row kh sits in buffer row r - 1 + kh - rbuf0).  Writes un-rectified
// pooled bf16 values into `xout` (planar map with halo, this section's pooled geometry) and
// each strip's first-column vertical maxima into `edge`.  `wslot`: conv0's staged weight set.
// The two conv rows of pooled row py+1 are read from LDS while those of row py are multiplied.
template <class S>
__device__ __forceinline__ void conv0_pool(const char* in, char* xout, char* edge, char* trash, const bf16x8 (&w0)[S::W0_FRAGS],
                                           const char* wslot, int pr0, int pr1, int rbuf0, int lane, int wave)
{
    const int g = lane >> 4, n = lane & 15;
    constexpr float SCALE = S::INKIND == IN_LDS ? 1.0f : 1.0f / 255.0f;
    constexpr bool FULL = S::W % 16 == 0;                 // no partial column strip
    floatx4 bv[S::FT];
#pragma unroll
    for (int j = 0; j < S::FT; ++j) bv[j] = *(const floatx4*)(wslot + S::W0_FRAGS * 1024 + (j * 4 + g) * 16) * (1.0f / SCALE);
    int koff[S::NK0];                                     // 3-channel frame: per-chunk offsets; planar: lane bases
    if constexpr (S::INKIND == IN_U8_C3) {
        // K slot s = kc*4 + g -> (kernel row s/2, pixel pair s%2); 8-byte cells
#pragma unroll
        for (int kc = 0; kc < 2; ++kc) {
            int s = kc * 4 + g;
            if (s > 5) s = 0;
            koff[kc] = (s >> 1) * S::IPITCH + (s & 1) * 2;
        }
    } else {
        KMap<S::CIN>::lane_bases(koff, g, S::IPLANE, S::IPITCH);
    }
    const int npr = pr1 - pr0;
    const floatx4 NEG = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};

    // Work split: the NCS * npr (column strip, pooled row) pairs, strip-major, cut into one run per wavefront; a
    // run that crosses a strip boundary becomes two units.  Each unit recomputes the conv row above its first
    // pooled row, so long runs keep that overhead small.
    const int nq = S::NCS * npr;
    const int q0 = wave * nq / RN_WAVES, q1 = (wave + 1) * nq / RN_WAVES;
#pragma unroll 1
    for (int q = q0; q < q1;) {
        const int cs = q / npr, pb0 = pr0 + q % npr;
        const int pb1 = min(pr0 + npr, pb0 + (q1 - q));
        q += pb1 - pb0;
        const int col = cs * 16 + n;
        const bool live = FULL || col < S::W;
        const int colc = live ? col : S::W - 1;
        // cell index of conv row r, tap (0,0): (r - 1 - rbuf0) * IPITCH + colc
        const int cbase = colc - (1 + rbuf0) * S::IPITCH;
        floatx4 top[S::FT];
        // a second fragment set (loads a whole iteration ahead) only where the registers allow it
        constexpr bool TWO = S::W0_FRAGS * 4 + S::KC0 * 32 <= 136;
        bf16x8 fa[S::KC0], fb[S::KC0], ga[TWO ? S::KC0 : 1], gb[TWO ? S::KC0 : 1];
        const int rt = 2 * pb0 - S::PADH;
        if (rt >= 0) {
            conv0_load<S>(fa, in, cbase + rt * S::IPITCH, koff);
            conv0_mma<S>(top, fa, w0, bv);
        } else {
#pragma unroll
            for (int j = 0; j < S::FT; ++j) top[j] = NEG;
        }
        // Output addresses of this unit's first pooled row; they advance by one row per pooled row.  Lanes with
        // nothing to store (odd columns; all but column 0 for the edge) store into a per-lane trash cell, which
        // keeps the loop body free of branches.
        const int px = col >> 1;
        const bool wr_edge = n == 0 && cs > 0;
        const bool wr_pool = live && !(n & 1);
        char* xptr = wr_pool ? xout + ((pb0 + 1) * S::PITCH + px + 1) * 16 + (g >> 1) * (S::PLANE * 16) + (g & 1) * 8 : trash + lane * 8;
        char* eptr = wr_edge ? edge + ((cs * S::PH + pb0) * S::C + g * 4) * 2 : trash + lane * 8;
        const int xstep = wr_pool ? S::PITCH * 16 : 0, estep = wr_edge ? S::C * 2 : 0;
        const int xj = wr_pool ? 2 * S::PLANE * 16 : 0, ej = wr_edge ? 32 : 0;

        // rows of pooled row py: mid = 2 py - PADH + 1 (always inside the image), bot = mid + 1 (below the image for
        // the map's last pooled row when the height is even: pool_row then leaves it out).  The lane bases walk
        // down two rows per pooled row; requests past the unit's end read rows that are never used (past the
        // map's end: whatever LDS holds behind it).
        const char* pm[KMap<S::CIN>::NBASE];
#pragma unroll
        for (int q = 0; q < KMap<S::CIN>::NBASE; ++q) pm[q] = in + (cbase + (2 * pb0 - S::PADH + 1) * S::IPITCH + koff[q]) * 16;
        auto load_pair = [&](bf16x8 (&a)[S::KC0], bf16x8 (&c)[S::KC0]) {
            conv0_load_p<S, 0>(a, pm);
            conv0_load_p<S, 1>(c, pm);
#pragma unroll
            for (int q = 0; q < KMap<S::CIN>::NBASE; ++q) pm[q] += 2 * S::IPITCH * 16;
        };
        auto mma_pair = [&](floatx4 (&mid)[S::FT], floatx4 (&bot)[S::FT], const bf16x8 (&a)[S::KC0], const bf16x8 (&c)[S::KC0]) {
            conv0_mma<S>(mid, a, w0, bv);
            conv0_mma<S>(bot, c, w0, bv);
        };
        // `last`: the unit's last pooled row, whose bottom conv row may lie below the image
        const bool no_bot = 2 * (pb1 - 1) - S::PADH + 2 >= S::H;         // uniform
        auto pool_row = [&](const floatx4 (&mid)[S::FT], const floatx4 (&bot)[S::FT], bool last = false) {
#pragma unroll
            for (int j = 0; j < S::FT; ++j) {
                floatx4 v = max4(top[j], mid[j]);
                if (!(last && no_bot)) v = max4(v, bot[j]);
                if (SCALE != 1.0f) v = v * SCALE;
                if (!FULL && !live) v = NEG;
                *(bf16x4*)(eptr + j * ej) = to_bf16x4(v);
                const floatx4 h = hmax3_row16(v);
                *(bf16x4*)(xptr + j * xj) = to_bf16x4(h);
                top[j] = bot[j];
            }
            xptr += xstep;
            eptr += estep;
        };
        // One row's two conv rows multiplied while the previous row is pooled, interleaved by hand: after each
        // chunk's MFMAs one piece of the pooling (5 pieces per feature tile: vertical maximum, edge store,
        // horizontal maximum, store, top <- bot).  A wavefront's vector instructions issue under its own running
        // MFMAs; left as a block of MFMAs and a block of vector work, the SIMD's two wavefronts fall into step
        // after the phase's barrier and wait for the matrix pipe together, then for the vector unit together.
        auto mma_pool = [&](floatx4 (&mid)[S::FT], floatx4 (&bot)[S::FT], bf16x8 (&a)[S::KC0], bf16x8 (&c)[S::KC0],
                            const floatx4 (&pmid)[S::FT], const floatx4 (&pbot)[S::FT]) {
            using K = KMap<S::CIN>;
            constexpr int STEPS = 2 * S::KC0, NP = 5 * S::FT;
            floatx4 v[S::FT], h[S::FT];
            auto piece = [&](auto pc) {
                constexpr int j = decltype(pc)::value / 5, part = decltype(pc)::value % 5;
                if constexpr (part == 0) {
                    v[j] = max4(max4(top[j], pmid[j]), pbot[j]);
                    if (SCALE != 1.0f) v[j] = v[j] * SCALE;
                    if (!FULL && !live) v[j] = NEG;
                } else if constexpr (part == 1) {
                    *(bf16x4*)(eptr + j * ej) = to_bf16x4(v[j]);
                } else if constexpr (part == 2) {
                    h[j] = hmax3_row16(v[j]);
                } else if constexpr (part == 3) {
                    *(bf16x4*)(xptr + j * xj) = to_bf16x4(h[j]);
                } else {
                    top[j] = pbot[j];
                }
            };
            static_for<STEPS>([&](auto st) {
                constexpr int s = decltype(st)::value, kc = s % S::KC0;
#pragma unroll
                for (int j = 0; j < S::FT; ++j) {
                    if constexpr (s < S::KC0) mid[j] = mfma16(w0[j * S::KC0 + kc], a[kc], kc == 0 ? bv[j] : mid[j]);
                    else bot[j] = mfma16(w0[j * S::KC0 + kc], c[kc], kc == 0 ? bv[j] : bot[j]);
                }
                // the fragment just multiplied is requested again for the next row of the sequence: a whole
                // mma_pool ahead of its use
                // (volatile: an ordinary load is free to move across the scheduling fences, and the compiler gathers
                // all ten in front of the next row's first MFMA, which then waits for them)
                if constexpr (s < S::KC0) a[kc] = lds_read_pinned(pm[K::kbase(kc)] + K::kimm(kc, S::IPITCH) * 16);
                else c[kc] = lds_read_pinned(pm[K::kbase(kc)] + (K::kimm(kc, S::IPITCH) + S::IPITCH) * 16);
                static_for<(s + 1) * NP / STEPS - s * NP / STEPS>([&](auto k) { piece(std::integral_constant<int, s * NP / STEPS + decltype(k)::value>{}); });
                SCHED_FENCE;
            });
            xptr += xstep;
            eptr += estep;
#pragma unroll
            for (int q = 0; q < K::NBASE; ++q) pm[q] += 2 * S::IPITCH * 16;
        };
        // Software pipeline over pooled rows: while row py is pooled (vector ALU), the matrix cores multiply row
        // py+1 and LDS delivers the fragments of row py+2 (py+3 with two fragment sets).  Accumulator sets
        // (m0, b0) / (m1, b1) and fragment sets alternate, hence two rows per iteration.
        // (32 input and output channels: fragments, weights and two accumulator sets exceed the register file;
        // those sections run the plain load -> multiply -> pool loop)
        constexpr bool SWP = S::W0_FRAGS * 4 + S::KC0 * 8 + S::FT * 16 <= 160;
        floatx4 m0[S::FT], b0[S::FT], m1[SWP ? S::FT : 1], b1[SWP ? S::FT : 1];
        if constexpr (!SWP) {
#pragma unroll 1
            for (int py = pb0; py < pb1; ++py) {
                load_pair(fa, fb);
                mma_pair(m0, b0, fa, fb);
                pool_row(m0, b0, py + 1 == pb1);
            }
        } else {
        auto& oa = pick_ref<TWO>(ga, fa);                                    // fragments of the odd rows
        auto& ob = pick_ref<TWO>(gb, fb);
        constexpr int LA = TWO ? 2 : 1;
        int py = pb0;
        load_pair(fa, fb);
        if constexpr (TWO) load_pair(ga, gb);
        mma_pair(m0, b0, fa, fb);
        load_pair(fa, fb);
#pragma unroll 1
        for (; py + 2 < pb1; py += 2) {
            mma_pool(m1, b1, oa, ob, m0, b0);
            mma_pool(m0, b0, fa, fb, m1, b1);
        }
        if (py + 1 < pb1) {
            mma_pair(m1, b1, oa, ob);
            pool_row(m0, b0);
            pool_row(m1, b1, true);
        } else {
            pool_row(m0, b0, true);
        }
        }
    }
}

// conv0 + pool for the 3-channel frame, without lane shifts: lane n of a unit owns POOLED column 16 sp + n
// and the three conv columns under its pooling window (2 px, 2 px + 1, 2 px + 2) come from three MFMA tiles
// whose B fragments sit one frame cell apart.  The 3-maximum is then lane-wise: every lane holds a pooled
// value, no neighbour columns are exchanged, and the map is complete when the phase ends.  Half as many
// vector instructions per pooled value as the shifted scheme, for 1.5 x the (cheap, K = 27) MFMAs.
// The map's last pooled column has no third conv column: its lanes read the second one twice.
//
// B fragments are aligned to PAIRS of frame-buffer rows: P(k) = buffer rows 2k, 2k+1; lane group g -> row
// 2k + (g >> 1), pixel pair g & 1 (two 4-channel cells).  The whole frame is resident (buffer row 0 = image
// row -1), so conv row r reads buffer rows r, r+1, r+2:
//   even r = 2k:   P(k) x fragment 0 (kernel rows 0 | 1)  +  P(k+1) x fragment 1 (kernel row 2 | zeros)
//   odd  r = 2k+1: P(k) x fragment 2 (zeros | kernel row 0)  +  P(k+1) x fragment 3 (kernel rows 1 | 2)
// Pooled row py (conv rows 2py, 2py+1, 2py+2; PADH == 0) therefore needs P(py), P(py+1), P(py+2) and each
// new pooled row reads ONE new pair per tile.  The pairs rotate through three register slots, hence the
// loop over pooled rows is unrolled by three.  The bottom pooled row has no third conv row.
template <class S>
__device__ __forceinline__ void conv0_pool3(const char* in, char* xout, const bf16x8 (&w0)[S::W0_FRAGS], const char* wslot,
                                            int lane, int wave)
{
    static_assert(S::INKIND == IN_U8_C3 && S::FT == 1 && S::W0_FRAGS == 4 && S::NSTRIPS == 1 && S::PW % 16 == 0 &&
                      S::PADH == 0 && S::H % 2 == 0,
                  "conv0_pool3: whole 3-channel frame, even height, pooled width a multiple of 16");
    const int g = lane >> 4, n = lane & 15;
    constexpr float SCALE = 1.0f / 255.0f;
    constexpr int ROWB = S::IPITCH * 8;                     // bytes per frame row (8-byte cells)
    const floatx4 bv = *(const floatx4*)(wslot + S::W0_FRAGS * 1024 + g * 16);
    const int koffp = (g >> 1) * S::IPITCH + (g & 1) * 2;
    typedef bf16x8 Pair[3];                                 // one row pair's fragments, per tile d
    constexpr int NSP = S::PW / 16;
    constexpr int nq = NSP * S::PH;
    const floatx4 ZERO = {0.f, 0.f, 0.f, 0.f};
    const int q0 = wave * nq / RN_WAVES, q1 = (wave + 1) * nq / RN_WAVES;
#pragma unroll 1
    for (int q = q0; q < q1;) {
        const int sp = q / S::PH, pb0 = q % S::PH;
        const int pb1 = min(S::PH, pb0 + (q1 - q));
        q += pb1 - pb0;
        const int px = sp * 16 + n;
        // pa: tiles d = 0, 1 (d = 1 one cell further: an immediate) of the pair the pointers sit on; pa2: tile d = 2
        const char* pa = in + (2 * pb0 * S::IPITCH + 2 * px + koffp) * 8;
        const char* pa2 = pa + (px == S::PW - 1 ? 8 : 16);
        int kp = pb0;                                        // pair the pointers sit on; the map's last pair is PH
        auto load_pair = [&](Pair& f) {
#pragma unroll
            for (int d = 0; d < 3; ++d) {
                const char* c = d < 2 ? pa + d * 8 : pa2;
                const bf16x4 lo = *(const bf16x4*)c, hi = *(const bf16x4*)(c + 8);
                f[d] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
            const bool more = kp < S::PH;                    // past the last pair: stay (those fragments are never used)
            pa += more ? 2 * ROWB : 0;
            pa2 += more ? 2 * ROWB : 0;
            kp += more ? 1 : 0;
        };
        // horizontal maximum over the three tiles of one conv row: PAR = 0 even row, 1 odd row
        auto conv_row = [&](auto par, const Pair& lo, const Pair& hi) {
            constexpr int P = decltype(par)::value;
            floatx4 acc[3];
#pragma unroll
            for (int d = 0; d < 3; ++d) {
                acc[d] = mfma16(w0[2 * P], lo[d], ZERO);
                acc[d] = mfma16(w0[2 * P + 1], hi[d], acc[d]);
            }
            return max4(max4(acc[0], acc[1]), acc[2]);
        };
        using EVEN = std::integral_constant<int, 0>;
        using ODD = std::integral_constant<int, 1>;
        Pair F[3];                                           // pair k lives in F[(k - pb0) % 3]
        load_pair(F[0]);
        load_pair(F[1]);
        floatx4 top = conv_row(EVEN{}, F[0], F[1]);
        load_pair(F[2]);
        char* xptr = xout + ((pb0 + 1) * S::PITCH + px + 1) * 16 + (g >> 1) * (S::PLANE * 16) + (g & 1) * 8;
        auto store_row = [&](floatx4 v) {
            *(bf16x4*)xptr = to_bf16x4(v * SCALE + bv);
            xptr += S::PITCH * 16;
        };
        auto row_step = [&](auto jj) {                       // pooled row py = pb0 + 3 i + J
            constexpr int J = decltype(jj)::value;
            const floatx4 hm = conv_row(ODD{}, F[J % 3], F[(J + 1) % 3]);
            const floatx4 hb = conv_row(EVEN{}, F[(J + 1) % 3], F[(J + 2) % 3]);
            load_pair(F[J % 3]);                             // pair py + 3 replaces pair py
            store_row(max4(max4(top, hm), hb));
            top = hb;
        };
        auto last_step = [&](auto jj) {                      // the map's bottom row: conv rows 2py, 2py+1 only
            constexpr int J = decltype(jj)::value;
            store_row(max4(top, conv_row(ODD{}, F[J % 3], F[(J + 1) % 3])));
        };
        using J0 = std::integral_constant<int, 0>; using J1 = std::integral_constant<int, 1>; using J2 = std::integral_constant<int, 2>;
        const int lim = min(pb1, S::PH - 1);
        int py = pb0;
#pragma unroll 1
        for (; py + 3 <= lim; py += 3) {
            row_step(J0{});
            row_step(J1{});
            row_step(J2{});
        }
        const int r = lim - py;
        if (r >= 1) row_step(J0{});
        if (r == 2) row_step(J1{});
        if (pb1 == S::PH) {
            if (r == 0) last_step(J0{});
            else if (r == 1) last_step(J1{});
            else last_step(J2{});
        }
    }
}

// conv0_pool3 for an XFUSED section: the same arithmetic, walked along the wavefront's tile chains (see
// SlideMap16).  x[i] receives tile i's pooled values (fp32, bias added), rout the planar map of ReLU(x).
template <class S>
__device__ __forceinline__ void conv0_pool3_x(const char* in, char* rout, const bf16x8 (&w0)[S::W0_FRAGS], const char* wslot,
                                              floatx4 (&x)[S::NT][S::FT], int lane, int wave)
{
    static_assert(S::XFUSED && S::FT == 1 && S::W0_FRAGS == 4 && S::NSTRIPS == 1 && S::PADH == 0 && S::H % 2 == 0,
                  "conv0_pool3_x: whole 3-channel frame, even height, sliding block scheme");
    using SM = SlideMap16;
    const int g = lane >> 4, n = lane & 15;
    constexpr float SCALE = 1.0f / 255.0f;
    constexpr int ROWB = S::IPITCH * 8;
    const floatx4 bv = *(const floatx4*)(wslot + S::W0_FRAGS * 1024 + g * 16);
    const int koffp = (g >> 1) * S::IPITCH + (g & 1) * 2;
    typedef bf16x8 Pair[3];
    const floatx4 ZERO = {0.f, 0.f, 0.f, 0.f};
    using EVEN = std::integral_constant<int, 0>;
    using ODD = std::integral_constant<int, 1>;
    auto conv_row = [&](auto par, const Pair& lo, const Pair& hi) {
        constexpr int P = decltype(par)::value;
        floatx4 acc[3];
#pragma unroll
        for (int d = 0; d < 3; ++d) {
            acc[d] = mfma16(w0[2 * P], lo[d], ZERO);
            acc[d] = mfma16(w0[2 * P + 1], hi[d], acc[d]);
        }
        return max4(max4(acc[0], acc[1]), acc[2]);
    };
    auto run_chain = [&](auto cc) {
        constexpr int c = decltype(cc)::value;
        constexpr int LEN = c == 0 ? SM::LEN0 : SM::LEN1, I0 = c == 0 ? 0 : SM::LEN0;
        int strip, row0, nt;
        SM::chain(wave, c, strip, row0, nt);
        const int px = strip * 16 + n;
        const char* pa = in + (2 * row0 * S::IPITCH + 2 * px + koffp) * 8;
        const char* pa2 = pa + (px == S::PW - 1 ? 8 : 16);
        int kp = row0;                                       // pair the pointers sit on; the map's last pair is PH
        auto load_pair = [&](Pair& f) {
#pragma unroll
            for (int d = 0; d < 3; ++d) {
                const char* cp = d < 2 ? pa + d * 8 : pa2;
                const bf16x4 lo = *(const bf16x4*)cp, hi = *(const bf16x4*)(cp + 8);
                f[d] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
            const bool more = kp < S::PH;                    // past the last pair: stay (those fragments are never used)
            pa += more ? 2 * ROWB : 0;
            pa2 += more ? 2 * ROWB : 0;
            kp += more ? 1 : 0;
        };
        Pair F[3];                                           // pair k lives in F[(k - row0) % 3]
        load_pair(F[0]);
        load_pair(F[1]);
        floatx4 top = conv_row(EVEN{}, F[0], F[1]);
        load_pair(F[2]);
        char* rptr = rout + ((row0 + 1) * S::PITCH + px + 1) * 16 + (g >> 1) * (S::PLANE * 16) + (g & 1) * 8;
#pragma unroll
        for (int pos = 0; pos < LEN; ++pos) {
            constexpr int dummy = 0; (void)dummy;
            if (pos < nt) {                                  // uniform
                floatx4 v;
                if (row0 + pos < S::PH - 1) {                // uniform: the map's bottom row has no third conv row
                    const floatx4 hm = conv_row(ODD{}, F[pos % 3], F[(pos + 1) % 3]);
                    const floatx4 hb = conv_row(EVEN{}, F[(pos + 1) % 3], F[(pos + 2) % 3]);
                    load_pair(F[pos % 3]);                   // pair py + 3 replaces pair py
                    v = max4(max4(top, hm), hb);
                    top = hb;
                } else {
                    v = max4(top, conv_row(ODD{}, F[pos % 3], F[(pos + 1) % 3]));
                }
                v = v * SCALE + bv;
                x[I0 + pos][0] = v;
                *(bf16x4*)rptr = relu_bf16x4(to_bf16x4(v));
                rptr += S::PITCH * 16;
            } else {
                x[I0 + pos][0] = ZERO;
            }
        }
    };
    run_chain(std::integral_constant<int, 0>{});
    run_chain(std::integral_constant<int, 1>{});
}

// Per-lane cell index (row * PITCH + column, plane 0, tap (0,0)) of the pixel this lane holds in each of
// the wavefront's tiles; pixels past the end of the map are clamped to the last one.  NWA = wavefronts
// that own tiles in this section.
// (row, column) of pixel t*16 + n of the pooled map, clamped to the last pixel.  The division runs on the
// tile's first pixel, which is uniform across the wavefront (scalar unit); lanes only wrap rows.
template <class S>
__device__ __forceinline__ void tile_pixel(int t, int n, int& y, int& xx)
{
    const int p0 = t * 16;
    y = p0 / S::PW;
    xx = p0 % S::PW + n;
#pragma unroll
    for (int k = 0; k < (15 + S::PW - 1) / S::PW; ++k)
        if (xx >= S::PW) { xx -= S::PW; ++y; }
    if (S::NPIX % 16 != 0 && y >= S::PH) { y = S::PH - 1; xx = S::PW - 1; }
}

// Pooled pixel (y, xx) that lane n holds in the wavefront's tile i (clamped into the map), whether the tile
// exists (uniform across the wavefront) and whether the lane's pixel does.
template <class S>
__device__ __forceinline__ void tile_ref(int wave, int i, int n, int& y, int& xx, bool& tile_ok, bool& lane_ok)
{
    if constexpr (S::V2) {
        TileMap1824::pixel(wave, i, n, y, xx, tile_ok);
        lane_ok = tile_ok;
    } else if constexpr (S::SLIDE) {
        const int c = i < SlideMap16::LEN0 ? 0 : 1, pos = i - (c ? SlideMap16::LEN0 : 0);
        int strip, row0, nt;
        SlideMap16::chain(wave, c, strip, row0, nt);
        tile_ok = lane_ok = pos < nt;
        y = row0 + (pos < nt ? pos : nt - 1);
        xx = strip * 16 + n;
    } else {
        const int t = wave + S::NWA * i;
        tile_ok = t < S::NTILES;
        lane_ok = S::NPIX % 16 == 0 ? tile_ok : t * 16 + n < S::NPIX;
        tile_pixel<S>(tile_ok ? t : S::NTILES - 1, n, y, xx);
    }
}

// Sliding-window 3x3 SAME conv 16 -> 16 (see SlideMap16).  Tiles are taken two at a time (an even row and
// the odd row below it) with independent accumulators, so their MFMA chains interleave; the fragments of
// the next pair are read while the current pair is multiplied.  Tiles past the end of a short chain are
// computed on whatever the map holds there and stored to `trash`.
template <class S, bool ADD_X, int OUT>
__device__ __forceinline__ void block_conv_slide16(const char* src, char* dst, char* trash, const char* wslot,
                                                   floatx4 (&x)[S::NT][S::FT], int lane, int wave)
{
    static_assert(S::FT == 1 && OUT != 2, "sliding block convolution: 16 channels, LDS output");
    using SM = SlideMap16;
    const int g = lane >> 4, n = lane & 15;
    bf16x8 w[SM::NFRAG];
    load_a_frags(w, wslot, lane);
    const floatx4 bv = *(const floatx4*)(wslot + SM::NFRAG * 1024 + g * 16);
    constexpr int ROWB = S::PITCH * 16;                                  // bytes per map row
    const int laneR = ((g & 1) * S::PLANE + (g >> 1) + n) * 16;
    const int laneE = ((g & 1) * S::PLANE + (g >> 1) * S::PITCH + 2 + n) * 16;
    const int laneD = (S::PITCH + 1 + n) * 16 + (g >> 1) * (S::PLANE * 16) + (g & 1) * 8;
    auto run_chain = [&](auto cc) {
        constexpr int c = decltype(cc)::value;
        constexpr int LEN = c == 0 ? SM::LEN0 : SM::LEN1, I0 = c == 0 ? 0 : SM::LEN0;
        int strip, row0, nt;
        SM::chain(wave, c, strip, row0, nt);
        const int cb = (row0 * S::PITCH + strip * 16) * 16;              // uniform
        const char* pR = src + cb + laneR;
        const char* pE = src + cb + laneE;
        char* pD = dst + cb + laneD;
        bf16x8 R[LEN + 2], E[LEN / 2 + 1];
#pragma unroll
        for (int r = 0; r < 4; ++r) R[r] = *(const bf16x8*)(pR + r * ROWB);
        E[0] = *(const bf16x8*)pE;
        E[1] = *(const bf16x8*)(pE + 2 * ROWB);
#pragma unroll
        for (int pp = 0; pp < LEN / 2; ++pp) {
            if (pp + 1 < LEN / 2) {
                R[2 * pp + 4] = *(const bf16x8*)(pR + (2 * pp + 4) * ROWB);
                R[2 * pp + 5] = *(const bf16x8*)(pR + (2 * pp + 5) * ROWB);
                E[pp + 2] = *(const bf16x8*)(pE + (2 * pp + 4) * ROWB);
            }
            floatx4 a0 = ADD_X ? x[I0 + 2 * pp][0] + bv : bv;
            floatx4 a1 = ADD_X ? x[I0 + 2 * pp + 1][0] + bv : bv;
            SCHED_FENCE;
            a0 = mfma16(w[0], R[2 * pp], a0);      a1 = mfma16(w[0], R[2 * pp + 1], a1);
            a0 = mfma16(w[1], R[2 * pp + 1], a0);  a1 = mfma16(w[1], R[2 * pp + 2], a1);
            a0 = mfma16(w[2], R[2 * pp + 2], a0);  a1 = mfma16(w[2], R[2 * pp + 3], a1);
            a0 = mfma16(w[3], E[pp], a0);          a1 = mfma16(w[5], E[pp], a1);
            a0 = mfma16(w[4], E[pp + 1], a0);      a1 = mfma16(w[6], E[pp + 1], a1);
            SCHED_FENCE;
            const bool ok = 2 * pp < nt;                                   // uniform; chains have even lengths
            char* d = ok ? pD + (2 * pp) * ROWB : trash;
            if (ADD_X) { x[I0 + 2 * pp][0] = a0; x[I0 + 2 * pp + 1][0] = a1; }
            const bf16x4 v0 = to_bf16x4(a0), v1 = to_bf16x4(a1);
            *(bf16x4*)d = OUT == 1 ? v0 : relu_bf16x4(v0);
            *(bf16x4*)(d + (ok ? ROWB : 0)) = OUT == 1 ? v1 : relu_bf16x4(v1);
        }
    };
    run_chain(std::integral_constant<int, 0>{});
    run_chain(std::integral_constant<int, 1>{});
}

// 3x3 SAME conv C -> C on the section's pooled map, this wavefront's tiles.
// src/dst: planar maps with halo.  OUT: 0 = store ReLU(v) to dst, 1 = store v
// to dst, 2 = store ReLU(v) to the global feature row.  The B fragments of tile
// i+1 are read from LDS while tile i's MFMAs run.
struct NoFiller {
    __device__ __forceinline__ void operator()() const {}
};
// `filler`: independent vector-ALU work that every wavefront runs once, placed behind the requests for the
// weight and first activation fragments so that it executes while those travel from LDS.
// NIMG > 1: the tiles of NIMG images, whose maps sit S::ACT_BYTES apart in src and in dst, share the phase (and
// the wavefront's weight fragments): tile i belongs to image i / NT.
template <class S, bool ADD_X, int OUT, class Filler = NoFiller, int NIMG = 1>
__device__ __forceinline__ void block_conv(const char* src, char* dst, const char* wslot, const int (&tb)[S::NT],
                                           floatx4 (&x)[NIMG * S::NT][S::FT], __bf16* const (&feat_rows)[NIMG], int lane, int wave,
                                           Filler filler = Filler{})
{
    static_assert(NIMG == 1 || S::NT == 1, "several images share a phase only with one tile per wavefront each");
    constexpr int NTT = NIMG * S::NT;
    constexpr int IMG_CELLS = S::ACT_BYTES / 16;           // cells between the two images' maps
    if (wave >= S::NWA) {                                  // uniform per wavefront
        filler();
        return;
    }
    const int g = lane >> 4, n = lane & 15;
    constexpr bool WHOLE = S::NPIX % 16 == 0;              // no partial last tile
    bf16x8 w[S::WB_FRAGS];
    floatx4 bv[S::FT];
    using K = KMap<S::C>;
    int lb[K::NBASE];
    K::lane_bases(lb, g, S::PLANE, S::PITCH);
    // destination of this lane's four channels, tile base excluded
    char* dstl = dst + ((S::PITCH + 1) * 16 + (g >> 1) * (S::PLANE * 16) + (g & 1) * 8);

    // Software pipeline over (tile, chunk), pinned with scheduling fences: the activation fragment of chunk
    // kc + AHEAD (of this tile or, past its end, of the next one) is requested right after the MFMAs of chunk
    // kc, into the register slot that chunk kc + AHEAD - KCB of this tile has already left.  During the first
    // tile the weight fragments travel the same way: every wavefront of the workgroup asks for its whole weight
    // operand at the same moment, and requesting it in consumption order lets the chain start after the first
    // few fragments instead of after all of them.  (The counter of outstanding LDS reads is 4 bits wide: with
    // every read issued up front, the first wait could not be told apart from waiting for half of them.)
    constexpr int AHEAD = S::KCB < 4 ? S::KCB - 1 : 4;
    static_assert(AHEAD >= 1 && AHEAD < S::KCB, "prefetch distance");
    bf16x8 bfr[S::KCB];
    auto tbv = [&](int i) { return tb[i % S::NT] + (i / S::NT) * IMG_CELLS; };
    auto request = [&](int i, int kc, bool with_w) {          // i, kc: compile-time after unrolling
        const int ii = i < NTT ? i : NTT - 1;                 // past the last tile: a valid address, value unused
        const char* pa = src + (tbv(ii) + lb[K::kbase(kc)]) * 16;
        if (with_w) {
#pragma unroll
            for (int j = 0; j < S::FT; ++j) w[j * S::KCB + kc] = *(const bf16x8*)(wslot + ((j * S::KCB + kc) * 64 + lane) * 16);
        }
        bfr[kc] = *(const bf16x8*)(pa + K::kimm(kc, S::PITCH) * 16);
    };
#pragma unroll
    for (int j = 0; j < S::FT; ++j) bv[j] = *(const floatx4*)(wslot + S::WB_FRAGS * 1024 + (j * 4 + g) * 16);
#pragma unroll
    for (int kc = 0; kc < AHEAD; ++kc) request(0, kc, true);
    if constexpr (!std::is_same<Filler, NoFiller>::value) {
        SCHED_FENCE;
        filler();
        SCHED_FENCE;
    }
#pragma unroll
    for (int i = 0; i < NTT; ++i) {
        const int t = wave + S::NWA * (i % S::NT);
        if (t >= S::NTILES) break;                         // (two images: one tile each, both exist or neither)
        floatx4 acc[S::FT];
#pragma unroll
        for (int j = 0; j < S::FT; ++j) acc[j] = ADD_X ? x[i][j] + bv[j] : bv[j];
#pragma unroll
        for (int kc = 0; kc < S::KCB; ++kc) {
            SCHED_FENCE;
#pragma unroll
            for (int j = 0; j < S::FT; ++j) acc[j] = mfma16(w[j * S::KCB + kc], bfr[kc], acc[j]);
            if (kc + AHEAD < S::KCB) request(i, kc + AHEAD, i == 0);
            else if (i + 1 < NTT) request(i + 1, kc + AHEAD - S::KCB, false);
        }
        SCHED_FENCE;
        const int p = t * 16 + n;
#pragma unroll
        for (int j = 0; j < S::FT; ++j) {
            if (ADD_X) x[i][j] = acc[j];
            if (WHOLE || p < S::NPIX) {
                const bf16x4 vb = to_bf16x4(acc[j]);
                const bf16x4 out = OUT == 1 ? vb : relu_bf16x4(vb);
                if (OUT == 2) *(bf16x4*)(feat_rows[i / S::NT] + (size_t)p * S::C + j * 16 + g * 4) = out;
                else *(bf16x4*)(dstl + tbv(i) * 16 + j * (2 * S::PLANE * 16)) = out;
            }
        }
    }
}

// 3x3 SAME conv 32 -> 32 on an 18 x 24 map laid out for TileMap1824, this wavefront's chain of up to four tiles.
// One instruction stream per wavefront, software-pipelined by hand (the order below is pinned with scheduling
// fences): the MFMAs of tile i run back to back, kernel rows 0, 1, 2, and between them issue
//   * the three fragment reads of tile i + 1's new window row, into the registers tile i's kernel row 0 has
//     just left (they then have six chunks' time to arrive),
//   * the epilogue of tile i - 1 (conversion, ReLU, store), a few instructions per chunk, and
//   * the start values of tile i + 1's accumulators.
// A wavefront's own vector instructions do issue under its running MFMAs (an MFMA occupies the issue port for
// 8 of its 16 cycles; measured: up to two vector instructions per MFMA are free), so the epilogue costs no time
// of its own and a wavefront running alone at the end of a phase still keeps the matrix pipe fed.
template <class S, bool ADD_X, int OUT, class Filler = NoFiller>
__device__ __forceinline__ void block_conv_v2(const char* src, char* dst, const char* wslot, const int (&tb)[4],
                                              floatx4 (&x)[4][2], int lane, int wave, Filler filler = Filler{})
{
    static_assert(S::FT == 2 && S::C == 32 && OUT != 2, "18 x 24 maps of 32 channels, LDS output");
    using TM = TileMap1824;
    const int g = lane >> 4;
    const int nt = TM::ntiles(wave);                                  // uniform
    const bool restart2 = TM::fresh(wave, 2);                         // uniform
    const int lb = g * S::PLANE;
    char* dstl = dst + ((S::PITCH + 1) * 16 + (g >> 1) * (S::PLANE * 16) + (g & 1) * 8);
    bf16x8 w[18];
    bf16x8 F[3][3];                                                   // window row (i + kh) % 3, kernel column kw
    floatx4 bv[2];
    auto wfrag = [&](int kc) {
        w[kc] = *(const bf16x8*)(wslot + (kc * 64 + lane) * 16);
        w[9 + kc] = *(const bf16x8*)(wslot + ((9 + kc) * 64 + lane) * 16);
    };
    auto frag = [&](int i, int kh, int kw) { return *(const bf16x8*)(src + (tb[i] + lb + kh * S::PITCH + kw) * 16); };
#pragma unroll
    for (int j = 0; j < 2; ++j) bv[j] = *(const floatx4*)(wslot + 18 * 1024 + (j * 4 + g) * 16);
    // tile 0: weights and fragments chunk by chunk in the order the chain consumes them, four chunks ahead
    constexpr int AHEAD = 4;
#pragma unroll
    for (int kc = 0; kc < AHEAD; ++kc) { wfrag(kc); F[kc / 3][kc % 3] = frag(0, kc / 3, kc % 3); }
    if constexpr (!std::is_same<Filler, NoFiller>::value) {
        SCHED_FENCE;
        filler();
        SCHED_FENCE;
    }
    floatx4 acc[2], nxt[2], fin[2];
    bf16x4 ob[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[j] = ADD_X ? x[0][j] + bv[j] : bv[j];
    auto store = [&](int i, int j, bf16x4 v) { *(bf16x4*)(dstl + tb[i] * 16 + j * (2 * S::PLANE * 16)) = v; };
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (i >= nt) break;                                            // uniform
        if (i == 2 && restart2) {                                      // uniform: a new chain, its first two window rows
#pragma unroll
            for (int q = 0; q < 6; ++q) F[(i + q / 3) % 3][q % 3] = frag(i, q / 3, q % 3);
        }
#pragma unroll
        for (int kc = 0; kc < 9; ++kc) {
            const int kh = kc / 3, kw = kc % 3;
            SCHED_FENCE;
            acc[0] = mfma16(w[kc], F[(i + kh) % 3][kw], acc[0]);
            acc[1] = mfma16(w[9 + kc], F[(i + kh) % 3][kw], acc[1]);
            if (i == 0 && kc + AHEAD < 9) { wfrag(kc + AHEAD); F[(kc + AHEAD) / 3][(kc + AHEAD) % 3] = frag(0, (kc + AHEAD) / 3, (kc + AHEAD) % 3); }
            if (kc == 2 && i + 1 < 4) {                                // tile i + 1's new row (a missing tile repeats the last one)
#pragma unroll
                for (int q = 0; q < 3; ++q) F[i % 3][q] = frag(i + 1, 2, q);
            }
            if (i > 0) {                                               // epilogue of tile i - 1
                if (kc == 3) ob[0] = to_bf16x4(fin[0]);
                if (kc == 4) store(i - 1, 0, OUT == 1 ? ob[0] : relu_bf16x4(ob[0]));
                if (kc == 5) ob[1] = to_bf16x4(fin[1]);
                if (kc == 6) store(i - 1, 1, OUT == 1 ? ob[1] : relu_bf16x4(ob[1]));
            }
            if (kc == 7 && i + 1 < 4) nxt[0] = ADD_X ? x[i + 1][0] + bv[0] : bv[0];
            if (kc == 8 && i + 1 < 4) nxt[1] = ADD_X ? x[i + 1][1] + bv[1] : bv[1];
        }
        SCHED_FENCE;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            fin[j] = acc[j];
            if (ADD_X) x[i][j] = acc[j];
            acc[j] = nxt[j];
        }
    }
    // the last tile's epilogue
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (i + 1 == nt) {                                             // uniform
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const bf16x4 vb = to_bf16x4(fin[j]);
                store(i, j, OUT == 1 ? vb : relu_bf16x4(vb));
            }
        }
    }
}

// conv0 of a CONVMAP section in block_conv's terms: a 3x3 SAME conv C -> C over the section's H x W input map,
// all wavefronts, output = the un-pooled, un-rectified conv map (planar, same geometry as the input).
template <class S>
struct ConvMapCfg {
    static constexpr int C = S::C, FT = S::FT, KCB = S::KC0, WB_FRAGS = S::W0_FRAGS;
    static constexpr int PH = S::H, PW = S::W, NPIX = PH * PW, NTILES = (NPIX + 15) / 16;
    static constexpr bool V2 = C == 32 && PH == 18 && PW == 24 && S::IPADX == 2 && RN_WAVES == 8;
    static constexpr int NWA = RN_WAVES, NT = V2 ? 4 : (NTILES + NWA - 1) / NWA;
    static constexpr int PITCH = S::IPITCH, PLANE = S::IPLANE, ACT_BYTES = S::CM_BYTES;
    static_assert(S::CONVMAP && S::IROWS == S::H + 2 && PLANE * (C / 8) * 16 == S::CM_BYTES, "conv map geometry");
};

template <class S, class Filler = NoFiller>
__device__ __forceinline__ void conv_map(const char* in, char* out, const char* wslot, int lane, int wave, Filler filler = Filler{})
{
    using CM = ConvMapCfg<S>;
    int tb[CM::NT];
    floatx4 unused[CM::NT][CM::FT];                        // block_conv reads x only when it adds it
    if constexpr (CM::V2) {
#pragma unroll
        for (int i = 0; i < CM::NT; ++i) {
            int y, xx;
            bool ok;
            TileMap1824::pixel(wave, i, lane & 15, y, xx, ok);
            tb[i] = y * CM::PITCH + xx;
        }
        block_conv_v2<CM, false, 1, Filler>(in, out, wslot, tb, unused, lane, wave, filler);
    } else {
#pragma unroll
        for (int i = 0; i < CM::NT; ++i) {
            const int t = wave + CM::NWA * i;
            int y, xx;
            tile_pixel<CM>(t < CM::NTILES ? t : CM::NTILES - 1, lane & 15, y, xx);
            tb[i] = y * CM::PITCH + xx;
        }
        __bf16* const no_rows[1] = {nullptr};
        block_conv<CM, false, 1, Filler>(in, out, wslot, tb, unused, no_rows, lane, wave, filler);
    }
}

// 3x3 / stride-2 maximum of a CONVMAP section's conv map at pooled pixel (y, xx) for the lane's four channels of
// feature tile j.  Window rows and columns that fall outside the map are clamped onto it (a repeated value
// does not change a maximum), which is the SAME padding of max-pooling.
template <class S>
__device__ __forceinline__ void pool_window(const char* cmap, int y, int xx, int g, bf16x4 (&v)[S::FT][9])
{
    using CM = ConvMapCfg<S>;
    int ro[3], co[3];
#pragma unroll
    for (int d = 0; d < 3; ++d) {
        const int r = 2 * y - S::PADH + d, c = 2 * xx + d;
        ro[d] = ((r < 0 ? 0 : (r > S::H - 1 ? S::H - 1 : r)) + 1) * CM::PITCH;
        co[d] = (c > S::W - 1 ? S::W - 1 : c) + 1;
    }
    const char* base = cmap + (g >> 1) * (CM::PLANE * 16) + (g & 1) * 8;
#pragma unroll
    for (int j = 0; j < S::FT; ++j)
#pragma unroll
        for (int d = 0; d < 9; ++d) v[j][d] = *(const bf16x4*)(base + (ro[d / 3] + co[d % 3]) * 16 + j * (2 * CM::PLANE * 16));
}

// zero the halo ring of a planar map of CG planes (PLANE cells apart), interior IH x IW
template <int CG, int IH, int IW, int PLANE, int PITCH = IW + 2>
__device__ __forceinline__ void zero_halo(char* buf, int tid)
{
    constexpr int ROWS = IH + 2;
    constexpr int RING = 2 * PITCH + 2 * IH;          // cells in one plane's ring (whole first and last rows)
    const bf16x8 z = {};
    for (int i = tid; i < CG * RING; i += RN_THREADS) {
        const int cg = i / RING, r = i % RING;
        int y, xx;
        if (r < PITCH) { y = 0; xx = r; }
        else if (r < 2 * PITCH) { y = ROWS - 1; xx = r - PITCH; }
        else { const int q = r - 2 * PITCH; y = 1 + (q >> 1); xx = (q & 1) ? IW + 1 : 0; }
        *(bf16x8*)(buf + (cg * PLANE + y * PITCH + xx) * 16) = z;
    }
}

// LDS layout shared by the sections of one network.
template <int B0_, int B1_, int EDGE_, int PERM_>
struct LdsMap {
    static constexpr int r256(int v) { return (v + 255) / 256 * 256; }
    static constexpr int BUF0 = 0;
    static constexpr int BUF1 = r256(B0_);
    static constexpr int EDGE = BUF1 + r256(B1_);
    static constexpr int NEUTRAL = EDGE + EDGE_;                   // 8 bytes below every activation: 'no edge column'
    static constexpr int TRASH = EDGE + r256(EDGE_ + 16);         // 512 B: where lanes with nothing to store write
    static constexpr int WSA = TRASH + 512;
    static constexpr int WSB_HI = WSA + WSLOT_BYTES;
    static constexpr int PERM = LDS_TOTAL - r256(PERM_);           // first layer's weights, resident for the whole kernel
    static constexpr int WSB_HI_CAP = PERM - WSB_HI;
    static constexpr int LOW_SLOT_AT = 36 * 1024;                  // maps of at most this size leave room for a weight slot behind them
    static constexpr int WSB_LO = BUF1 + LOW_SLOT_AT;              // inside buf1's tail: only while buf1 holds <= LOW_SLOT_AT bytes
    static constexpr int WSB_LO0 = BUF0 + LOW_SLOT_AT;             // inside buf0's tail, for sections whose input sits in buf1
    static_assert(WSB_LO0 + WSLOT_BYTES <= BUF1, "low weight slot must fit in buf0's tail");
    static_assert(WSB_HI_CAP >= 0, "LDS layout does not fit");
    static_assert(WSB_LO + WSLOT_BYTES <= EDGE, "low weight slot must fit in buf1's tail");
};

// x-read of a CONVMAP section, in two halves so that two images can share the block phases: pooled_x takes the
// 3x3/2 maximum of the conv map for this wavefront's tiles (x, and the tiles' cell indices tb); store_relu
// writes R = ReLU(x) into a planar map.
template <class S>
__device__ __forceinline__ void pooled_x(const char* cmap, int (&tb)[S::NT], floatx4 (&x)[S::NT][S::FT], bool (&ok)[S::NT],
                                         int lane, int wave)
{
    const int g = lane >> 4, n = lane & 15;
    if (wave >= S::NWA) return;
    bf16x4 wv[S::NT][S::FT][9];
#pragma unroll
    for (int i = 0; i < S::NT; ++i) {                      // all loads first
        int y, xx;
        bool tile_ok;
        tile_ref<S>(wave, i, n, y, xx, tile_ok, ok[i]);
        tb[i] = y * S::PITCH + xx;
        if (!tile_ok) break;
        pool_window<S>(cmap, y, xx, g, wv[i]);
    }
#pragma unroll
    for (int i = 0; i < S::NT; ++i) {
        if (wave + S::NWA * i >= S::NTILES) break;
#pragma unroll
        for (int j = 0; j < S::FT; ++j) {
            // nine-value maxima on bf16 pairs (packed fp16 maximum, exact for these values: see bf16x2_max), widened once
            uint2 m = __builtin_bit_cast(uint2, wv[i][j][0]);
#pragma unroll
            for (int d = 1; d < 9; ++d) {
                const uint2 w = __builtin_bit_cast(uint2, wv[i][j][d]);
                m.x = bf16x2_max(m.x, w.x);
                m.y = bf16x2_max(m.y, w.y);
            }
            x[i][j] = floatx4{bf16_lo_f32(m.x), bf16_hi_f32(m.x), bf16_lo_f32(m.y), bf16_hi_f32(m.y)};
        }
    }
}

template <class S>
__device__ __forceinline__ void store_relu(char* rmap, const int (&tb)[S::NT], const floatx4 (&x)[S::NT][S::FT],
                                           const bool (&ok)[S::NT], int lane, int wave)
{
    const int g = lane >> 4;
    if (wave >= S::NWA) return;
    const int loff = (S::PITCH + 1) * 16 + (g >> 1) * (S::PLANE * 16) + (g & 1) * 8;
#pragma unroll
    for (int i = 0; i < S::NT; ++i) {
        if (wave + S::NWA * i >= S::NTILES) break;
#pragma unroll
        for (int j = 0; j < S::FT; ++j)
            if (ok[i]) *(bf16x4*)(rmap + tb[i] * 16 + loff + j * (2 * S::PLANE * 16)) = relu_bf16x4(to_bf16x4(x[i][j]));
    }
}

// Weight sets are numbered along one image: S1.block1.a = 0 ... (the first layer's set is resident).  Set q
// lives in slot A when q is even, else in slot B; B is the high slot while the consuming section keeps its maps
// full size (section 1) and otherwise the low slot inside the unused tail of buf1, or of buf0 when the
// consuming section's input sits in buf1 (INB: it follows an XFUSED section).
template <class M, class S, bool INB>
constexpr int wslot(int q)
{
    return (q & 1) == 0 ? M::WSA : (S::ACT_BYTES > M::LOW_SLOT_AT ? M::WSB_HI : (INB ? M::WSB_LO0 : M::WSB_LO));
}

// One section for one image.
//   J0: number of this section's conv0 weight set (-1: the resident first-layer set); its blocks use J0+1..J0+4.
//   SN / nsw: the next section (its conv0 set is staged from here); NSETS: sets per image.
//   Staging rule: the phase that uses set j starts the asynchronous load of set j+1 into the other slot and
//   waits for it just before its closing barrier (the x-read phase uses no set and stages nothing).
// On entry (INKIND == IN_LDS) buf0 holds the previous section's un-rectified output as a planar map with
// halo; on exit (not LAST) buf0 holds this section's.  LAST writes ReLU(x) to feat_row.
template <class S, class SN, class M, bool LAST, int SI, int J0, int NSETS, bool INB, class PreT>
__device__ __forceinline__ void run_section(char* lds, const SecWeights& sw, const SecWeights& nsw,
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
    // Buffer roles.  Normally conv0 reads buf0 and pools into buf1, the x-read phase moves ReLU(x) to buf0, and
    // the blocks alternate R (buf0) -> U (buf1) -> R.  INB: the input sits in buf1 (the previous section was
    // XFUSED), conv0 pools into buf0 and the x-read phase rectifies in place.  XFUSED: conv0 leaves R in buf1
    // and the blocks run buf1 -> buf0 -> buf1, so this section's output lands in buf1.
    static_assert(!INB || (S::INKIND == IN_LDS && !S::CONVMAP && !S::XFUSED && (J0 < 0 || J0 % 2 == 0)), "input in buf1: strip-pooled LDS sections only");
    char* cin = INB ? buf1 : buf0;
    char* pool = INB ? buf0 : buf1;
    char* bufR = S::XFUSED ? buf1 : buf0;
    char* bufU = S::XFUSED ? buf0 : buf1;
    constexpr int QB = J0 + 1;                                   // set number of block1.a
    constexpr int SLOT_C0 = J0 < 0 ? M::PERM : wslot<M, S, INB>(J0);
    static_assert(S::ACT_BYTES <= M::LOW_SLOT_AT || S::WB_SET * 1024 <= M::WSB_HI_CAP, "block weights do not fit the high slot");
    static_assert(S::WB_SET * 1024 <= WSLOT_BYTES && S::W0_SET * 1024 <= WSLOT_BYTES, "weight set larger than a slot");
    static_assert(LAST || (QB + 4) % 2 == 0 || SN::ACT_BYTES <= M::LOW_SLOT_AT || SN::W0_SET * 1024 <= M::WSB_HI_CAP, "next conv0 set does not fit");
    // set q (relative to this section: 0 = block1.a ... 3 = block2.b, 4 = next conv0)
    auto stage = [&](auto rel) {
        constexpr int r = decltype(rel)::value;
        constexpr int q = QB + r;
        if constexpr (q < NSETS) {
            if constexpr (r < 4) stage_set<S::WB_SET>(sw.wb[r], lds + wslot<M, S, INB>(q), lane, wave);
            else stage_set<SN::W0_SET>(nsw.w0, lds + wslot<M, SN, S::XFUSED>(q), lane, wave);
        }
    };
    using I0 = std::integral_constant<int, 0>; using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>; using I3 = std::integral_constant<int, 3>;
    using I4 = std::integral_constant<int, 4>;
    floatx4 x[S::NT][S::FT];

    // ---------------- conv0 + max-pool ----------------
    {
        stage(I0{});                                             // this phase uses set J0: stage J0 + 1
        if constexpr (!S::CONVMAP) zero_halo<S::C / 8, S::PH, S::PW, S::PLANE, S::PITCH>(pool, tid);
        bf16x8 w0[S::CONVMAP ? 1 : S::W0_FRAGS];
        if constexpr (S::CONVMAP) {
            conv_map<S>(buf0, buf1, lds + SLOT_C0, lane, wave);     // buf1 <- the full-resolution conv map
        } else if constexpr (S::INKIND == IN_LDS) {
            load_a_frags(w0, lds + SLOT_C0, lane);
            conv0_pool<S>(cin, pool, edge, lds + M::TRASH, w0, lds + SLOT_C0, 0, S::PH, -1, lane, wave);
        } else {
            // Strips: strip 0 is already in buf0 (the previous image's last phase or the kernel prologue put it
            // there).  With several strips the loads run TWO strips ahead, alternating between the caller's
            // register set (even strips) and a second one (odd strips): one strip's convolution is several
            // times shorter than a trip to memory.
            constexpr bool TWO_AHEAD = S::NSTRIPS > 1 && S::NSTRIPS % 2 == 0;
            PreT pre_odd;
            auto one_strip = [&](int strip, PreT& mine) {          // `mine`: the register set strips of this parity use
                if (strip > 0) prefetch_commit<S>(mine, buf0, strip, tid);
                if constexpr (TWO_AHEAD) {
                    if (strip == 0) prefetch_issue<S>(pre_odd, obs_img, 1, tid);
                    if (strip + 2 < S::NSTRIPS) prefetch_issue<S>(mine, obs_img, strip + 2, tid);
                } else {
                    if (strip + 1 < S::NSTRIPS) prefetch_issue<S>(mine, obs_img, strip + 1, tid);
                }
                if (strip > 0) lds_barrier();
                if (strip == 0) load_a_frags(w0, lds + SLOT_C0, lane);
                int pr0, pr1, r0, r1;
                strip_rows<S>(strip, pr0, pr1, r0, r1);
                if constexpr (S::XFUSED) conv0_pool3_x<S>(buf0, buf1, w0, lds + SLOT_C0, x, lane, wave);
                else if constexpr (S::POOL3) conv0_pool3<S>(buf0, buf1, w0, lds + SLOT_C0, lane, wave);
                else conv0_pool<S>(buf0, buf1, edge, lds + M::TRASH, w0, lds + SLOT_C0, pr0, pr1, r0 - 1, lane, wave);
                if (strip + 1 < S::NSTRIPS) lds_barrier();
            };
            if constexpr (TWO_AHEAD) {
#pragma unroll 1
                for (int strip = 0; strip < S::NSTRIPS; strip += 2) {
                    one_strip(strip, pre);
                    one_strip(strip + 1, pre_odd);
                }
            } else {
#pragma unroll 1
                for (int strip = 0; strip < S::NSTRIPS; ++strip) one_strip(strip, pre);
            }
        }
        stage_wait();
        lds_barrier();
    }

    // ---------------- x <- pooled map (+ edge columns); R = ReLU(x) ----------------
    int tb[S::NT];                                     // per tile: cell index of the lane's pixel (tap (0,0), plane 0)
    if constexpr (!S::XFUSED) {
        // INB: R replaces the pooled values in buf0 cell by cell (a lane reads and writes only its own cells and
        // the halo is already zero); buf1 gets the zero halo the first block's output needs
        zero_halo<S::C / 8, S::PH, S::PW, S::PLANE, S::PITCH>(INB ? buf1 : buf0, tid);
        if constexpr (S::CONVMAP) {
            bool ok[S::NT];
            pooled_x<S>(buf1, tb, x, ok, lane, wave);   // x = 3x3/2 maximum of the conv map in buf1
            store_relu<S>(buf0, tb, x, ok, lane, wave);
        } else if (wave < S::NWA) {
            const int loff = (S::PITCH + 1) * 16 + (g >> 1) * (S::PLANE * 16) + (g & 1) * 8;
            bf16x4 pv[S::NT][S::FT], ev[S::NT][S::FT];
            bool ok[S::NT];
#pragma unroll
            for (int i = 0; i < S::NT; ++i) {          // all loads first
                int y, xx;
                bool tile_ok;
                tile_ref<S>(wave, i, n, y, xx, tile_ok, ok[i]);
                tb[i] = y * S::PITCH + xx;
                if (!S::SLIDE && !tile_ok) break;
                // the pooled value of a strip's last column lacks its right neighbour: it is the next strip's edge
                // column; every other lane reads the neutral cell instead
                const bool fix = !S::POOL3 && (xx & 7) == 7 && xx + 1 < S::PW;
                const int eoff = fix ? M::EDGE + (((((xx + 1) >> 3) * S::PH + y) * S::C + g * 4) * 2) : M::NEUTRAL;
                const int ejmp = fix ? 32 : 0;
                const int off = tb[i] * 16 + loff;
#pragma unroll
                for (int j = 0; j < S::FT; ++j) {
                    pv[i][j] = *(const bf16x4*)(pool + off + j * (2 * S::PLANE * 16));
                    if constexpr (!S::POOL3) ev[i][j] = *(const bf16x4*)(lds + eoff + j * ejmp);
                }
            }
#pragma unroll
            for (int i = 0; i < S::NT; ++i) {
                if (!S::SLIDE && wave + S::NWA * i >= S::NTILES) break;
                const int off = tb[i] * 16 + loff;
#pragma unroll
                for (int j = 0; j < S::FT; ++j) {
                    bf16x4 r;
                    if constexpr (S::POOL3) {
                        x[i][j] = to_floatx4(pv[i][j]);
                        r = pv[i][j];
                    } else {
                        // maximum on the bf16 pairs (bf16x2_max), widened once; R needs no conversion back
                        const uint2 a = __builtin_bit_cast(uint2, pv[i][j]), e = __builtin_bit_cast(uint2, ev[i][j]);
                        const uint2 m = {bf16x2_max(a.x, e.x), bf16x2_max(a.y, e.y)};
                        x[i][j] = floatx4{bf16_lo_f32(m.x), bf16_hi_f32(m.x), bf16_lo_f32(m.y), bf16_hi_f32(m.y)};
                        r = __builtin_bit_cast(bf16x4, m);
                    }
                    // a short chain's missing tiles rewrite its last tile with the same values
                    if (S::SLIDE || ok[i]) *(bf16x4*)(buf0 + off + j * (2 * S::PLANE * 16)) = relu_bf16x4(r);
                }
            }
        }
        lds_barrier();
    }
    __bf16* const feat_rows[1] = {feat_row};
    auto conv = [&](auto add_x, auto out, const char* src, char* dst, const char* ws, auto filler) {
        constexpr bool ADD_X = decltype(add_x)::value;
        constexpr int OUT = decltype(out)::value;
        if constexpr (S::SLIDE) {
            filler();
            block_conv_slide16<S, ADD_X, OUT>(src, dst, lds + M::TRASH + lane * 8, ws, x, lane, wave);
        } else if constexpr (S::V2) {
            block_conv_v2<S, ADD_X, OUT>(src, dst, ws, tb, x, lane, wave, filler);
        } else {
            block_conv<S, ADD_X, OUT>(src, dst, ws, tb, x, feat_rows, lane, wave, filler);
        }
    };
    using BF = std::false_type; using BT = std::true_type;

    // ---------------- residual blocks ----------------
    // The last section's maps are small and the next frame sits in registers: its rows that land behind
    // those maps in buf0 are converted a slice per block phase (the wavefronts mostly wait for LDS here), the
    // rest in the last phase, when buf0 is free.
    using PS = typename PreT::Sec;
    constexpr bool SLICED = LAST && PS::INKIND == IN_U8_C3 && PS::NSTRIPS == 1 && PS::PRE_N == 4 &&
                            S::ACT_BYTES <= PS::PRE_SPLIT_BYTES;
    auto slice = [&](auto part) {
        return [&pre, buf0, tid]() {
            if constexpr (SLICED) prefetch_commit<PS, decltype(part)::value>(pre, buf0, 0, tid);
        };
    };
    stage(I1{});
    // U's buffer held the conv map (CONVMAP) or the frame (XFUSED) until now: its halo ring is zeroed while
    // this phase fills its interior
    if constexpr (S::CONVMAP || S::XFUSED) zero_halo<S::C / 8, S::PH, S::PW, S::PLANE, S::PITCH>(bufU, tid);
    conv(BF{}, I0{}, bufR, bufU, lds + wslot<M, S, INB>(QB), slice(I1{}));
    stage_wait();
    lds_barrier();
    stage(I2{});
    conv(BT{}, I0{}, bufU, bufR, lds + wslot<M, S, INB>(QB + 1), slice(I2{}));
    stage_wait();
    lds_barrier();
    stage(I3{});
    conv(BF{}, I0{}, bufR, bufU, lds + wslot<M, S, INB>(QB + 2), slice(I3{}));
    stage_wait();
    lds_barrier();
    if constexpr (!LAST) stage(I4{});
    conv(BT{}, std::integral_constant<int, LAST ? 2 : 1>{}, bufU, bufR, lds + wslot<M, S, INB>(QB + 3), NoFiller{});
    // The last layer writes to global memory, so buf0 is free: the next frame's first strip (prefetched into
    // registers before this section) is converted into it here, under this phase's barrier.
    if constexpr (LAST) prefetch_commit<PS, SLICED ? 0 : -1>(pre, buf0, 0, tid);
    stage_wait();
    lds_barrier();
}

// ---- several images through the last section's block phases together ----
// The last section's maps are small (7 tiles of 16 pixels on the 9 x 12 map): a block phase there is mostly the
// price of every wavefront fetching the layer's whole weight operand, the barrier and the operand latencies, for
// one tile of work.  A workgroup therefore takes its images in groups: every member runs through sections 1 and
// 2 and the last section's conv0 and pooling; the residual streams of all but the last member then wait in 8
// registers per lane each, and the four block convolutions run once for the whole group, one tile per image and
// wavefront on one set of weight fragments.
//   last_front_first: conv0 + pooling of a waiting member; no R map is written yet.  The next member's frame
//     (prefetched into `pre`) is converted into buf0, which is free once conv0 has read it.
//   last_group: conv0 + pooling of the last member, R maps of all (buf0 + k * ACT_BYTES), the block phases on
//     all, features of all to global memory; the next group's first frame is converted into buf0 in slices
//     behind the block phases' fragment requests, above the R maps, and below them in the last phase.
template <class S, class M, int J0, class PreT>
__device__ __forceinline__ void last_front_first(char* lds, floatx4 (&xa)[S::NT][S::FT], PreT& pre, int tid)
{
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    char* buf0 = lds + M::BUF0;
    char* buf1 = lds + M::BUF1;
    conv_map<S>(buf0, buf1, lds + wslot<M, S, false>(J0), lane, wave);
    lds_barrier();
    int tb[S::NT];
    bool ok[S::NT];
    pooled_x<S>(buf1, tb, xa, ok, lane, wave);
    prefetch_commit<typename PreT::Sec>(pre, buf0, 0, tid);
    lds_barrier();
}

template <class S, class M, int J0, int NSETS, int N, int NQ, class PreT>
__device__ __forceinline__ void last_group(char* lds, const SecWeights& sw, const floatx4 (&xq)[NQ][S::NT][S::FT], PreT& pre,
                                           __bf16* __restrict__ feat0, size_t feat_step, int tid)
{
    // image k of the group (k = 0 .. N-2) waits in xq[N-2-k] (the most recent one in xq[0]); image N-1 is the
    // one whose section-2 output sits in buf0 now; image k's features go to feat0 + k * feat_step
    static_assert(N >= 2 && N - 1 <= NQ, "group size");
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    char* buf0 = lds + M::BUF0;
    char* buf1 = lds + M::BUF1;
    using PS = typename PreT::Sec;
    constexpr int QB = J0 + 1;
    constexpr int IMG = S::ACT_BYTES;                      // distance between two images' maps
    constexpr int LIMIT = N * IMG;                         // the frame's cells below this byte wait for the last phase
    static_assert(S::CONVMAP && S::NT == 1 && N * IMG <= M::LOW_SLOT_AT, "groups: small conv-map sections, one tile per wavefront");
    static_assert(PS::INKIND == IN_U8_C3 && PS::NSTRIPS == 1 && PS::PRE_N == 4, "groups: whole 3-channel frame in four items per thread");
    auto stage = [&](auto rel) {
        constexpr int r = decltype(rel)::value;
        static_assert(QB + r < NSETS, "set number");
        stage_set<S::WB_SET>(sw.wb[r], lds + wslot<M, S, false>(QB + r), lane, wave);
    };
    auto halos = [&](char* buf) {
#pragma unroll
        for (int k = 0; k < N; ++k) zero_halo<S::C / 8, S::PH, S::PW, S::PLANE, S::PITCH>(buf + k * IMG, tid);
    };
    using I0 = std::integral_constant<int, 0>; using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>; using I3 = std::integral_constant<int, 3>;

    // conv0 of the last image
    stage(I0{});
    conv_map<S>(buf0, buf1, lds + wslot<M, S, false>(J0), lane, wave);
    stage_wait();
    lds_barrier();
    // pooled x of the last image; R of all
    floatx4 x[N * S::NT][S::FT];
    int tb[S::NT];
    bool ok[S::NT];
    {
        floatx4 xb[S::NT][S::FT];
        pooled_x<S>(buf1, tb, xb, ok, lane, wave);
        halos(buf0);
#pragma unroll
        for (int k = 0; k < N - 1; ++k) {
            store_relu<S>(buf0 + k * IMG, tb, xq[N - 2 - k], ok, lane, wave);
#pragma unroll
            for (int j = 0; j < S::FT; ++j) x[k][j] = xq[N - 2 - k][0][j];
        }
        store_relu<S>(buf0 + (N - 1) * IMG, tb, xb, ok, lane, wave);
#pragma unroll
        for (int j = 0; j < S::FT; ++j) x[N - 1][j] = xb[0][j];
    }
    lds_barrier();
    // block phases on all images
    __bf16* feats[N];
#pragma unroll
    for (int k = 0; k < N; ++k) feats[k] = feat0 + k * feat_step;
    auto slice = [&](auto part) {
        return [&pre, buf0, tid]() { prefetch_commit<PS, decltype(part)::value, LIMIT>(pre, buf0, 0, tid); };
    };
    stage(I1{});
    halos(buf1);                                           // held the conv map until now
    block_conv<S, false, 0, decltype(slice(I1{})), N>(buf0, buf1, lds + wslot<M, S, false>(QB), tb, x, feats, lane, wave, slice(I1{}));
    stage_wait();
    lds_barrier();
    stage(I2{});
    block_conv<S, true, 0, decltype(slice(I2{})), N>(buf1, buf0, lds + wslot<M, S, false>(QB + 1), tb, x, feats, lane, wave, slice(I2{}));
    stage_wait();
    lds_barrier();
    stage(I3{});
    block_conv<S, false, 0, decltype(slice(I3{})), N>(buf0, buf1, lds + wslot<M, S, false>(QB + 2), tb, x, feats, lane, wave, slice(I3{}));
    stage_wait();
    lds_barrier();
    block_conv<S, true, 2, NoFiller, N>(buf1, buf0, lds + wslot<M, S, false>(QB + 3), tb, x, feats, lane, wave);
    prefetch_commit<PS, 0, LIMIT>(pre, buf0, 0, tid);      // buf0's maps are dead: the rest of the frame and its halo
    lds_barrier();
}

template <class S1, class S2, class S3>
struct Net3 {
    static constexpr int mx(int a, int b) { return a > b ? a : b; }
    static constexpr int B0 = mx(mx(mx(S1::ACT_BYTES, S1::IN_BYTES), mx(S2::ACT_BYTES, S2::IN_BYTES)), mx(S3::ACT_BYTES, S3::IN_BYTES));
    static constexpr int B1 = mx(mx(S1::ACT_BYTES, S2::ACT_BYTES), S3::ACT_BYTES);
    static constexpr int EDGE = mx(mx(S1::EDGE_BYTES, S2::EDGE_BYTES), S3::EDGE_BYTES);
    using M = LdsMap<B0, B1, EDGE, S1::W0_SET * 1024>;
    static constexpr int NSETS = 14;
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
    if (tid == 0) {   // the neutral edge cell
        *(uint2*)(lds + M::NEUTRAL) = uint2{BF16X2_LOWEST, BF16X2_LOWEST};
    }
    // the resident first-layer weight set
    stage_set<S1::W0_SET>(a.sec[0].w0, lds + M::PERM, tid & 63, __builtin_amdgcn_readfirstlane(tid >> 6));
    Prefetch<S1> pre;
    prefetch_issue<S1>(pre, a.obs + FRAME * blockIdx.x, 0, tid);
    prefetch_commit<S1>(pre, lds + M::BUF0, 0, tid);
    stage_wait();
    lds_barrier();
    // Images in groups of up to NG where the last section allows it (see last_group): the members of a group run
    // one after the other through ONE copy of the code of sections 1 and 2; all but the last then do the last
    // section's conv0 and pooling and wait, the last one finishes the group.  A group of one takes the plain path.
    constexpr int NG = (S3::CONVMAP && S3::NT == 1 && !S2::XFUSED && S1::INKIND == IN_U8_C3 && S1::NSTRIPS == 1 && S1::PRE_N == 4)
                           ? RN_GROUP : 1;
    static_assert(NG == 1 || NG * S3::ACT_BYTES <= M::LOW_SLOT_AT, "the group's maps must leave the low weight slot free");
    const int grid = (int)gridDim.x;
    floatx4 xq[NG > 1 ? NG - 1 : 1][S3::NT][S3::FT];                   // pooled x of the waiting members, most recent first
    for (int img = blockIdx.x; img < a.B; img += NG * grid) {
        int n = 1;                                                     // members of this group (uniform over the workgroup)
        while (n < NG && img + n * grid < a.B) ++n;
        for (int k = 0; k < n; ++k) {
            const int cur = img + k * grid;
            const uint8_t* obs_img = a.obs + FRAME * cur;
            __bf16* feat_row = a.feat + (size_t)cur * a.ldf;
            run_section<S1, S2, M, false, 0, -1, N::NSETS, false>(lds, a.sec[0], a.sec[1], obs_img, pre, feat_row, tid);
            run_section<S2, S3, M, false, 1, 4, N::NSETS, S1::XFUSED>(lds, a.sec[1], a.sec[2], obs_img, pre, feat_row, tid);
            // the next frame's bytes travel while the last section computes (unconditional load address)
            const int nxt = k + 1 < n ? cur + grid : (img + NG * grid < a.B ? img + NG * grid : cur);
            prefetch_issue<S1>(pre, a.obs + FRAME * nxt, 0, tid);
            if (n == 1) {
                run_section<S3, S3, M, true, 2, 9, N::NSETS, S2::XFUSED>(lds, a.sec[2], a.sec[2], obs_img, pre, feat_row, tid);
            } else if constexpr (NG > 1) {
                __bf16* feat0 = a.feat + (size_t)img * a.ldf;
                const size_t fstep = (size_t)grid * a.ldf;
                if (k + 1 < n) {
#pragma unroll
                    for (int q = NG - 2; q > 0; --q)
#pragma unroll
                        for (int j = 0; j < S3::FT; ++j) xq[q][0][j] = xq[q - 1][0][j];
                    last_front_first<S3, M, 9>(lds, xq[0], pre, tid);
                } else if (n == 2) {
                    last_group<S3, M, 9, N::NSETS, 2, NG - 1>(lds, a.sec[2], xq, pre, feat0, fstep, tid);
                } else if constexpr (NG >= 3) {
                    if (n == 3) last_group<S3, M, 9, N::NSETS, 3, NG - 1>(lds, a.sec[2], xq, pre, feat0, fstep, tid);
                    else if constexpr (NG >= 4) last_group<S3, M, 9, N::NSETS, 4, NG - 1>(lds, a.sec[2], xq, pre, feat0, fstep, tid);
                }
            }
        }
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
    static constexpr int NSETS = 19;
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
    if (tid == 0) {   // the neutral edge cell
        *(uint2*)(lds + M::NEUTRAL) = uint2{BF16X2_LOWEST, BF16X2_LOWEST};
    }
    stage_set<S1::W0_SET>(a.sec[0].w0, lds + M::PERM, tid & 63, __builtin_amdgcn_readfirstlane(tid >> 6));
    Prefetch<S1> pre;
    prefetch_issue<S1>(pre, a.obs + FRAME * blockIdx.x, 0, tid);
    prefetch_commit<S1>(pre, lds + M::BUF0, 0, tid);
    stage_wait();
    lds_barrier();
    for (int img = blockIdx.x; img < a.B; img += gridDim.x) {
        const uint8_t* obs_img = a.obs + FRAME * img;
        __bf16* feat_row = a.feat + (size_t)img * a.ldf;
        run_section<S1, S2, M, false, 0, -1, N::NSETS, false>(lds, a.sec[0], a.sec[1], obs_img, pre, feat_row, tid);
        run_section<S2, S3, M, false, 1, 4, N::NSETS, S1::XFUSED>(lds, a.sec[1], a.sec[2], obs_img, pre, feat_row, tid);
        const int nimg = img + (int)gridDim.x < a.B ? img + (int)gridDim.x : img;
        run_section<S3, S4, M, false, 2, 9, N::NSETS, S2::XFUSED>(lds, a.sec[2], a.sec[3], obs_img, pre, feat_row, tid);
        prefetch_issue<S1>(pre, a.obs + FRAME * nimg, 0, tid);
        run_section<S4, S4, M, true, 3, 14, N::NSETS, S3::XFUSED>(lds, a.sec[3], a.sec[3], obs_img, pre, feat_row, tid);
    }
}

}  // namespace seedinf
