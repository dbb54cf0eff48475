// bf16 MFMA GEMM for the dense layers at large batch: operands staged through LDS.
//
// Same contract as gemm_bf16.h (packed weight fragments in A, activation rows in B, the same epilogues), for
// batches large enough to fill the chip with big tiles.  A workgroup of 8 wavefronts owns RG*64 rows x FG*64
// features; every wavefront owns a 64 x 64 sub-tile (4 row tiles x 4 feature tiles, 16 MFMAs per 8 fragments)
// and, with KG = 2, every second K chunk of it (the two partial sums meet in LDS at the end).
//
// K is walked in stages of two chunks (64 values of k).  A stage's fragments travel global -> LDS with
// asynchronous loads, one instruction per kilobyte.  Weight fragments are contiguous in global memory and land
// in lane order.  Activation rows are fetched whole-segment-wise: four (bf16) or eight (fp32) consecutive lanes
// fetch the 64 or 128 contiguous bytes that one row contributes to a chunk (a lane-per-row fetch would cost the
// texture path four times as many cycles), rotated within the row so that the 16-byte reads that rebuild the
// MFMA operand (lane n + 16 g: row n, k = 8 g .. 8 g + 7) hit every LDS bank once.  fp32 rows (the recurrent
// state) are converted to bf16 when read.  NSLOT LDS slots: while stage i is multiplied, stages i + 1 ..
// i + NSLOT - 1 are in flight; one barrier per stage.
//
// KG = 8 (long K, few output tiles: the linear layer after the torso): the eight wavefronts share one 64 x 64
// tile and each takes every eighth chunk.  Nothing is shared between them, so each runs private rings in its
// own 20 KiB of LDS (three slots of activation fragments, two of weight fragments) with no barrier inside the
// K loop; the staging buys the coalesced row fetch and loads that need no registers.  The eight partial tiles meet in LDS and four wavefronts finish one row
// tile each.  (Splitting K over workgroups instead costs more than it saves here: partial sums that cross the
// chip's L2 slices need device-scope fences, each of which writes back and invalidates a whole slice.)
#pragma once
#include "gemm_bf16.h"

namespace seedinf {

constexpr int GL_THREADS = 512;
// Rows from which the dense layers run these kernels with their 64 x 64 sub-tiles per wavefront; below, the
// direct kernels' smaller tiles fill the chip better.
constexpr int GL_MIN_ROWS = 2048;

template <int FG, int RG, int KG, bool XF32>
struct GemmLdsCfg {
    static constexpr int SC = KG > 2 ? KG : 2;          // chunks per stage
    static constexpr int NXF = RG * 4 * SC;             // activation fragments per stage: (row tile, chunk)
    static constexpr int NWF = FG * 4 * SC;             // weight fragments per stage: (feature tile, chunk)
    static constexpr int XFB = XF32 ? 2048 : 1024;      // LDS bytes per activation fragment
    static constexpr int W_OFF = NXF * XFB;
    static constexpr int SLOT = W_OFF + NWF * 1024;
    static constexpr int CB = (NXF + NWF) / 8;          // loads per wavefront, stage of bf16 rows
    static constexpr int CF = (2 * NXF + NWF) / 8;      // stage of fp32 rows
    static constexpr int EXCH = KG == 1 ? 0 : (KG == 2 ? 8 * 8 : 8 * 16) * 1024;   // partial tiles handed over at the end
    static constexpr int NSLOT = KG == 8 ? 2 : (4 * SLOT <= 128 * 1024 ? 4 : (3 * SLOT <= 144 * 1024 ? 3 : 2));
    static constexpr int LDS_BYTES = KG == 8 ? 8 * 20480 : (NSLOT * SLOT > EXCH ? NSLOT * SLOT : EXCH);
    static_assert(FG * RG * KG == 8, "8 wavefronts");
    static_assert((NXF + NWF) % 8 == 0 && (2 * NXF + NWF) % 8 == 0, "a stage's loads divide evenly over 8 wavefronts");
    static_assert(!XF32 || SC == 2, "fp32 rows: stages of two chunks (a stage never straddles the two segments)");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
};

template <int N>
__device__ __forceinline__ void wait_outstanding()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int FG, int RG, int KG, int EPI, bool XF32>
__global__ __launch_bounds__(GL_THREADS) void gemm_bf16_lds_kernel(GemmArgs p)
{
    using C = GemmLdsCfg<FG, RG, KG, XF32>;
    static_assert(KG == 1 || KG == 2 || (KG == 8 && EPI == EPI_RELU), "K groups");
    extern __shared__ __attribute__((aligned(16))) char gl_lds[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)gl_lds;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, n = lane & 15;
    const int kg = wave % KG, rg = (wave / KG) % RG, fg = wave / (KG * RG);
    const int r0 = blockIdx.x * (RG * 64);
    const int wt = blockIdx.y * FG + fg;                 // the wavefront's tile group along features
    const bool active = wt * 4 < p.n_ftiles;             // uniform
    const int kct = p.kc1 + ((p.k2 + 31) >> 5);
    const int nst = (kct + C::SC - 1) / C::SC;

    floatx4 acc[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[r][j] = floatx4{0.f, 0.f, 0.f, 0.f};
    bool fresh[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = min(r0 + rg * 64 + r * 16 + n, p.rows - 1);
        fresh[r] = EPI == EPI_LSTM && p.done && p.done[row];
    }

    // asynchronous loads of stage st into its slot; instruction q of the stage belongs to wavefront q % 8
    auto issue = [&](int st) {
        const int kc_a = C::SC * st;
        const bool f32 = XF32 && kc_a >= p.kc1;          // uniform (kc1 is even)
        const uint32_t sb = lds0 + (st % C::NSLOT) * C::SLOT;
        const int nxi = f32 ? 2 * C::NXF : C::NXF;
#pragma unroll
        for (int jj = 0; jj < (XF32 ? C::CF : C::CB); ++jj) {
            if (jj >= (f32 ? C::CF : C::CB)) break;      // uniform
            const int q = wave + 8 * jj;
            if (q < nxi) {
                const int fidx = f32 ? q >> 1 : q, half = f32 ? q & 1 : 0;
                const int rt = fidx / C::SC, c = fidx % C::SC;
                const int kc = min(kc_a + c, kct - 1);   // past the end: the last chunk again (never multiplied)
                const void* src;
                if (!f32) {
                    // lane L: row L / 4 of the tile, 16-byte piece (L % 4 - L / 16) mod 4 of the row's 64 bytes
                    const int row = min(r0 + rt * 16 + (lane >> 2), p.rows - 1);
                    const int piece = (lane - (lane >> 4)) & 3;
                    src = p.x1 + (size_t)row * p.ld1 + kc * 32 + piece * 8;
                } else {
                    // instruction `half`: rows 8 half .. 8 half + 7; lane L: row L / 8 of those, piece
                    // (L % 8 - row / 2) mod 8 of the row's 128 bytes
                    const int nr = half * 8 + (lane >> 3);
                    const int row = min(r0 + rt * 16 + nr, p.rows - 1);
                    const int piece = (lane - (nr >> 1)) & 7;
                    int col = (kc - p.kc1) * 32 + piece * 4;
                    col = col + 4 <= p.k2 ? col : 0;     // columns past the end: any valid address, zeroed when read
                    src = p.x2 + (size_t)row * p.ld2 + col;
                }
                g2lds16(src, sb + fidx * C::XFB + half * 1024);
            } else {
                const int e = q - nxi;
                const int c = e % C::SC;
                const int kc = min(kc_a + c, kct - 1);
                const int ft = min((int)(blockIdx.y * FG * 4) + e / C::SC, p.n_ftiles - 1);
                g2lds16(p.wp + ((size_t)ft * kct + kc) * 64 + lane, sb + C::W_OFF + e * 1024);
            }
        }
    };
    auto multiply = [&](int st) {
        const int kc_a = C::SC * st;
        const bool f32 = XF32 && kc_a >= p.kc1;
        const char* sb = gl_lds + (st % C::NSLOT) * C::SLOT;
        // where this lane's operand pieces sit inside a fragment's LDS image (see issue())
        const int cell_b = 4 * n + ((g + (n >> 2)) & 3);
        const int cell_lo = (n >> 3) * 64 + 8 * (n & 7) + ((2 * g + (n >> 1)) & 7);
        const int cell_hi = (n >> 3) * 64 + 8 * (n & 7) + ((2 * g + 1 + (n >> 1)) & 7);
#pragma unroll
        for (int cc = 0; cc < C::SC / KG; ++cc) {
            const int c = KG == 1 ? cc : kg;
            const int kc = kc_a + c;
            if (kc >= kct) continue;                     // uniform
            bf16x8 a[4], b[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) a[j] = *(const bf16x8*)(sb + C::W_OFF + (((fg * 4 + j) * C::SC + c) * 64 + lane) * 16);
            if (!f32) {
#pragma unroll
                for (int r = 0; r < 4; ++r) b[r] = *(const bf16x8*)(sb + ((rg * 4 + r) * C::SC + c) * C::XFB + cell_b * 16);
            } else {
                const bool colok = (kc - p.kc1) * 32 + g * 8 + 8 <= p.k2;
                const floatx4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const char* f = sb + ((rg * 4 + r) * C::SC + c) * C::XFB;
                    const floatx4 lo = *(const floatx4*)(f + cell_lo * 16), hi = *(const floatx4*)(f + cell_hi * 16);
                    const bool ok = colok && !fresh[r];
                    b[r] = to_bf16x8(ok ? lo : z, ok ? hi : z);
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[r][j] = mfma16(a[j], b[r], acc[r][j]);
        }
    };

    if constexpr (KG == 8) {
        // private rings: wavefront w owns chunks w, w + 8, ...; 20 KiB of LDS each: three slots of 4 activation
        // fragments (those come from HBM, the longer wait) and two slots of 4 weight fragments
        const int ni = (kct - wave + 7) / 8;
        const int cell_b = 4 * n + ((g + (n >> 2)) & 3);
        const int piece = (lane - (lane >> 4)) & 3;
        auto issue_x = [&](int i) {
            const int kc = wave + 8 * i;
            const uint32_t sb = lds0 + wave * 20480 + (i % 3) * 4096;
#pragma unroll
            for (int rt = 0; rt < 4; ++rt) {
                const int row = min(r0 + rt * 16 + (lane >> 2), p.rows - 1);
                g2lds16(p.x1 + (size_t)row * p.ld1 + kc * 32 + piece * 8, sb + rt * 1024);
            }
        };
        auto issue_w = [&](int i) {
            const int kc = wave + 8 * i;
            const uint32_t sb = lds0 + wave * 20480 + 12288 + (i & 1) * 4096;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int ft = min(wt * 4 + j, p.n_ftiles - 1);
                g2lds16(p.wp + ((size_t)ft * kct + kc) * 64 + lane, sb + j * 1024);
            }
        };
        // issue order: x(0) x(1) w(0) | x(2) w(1) | x(3) w(2) | ...: when chunk i is due, x(i + 2) and w(i + 1)
        // (8 loads) are the only ones issued after its own
        if (ni > 0) issue_x(0);
        if (ni > 1) issue_x(1);
        if (ni > 0) issue_w(0);
        for (int i = 0; i < ni; ++i) {
            // (the slots written now were last read for chunk i - 1, whose MFMAs have been issued)
            if (i + 2 < ni) issue_x(i + 2);
            if (i + 1 < ni) issue_w(i + 1);
            if (i + 2 < ni) wait_outstanding<8>();
            else if (i + 1 < ni) wait_outstanding<4>();
            else stage_wait();
            const char* xb = gl_lds + wave * 20480 + (i % 3) * 4096;
            const char* wb = gl_lds + wave * 20480 + 12288 + (i & 1) * 4096;
            bf16x8 a[4], b[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) a[j] = *(const bf16x8*)(wb + (j * 64 + lane) * 16);
#pragma unroll
            for (int r = 0; r < 4; ++r) b[r] = *(const bf16x8*)(xb + (r * 64 + cell_b) * 16);
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[r][j] = mfma16(a[j], b[r], acc[r][j]);
        }
    } else {
    // Loads complete in the order issued, so "at most N outstanding" with N = the loads of the NSLOT - 2 stages
    // issued after stage st means stage st has landed (N counts bf16 stages, the smaller kind: never too lax).
    // Near the end fewer stages are behind st and the wait drains everything.
    constexpr int AHEAD = C::NSLOT - 1;
#pragma unroll
    for (int i = 0; i < AHEAD; ++i)
        if (i < nst) issue(i);
    for (int st = 0; st < nst; ++st) {
        if (st + AHEAD - 1 < nst) wait_outstanding<(AHEAD - 1) * C::CB>();
        else stage_wait();
        __syncthreads();                                 // everybody's loads of stage st have landed, and everybody has left stage st - 1
        if (st + AHEAD < nst) issue(st + AHEAD);
        if (active) multiply(st);
    }
    }
    __syncthreads();                                     // LDS is free

    if constexpr (KG == 1) {
        if (active) gemm_epilogue<4, EPI>(p, acc, -1, wt, r0 + rg * 64, lane);
    } else if constexpr (KG == 2) {
        // the partners (wave ^ 1) swap halves: K group 0 finishes row tiles 0, 1, K group 1 row tiles 2, 3
        floatx4* ex = (floatx4*)gl_lds;                  // [wave][2][4][64]
        floatx4 fin[2][4];
        auto swap_halves = [&](auto keep0) {
            constexpr int K0 = decltype(keep0)::value, S0 = 2 - K0;
#pragma unroll
            for (int rr = 0; rr < 2; ++rr)
#pragma unroll
                for (int j = 0; j < 4; ++j) ex[((wave * 2 + rr) * 4 + j) * 64 + lane] = acc[S0 + rr][j];
            __syncthreads();
#pragma unroll
            for (int rr = 0; rr < 2; ++rr)
#pragma unroll
                for (int j = 0; j < 4; ++j) fin[rr][j] = acc[K0 + rr][j] + ex[(((wave ^ 1) * 2 + rr) * 4 + j) * 64 + lane];
        };
        if (kg == 0) swap_halves(std::integral_constant<int, 0>{});
        else swap_halves(std::integral_constant<int, 2>{});
        if (active) gemm_epilogue<2, EPI>(p, fin, -1, wt, r0 + rg * 64 + kg * 32, lane);
    } else {
        // eight partial tiles: everybody writes all 16 of its accumulators, wavefront r < 4 sums row tile r
        floatx4* ex = (floatx4*)gl_lds;                  // [wave][4][4][64]
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int j = 0; j < 4; ++j) ex[((wave * 4 + r) * 4 + j) * 64 + lane] = acc[r][j];
        __syncthreads();
        if (wave >= 4 || !active) return;
        floatx4 fin[1][4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            floatx4 t = ex[((0 * 4 + wave) * 4 + j) * 64 + lane];
#pragma unroll
            for (int w2 = 1; w2 < 8; ++w2) t += ex[((w2 * 4 + wave) * 4 + j) * 64 + lane];
            fin[0][j] = t;
        }
        gemm_epilogue<1, EPI>(p, fin, -1, wt, r0 + wave * 16, lane);
    }
}

template <int EPI>
inline hipError_t gemm_lds_set_attributes()
{
    hipError_t e = hipSuccess;
    auto set = [&](const void* f, int bytes) {
        if (e == hipSuccess) e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    };
    if constexpr (EPI == EPI_RELU) set((const void*)gemm_bf16_lds_kernel<1, 1, 8, EPI, false>, GemmLdsCfg<1, 1, 8, false>::LDS_BYTES);
    set((const void*)gemm_bf16_lds_kernel<4, 1, 2, EPI, true>, GemmLdsCfg<4, 1, 2, true>::LDS_BYTES);
    set((const void*)gemm_bf16_lds_kernel<4, 2, 1, EPI, true>, GemmLdsCfg<4, 2, 1, true>::LDS_BYTES);
    return e;
}

}  // namespace seedinf
