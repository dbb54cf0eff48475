// bf16 MFMA GEMMs for the dense layers at large batch: operands staged through LDS.
//
// Same contract as gemm_bf16.h (packed weight fragments in A, activation rows in B, the same epilogues), for
// batches large enough to fill the chip with big tiles: 8 wavefronts per workgroup, every wavefront a 64 x 64
// sub-tile (4 row tiles x 4 feature tiles, 16 MFMAs per 8 fragments).
//
// What the staging buys is the activation fetch.  Fragments travel global -> LDS with asynchronous loads, one
// instruction per kilobyte, and activation rows are fetched whole-segment-wise: four (bf16) or eight (fp32)
// consecutive lanes fetch the 64 or 128 contiguous bytes that one row contributes to a chunk (a lane-per-row
// fetch would cost the texture path four times as many cycles), rotated within the row so that the 16-byte
// reads that rebuild the MFMA operand (lane n + 16 g: row n, k = 8 g .. 8 g + 7) hit every LDS bank once.  fp32
// rows (the recurrent state) are converted to bf16 when read.
//
// Two kernels:
//   gemm_bf16_xw_kernel<FG, RG, KG, EPI, XF32> (KG = 1, 2): a workgroup owns RG*64 rows x FG*64 features; with
//     KG = 2 a wavefront takes every second K chunk of its sub-tile and the two partial sums meet in LDS at the
//     end.  Activations go through a four-slot LDS ring with one barrier per stage of two chunks; a wavefront's
//     weight fragments go straight into its registers.
//   gemm_bf16_k8_kernel<EPI> (long K, few output tiles: the linear layer after the torso): the eight wavefronts
//     share one 64 x 64 tile and each takes every eighth chunk.  Nothing is shared between them, so each runs
//     private rings in its own 20 KiB of LDS (three slots of activation fragments, two of weight fragments)
//     with no barrier inside the K loop.  The eight partial tiles meet in LDS and four wavefronts finish one
//     row tile each.  (Splitting K over workgroups instead costs more than it saves here: partial sums that
//     cross the chip's L2 slices need device-scope fences, each of which writes back and invalidates a whole
//     slice.)
#pragma once
#include "gemm_bf16.h"

namespace seedinf {

constexpr int GL_THREADS = 512;
// Rows from which the dense layers run these kernels with their 64 x 64 sub-tiles per wavefront; below, the
// direct kernels' smaller tiles fill the chip better (measured: the Atari agent's step at 1536 rows 132 -> 104 us
// with these kernels, the same at 1024 rows 85 -> 90 us).
constexpr int GL_MIN_ROWS = 1536;
constexpr int GL_K8_LDS_BYTES = 8 * 20480;              // private rings; the 128 KiB of partial tiles reuse them

template <int N>
__device__ __forceinline__ void wait_outstanding()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int EPI>
__global__ __launch_bounds__(GL_THREADS) void gemm_bf16_k8_kernel(GemmArgs p)
{
    static_assert(EPI == EPI_RELU, "the K-split tile has the plain epilogue only");
    extern __shared__ __attribute__((aligned(16))) char gl_lds[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)gl_lds;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, n = lane & 15;
    const int r0 = blockIdx.x * 64;
    const int wt = blockIdx.y;                           // the workgroup's tile group along features
    const int kct = p.kc1;

    floatx4 acc[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[r][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    // wavefront w owns chunks w, w + 8, ...; 20 KiB of LDS each: three slots of 4 activation fragments (those
    // come from HBM, the longer wait) and two slots of 4 weight fragments
    const int ni = (kct - wave + 7) / 8;
    const int cell_b = 4 * n + ((g + (n >> 2)) & 3);     // where this lane's operand piece sits in a fragment's LDS image
    const int piece = (lane - (lane >> 4)) & 3;          // lane L fetches row L / 4, 16-byte piece (L % 4 - L / 16) mod 4
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
    // (8 loads) are the only ones issued after its own, and loads complete in the order issued
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
    __syncthreads();                                     // LDS is free

    // eight partial tiles: everybody writes all 16 of its accumulators, wavefront r < 4 sums row tile r
    floatx4* ex = (floatx4*)gl_lds;                      // [wave][4][4][64]
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int j = 0; j < 4; ++j) ex[((wave * 4 + r) * 4 + j) * 64 + lane] = acc[r][j];
    __syncthreads();
    if (wave >= 4) return;
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

// ---- activations through a shared LDS ring, weights straight into registers ----
// A wavefront's weight fragments are its own (nobody else in the workgroup multiplies by them) and already sit in
// MFMA lane order in global memory, one contiguous kilobyte each: they are loaded directly into registers, PF
// stages ahead of their use.  Only the activation rows, which the feature groups share and which need the
// coalesced whole-segment fetch, go through LDS: a stage is 8-32 KiB instead of 48-64, four slots fit, and a
// wavefront issues one to four asynchronous loads per stage instead of five to eight (their issue blocks the
// wavefront: with the weights in the same ring the K loop ran at a third of the rate operands can be delivered).
template <int FG, int RG, int KG, bool XF32>
struct GemmXwCfg {
    static constexpr int SC = 2;                        // chunks per stage
    static constexpr int NXF = RG * 4 * SC;             // activation fragments per stage: (row tile, chunk)
    static constexpr int XFB = XF32 ? 2048 : 1024;      // LDS bytes per activation fragment
    static constexpr int SLOT = NXF * XFB;
    static constexpr int CB = NXF / 8;                  // asynchronous loads per wavefront, stage of bf16 rows
    static constexpr int CF = 2 * NXF / 8;              // stage of fp32 rows
    static constexpr int NSLOT = 4;
    static constexpr int NPW = SC / KG;                 // chunks per stage and wavefront
    static constexpr int PF = KG == 2 ? 2 : 1;          // stages between a weight fragment's load and its use
    static constexpr int EXCH = KG == 1 ? 0 : 8 * 8 * 1024;   // partial tiles handed over at the end
    static constexpr int LDS_BYTES = NSLOT * SLOT > EXCH ? NSLOT * SLOT : EXCH;
    static_assert(FG * RG * KG == 8 && (KG == 1 || KG == 2), "8 wavefronts, K over one or two of them");
    static_assert(NXF % 8 == 0 && PF < NSLOT - 1, "a stage's loads divide evenly over 8 wavefronts");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
};

template <int FG, int RG, int KG, int EPI, bool XF32>
__global__ __launch_bounds__(GL_THREADS) void gemm_bf16_xw_kernel(GemmArgs p)
{
    using C = GemmXwCfg<FG, RG, KG, XF32>;
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
    const bf16x8* wsrc[4];                               // the wavefront's four feature tiles, this lane's 16 bytes of chunk 0
#pragma unroll
    for (int j = 0; j < 4; ++j) wsrc[j] = p.wp + (size_t)min(wt * 4 + j, p.n_ftiles - 1) * kct * 64 + lane;

    // asynchronous loads of stage st's activation fragments into its slot; instruction q belongs to wavefront q % 8
    auto issue_x = [&](int st) {
        const int kc_a = C::SC * st;
        const bool f32 = XF32 && kc_a >= p.kc1;          // uniform (kc1 is even)
        const uint32_t sb = lds0 + (st % C::NSLOT) * C::SLOT;
#pragma unroll
        for (int jj = 0; jj < (XF32 ? C::CF : C::CB); ++jj) {
            if (jj >= (f32 ? C::CF : C::CB)) break;      // uniform
            const int q = wave + 8 * jj;
            const int fidx = f32 ? q >> 1 : q, half = f32 ? q & 1 : 0;
            const int rt = fidx / C::SC, c = fidx % C::SC;
            const int kc = min(kc_a + c, kct - 1);       // past the end: the last chunk again (never multiplied)
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
                col = col + 4 <= p.k2 ? col : 0;         // columns past the end: any valid address, zeroed when read
                src = p.x2 + (size_t)row * p.ld2 + col;
            }
            g2lds16(src, sb + fidx * C::XFB + half * 1024);
        }
    };
    auto load_w = [&](int st, bf16x8 (&w)[C::NPW][4]) {
#pragma unroll
        for (int cc = 0; cc < C::NPW; ++cc) {
            const int kc = min(C::SC * st + (KG == 1 ? cc : kg), kct - 1);
#pragma unroll
            for (int j = 0; j < 4; ++j) w[cc][j] = wsrc[j][(size_t)kc * 64];
        }
    };
    auto multiply = [&](int st, const bf16x8 (&w)[C::NPW][4]) {
        const int kc_a = C::SC * st;
        const bool f32 = XF32 && kc_a >= p.kc1;
        const char* sb = gl_lds + (st % C::NSLOT) * C::SLOT;
        // where this lane's operand pieces sit inside a fragment's LDS image (see issue_x())
        const int cell_b = 4 * n + ((g + (n >> 2)) & 3);
        const int cell_lo = (n >> 3) * 64 + 8 * (n & 7) + ((2 * g + (n >> 1)) & 7);
        const int cell_hi = (n >> 3) * 64 + 8 * (n & 7) + ((2 * g + 1 + (n >> 1)) & 7);
#pragma unroll
        for (int cc = 0; cc < C::NPW; ++cc) {
            const int c = KG == 1 ? cc : kg;
            const int kc = kc_a + c;
            if (kc >= kct) continue;                     // uniform
            bf16x8 b[4];
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
                for (int j = 0; j < 4; ++j) acc[r][j] = mfma16(w[cc][j], b[r], acc[r][j]);
        }
    };

    // Loads complete in the order issued.  In the steady state the loads a wavefront issues after stage st's
    // activation loads are the weight loads of AHEAD iterations and the activation loads of AHEAD - 1 (counted
    // as bf16 stages, the smaller kind: never too lax), so "at most that many outstanding" means stage st has
    // landed.  The first iteration collects everything the prologue issued (stages 0 .. AHEAD - 1), the last
    // ones, where fewer loads follow, drain everything; so do wavefronts without feature tiles, which load no weights.
    constexpr int AHEAD = C::NSLOT - 1, R = C::PF + 1;
    constexpr int LATER = AHEAD * C::NPW * 4 + (AHEAD - 1) * C::CB;
    bf16x8 wr[R][C::NPW][4];
#pragma unroll
    for (int i = 0; i < AHEAD; ++i)
        if (i < nst) issue_x(i);
#pragma unroll
    for (int i = 0; i < C::PF; ++i)
        if (active && i < nst) load_w(i, wr[i]);
    for (int st0 = 0; st0 < nst; st0 += R) {
#pragma unroll
        for (int u = 0; u < R; ++u) {
            const int st = st0 + u;
            if (st >= nst) break;                        // uniform
            if (st == 0 || !active || st + AHEAD - 1 >= nst) stage_wait();
            else if (st >= AHEAD) wait_outstanding<LATER>();
            __syncthreads();                             // everybody's loads of stage st have landed, and everybody has left stage st - 1
            if (st + AHEAD < nst) issue_x(st + AHEAD);
            if (active && st + C::PF < nst) load_w(st + C::PF, wr[(u + C::PF) % R]);
            if (active) multiply(st, wr[u]);
        }
    }
    __syncthreads();                                     // LDS is free

    if constexpr (KG == 1) {
        if (active) gemm_epilogue<4, EPI>(p, acc, -1, wt, r0 + rg * 64, lane);
    } else {
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
    }
}

template <int EPI>
inline hipError_t gemm_lds_set_attributes()
{
    hipError_t e = hipSuccess;
    auto set = [&](const void* f, int bytes) {
        if (e == hipSuccess) e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    };
    if constexpr (EPI == EPI_RELU) set((const void*)gemm_bf16_k8_kernel<EPI>, GL_K8_LDS_BYTES);
    set((const void*)gemm_bf16_xw_kernel<4, 1, 2, EPI, true>, GemmXwCfg<4, 1, 2, true>::LDS_BYTES);
    set((const void*)gemm_bf16_xw_kernel<4, 2, 1, EPI, true>, GemmXwCfg<4, 2, 1, true>::LDS_BYTES);
    return e;
}

}  // namespace seedinf
