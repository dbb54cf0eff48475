// bf16 MFMA GEMM for the dense layers: Y[row, f] = sum_k X[row, k] * W[k, f].
//
// Weights are pre-packed on the host into A-operand fragments:
//   Wp[ftile][kchunk][lane][8], lane -> feature ftile*16 + lane%16,
//   k = kchunk*32 + 8*(lane/16) + e; padded with zeros to whole tiles/chunks.
// Activations are read straight from their row-major bf16 (or fp32, converted
// on load) buffer as B-operand fragments: 16 bytes per lane.
// Two kernels, chosen by the length of K:
//   gemm_bf16_kernel (short K, the recurrent core): a wavefront owns 4 feature
//     tiles x RT row tiles and walks all of K; the block's 4 wavefronts differ
//     in their feature tiles.
//   gemm_bf16_splitk_kernel (long K, the linear layer after the torso): the
//     block's 4 wavefronts share ONE output tile of RT*16 rows x 64 features
//     and split K between them.  That layer has few outputs and a long K, so
//     splitting rows or features further would have every compute unit re-read
//     the whole weight matrix.  4 or 8 wavefronts per block: each walks its
//     share of K with three stages of loads in flight, the partial sums meet
//     in LDS, and wavefront r finishes row tile r.
//
// Epilogues:
//   EPI_RELU : y = max(acc + bias, 0) stored as bf16 and/or fp32
//   EPI_LSTM : the 4 feature tiles of a group are the i, f, g, o gates of the
//              same 16 units; adds bias, the gathered previous-action row and
//              reward * reward-row (all fp32), then the LSTM cell update
//              (Appendix A.3.1: the core also sees the one-hot previous action
//              and the previous reward).
#pragma once
#include "bf16_common.h"

namespace seedinf {

enum { EPI_RELU = 0, EPI_LSTM = 1 };

struct GemmArgs {
    const __bf16* x1; int ld1; int kc1;      // first K segment: kc1 chunks of 32 from bf16 rows
    const float* x2; int ld2; int k2;        // second K segment (fp32 rows, converted on load), k2 valid columns; kc2 = ceil(k2/32)
    const bf16x8* wp;                        // packed weights, kc1 + kc2 chunks per feature tile
    int n_ftiles;                            // feature tiles that exist in wp
    int rows;                                // batch rows
    // EPI_RELU
    const float* bias_pad;                   // [n_ftiles*16]
    __bf16* y_bf16; int ldy_bf16;            // optional
    float* y_f32; int ldy_f32; int n_out;    // optional; only f < n_out stored
    // EPI_LSTM
    const float* lstm_w;                     // flat fp32 [F+A+1+Hn][4Hn]
    const float* lstm_b;                     // [4Hn]
    const int32_t* prev_action; const float* prev_reward;
    const float* c_in; float* h_out; float* c_out;
    int F, A, Hn;
    const uint8_t* done;                     // [rows] or nullptr: non-zero = the row's cell starts from the zero state
};

// Gate non-linearities from the hardware exponential and reciprocal (about 1 ulp each): a handful of
// instructions instead of the library routines' dozens, and both saturate correctly (exp -> inf gives
// reciprocal 0).  tanh v = 1 - 2 / (1 + e^(2v)): absolute error ~1e-7 near 0, far inside this mode's tolerance.
__device__ __forceinline__ float sigmoidf_(float v) { return __builtin_amdgcn_rcpf(1.0f + __expf(-v)); }
__device__ __forceinline__ float tanhf_(float v) { return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __expf(2.0f * v)); }

// Epilogue of one block tile: row tiles r with (only_r < 0 || r == only_r); wt = the tile group along features.
template <int RT, int EPI>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& p, floatx4 (&acc)[RT][4], int only_r, int wt, int r0, int lane)
{
    const int g = lane >> 4, n = lane & 15;
    const int ft0 = wt * 4;
    if constexpr (EPI == EPI_RELU) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (ft0 + j >= p.n_ftiles) break;
            const int f = (ft0 + j) * 16 + g * 4;
            const floatx4 bv = *(const floatx4*)(p.bias_pad + f);
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                const int row = r0 + r * 16 + n;
                if ((only_r >= 0 && r != only_r) || row >= p.rows) continue;
                floatx4 v = relu4(acc[r][j] + bv);
                if (p.y_bf16) *(bf16x4*)(p.y_bf16 + (size_t)row * p.ldy_bf16 + f) = to_bf16x4(v);
                if (p.y_f32) {
                    float* d = p.y_f32 + (size_t)row * p.ldy_f32 + f;
                    if (f + 4 <= p.n_out) *(floatx4*)d = v;
                    else
                        for (int i = 0; i < 4; ++i)
                            if (f + i < p.n_out) d[i] = v[i];
                }
            }
        }
    } else {
        // tile group wt = unit tile; feature tile j = gate j of units wt*16 .. wt*16+15
        // Two rounds of loads for all row tiles together, then the arithmetic and the stores: written row tile by
        // row tile, each tile's loads stay behind the previous tile's stores (they may alias as far as the
        // compiler knows) and the epilogue is a chain of two trips to memory per tile.
        const int Hn = p.Hn, G4 = 4 * p.Hn;
        const int u = wt * 16 + g * 4;                  // this lane's 4 consecutive units
        floatx4 bg[4], wr[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            bg[j] = *(const floatx4*)(p.lstm_b + j * Hn + u);
            wr[j] = *(const floatx4*)(p.lstm_w + (size_t)(p.F + p.A) * G4 + j * Hn + u);
        }
        int act[RT];
        float rew[RT];
        bool fresh[RT];
        floatx4 c0[RT];
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            const int row = min(r0 + r * 16 + n, p.rows - 1);
            act[r] = p.prev_action[row];
            rew[r] = p.prev_reward[row];
            fresh[r] = p.done && p.done[row];
            c0[r] = *(const floatx4*)(p.c_in + (size_t)row * Hn + u);
        }
        // second round: the previous actions' weight rows (from a clamped index: whether a row counts is decided below)
        floatx4 wa[RT][4];
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            const int aa = min(max(act[r], 0), p.A - 1);
#pragma unroll
            for (int j = 0; j < 4; ++j) wa[r][j] = *(const floatx4*)(p.lstm_w + (size_t)(p.F + aa) * G4 + j * Hn + u);
        }
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            const int row = r0 + r * 16 + n;
            if ((only_r >= 0 && r != only_r) || row >= p.rows) continue;
            const int a = act[r];
            floatx4 pre[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                pre[j] = acc[r][j] + bg[j] + rew[r] * wr[j];
                if (a >= 0 && a < p.A) pre[j] += wa[r][j];
            }
            floatx4 cp = c0[r];
            if (fresh[r]) cp = floatx4{0.f, 0.f, 0.f, 0.f};
            floatx4 cn, hn;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                cn[i] = sigmoidf_(pre[1][i]) * cp[i] + sigmoidf_(pre[0][i]) * tanhf_(pre[2][i]);
                hn[i] = sigmoidf_(pre[3][i]) * tanhf_(cn[i]);
            }
            *(floatx4*)(p.c_out + (size_t)row * Hn + u) = cn;
            *(floatx4*)(p.h_out + (size_t)row * Hn + u) = hn;
        }
    }
}

// The LSTM epilogue's operands for one row tile, requested before the K loop so that their trips to memory run
// beside the loop's own (taken one after another - flags, then weights, then the action row, then the cell -
// the kernel is a chain of four memory latencies around a microsecond of arithmetic).
struct LstmOperands {
    floatx4 bg[4], wr[4], wa[4], c0;
    int a;
    float rew;
    bool fresh;
};

// first round: everything whose address is known at once (`row` already clamped into the batch)
__device__ __forceinline__ void lstm_prefetch(const GemmArgs& p, LstmOperands& o, int wt, int row, int g)
{
    const int Hn = p.Hn, G4 = 4 * p.Hn;
    const int u = wt * 16 + g * 4;
    o.a = p.prev_action[row];
    o.rew = p.prev_reward[row];
    o.fresh = p.done && p.done[row];
    o.c0 = *(const floatx4*)(p.c_in + (size_t)row * Hn + u);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        o.bg[j] = *(const floatx4*)(p.lstm_b + j * Hn + u);
        o.wr[j] = *(const floatx4*)(p.lstm_w + (size_t)(p.F + p.A) * G4 + j * Hn + u);
    }
}

// second round: the previous action's weight row (from a clamped index: an action outside the range adds nothing,
// which the epilogue decides, not this load)
__device__ __forceinline__ void lstm_prefetch_action(const GemmArgs& p, LstmOperands& o, int wt, int g)
{
    const int Hn = p.Hn, G4 = 4 * p.Hn;
    const int u = wt * 16 + g * 4;
    const int aa = min(max(o.a, 0), p.A - 1);
#pragma unroll
    for (int j = 0; j < 4; ++j) o.wa[j] = *(const floatx4*)(p.lstm_w + (size_t)(p.F + aa) * G4 + j * Hn + u);
}

// gates and cell of one row from prefetched operands: the arithmetic of gemm_epilogue's LSTM branch, term by term
__device__ __forceinline__ void lstm_epilogue_row(const GemmArgs& p, const floatx4 (&acc)[4], const LstmOperands& o, int wt, int row, int g)
{
    const int Hn = p.Hn;
    const int u = wt * 16 + g * 4;
    floatx4 pre[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        pre[j] = acc[j] + o.bg[j] + o.rew * o.wr[j];
        if (o.a >= 0 && o.a < p.A) pre[j] += o.wa[j];
    }
    floatx4 c0 = o.c0;
    if (o.fresh) c0 = floatx4{0.f, 0.f, 0.f, 0.f};
    floatx4 cn, hn;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        cn[i] = sigmoidf_(pre[1][i]) * c0[i] + sigmoidf_(pre[0][i]) * tanhf_(pre[2][i]);
        hn[i] = sigmoidf_(pre[3][i]) * tanhf_(cn[i]);
    }
    *(floatx4*)(p.c_out + (size_t)row * Hn + u) = cn;
    *(floatx4*)(p.h_out + (size_t)row * Hn + u) = hn;
}

// K loop over the chunks [kb, ke) of one source segment, branch-free inside: NST rotating fragment sets keep
// NST-1 stages of loads in flight while one is multiplied (these loops are bound by load latency and L1
// capacity, so bytes in flight and whole cache lines are what counts).  A stage is CPS consecutive chunks: with
// bf16 rows a chunk is 64 bytes of a row, so CPS = 2 (and an even kb) makes every activation load pair use a
// whole 128-byte line while it is in L1.  F32: the activations of this segment are fp32 rows (converted when
// multiplied; one chunk is a whole line), chunk numbering inside the segment starts at `seg0`, and only columns
// < kvalid exist.
template <int RT, int NST, int CPS, bool F32, int FT = 4>
__device__ __forceinline__ void gemm_k_loop(floatx4 (&acc)[RT][FT], const bf16x8* const (&wl)[FT], const void* xbase, int ld,
                                            const int (&rowi)[RT], int kb, int ke, int seg0, int kvalid, int g,
                                            const bool (&zero_row)[RT])
{
    if (kb >= ke) return;
    struct Stage {
        bf16x8 a[CPS][FT];
        bf16x8 b[CPS][F32 ? 1 : RT];
        floatx4 f[CPS][F32 ? RT : 1][2];
    };
    Stage st[NST];
    auto load = [&](Stage& s, int k0) {                // chunks k0 .. k0+CPS-1; past the end: the last chunk again
#pragma unroll
        for (int c = 0; c < CPS; ++c) {
            const int kc = k0 + c < ke ? k0 + c : ke - 1;
#pragma unroll
            for (int j = 0; j < FT; ++j) s.a[c][j] = wl[j][(size_t)kc * 64];
            if constexpr (!F32) {
                const __bf16* x = (const __bf16*)xbase;
#pragma unroll
                for (int r = 0; r < RT; ++r)
                    s.b[c][r] = *(const bf16x8*)(x + (size_t)rowi[r] * ld + (kc - seg0) * 32 + g * 8);
            } else {
                const float* x = (const float*)xbase;
                int k = (kc - seg0) * 32 + g * 8;
                k = k + 8 <= kvalid ? k : 0;           // columns past the end: any valid address, zeroed when used
#pragma unroll
                for (int r = 0; r < RT; ++r) {
                    const float* q = x + (size_t)rowi[r] * ld + k;
                    s.f[c][r][0] = *(const floatx4*)q;
                    s.f[c][r][1] = *(const floatx4*)(q + 4);
                }
            }
        }
    };
    auto mma1 = [&](const Stage& s, int c, int kc) {
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            bf16x8 b;
            if constexpr (!F32) {
                b = s.b[c][r];
            } else {
                const bool ok = (kc - seg0) * 32 + g * 8 + 8 <= kvalid && !zero_row[r];
                const floatx4 z = {0.f, 0.f, 0.f, 0.f};
                b = to_bf16x8(ok ? s.f[c][r][0] : z, ok ? s.f[c][r][1] : z);
            }
#pragma unroll
            for (int j = 0; j < FT; ++j) acc[r][j] = mfma16(s.a[c][j], b, acc[r][j]);
        }
    };
#pragma unroll
    for (int i = 0; i < NST - 1; ++i) load(st[i], kb + i * CPS);
    int kc = kb;
    for (; kc + NST * CPS <= ke; kc += NST * CPS) {
#pragma unroll
        for (int i = 0; i < NST; ++i) {
            load(st[(i + NST - 1) % NST], kc + (i + NST - 1) * CPS);
#pragma unroll
            for (int c = 0; c < CPS; ++c) mma1(st[i], c, kc + i * CPS + c);
        }
    }
    // fewer than NST * CPS chunks are left; the first NST - 1 stages of them are already loaded, and a last
    // partial stage (CPS > 1: e.g. five chunks left of six) is loaded now
    if (CPS > 1 && kc + (NST - 1) * CPS < ke) load(st[NST - 1], kc + (NST - 1) * CPS);   // uniform
#pragma unroll
    for (int i = 0; i < (CPS > 1 ? NST : NST - 1); ++i)
#pragma unroll
        for (int c = 0; c < CPS; ++c)
            if (kc + i * CPS + c < ke) mma1(st[i], c, kc + i * CPS + c);
}

// ---- short K: the block's 4 wavefronts take different feature-tile groups, each walks all of K ----
template <int RT, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmArgs p)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, n = lane & 15;
    const int wt = blockIdx.y * 4 + wave;              // wavefront's tile group along features
    const int ft0 = wt * 4;
    if (ft0 >= p.n_ftiles) return;                     // uniform per wavefront
    const int r0 = blockIdx.x * (RT * 16);
    const int kc2 = (p.k2 + 31) >> 5;
    const int kct = p.kc1 + kc2;

    floatx4 acc[RT][4];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[r][j] = floatx4{0.f, 0.f, 0.f, 0.f};
    int rowi[RT];
#pragma unroll
    for (int r = 0; r < RT; ++r) rowi[r] = min(r0 + r * 16 + n, p.rows - 1);
    const bf16x8* wl[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) wl[j] = p.wp + ((size_t)min(ft0 + j, p.n_ftiles - 1) * kct) * 64 + lane;

    // rows that start a new episode contribute no recurrent input (the fp32 segment is the previous h)
    bool fresh[RT];
#pragma unroll
    for (int r = 0; r < RT; ++r) fresh[r] = EPI == EPI_LSTM && p.done && p.done[rowi[r]];
    gemm_k_loop<RT, 3, 2, false>(acc, wl, p.x1, p.ld1, rowi, 0, p.kc1, 0, 0, g, fresh);
    gemm_k_loop<RT, 3, 1, true>(acc, wl, p.x2, p.ld2, rowi, p.kc1, kct, p.kc1, p.k2, g, fresh);
    gemm_epilogue<RT, EPI>(p, acc, -1, wt, r0, lane);
}

// ---- long K: the block's 4 wavefronts share one output tile and split K ----
// FT = feature tiles of the output tile: 4 (a whole group, every epilogue), or 2 or 1 (EPI_RELU only: small
// batches, where 16 x 32 or 16 x 16 tiles put two or four times as many compute units to work on the weight matrix).
template <int RT, int EPI, int NW, int FT = 4>
__global__ __launch_bounds__(NW * 64) void gemm_bf16_splitk_kernel(GemmArgs p)
{
    static_assert(NW == 4 || NW == 8, "4 or 8 wavefronts share the output tile");
    static_assert(FT == 4 || ((FT == 1 || FT == 2) && EPI == EPI_RELU), "whole gate groups for the LSTM epilogue");
    extern __shared__ __attribute__((aligned(16))) char gemm_lds[];     // partial sums [wave][row tile][feature tile][lane]
    floatx4* part = (floatx4*)gemm_lds;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, n = lane & 15;
    const int wt = blockIdx.y;                         // the block's tile group (FT = 4) or tile (FT = 1) along features
    const int ft0 = wt * FT;
    const int r0 = blockIdx.x * (RT * 16);
    const int kc2 = (p.k2 + 31) >> 5;
    const int kct = p.kc1 + kc2;
    // this wavefront's K chunks: an NW-th of K cut at even chunks (whole 128-byte lines of the bf16 rows)
    const int kpairs = (kct + 1) / 2;
    const int k0 = 2 * (wave * kpairs / NW), k1 = min(2 * ((wave + 1) * kpairs / NW), kct);

    floatx4 acc[RT][FT];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int j = 0; j < FT; ++j) acc[r][j] = floatx4{0.f, 0.f, 0.f, 0.f};
    int rowi[RT];
#pragma unroll
    for (int r = 0; r < RT; ++r) rowi[r] = min(r0 + r * 16 + n, p.rows - 1);
    const bf16x8* wl[FT];
#pragma unroll
    for (int j = 0; j < FT; ++j) wl[j] = p.wp + ((size_t)min(ft0 + j, p.n_ftiles - 1) * kct) * 64 + lane;

    // the wavefront that will finish row tile `wave` requests that tile's epilogue operands now
    // (tiles of up to two row tiles: with four the kernel has no registers to spare and the operands are fetched
    // by the epilogue itself)
    constexpr bool LSTM_AHEAD = EPI == EPI_LSTM && RT <= 2;
    LstmOperands lo;
    const bool finisher = LSTM_AHEAD && wave < RT;                           // uniform
    const int lrow = min(r0 + wave * 16 + n, p.rows - 1);
    if constexpr (LSTM_AHEAD)
        if (finisher) lstm_prefetch(p, lo, wt, lrow, g);
    bool fresh[RT];
#pragma unroll
    for (int r = 0; r < RT; ++r) fresh[r] = EPI == EPI_LSTM && p.done && p.done[rowi[r]];
    gemm_k_loop<RT, 3, 2, false, FT>(acc, wl, p.x1, p.ld1, rowi, k0, min(k1, p.kc1), 0, 0, g, fresh);
    gemm_k_loop<RT, 3, 1, true, FT>(acc, wl, p.x2, p.ld2, rowi, max(k0, p.kc1), k1, p.kc1, p.k2, g, fresh);
    if constexpr (LSTM_AHEAD)
        if (finisher) lstm_prefetch_action(p, lo, wt, g);                 // in flight across the reduction below

    // K reduction through LDS.  With 8 wavefronts the upper four first hand everything to the lower four.
    if constexpr (NW == 8) {
        if (wave >= 4) {
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int j = 0; j < FT; ++j) part[(((wave - 4) * RT + r) * 4 + j) * 64 + lane] = acc[r][j];
        }
        __syncthreads();
        if (wave >= 4) return;
#pragma unroll
        for (int r = 0; r < RT; ++r)
#pragma unroll
            for (int j = 0; j < FT; ++j) acc[r][j] += part[((wave * RT + r) * 4 + j) * 64 + lane];
        // (wavefront w has read only region w of the buffer, the region it writes next; the barrier below
        // counts the four wavefronts that are still alive)
    }
    // Wavefront r keeps row tile r, the others hand theirs over
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        if (r == wave) continue;                       // uniform
#pragma unroll
        for (int j = 0; j < FT; ++j) part[((wave * RT + r) * 4 + j) * 64 + lane] = acc[r][j];
    }
    __syncthreads();
    if (wave >= RT) return;
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        if (r != wave) continue;                       // uniform
#pragma unroll
        for (int w2 = 0; w2 < 4; ++w2) {
            if (w2 == r) continue;
#pragma unroll
            for (int j = 0; j < FT; ++j) acc[r][j] += part[((w2 * RT + r) * 4 + j) * 64 + lane];
        }
    }
    if constexpr (LSTM_AHEAD) {
#pragma unroll
        for (int r = 0; r < RT; ++r)
            if (r == wave && r0 + r * 16 + n < p.rows) lstm_epilogue_row(p, acc[r], lo, wt, r0 + r * 16 + n, g);
    } else if constexpr (FT == 4) {
        gemm_epilogue<RT, EPI>(p, acc, wave, wt, r0, lane);
    } else {
        // one or two feature tiles: bias, ReLU, store (row tile `wave` of this wavefront)
#pragma unroll
        for (int j = 0; j < FT; ++j) {
            if (ft0 + j >= p.n_ftiles) break;              // uniform
            const int f = (ft0 + j) * 16 + g * 4;
            const floatx4 bv = *(const floatx4*)(p.bias_pad + f);
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                const int row = r0 + r * 16 + n;
                if (r != wave || row >= p.rows) continue;
                const floatx4 v = relu4(acc[r][j] + bv);
                if (p.y_bf16) *(bf16x4*)(p.y_bf16 + (size_t)row * p.ldy_bf16 + f) = to_bf16x4(v);
                if (p.y_f32) {
                    float* d = p.y_f32 + (size_t)row * p.ldy_f32 + f;
                    if (f + 4 <= p.n_out) *(floatx4*)d = v;
                    else
                        for (int i = 0; i < 4; ++i)
                            if (f + i < p.n_out) d[i] = v[i];
                }
            }
        }
    }
}

// bf16 rows -> fp32 rows (diagnostic tap)
__global__ __launch_bounds__(256) void bf16_rows_to_f32_kernel(const __bf16* __restrict__ x, int ldx, float* __restrict__ y,
                                                               int n_cols, size_t total)
{
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    size_t row = idx / n_cols;
    int col = (int)(idx % n_cols);
    y[idx] = (float)x[row * ldx + col];
}

}  // namespace seedinf
