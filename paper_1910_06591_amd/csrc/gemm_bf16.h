// bf16 MFMA GEMM for the dense layers: Y[row, f] = sum_k X[row, k] * W[k, f].
//
// Weights are pre-packed on the host into A-operand fragments:
//   Wp[ftile][kchunk][lane][8], lane -> feature ftile*16 + lane%16,
//   k = kchunk*32 + 8*(lane/16) + e; padded with zeros to whole tiles/chunks.
// Activations are read straight from their row-major bf16 (or fp32, converted
// on load) buffer as B-operand fragments: 16 bytes per lane.
// One wavefront owns 4 feature tiles x RT row tiles; a block is 4 wavefronts
// that differ in their feature tiles.  K is walked in chunks of 32.
//
// Epilogues:
//   EPI_RELU : y = max(acc + bias, 0) stored as bf16 and/or fp32
//   EPI_LSTM : the wavefront's 4 feature tiles are the i, f, g, o gates of the
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
};

__device__ __forceinline__ float sigmoidf_(float v) { return 1.0f / (1.0f + expf(-v)); }

template <int RT, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmArgs p)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
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

    // K loop, software-pipelined: the fragments of chunk kc+1 are loaded while chunk kc is multiplied
    auto load_chunk = [&](bf16x8 (&a)[4], bf16x8 (&b)[RT], int kc) {
#pragma unroll
        for (int j = 0; j < 4; ++j) a[j] = wl[j][(size_t)kc * 64];
        if (kc < p.kc1) {
#pragma unroll
            for (int r = 0; r < RT; ++r)
                b[r] = *(const bf16x8*)(p.x1 + (size_t)rowi[r] * p.ld1 + kc * 32 + g * 8);
        } else {
            const int k = (kc - p.kc1) * 32 + g * 8;
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                floatx4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
                if (k + 8 <= p.k2) {
                    const float* s = p.x2 + (size_t)rowi[r] * p.ld2 + k;
                    lo = *(const floatx4*)s;
                    hi = *(const floatx4*)(s + 4);
                }
                b[r] = to_bf16x8(lo, hi);
            }
        }
    };
    auto mma_chunk = [&](const bf16x8 (&a)[4], const bf16x8 (&b)[RT]) {
#pragma unroll
        for (int r = 0; r < RT; ++r)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[r][j] = mfma16(a[j], b[r], acc[r][j]);
    };
    {
        bf16x8 a0[4], b0[RT], a1[4], b1[RT];
        load_chunk(a0, b0, 0);
        int kc = 0;
        for (; kc + 2 <= kct; kc += 2) {
            load_chunk(a1, b1, kc + 1);
            mma_chunk(a0, b0);
            load_chunk(a0, b0, kc + 2 < kct ? kc + 2 : kct - 1);
            mma_chunk(a1, b1);
        }
        if (kc < kct) mma_chunk(a0, b0);
    }

    if constexpr (EPI == EPI_RELU) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (ft0 + j >= p.n_ftiles) break;
            const int f = (ft0 + j) * 16 + g * 4;
            const floatx4 bv = *(const floatx4*)(p.bias_pad + f);
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                const int row = r0 + r * 16 + n;
                if (row >= p.rows) continue;
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
        // wavefront wt = unit tile; feature tile j = gate j of units wt*16 .. wt*16+15
        const int Hn = p.Hn, G4 = 4 * p.Hn;
        const int u = wt * 16 + g * 4;                  // this lane's 4 consecutive units
        floatx4 bg[4], wr[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            bg[j] = *(const floatx4*)(p.lstm_b + j * Hn + u);
            wr[j] = *(const floatx4*)(p.lstm_w + (size_t)(p.F + p.A) * G4 + j * Hn + u);
        }
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            const int row = r0 + r * 16 + n;
            if (row >= p.rows) continue;
            const int a = p.prev_action[row];
            const float rew = p.prev_reward[row];
            floatx4 pre[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                pre[j] = acc[r][j] + bg[j] + rew * wr[j];
                if (a >= 0 && a < p.A) pre[j] += *(const floatx4*)(p.lstm_w + (size_t)(p.F + a) * G4 + j * Hn + u);
            }
            const floatx4 c0 = *(const floatx4*)(p.c_in + (size_t)row * Hn + u);
            floatx4 cn, hn;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                cn[i] = sigmoidf_(pre[1][i]) * c0[i] + sigmoidf_(pre[0][i]) * tanhf(pre[2][i]);
                hn[i] = sigmoidf_(pre[3][i]) * tanhf(cn[i]);
            }
            *(floatx4*)(p.c_out + (size_t)row * Hn + u) = cn;
            *(floatx4*)(p.h_out + (size_t)row * Hn + u) = hn;
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
