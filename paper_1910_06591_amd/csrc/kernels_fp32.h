// Generic fp32 kernels: every layer of either torso, the recurrent core and the
// hidden layers of the dueling heads, for any valid arch.  These are the
// SEED_PRECISION_FP32 path (plain vector ALU arithmetic, fp32 accumulation).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace seedinf {

__device__ __forceinline__ float load_in(const uint8_t* p, size_t i) { return (float)p[i] / 255.0f; }
__device__ __forceinline__ float load_in(const float* p, size_t i) { return p[i]; }

// 2-D cross-correlation, NHWC, weights [kh][kw][cin][cout]; one thread per
// output element, cout fastest so weight reads coalesce.  Options: rectify the
// input on load, add a residual (same shape as the output), rectify the output.
// uint8 input is scaled by 1/255 on load (first layer).
template <typename TIn>
__global__ __launch_bounds__(256) void conv2d_f32_kernel(
    const TIn* __restrict__ x, const float* __restrict__ w, const float* __restrict__ bias,
    const float* resid, float* y, int B, int H, int W, int Cin, int OH, int OW, int Cout, int k,
    int stride, int pad, int relu_in, int relu_out)
{
    const size_t total = (size_t)B * OH * OW * Cout;
    // grid-stride: the launch caps its grid, so any batch the workspace can hold stays within the launch limits
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    int co = (int)(idx % Cout);
    size_t t = idx / Cout;
    int ow = (int)(t % OW); t /= OW;
    int oh = (int)(t % OH);
    int b = (int)(t / OH);
    const size_t img = (size_t)b * H * W * Cin;
    // four independent partial sums over the input channels: a single chain would wait out a load per term
    float a0 = bias[co], a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
    auto term = [&](size_t xi, const float* wq) {
        float v = load_in(x, xi);
        if (relu_in) v = fmaxf(v, 0.0f);
        return v * wq[0];
    };
    // taps inside the image: [kh0, kh1) x [kw0, kw1) (loops without early exits can be unrolled, which is what
    // lets the loads of several taps be in flight together)
    const int kh0 = max(0, pad - oh * stride), kh1 = min(k, H + pad - oh * stride);
    const int kw0 = max(0, pad - ow * stride), kw1 = min(k, W + pad - ow * stride);
    for (int kh = kh0; kh < kh1; ++kh) {
        int ih = oh * stride + kh - pad;
#pragma unroll 4
        for (int kw = kw0; kw < kw1; ++kw) {
            int iw = ow * stride + kw - pad;
            size_t xo = img + ((size_t)ih * W + iw) * Cin;
            const float* wp = w + ((size_t)(kh * k + kw) * Cin) * Cout + co;
            int ci = 0;
            for (; ci + 3 < Cin; ci += 4) {
                a0 += term(xo + ci, wp + (size_t)ci * Cout);
                a1 += term(xo + ci + 1, wp + (size_t)(ci + 1) * Cout);
                a2 += term(xo + ci + 2, wp + (size_t)(ci + 2) * Cout);
                a3 += term(xo + ci + 3, wp + (size_t)(ci + 3) * Cout);
            }
            for (; ci < Cin; ++ci) a0 += term(xo + ci, wp + (size_t)ci * Cout);
        }
    }
    float acc = (a0 + a1) + (a2 + a3);
    if (resid) acc += resid[idx];
    if (relu_out) acc = fmaxf(acc, 0.0f);
    y[idx] = acc;
    }
}

// 3x3 / stride 2 max-pool with SAME geometry; cells outside the image are skipped.
__global__ __launch_bounds__(256) void maxpool3x3s2_f32_kernel(
    const float* __restrict__ x, float* __restrict__ y, int B, int H, int W, int C, int OH, int OW,
    int pad_h, int pad_w, int relu_out)
{
    const size_t total = (size_t)B * OH * OW * C;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    int c = (int)(idx % C);
    size_t t = idx / C;
    int ow = (int)(t % OW); t /= OW;
    int oh = (int)(t % OH);
    int b = (int)(t / OH);
    float m = -INFINITY;
    for (int i = 0; i < 3; ++i) {
        int ih = oh * 2 + i - pad_h;
        if (ih < 0 || ih >= H) continue;
        for (int j = 0; j < 3; ++j) {
            int iw = ow * 2 + j - pad_w;
            if (iw < 0 || iw >= W) continue;
            m = fmaxf(m, x[(((size_t)b * H + ih) * W + iw) * C + c]);
        }
    }
    if (relu_out) m = fmaxf(m, 0.0f);
    y[idx] = m;
    }
}

__global__ __launch_bounds__(256) void relu_f32_kernel(const float* __restrict__ x, float* __restrict__ y, size_t n)
{
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (size_t)gridDim.x * blockDim.x)
        y[idx] = fmaxf(x[idx], 0.0f);
}

// y[b, o] = act(bias[o] + sum_i x[b, i] * w[i, o]).  One wavefront per (row, 64-output group) would idle at
// small B and wait out one load per term, so the reduction dimension is split over the 16 wavefronts of a block
// (combined through LDS in a fixed order) and every lane keeps four independent partial sums.
constexpr int DENSE_F32_WAVES = 16;
__global__ __launch_bounds__(DENSE_F32_WAVES * 64) void dense_f32_kernel(
    const float* __restrict__ x, const float* __restrict__ w, const float* __restrict__ bias,
    float* __restrict__ y, int n_in, int n_out, int ldx, int ldy, int relu_out)
{
    __shared__ float part[DENSE_F32_WAVES][64];
    int b = blockIdx.x;
    int lane = threadIdx.x & 63;
    int o = blockIdx.y * 64 + lane;
    int q = threadIdx.x >> 6;
    float acc = 0.0f;
    if (o < n_out) {
        const float* xr = x + (size_t)b * ldx;
        constexpr int Q = DENSE_F32_WAVES;
        float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
        int i = q;
        for (; i + 3 * Q < n_in; i += 4 * Q) {
            a0 = fmaf(xr[i], w[(size_t)i * n_out + o], a0);
            a1 = fmaf(xr[i + Q], w[(size_t)(i + Q) * n_out + o], a1);
            a2 = fmaf(xr[i + 2 * Q], w[(size_t)(i + 2 * Q) * n_out + o], a2);
            a3 = fmaf(xr[i + 3 * Q], w[(size_t)(i + 3 * Q) * n_out + o], a3);
        }
        for (; i < n_in; i += Q) a0 = fmaf(xr[i], w[(size_t)i * n_out + o], a0);
        acc = (a0 + a1) + (a2 + a3);
    }
    part[q][lane] = acc;
    __syncthreads();
    if (q == 0 && o < n_out) {
        float s = bias[o];
#pragma unroll
        for (int j = 0; j < DENSE_F32_WAVES; ++j) s += part[j][lane];
        if (relu_out) s = fmaxf(s, 0.0f);
        y[(size_t)b * ldy + o] = s;
    }
}

__device__ __forceinline__ float sigmoid_f32(float v) { return 1.0f / (1.0f + expf(-v)); }

// One LSTM step in fp32.  Thread (b, j) accumulates the four gate
// pre-activations of unit j over [features | gathered action row | reward row |
// h rows] and applies the cell update.  W is [F + A + 1 + Hn][4 Hn], column
// blocks input | forget | cell | output.
__global__ __launch_bounds__(256) void lstm_f32_kernel(
    const float* __restrict__ feat, const int32_t* __restrict__ prev_action,
    const float* __restrict__ prev_reward, const float* __restrict__ h_in,
    const float* __restrict__ c_in, const float* __restrict__ w, const float* __restrict__ bias,
    float* __restrict__ h_out, float* __restrict__ c_out, int B, int F, int A, int Hn,
    const uint8_t* __restrict__ done)
{
    int j = blockIdx.y * blockDim.x + threadIdx.x;
    int b = blockIdx.x;
    if (j >= Hn) return;
    // a row that starts a new episode runs the cell from the zero state (Section 3: termination flags)
    const bool fresh = done && done[b];
    const int G = 4 * Hn;
    float gi = bias[j], gf = bias[Hn + j], gg = bias[2 * Hn + j], go = bias[3 * Hn + j];
    const float* fr = feat + (size_t)b * F;
    for (int i = 0; i < F; ++i) {
        float v = fr[i];
        const float* wr = w + (size_t)i * G + j;
        gi = fmaf(v, wr[0], gi); gf = fmaf(v, wr[Hn], gf); gg = fmaf(v, wr[2 * Hn], gg); go = fmaf(v, wr[3 * Hn], go);
    }
    int a = prev_action[b];
    if (a >= 0 && a < A) {
        const float* wr = w + (size_t)(F + a) * G + j;
        gi += wr[0]; gf += wr[Hn]; gg += wr[2 * Hn]; go += wr[3 * Hn];
    }
    {
        float r = prev_reward[b];
        const float* wr = w + (size_t)(F + A) * G + j;
        gi = fmaf(r, wr[0], gi); gf = fmaf(r, wr[Hn], gf); gg = fmaf(r, wr[2 * Hn], gg); go = fmaf(r, wr[3 * Hn], go);
    }
    const float* hr = h_in + (size_t)b * Hn;
    for (int i = 0; i < Hn && !fresh; ++i) {
        float v = hr[i];
        const float* wr = w + (size_t)(F + A + 1 + i) * G + j;
        gi = fmaf(v, wr[0], gi); gf = fmaf(v, wr[Hn], gf); gg = fmaf(v, wr[2 * Hn], gg); go = fmaf(v, wr[3 * Hn], go);
    }
    float cn = sigmoid_f32(gf) * (fresh ? 0.0f : c_in[(size_t)b * Hn + j]) + sigmoid_f32(gi) * tanhf(gg);
    c_out[(size_t)b * Hn + j] = cn;
    h_out[(size_t)b * Hn + j] = sigmoid_f32(go) * tanhf(cn);
}

// Conversions used by the diagnostic tap.
__global__ __launch_bounds__(256) void copy_f32_kernel(const float* __restrict__ x, float* __restrict__ y, size_t n)
{
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (size_t)gridDim.x * blockDim.x)
        y[idx] = x[idx];
}

}  // namespace seedinf
