// Generic fp32 kernels: every layer of either torso, the recurrent core and the
// hidden layers of the dueling heads, for any valid arch.  These are the
// SEED_PRECISION_FP32 path (plain vector ALU arithmetic, fp32 accumulation).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace seedinf {

// raw input values: uint8 frames are scaled by 1/255 after the sum (first layer), not per term
__device__ __forceinline__ float load_raw(const uint8_t* p, size_t i) { return (float)p[i]; }
__device__ __forceinline__ float load_raw(const float* p, size_t i) { return p[i]; }
template <typename T> __device__ __forceinline__ float input_scale() { return 1.0f; }
template <> __device__ __forceinline__ float input_scale<uint8_t>() { return 1.0f / 255.0f; }

// Flat work-item index -> (slice, image, row, column, channel group) with channel group and slice fastest.  32-bit
// arithmetic whenever the launch's item count allows it (uniform): a 64-bit division is about a hundred
// instructions, and at small batch these kernels' time is the length of one lane's instruction stream.
template <int KS>
__device__ __forceinline__ void conv_f32_decode(size_t idx, size_t total, int OH, int OW, int CG, int& sl, size_t& o, int& b, int& oh,
                                                int& ow, int& cg)
{
    if (total < ((size_t)1 << 32)) {
        const unsigned i = (unsigned)idx;
        sl = (int)(i % KS);
        const unsigned oo = i / KS;
        o = oo;
        cg = (int)(oo % (unsigned)CG);
        unsigned t = oo / (unsigned)CG;
        ow = (int)(t % (unsigned)OW); t /= (unsigned)OW;
        oh = (int)(t % (unsigned)OH);
        b = (int)(t / (unsigned)OH);
    } else {
        sl = (int)(idx % KS);
        o = idx / KS;
        cg = (int)(o % CG);
        size_t t = o / CG;
        ow = (int)(t % OW); t /= OW;
        oh = (int)(t % OH);
        b = (int)(t / OH);
    }
}

// 2-D cross-correlation, NHWC, weights [kh][kw][cin][cout].  KS adjacent lanes share one output element and split
// the k * k taps between them (cout next fastest, so weight reads still coalesce in runs); the partial sums meet
// in a butterfly whose result does not depend on the lane.  A thread per output walks all k * k * cin terms as a
// chain of trips to memory.  KS is a constant, so a row's result never depends on what else is in the batch.
// Options: rectify the input on load, add a residual (same shape as the output), rectify the output.  uint8
// input (first layer) is scaled by 1/255 after the sum.
constexpr int CONV_F32_KS = 4;
template <typename TIn, int KS = CONV_F32_KS>
__global__ __launch_bounds__(256) void conv2d_f32_kernel(
    const TIn* __restrict__ x, const float* __restrict__ w, const float* __restrict__ bias,
    const float* resid, float* y, int B, int H, int W, int Cin, int OH, int OW, int Cout, int k,
    int stride, int pad, int relu_in, int relu_out)
{
    const size_t total = (size_t)B * OH * OW * Cout * KS;              // a multiple of KS: the lanes of a group leave together
    const int T = k * k;
    // grid-stride: the launch caps its grid, so any batch the workspace can hold stays within the launch limits
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    int sl, b, oh, ow, co;
    size_t oidx;
    conv_f32_decode<KS>(idx, total, OH, OW, Cout, sl, oidx, b, oh, ow, co);
    const size_t img = (size_t)b * H * W * Cin;
    // four independent partial sums over the input channels: a single chain would wait out a load per term
    float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
    // this lane's taps; a tap outside the image reads a clamped pixel and counts as zero (no branch in the loop,
    // so that it unrolls and the loads of several taps are in flight together)
    const int t0 = sl * T / KS, t1 = (sl + 1) * T / KS;
#pragma unroll 4
    for (int tp = t0; tp < t1; ++tp) {
        const int kh = tp / k, kw = tp - kh * k;
        const int ih = oh * stride + kh - pad, iw = ow * stride + kw - pad;
        const bool ok = ih >= 0 && ih < H && iw >= 0 && iw < W;
        const size_t xo = img + ((size_t)min(max(ih, 0), H - 1) * W + min(max(iw, 0), W - 1)) * Cin;
        const float* wp = w + ((size_t)tp * Cin) * Cout + co;
        auto term = [&](size_t xi, const float* wq) {
            float v = load_raw(x, xi);
            if (relu_in) v = fmaxf(v, 0.0f);
            return (ok ? v : 0.0f) * wq[0];
        };
        int ci = 0;
        for (; ci + 3 < Cin; ci += 4) {
            a0 += term(xo + ci, wp + (size_t)ci * Cout);
            a1 += term(xo + ci + 1, wp + (size_t)(ci + 1) * Cout);
            a2 += term(xo + ci + 2, wp + (size_t)(ci + 2) * Cout);
            a3 += term(xo + ci + 3, wp + (size_t)(ci + 3) * Cout);
        }
        for (; ci < Cin; ++ci) a0 += term(xo + ci, wp + (size_t)ci * Cout);
    }
    float part = (a0 + a1) + (a2 + a3);
#pragma unroll
    for (int m = 1; m < KS; m <<= 1) part += __shfl_xor(part, m);
    if (sl == 0) {
        float acc = bias[co] + part * input_scale<TIn>();
        if (resid) acc += resid[oidx];
        if (relu_out) acc = fmaxf(acc, 0.0f);
        y[oidx] = acc;
    }
    }
}

// The same for layers whose channel counts are multiples of four (and whose operands are aligned for it).  A lane
// takes FOUR consecutive output channels of a pixel, so a term's weights are one 16-byte load and its input value
// serves four sums, and the input's channels come four at a time (one dword of a uint8 frame, 16 bytes of an fp32
// map).  The k * k taps are split over the block's eight WAVEFRONTS, not over lanes: a wavefront's taps are then
// uniform, their index arithmetic runs on the scalar unit, and a lane's instruction stream - whose length is this
// kernel's time at small batch, where a SIMD holds a single wavefront - shrinks to a few adds, the loads and the
// multiply-adds per term.  A block is 64 (pixel, channel group) items of one image; the eight partial sums meet in
// LDS in a fixed order.  Which of the two kernels runs depends on the layer and the buffers' alignment only.
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ f32x4 load_raw4(const uint8_t* p, int i)
{
    const uint32_t v = *(const uint32_t*)(p + i);
    return f32x4{(float)(v & 0xff), (float)((v >> 8) & 0xff), (float)((v >> 16) & 0xff), (float)(v >> 24)};
}
__device__ __forceinline__ f32x4 load_raw4(const float* p, int i) { return *(const f32x4*)(p + i); }

// requires Cin % 4 == 0, Cout % 4 == 0, OH * OW * Cout / 4 and H * W * Cin below 2^31, 16-byte aligned w, bias, y, resid
// and fp32 x (4-byte aligned uint8 x).  Grid: (ceil(OH * OW * Cout / 4 / 64), min(B, 65535)).
constexpr int CONV_F32_V4_WAVES = 8;
template <typename TIn>
__global__ __launch_bounds__(CONV_F32_V4_WAVES * 64) void conv2d_f32_v4_kernel(
    const TIn* __restrict__ x, const float* __restrict__ w, const float* __restrict__ bias,
    const float* resid, float* y, int B, int H, int W, int Cin, int OH, int OW, int Cout, int k,
    int stride, int pad, int relu_in, int relu_out)
{
    constexpr int KS = CONV_F32_V4_WAVES;
    __shared__ f32x4 red[KS - 1][64];
    const int lane = threadIdx.x & 63;
    const int sl = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int CG = Cout >> 2, per_img = OH * OW * CG;
    const int item = blockIdx.x * 64 + lane;
    const bool live = item < per_img;
    const int it = live ? item : per_img - 1;
    const int cg = it % CG, pix = it / CG;
    const int ow = pix % OW, oh = pix / OW;
    const int co = cg * 4;
    const int ih0 = oh * stride - pad, iw0 = ow * stride - pad;
    const int T = k * k;
    const int t0 = sl * T / KS, t1 = (sl + 1) * T / KS;                  // this wavefront's taps
    const int C4 = Cin >> 2, nitems = (t1 - t0) * C4;
    const float* wl = w + co;
    for (int b = blockIdx.y; b < B; b += gridDim.y) {
        const TIn* ximg = x + (size_t)b * H * W * Cin;
        f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
        // (tap, four input channels) items, U at a time: all their loads are issued - from clamped, valid
        // addresses; an item past the end or outside the image counts as zero - before the first is used
        constexpr int U = 8;
        for (int f0 = 0; f0 < nitems; f0 += U) {
            f32x4 v[U], wv[U][4];
            bool ok[U];
#pragma unroll
            for (int j = 0; j < U; ++j) {
                const int f = min(f0 + j, nitems - 1);                  // uniform, like everything derived from it
                const int tp = t0 + f / C4, ci = (f % C4) * 4;
                const int kh = tp / k, kw = tp - kh * k;
                const int ih = ih0 + kh, iw = iw0 + kw;
                ok[j] = f0 + j < nitems && ih >= 0 && ih < H && iw >= 0 && iw < W;
                v[j] = load_raw4(ximg, (min(max(ih, 0), H - 1) * W + min(max(iw, 0), W - 1)) * Cin + ci);
                const float* wp = wl + (size_t)(tp * Cin + ci) * Cout;
#pragma unroll
                for (int c = 0; c < 4; ++c) wv[j][c] = *(const f32x4*)(wp + c * Cout);
            }
#pragma unroll
            for (int j = 0; j < U; ++j) {
                f32x4 vv = v[j];
                if (relu_in) vv = f32x4{fmaxf(vv[0], 0.0f), fmaxf(vv[1], 0.0f), fmaxf(vv[2], 0.0f), fmaxf(vv[3], 0.0f)};
                if (!ok[j]) vv = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int c = 0; c < 4; ++c) acc += vv[c] * wv[j][c];
            }
        }
        if (sl > 0) red[sl - 1][lane] = acc;
        __syncthreads();
        if (sl == 0 && live) {
#pragma unroll
            for (int q = 0; q < KS - 1; ++q) acc += red[q][lane];
            const size_t at = ((size_t)b * per_img + item) * 4;          // = ((b * OH + oh) * OW + ow) * Cout + co
            f32x4 out = *(const f32x4*)(bias + co) + acc * input_scale<TIn>();
            if (resid) out += *(const f32x4*)(resid + at);
            if (relu_out) out = f32x4{fmaxf(out[0], 0.0f), fmaxf(out[1], 0.0f), fmaxf(out[2], 0.0f), fmaxf(out[3], 0.0f)};
            *(f32x4*)(y + at) = out;
        }
        __syncthreads();                                                // `red` is reused by the next image
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

// y[b, o] = act(bias[o] + sum_i x[b, i] * w[i, o]).  A block takes one row and DENSE_F32_COLS outputs; the
// reduction dimension is split 64 ways - over the block's 16 wavefronts and, inside a wavefront, over the four
// groups of 16 lanes - and every lane keeps four independent partial sums, so a lane's chain of trips to memory
// is n_in / 256 long (the time of this kernel at small batch is that chain, not the bytes).  The partial sums meet
// in a fixed order (lane groups by butterfly, wavefronts through LDS).
constexpr int DENSE_F32_WAVES = 16, DENSE_F32_COLS = 16;
__global__ __launch_bounds__(DENSE_F32_WAVES * 64) void dense_f32_kernel(
    const float* __restrict__ x, const float* __restrict__ w, const float* __restrict__ bias,
    float* __restrict__ y, int n_in, int n_out, int ldx, int ldy, int relu_out)
{
    __shared__ float part[DENSE_F32_WAVES][DENSE_F32_COLS];
    const int b = blockIdx.x;
    const int lane = threadIdx.x & 63, col = lane & 15, sub = lane >> 4;
    const int o = blockIdx.y * DENSE_F32_COLS + col;
    const int oc = min(o, n_out - 1);                  // lanes past the last output compute it again and store nothing
    const int q = threadIdx.x >> 6;
    const float* xr = x + (size_t)b * ldx;
    constexpr int Q = DENSE_F32_WAVES * 4;
    float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
    int i = q * 4 + sub;
    for (; i + 3 * Q < n_in; i += 4 * Q) {
        a0 = fmaf(xr[i], w[(size_t)i * n_out + oc], a0);
        a1 = fmaf(xr[i + Q], w[(size_t)(i + Q) * n_out + oc], a1);
        a2 = fmaf(xr[i + 2 * Q], w[(size_t)(i + 2 * Q) * n_out + oc], a2);
        a3 = fmaf(xr[i + 3 * Q], w[(size_t)(i + 3 * Q) * n_out + oc], a3);
    }
    for (; i < n_in; i += Q) a0 = fmaf(xr[i], w[(size_t)i * n_out + oc], a0);
    float acc = (a0 + a1) + (a2 + a3);
    acc += __shfl_xor(acc, 16);
    acc += __shfl_xor(acc, 32);
    if (sub == 0) part[q][col] = acc;
    __syncthreads();
    if (q == 0 && sub == 0 && o < n_out) {
        float s = bias[o];
#pragma unroll
        for (int j = 0; j < DENSE_F32_WAVES; ++j) s += part[j][col];
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
