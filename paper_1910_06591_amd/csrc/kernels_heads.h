// Output heads and action selection, fp32, one wavefront per batch row.
//
// The last linear maps (core -> logits/value, or dueling hidden -> advantage /
// value) are short dot products over n <= 8192 inputs and A <= 64 outputs: the
// 64 lanes split into 64/P groups (P = power of two >= A), lane (g, a) sums
// the inputs i = g, g + 64/P, ... for output a, and the groups are combined with
// xor-shuffles.  Softmax, the dueling mean and the (Gumbel-)argmax are row
// reductions over the first P lanes, again by shuffles: no LDS, no atomics, so
// results are bit-reproducible run to run.
#pragma once
#include <hip/hip_runtime.h>

#include <cfloat>
#include <cstdint>

namespace seedinf {

struct HeadsArgs {
    const float* vec_a; int ld_a;    // [B, n] input of the A action outputs
    const float* vec_v; int ld_v;    // [B, n] input of the value output
    const float* w_a;                // [n][A]
    const float* b_a;                // [A]
    const float* w_v;                // [n]
    const float* b_v;                // [1]
    const float* uniforms;           // [B, A] or nullptr (greedy)
    const float* epsilon;            // [B] or nullptr: epsilon-greedy exploration (Appendix A.3.1)
    const float* explore_u;          // [B, 2] uniforms in [0,1): explore iff u0 < epsilon, action floor(u1 * A)
    int32_t* action;                 // [B]
    float* logits;                   // [B, A]
    float* value;                    // [B]
    float* probs;                    // [B, A] or nullptr
    int n, A, B;
    int dueling;                     // 1: logits = V + Adv - mean(Adv)
};

// Everything after the dot products: `acc` = this lane's action output before the bias (already summed over
// the lane groups), `val` = the value output.  Bias, dueling combination, softmax, (Gumbel-)argmax, exploration.
template <int P>
__device__ __forceinline__ void heads_finish(const HeadsArgs& p, int row, int lane, float acc, float val)
{
    const int a = lane & (P - 1);
    const bool live = a < p.A;
    float out = live ? acc + p.b_a[a] : 0.0f;

    if (p.dueling) {
        float s = out;                            // dead lanes hold 0
#pragma unroll
        for (int off = P / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
        out = live ? val + out - s / (float)p.A : 0.0f;
    }

    if (lane < p.A) p.logits[(size_t)row * p.A + lane] = out;
    if (lane == 0) p.value[row] = val;

    if (p.probs) {
        float m = live ? out : -INFINITY;
#pragma unroll
        for (int off = P / 2; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
        float e = live ? expf(out - m) : 0.0f;
        float s = e;
#pragma unroll
        for (int off = P / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
        if (lane < p.A) p.probs[(size_t)row * p.A + lane] = e / s;
    }

    // selection: argmax of logits (+ Gumbel noise), lowest index wins ties
    float key = live ? out : -INFINITY;
    if (p.uniforms && live) {
        float u = p.uniforms[(size_t)row * p.A + a];
        u = fminf(fmaxf(u, FLT_MIN), 1.0f - 5.9604644775390625e-8f);
        key = out - logf(-logf(u));
    }
    int best = a;
#pragma unroll
    for (int off = P / 2; off > 0; off >>= 1) {
        float ok = __shfl_xor(key, off, 64);
        int ob = __shfl_xor(best, off, 64);
        if (ok > key || (ok == key && ob < best)) { key = ok; best = ob; }
    }
    if (lane == 0) {
        if (p.epsilon && p.explore_u[2 * (size_t)row] < p.epsilon[row]) {
            const int r = (int)floorf(p.explore_u[2 * (size_t)row + 1] * (float)p.A);
            best = r < 0 ? 0 : (r > p.A - 1 ? p.A - 1 : r);
        }
        p.action[row] = best;
    }
}

template <int P>
__global__ __launch_bounds__(256) void heads_select_kernel(HeadsArgs p)
{
    constexpr int G = 64 / P;
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= p.B) return;                      // whole wavefront leaves together
    const int a = lane & (P - 1);
    const int g = lane / P;
    const bool live = a < p.A;

    // action outputs
    float acc = 0.0f;
    {
        const float* v = p.vec_a + (size_t)row * p.ld_a;
        if (live) {
            // eight independent partial sums keep sixteen loads in flight per lane (the loop is bound by load
            // latency: its weights do not fit the first-level cache); the summation order is fixed, so results
            // stay reproducible
            float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            int i = g;
            for (; i + 7 * G < p.n; i += 8 * G) {
#pragma unroll
                for (int u = 0; u < 8; ++u) s[u] = fmaf(v[i + u * G], p.w_a[(size_t)(i + u * G) * p.A + a], s[u]);
            }
            for (; i < p.n; i += G) s[0] = fmaf(v[i], p.w_a[(size_t)i * p.A + a], s[0]);
            acc = ((s[0] + s[1]) + (s[2] + s[3])) + ((s[4] + s[5]) + (s[6] + s[7]));
        }
    }
#pragma unroll
    for (int off = P; off < 64; off <<= 1) acc += __shfl_xor(acc, off, 64);

    // value output: all 64 lanes share the dot product
    float vacc = 0.0f;
    {
        const float* v = p.vec_v + (size_t)row * p.ld_v;
        float t[4] = {0.f, 0.f, 0.f, 0.f};
        int i = lane;
        for (; i + 3 * 64 < p.n; i += 4 * 64) {
#pragma unroll
            for (int u = 0; u < 4; ++u) t[u] = fmaf(v[i + u * 64], p.w_v[i + u * 64], t[u]);
        }
        for (; i < p.n; i += 64) t[0] = fmaf(v[i], p.w_v[i], t[0]);
        vacc = (t[0] + t[1]) + (t[2] + t[3]);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) vacc += __shfl_xor(vacc, off, 64);
    heads_finish<P>(p, row, lane, acc, vacc + p.b_v[0]);
}

// The same heads for n = KS * (64 / P) * NPL inputs with NPL <= 64: every lane keeps its NPL action weights (and
// its share of the value weights) in registers and the workgroup walks several rows.  A wavefront fetches its
// slice of a row with ONE coalesced 16-byte load per lane and hands the values round through its own strip of
// LDS, where the lanes of a group read the same addresses (a broadcast).  (Fetched directly, 16 bytes per lane
// with 64 / G lanes on one address, the loads cost the texture path ~45 cycles each and were the kernel's
// whole time: 21.9 -> 12.7 us for the 512-input dueling heads at B = 4096, 7.5 -> 6.1 us for the policy heads.)
// KS wavefronts share a row, each taking a contiguous KS-th of the inputs (lane (g, a) of slice ks: inputs
// (ks * G + g) * NPL .. + NPL - 1); their partial sums meet in LDS in slice order and the slice-0 wavefront
// finishes the row.  Needs 16-byte aligned rows.
typedef float heads_f4 __attribute__((ext_vector_type(4)));
template <int P, int NPL, int KS>
__global__ __launch_bounds__(256) void heads_rows_kernel(HeadsArgs p)
{
    constexpr int G = 64 / P, NS = G * NPL, NV = NS / 64, RPB = 4 / KS;      // NS: inputs per slice; RPB: rows per pass
    static_assert(NPL % 4 == 0 && NS % 64 == 0 && (KS == 1 || KS == 2 || KS == 4), "inputs per lane");
    __shared__ float part[2][4][64];                     // [acc | value][wavefront][lane]
    __shared__ heads_f4 stage[4][NS / 4];                // per wavefront: its slice of the current row
    __shared__ heads_f4 stagev[4][NS / 4];               // ... and of the value output's input row where that is another one
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ks = wave % KS, rs = wave / KS;
    const int a = lane & (P - 1);
    const int g = lane / P;
    const bool live = a < p.A;
    const int i0 = ks * NS + g * NPL;                    // this lane's first action input
    float w[NPL], wv[NV];
#pragma unroll
    for (int k = 0; k < NPL; ++k) w[k] = live ? p.w_a[(size_t)(i0 + k) * p.A + a] : 0.0f;
#pragma unroll
    for (int k = 0; k < NV; ++k) wv[k] = p.w_v[ks * NS + lane + 64 * k];
    const float bv = p.b_v[0];
    const bool shared_in = p.vec_v == p.vec_a && p.ld_v == p.ld_a;         // policy heads: one input row for both
    for (int base = blockIdx.x * RPB; base < p.B; base += gridDim.x * RPB) {        // uniform per workgroup
        const int row = base + rs;
        float acc = 0.0f, vacc = 0.0f;
        if (row < p.B) {                                 // uniform per wavefront
            // the wavefront's NS inputs of this row: one coalesced 16-byte load per lane, handed round through the
            // wavefront's own LDS strip (the lanes of a group then read the same addresses: a broadcast)
            if (4 * lane < NS) {
                stage[wave][lane] = *(const heads_f4*)(p.vec_a + (size_t)row * p.ld_a + ks * NS + 4 * lane);
                if (!shared_in) stagev[wave][lane] = *(const heads_f4*)(p.vec_v + (size_t)row * p.ld_v + ks * NS + 4 * lane);
            }
            __builtin_amdgcn_wave_barrier();             // (one wavefront: its LDS accesses complete in program order)
            const heads_f4* v = &stage[wave][g * (NPL / 4)];
            float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
            for (int k = 0; k < NPL / 4; ++k) {
                const heads_f4 x = v[k];
                s0 = fmaf(x[0], w[4 * k], s0);
                s1 = fmaf(x[1], w[4 * k + 1], s1);
                s2 = fmaf(x[2], w[4 * k + 2], s2);
                s3 = fmaf(x[3], w[4 * k + 3], s3);
            }
            acc = (s0 + s1) + (s2 + s3);
#pragma unroll
            for (int off = P; off < 64; off <<= 1) acc += __shfl_xor(acc, off, 64);
            const float* vv = (const float*)(shared_in ? stage[wave] : stagev[wave]);
#pragma unroll
            for (int k = 0; k < NV; ++k) vacc = fmaf(vv[lane + 64 * k], wv[k], vacc);
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) vacc += __shfl_xor(vacc, off, 64);
        }
        if constexpr (KS > 1) {
            part[0][wave][lane] = acc;
            part[1][wave][lane] = vacc;
            __syncthreads();
            if (ks == 0) {
#pragma unroll
                for (int q = 1; q < KS; ++q) {
                    acc += part[0][wave + q][lane];
                    vacc += part[1][wave + q][lane];
                }
            }
            __syncthreads();                             // the partial sums are read before the next pass overwrites them
        }
        if (ks == 0 && row < p.B) heads_finish<P>(p, row, lane, acc, vacc + bv);
    }
}

}  // namespace seedinf
