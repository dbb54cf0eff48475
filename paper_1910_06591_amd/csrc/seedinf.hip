// libseedinf host side: C ABI, validation, weight upload/repack, workspace and
// the per-step kernel sequence.  See include/seedinf.h for the contract.
#include <hip/hip_runtime.h>

#include <algorithm>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "../../include/seedinf.h"
#include "plan.h"
#include "host_pool.h"
#include "kernels_fp32.h"
#include "kernels_heads.h"
#include "bf16_path.h"

using namespace seedinf;

struct seed_infer {
    Plan plan;
    int device = -1;
    float* d_w = nullptr;          // canonical flat fp32 weights the steps read: d_w_set[active]
    float* d_w_set[2] = {nullptr, nullptr};   // two copies: a weight update fills the idle one and flips
    int active = 0;
    char* staging[2] = {nullptr, nullptr};     // pinned host buffers weight updates are staged in, used alternately
    size_t staging_bytes = 0;
    hipEvent_t staged[2] = {nullptr, nullptr}; // recorded after the copy that reads staging[i]
    int stage_next = 0;
    // weight updates travel on a stream of the handle's own, so that an upload runs beside the steps already
    // enqueued on the caller's stream (they read the other copy) instead of behind them
    hipStream_t up_stream = nullptr;
    hipEvent_t uploaded[2] = {nullptr, nullptr};  // recorded on up_stream behind the update of copy i; the caller's stream waits for it
    hipEvent_t retired[2] = {nullptr, nullptr};   // recorded on the caller's stream when copy i stopped being the active one
    bool retired_set[2] = {false, false};
    float* d_act[2] = {nullptr, nullptr};   // fp32 ping-pong activations (fp32 mode)
    float* d_fc = nullptr;         // [max_batch, fc_units] fp32 (fp32 mode)
    float* d_hid = nullptr;        // [max_batch, 2*head_hidden] dueling hidden, fp32
    float* d_roll = nullptr;       // recurrent archs: 4 x [max_batch, lstm_units]: every step's h of an unroll, then two c buffers
    const float* feat_f32 = nullptr;   // where the last fp32-mode step left the torso features
    Bf16State* bf = nullptr;       // everything the bf16 path owns
    HostPool* pool = nullptr;      // host threads for the large copies (weight updates, the batcher's frames); made on first use
    std::vector<hipEvent_t> ev;    // profiling: 2 events per slot (empty = profiling off)
    int ev_used = 0;
    std::string err;
};

static thread_local std::string g_create_err;

// The handle's host threads (seven workers + the caller), started by the first large copy; nullptr if they cannot
// be started (the copies then run on the calling thread).
static HostPool* host_pool(seed_infer* h);

// ---- workspace in the library's static device array (seed_infer_step_static) ----
// Device memory beyond a step's inputs and outputs: the activations between the kernels.  The handle's own copy is
// allocated at creation; this one is part of the loaded code object, one instance per GPU.
static __device__ __align__(256) unsigned char seed_static_scratch[SEED_STATIC_SCRATCH_BYTES];

constexpr int SEED_MAX_DEVICES = 64;
static void* g_scratch_ptr[SEED_MAX_DEVICES] = {};    // device address of seed_static_scratch on each GPU

// Address of the current device's instance of the array; looked up once per device (no allocation).
static hipError_t scratch_address(int dev, void** out)
{
    if (dev < 0 || dev >= SEED_MAX_DEVICES) return hipErrorInvalidDevice;
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(seed_static_scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}


#define HIP_TRY(h, expr)                                                              \
    do {                                                                              \
        hipError_t e_ = (expr);                                                       \
        if (e_ != hipSuccess) {                                                       \
            (h)->err = std::string(#expr) + ": " + hipGetErrorString(e_);             \
            return e_ == hipErrorOutOfMemory ? SEED_ERR_OOM : SEED_ERR_DEVICE;        \
        }                                                                             \
    } while (0)

static HostPool* host_pool(seed_infer* h)
{
    if (!h->pool) {
        try {
            h->pool = new HostPool(7);
        } catch (...) {
            h->pool = nullptr;
        }
    }
    return h->pool;
}

extern "C" size_t seed_infer_weight_count(const seed_arch_t* arch)
{
    Plan p;
    std::string err;
    if (make_plan(arch, p, err) != SEED_OK) return 0;
    return p.n_weights;
}

extern "C" size_t seed_infer_torso_features(const seed_arch_t* arch)
{
    Plan p;
    std::string err;
    if (make_plan(arch, p, err) != SEED_OK) return 0;
    return p.flat;
}

static seed_status_t validate_impl(const seed_arch_t* arch, Plan& p, std::string& err)
{
    seed_status_t st = make_plan(arch, p, err);
    if (st != SEED_OK) return st;
    if (arch->precision == SEED_PRECISION_BF16) return bf16_supported(p, err);
    return SEED_OK;
}

extern "C" seed_status_t seed_infer_validate(const seed_arch_t* arch)
{
    Plan p;
    g_create_err.clear();
    return validate_impl(arch, p, g_create_err);
}

extern "C" const char* seed_infer_last_error(const seed_infer_t* h)
{
    return h ? h->err.c_str() : g_create_err.c_str();
}

static void free_all(seed_infer* h)
{
    if (!h) return;
    if (h->bf) { bf16_destroy(h->bf); h->bf = nullptr; }
    for (hipEvent_t e : h->ev) (void)hipEventDestroy(e);
    delete h->pool;
    if (h->up_stream) { (void)hipStreamSynchronize(h->up_stream); (void)hipStreamDestroy(h->up_stream); }
    for (int i = 0; i < 2; ++i) {
        if (h->uploaded[i]) (void)hipEventDestroy(h->uploaded[i]);
        if (h->retired[i]) (void)hipEventDestroy(h->retired[i]);
        if (h->staged[i]) (void)hipEventDestroy(h->staged[i]);
        if (h->staging[i]) (void)hipHostFree(h->staging[i]);
    }
    if (h->d_w_set[0]) (void)hipFree(h->d_w_set[0]);
    if (h->d_w_set[1]) (void)hipFree(h->d_w_set[1]);
    if (h->d_act[0]) (void)hipFree(h->d_act[0]);
    if (h->d_act[1]) (void)hipFree(h->d_act[1]);
    if (h->d_fc) (void)hipFree(h->d_fc);
    if (h->d_hid) (void)hipFree(h->d_hid);
    if (h->d_roll) (void)hipFree(h->d_roll);
    delete h;
}

extern "C" void seed_infer_destroy(seed_infer_t* h) { free_all(h); }

static seed_status_t create_impl(seed_infer* h, const float* weights_host)
{
    const Plan& p = h->plan;
    const seed_arch_t& a = p.arch;
    HIP_TRY(h, hipGetDevice(&h->device));
    HIP_TRY(h, hipMalloc(&h->d_w_set[0], p.n_weights * sizeof(float)));
    HIP_TRY(h, hipMalloc(&h->d_w_set[1], p.n_weights * sizeof(float)));
    h->d_w = h->d_w_set[0];
    HIP_TRY(h, hipMemcpy(h->d_w, weights_host, p.n_weights * sizeof(float), hipMemcpyHostToDevice));
    const size_t mb = (size_t)a.max_batch;
    if (a.head == SEED_HEAD_DUELING_Q) HIP_TRY(h, hipMalloc(&h->d_hid, mb * 2 * a.head_hidden * sizeof(float)));
    if (a.lstm_units > 0) HIP_TRY(h, hipMalloc(&h->d_roll, 4 * mb * a.lstm_units * sizeof(float)));
    if (a.precision == SEED_PRECISION_FP32) {
        HIP_TRY(h, hipMalloc(&h->d_act[0], mb * p.max_act * sizeof(float)));
        HIP_TRY(h, hipMalloc(&h->d_act[1], mb * p.max_act * sizeof(float)));
        HIP_TRY(h, hipMalloc(&h->d_fc, mb * a.fc_units * sizeof(float)));
    } else {
        seed_status_t st = bf16_create(p, h->d_w, &h->bf, h->err);
        if (st != SEED_OK) return st;
    }
    // staging for weight updates, allocated here so that seed_infer_set_weights allocates nothing
    h->staging_bytes = p.n_weights * sizeof(float);
    for (int i = 0; i < 2; ++i) {
        HIP_TRY(h, hipHostMalloc((void**)&h->staging[i], h->staging_bytes, hipHostMallocDefault));
        HIP_TRY(h, hipEventCreateWithFlags(&h->staged[i], hipEventDisableTiming));
        HIP_TRY(h, hipEventCreateWithFlags(&h->retired[i], hipEventDisableTiming));
        HIP_TRY(h, hipEventCreateWithFlags(&h->uploaded[i], hipEventDisableTiming));
    }
    HIP_TRY(h, hipStreamCreateWithFlags(&h->up_stream, hipStreamNonBlocking));        // default priority
    void* scratch = nullptr;                   // seed_infer_step_static's workspace on this device
    HIP_TRY(h, scratch_address(h->device, &scratch));
    HIP_TRY(h, hipDeviceSynchronize());
    return SEED_OK;
}

extern "C" seed_status_t seed_infer_create(const seed_arch_t* arch, const float* weights_host,
                                           size_t n_weights, seed_infer_t** out)
{
    g_create_err.clear();
    if (!out) { g_create_err = "out is NULL"; return SEED_ERR_INVALID_ARG; }
    seed_infer* h = new (std::nothrow) seed_infer;
    if (!h) { g_create_err = "host allocation failed"; return SEED_ERR_OOM; }
    seed_status_t st = validate_impl(arch, h->plan, g_create_err);
    if (st == SEED_OK && !weights_host) { g_create_err = "weights_host is NULL"; st = SEED_ERR_INVALID_ARG; }
    if (st == SEED_OK && n_weights != h->plan.n_weights) {
        char msg[128];
        snprintf(msg, sizeof msg, "n_weights is %zu, this arch has %zu", n_weights, h->plan.n_weights);
        g_create_err = msg;
        st = SEED_ERR_INVALID_ARG;
    }
    if (st != SEED_OK) { delete h; return st; }
    st = create_impl(h, weights_host);
    if (st != SEED_OK) {
        g_create_err = h->err;
        free_all(h);
        return st;
    }
    *out = h;
    return SEED_OK;
}

// Blocks of `per` threads for n elements, capped at 2^22 (the elementwise kernels stride over what is left): a
// launch's thread count stays far below 2^32 whatever the batch.
static inline unsigned blocks_for(size_t n, unsigned per = 256)
{
    const size_t b = (n + per - 1) / per;
    return (unsigned)(b < ((size_t)1 << 22) ? b : ((size_t)1 << 22));
}

static bool overlaps(const void* a, size_t na, const void* b, size_t nb)
{
    const char* pa = (const char*)a;
    const char* pb = (const char*)b;
    return pa < pb + nb && pb < pa + na;
}

template <typename TIn>
static void launch_conv_f32(hipStream_t s, const TIn* x, const float* w, const ConvLayer& c, const float* resid,
                            float* y, int B, int relu_in, int relu_out)
{
    // four output channels per lane where the layer and the buffers allow 16-byte weight and activation accesses
    auto aligned = [](const void* q, size_t a) { return ((uintptr_t)q & (a - 1)) == 0; };
    const size_t per_img = (size_t)c.OH * c.OW * (c.Cout / 4), in_img = (size_t)c.H * c.W * c.Cin;
    const bool v4 = c.Cout % 4 == 0 && c.Cin % 4 == 0 && per_img < ((size_t)1 << 31) && in_img < ((size_t)1 << 31) &&
                    (size_t)c.k * c.k * c.Cin < ((size_t)1 << 24) && aligned(w + c.w_off, 16) && aligned(w + c.b_off, 16) &&
                    aligned(x, sizeof(TIn) * 4) && aligned(y, 16) && (!resid || aligned(resid, 16));
    if (v4) {
        hipLaunchKernelGGL((conv2d_f32_v4_kernel<TIn>), dim3((unsigned)((per_img + 63) / 64), (unsigned)(B < 65535 ? B : 65535)), dim3(CONV_F32_V4_WAVES * 64), 0,
                           s, x, w + c.w_off, w + c.b_off, resid, y, B, c.H, c.W, c.Cin, c.OH, c.OW, c.Cout, c.k, c.stride, c.pad, relu_in,
                           relu_out);
    } else {
        size_t total = (size_t)B * c.OH * c.OW * c.Cout * CONV_F32_KS;
        hipLaunchKernelGGL((conv2d_f32_kernel<TIn>), dim3(blocks_for(total)), dim3(256), 0, s, x, w + c.w_off, w + c.b_off,
                           resid, y, B, c.H, c.W, c.Cin, c.OH, c.OW, c.Cout, c.k, c.stride, c.pad, relu_in, relu_out);
    }
}

// fp32 torso + linear layer.  Leaves the rectified linear output in h->d_fc.
static void torso_fc_f32(seed_infer* h, hipStream_t s, int B, const uint8_t* obs)
{
    const Plan& p = h->plan;
    const float* w = h->d_w;
    float* cur = nullptr;
    if (p.arch.torso == SEED_TORSO_CONV_STACK) {
        for (size_t l = 0; l < p.convs.size(); ++l) {
            float* dst = h->d_act[l & 1];
            if (l == 0) launch_conv_f32<uint8_t>(s, obs, w, p.convs[l], nullptr, dst, B, 0, 1);
            else launch_conv_f32<float>(s, cur, w, p.convs[l], nullptr, dst, B, 0, 1);
            cur = dst;
        }
    } else {
        float* a0 = h->d_act[0];
        float* a1 = h->d_act[1];
        for (size_t si = 0; si < p.sections.size(); ++si) {
            const Section& sec = p.sections[si];
            if (si == 0) launch_conv_f32<uint8_t>(s, obs, w, sec.conv0, nullptr, a0, B, 0, 0);
            else launch_conv_f32<float>(s, a1, w, sec.conv0, nullptr, a0, B, 0, 0);
            const ConvLayer& c0 = sec.conv0;
            size_t total = (size_t)B * sec.PH * sec.PW * c0.Cout;
            hipLaunchKernelGGL(maxpool3x3s2_f32_kernel, dim3(blocks_for(total)), dim3(256), 0, s, a0, a1, B, c0.OH, c0.OW,
                               c0.Cout, sec.PH, sec.PW, sec.pool_pad_h, sec.pool_pad_w, 0);
            const bool last_sec = si + 1 == p.sections.size();
            for (int blk = 0; blk < 2; ++blk) {
                launch_conv_f32<float>(s, a1, w, sec.block[2 * blk], nullptr, a0, B, 1, 0);
                // x <- x + conv_b(ReLU(t)); the torso's closing ReLU rides on the very last block
                launch_conv_f32<float>(s, a0, w, sec.block[2 * blk + 1], a1, a1, B, 1, last_sec && blk == 1);
            }
        }
        cur = a1;
    }
    h->feat_f32 = cur;
    const seed_arch_t& a = p.arch;
    hipLaunchKernelGGL(dense_f32_kernel, dim3(B, (a.fc_units + DENSE_F32_COLS - 1) / DENSE_F32_COLS), dim3(DENSE_F32_WAVES * 64), 0, s, cur, w + p.fc_w, w + p.fc_b,
                       h->d_fc, (int)p.flat, a.fc_units, (int)p.flat, a.fc_units, 1);
}

template <int P>
static void launch_heads_p(hipStream_t s, const HeadsArgs& ha)
{
    hipLaunchKernelGGL(heads_select_kernel<P>, dim3((ha.B + 3) / 4), dim3(256), 0, s, ha);
}

// The register-resident variant for n = KS * (64 / P) * NPL inputs (NPL = 32 or 64; KS = 1, 2 or 4 wavefronts per
// row) with 16-byte aligned input rows; the choice depends on the network and the buffers' alignment only,
// never on B, so a row's result does not depend on the batch it travels in.  At most 1024 workgroups (four per
// compute unit, which hides each row's load latency): at large B every workgroup walks several rows with its weights in registers.
template <int P>
static bool launch_heads_rows(hipStream_t s, const HeadsArgs& ha)
{
    constexpr int G = 64 / P;
    const bool aligned = ((uintptr_t)ha.vec_a % 16 == 0) && ha.ld_a % 4 == 0 && ((uintptr_t)ha.vec_v % 16 == 0) && ha.ld_v % 4 == 0;
    if (!aligned || ha.n % 64 != 0) return false;
    auto go = [&](auto npl, auto ksc) {
        constexpr int NPL = decltype(npl)::value, KS = decltype(ksc)::value, RPB = 4 / KS;
        const int grid = std::min((ha.B + RPB - 1) / RPB, 1024);
        hipLaunchKernelGGL((heads_rows_kernel<P, NPL, KS>), dim3(grid), dim3(256), 0, s, ha);
    };
    using N32 = std::integral_constant<int, 32>; using N64 = std::integral_constant<int, 64>;
    using K1 = std::integral_constant<int, 1>; using K2 = std::integral_constant<int, 2>; using K4 = std::integral_constant<int, 4>;
    if (ha.n == G * 32) go(N32{}, K1{});
    else if (ha.n == G * 64) go(N64{}, K1{});
    else if (ha.n == 2 * G * 64) go(N64{}, K2{});
    else if (ha.n == 4 * G * 64) go(N64{}, K4{});
    else return false;
    return true;
}

static void launch_heads(hipStream_t s, const HeadsArgs& ha)
{
    int A = ha.A;
    if (A <= 2) launch_heads_p<2>(s, ha);
    else if (A <= 4) launch_heads_p<4>(s, ha);
    else if (A <= 8) { if (!launch_heads_rows<8>(s, ha)) launch_heads_p<8>(s, ha); }
    else if (A <= 16) { if (!launch_heads_rows<16>(s, ha)) launch_heads_p<16>(s, ha); }
    else if (A <= 32) { if (!launch_heads_rows<32>(s, ha)) launch_heads_p<32>(s, ha); }
    else launch_heads_p<64>(s, ha);
}

// Torso and linear layer over B rows (rows of the handle's linear-layer buffers).
static seed_status_t run_torso_fc(seed_infer* h, hipStream_t s, int B, const uint8_t* obs)
{
    const Plan& p = h->plan;
    const bool prof = !h->ev.empty() && h->ev_used < SEED_PROFILE_SLOTS;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    if (prof) { ev0 = h->ev[2 * h->ev_used]; ev1 = h->ev[2 * h->ev_used + 1]; ++h->ev_used; }
    if (p.arch.precision == SEED_PRECISION_FP32) {
        if (prof) HIP_TRY(h, hipEventRecord(ev0, s));
        torso_fc_f32(h, s, B, obs);
        if (prof) HIP_TRY(h, hipEventRecord(ev1, s));
        HIP_TRY(h, hipGetLastError());
        return SEED_OK;
    }
    return bf16_torso_fc(h->bf, p, h->d_w, s, B, obs, ev0, ev1, h->err);
}

// Recurrent core, heads and action selection for the B rows that start at row `row0` of the linear layer's
// output; every pointer argument already names those rows' own data.
// `phases`: CORE = the recurrent step (rows row0 .. row0 + B of the linear layer's output -> h_out, c_out), HEADS =
// dueling hidden layers, output heads and action selection on the core's output.  A T-step unroll runs CORE per
// step and HEADS once over all T * B rows (h_out then holds every step's output, row0 = 0).
enum { PHASE_CORE = 1, PHASE_HEADS = 2, PHASE_BOTH = 3 };
static seed_status_t run_core_heads(seed_infer* h, hipStream_t s, int row0, int B, const int32_t* prev_action,
                                    const float* prev_reward, const float* h_in, const float* c_in, const uint8_t* done,
                                    float* h_out, float* c_out, const float* uniforms, const float* epsilon,
                                    const float* explore_u, int32_t* action_out, float* logits_out, float* value_out,
                                    float* probs_out, int phases = PHASE_BOTH)
{
    const Plan& p = h->plan;
    const seed_arch_t& a = p.arch;
    const float* w = h->d_w;
    const bool rec = a.lstm_units > 0;
    const float* core = nullptr;       // fp32 [B, p.core]
    int ld_core = p.core;
    if (a.precision == SEED_PRECISION_FP32) {
        const float* fc = h->d_fc + (size_t)row0 * a.fc_units;
        core = fc;
        if (rec) {
            if (phases & PHASE_CORE)
                hipLaunchKernelGGL(lstm_f32_kernel, dim3(B, (a.lstm_units + 255) / 256), dim3(256), 0, s, fc, prev_action,
                                   prev_reward, h_in, c_in, w + p.lstm_w, w + p.lstm_b, h_out, c_out, B, a.fc_units,
                                   a.num_actions, a.lstm_units, done);
            core = h_out;
        }
        if (a.head == SEED_HEAD_DUELING_Q && (phases & PHASE_HEADS)) {
            int hid = a.head_hidden;
            hipLaunchKernelGGL(dense_f32_kernel, dim3(B, (hid + DENSE_F32_COLS - 1) / DENSE_F32_COLS), dim3(DENSE_F32_WAVES * 64), 0, s, core, w + p.v1_w, w + p.v1_b,
                               h->d_hid, p.core, hid, ld_core, 2 * hid, 1);
            hipLaunchKernelGGL(dense_f32_kernel, dim3(B, (hid + DENSE_F32_COLS - 1) / DENSE_F32_COLS), dim3(DENSE_F32_WAVES * 64), 0, s, core, w + p.a1_w, w + p.a1_b,
                               h->d_hid + hid, p.core, hid, ld_core, 2 * hid, 1);
        }
    } else {
        seed_status_t st = bf16_core(h->bf, p, w, s, row0, B, prev_action, prev_reward, h_in, c_in, done, h_out, c_out,
                                     h->d_hid, &core, &ld_core, h->err, (phases & PHASE_CORE) != 0, (phases & PHASE_HEADS) != 0);
        if (st != SEED_OK) return st;
    }
    if (!(phases & PHASE_HEADS)) {
        HIP_TRY(h, hipGetLastError());
        return SEED_OK;
    }

    HeadsArgs ha{};
    ha.n = p.core; ha.A = a.num_actions; ha.B = B;
    ha.uniforms = uniforms; ha.epsilon = epsilon; ha.explore_u = explore_u; ha.action = action_out; ha.logits = logits_out; ha.value = value_out; ha.probs = probs_out;
    if (a.head == SEED_HEAD_POLICY_VALUE) {
        ha.vec_a = core; ha.ld_a = ld_core; ha.vec_v = core; ha.ld_v = ld_core;
        ha.w_a = w + p.pol_w; ha.b_a = w + p.pol_b; ha.w_v = w + p.val_w; ha.b_v = w + p.val_b;
        ha.dueling = 0;
    } else {
        int hid = a.head_hidden;
        ha.n = hid;
        ha.vec_v = h->d_hid; ha.ld_v = 2 * hid; ha.vec_a = h->d_hid + hid; ha.ld_a = 2 * hid;
        ha.w_a = w + p.a2_w; ha.b_a = w + p.a2_b; ha.w_v = w + p.v2_w; ha.b_v = w + p.v2_b;
        ha.dueling = 1;
    }
    launch_heads(s, ha);
    HIP_TRY(h, hipGetLastError());
    return SEED_OK;
}

// The kernels move frames and recurrent state 16 bytes per lane.
template <class... P>
static bool misaligned16(P... ptrs)
{
    return (((uintptr_t)ptrs | ...) & 15) != 0;
}

extern "C" seed_status_t seed_infer_step(seed_infer_t* h, int32_t B, const uint8_t* obs,
                                         const int32_t* prev_action, const float* prev_reward,
                                         const float* h_in, const float* c_in, const float* uniforms,
                                         int32_t* action_out, float* logits_out, float* value_out,
                                         float* h_out, float* c_out, float* probs_out, void* hip_stream)
{
    return seed_infer_step_ext(h, B, obs, prev_action, prev_reward, h_in, c_in, uniforms, nullptr, action_out, logits_out,
                               value_out, h_out, c_out, probs_out, hip_stream);
}

// The per-step workspace pointers of a handle.
struct WorkspacePtrs {
    float* d_act[2]; float* d_fc; float* d_hid;
    __bf16* bact[2]; __bf16* lw_c0; __bf16* lw_r; __bf16* lw_u; float* lw_x;
    __bf16* feat; __bf16* fc_bf16; float* fc_f32;
};

static WorkspacePtrs workspace_get(const seed_infer* h)
{
    WorkspacePtrs w{};
    w.d_act[0] = h->d_act[0]; w.d_act[1] = h->d_act[1]; w.d_fc = h->d_fc; w.d_hid = h->d_hid;
    if (const Bf16State* b = h->bf) {
        w.bact[0] = b->act[0]; w.bact[1] = b->act[1]; w.lw_c0 = b->lw_c0; w.lw_r = b->lw_r; w.lw_u = b->lw_u; w.lw_x = b->lw_x;
        w.feat = b->feat; w.fc_bf16 = b->fc_bf16; w.fc_f32 = b->fc_f32;
    }
    return w;
}

static void workspace_set(seed_infer* h, const WorkspacePtrs& w)
{
    h->d_act[0] = w.d_act[0]; h->d_act[1] = w.d_act[1]; h->d_fc = w.d_fc; h->d_hid = w.d_hid;
    if (Bf16State* b = h->bf) {
        b->act[0] = w.bact[0]; b->act[1] = w.bact[1]; b->lw_c0 = w.lw_c0; b->lw_r = w.lw_r; b->lw_u = w.lw_u; b->lw_x = w.lw_x;
        b->feat = w.feat; b->fc_bf16 = w.fc_bf16; b->fc_f32 = w.fc_f32;
    }
}

// Lay a step's workspace for B rows out from `base` (the same pieces seed_infer_create allocates for max_batch
// rows); returns the bytes it takes.  With base == nullptr only the size is computed.
static size_t workspace_carve(const seed_infer* h, int B, char* base, WorkspacePtrs& w)
{
    const Plan& p = h->plan;
    const seed_arch_t& a = p.arch;
    const size_t rows = (size_t)B;
    size_t off = 0;
    auto take = [&](size_t bytes) { char* at = base ? base + off : nullptr; off += (bytes + 255) / 256 * 256; return at; };
    w = WorkspacePtrs{};
    if (a.head == SEED_HEAD_DUELING_Q) w.d_hid = (float*)take(rows * 2 * a.head_hidden * sizeof(float));
    if (a.precision == SEED_PRECISION_FP32) {
        w.d_act[0] = (float*)take(rows * p.max_act * sizeof(float));
        w.d_act[1] = (float*)take(rows * p.max_act * sizeof(float));
        w.d_fc = (float*)take(rows * a.fc_units * sizeof(float));
        return off;
    }
    const Bf16State* b = h->bf;
    if (a.torso == SEED_TORSO_CONV_STACK && p.convs.size() > 1 && !b->stack_fused) {
        size_t m = 0;
        for (size_t l = 0; l + 1 < p.convs.size(); ++l) m = std::max(m, (size_t)p.convs[l].OH * p.convs[l].OW * p.convs[l].Cout);
        w.bact[0] = (__bf16*)take(rows * m * 2);
        w.bact[1] = (__bf16*)take(rows * m * 2);
    }
    if (a.torso == SEED_TORSO_RESNET && b->torso_kind == TORSO_NONE) {
        size_t m0 = 0, m1 = 0;
        for (const Section& sec : p.sections) {
            m0 = std::max(m0, (size_t)sec.conv0.OH * sec.conv0.OW * sec.conv0.Cout);
            m1 = std::max(m1, (size_t)sec.PH * sec.PW * sec.conv0.Cout);
        }
        w.lw_c0 = (__bf16*)take(rows * m0 * 2);
        w.lw_r = (__bf16*)take(rows * m1 * 2);
        w.lw_u = (__bf16*)take(rows * m1 * 2);
        w.lw_x = (float*)take(rows * m1 * 4);
    }
    w.feat = (__bf16*)take(rows * b->ldf * 2);
    w.fc_bf16 = (__bf16*)take(rows * b->ldfc * 2);
    w.fc_f32 = (float*)take(rows * a.fc_units * 4);
    return off;
}

__global__ __launch_bounds__(256) void zero_fill16_kernel(uint4* __restrict__ p, size_t n16)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
        p[i] = uint4{0u, 0u, 0u, 0u};
}

static seed_status_t step_impl(seed_infer_t* h, int32_t B, const uint8_t* obs,
                               const int32_t* prev_action, const float* prev_reward,
                               const float* h_in, const float* c_in, const float* uniforms,
                               const seed_step_ext_t* ext,
                               int32_t* action_out, float* logits_out, float* value_out,
                               float* h_out, float* c_out, float* probs_out, void* hip_stream, bool static_ws)
{
    if (!h) return SEED_ERR_INVALID_ARG;
    const Plan& p = h->plan;
    const seed_arch_t& a = p.arch;
    auto fail = [&](seed_status_t st, const char* m) { h->err = m; return st; };
    if (B < 0) return fail(SEED_ERR_INVALID_ARG, "B is negative");
    if (B > a.max_batch) return fail(SEED_ERR_BATCH_TOO_LARGE, "B exceeds max_batch");
    if (B == 0) return SEED_OK;
    if (!obs || !action_out || !logits_out || !value_out) return fail(SEED_ERR_INVALID_ARG, "obs, action_out, logits_out and value_out are required");
    const bool rec = a.lstm_units > 0;
    if (rec && (!prev_action || !prev_reward || !h_in || !c_in || !h_out || !c_out))
        return fail(SEED_ERR_INVALID_ARG, "a recurrent arch needs prev_action, prev_reward, h_in, c_in, h_out and c_out");
    if (!rec && (prev_action || prev_reward || h_in || c_in || h_out || c_out))
        return fail(SEED_ERR_INVALID_ARG, "a feed-forward arch takes no recurrent arguments (pass NULL)");
    if (a.select == SEED_SELECT_GUMBEL && !uniforms) return fail(SEED_ERR_INVALID_ARG, "Gumbel-max selection needs uniforms");
    if (a.select == SEED_SELECT_GREEDY && uniforms) return fail(SEED_ERR_INVALID_ARG, "greedy selection takes no uniforms (pass NULL)");
    if (misaligned16(obs, h_in, c_in, h_out, c_out))
        return fail(SEED_ERR_INVALID_ARG, "obs, h_in, c_in, h_out and c_out must be 16-byte aligned");
    const uint8_t* done = nullptr;
    const float* epsilon = nullptr;
    const float* explore_u = nullptr;
    if (ext) {
        if (ext->struct_size != sizeof(seed_step_ext_t)) return fail(SEED_ERR_INVALID_ARG, "ext->struct_size is not sizeof(seed_step_ext_t)");
        done = ext->done; epsilon = ext->epsilon; explore_u = ext->explore_uniforms;
        if (done && !rec) return fail(SEED_ERR_INVALID_ARG, "done flags need a recurrent arch");
        if ((epsilon == nullptr) != (explore_u == nullptr)) return fail(SEED_ERR_INVALID_ARG, "epsilon and explore_uniforms must be given together");
    }
    if (rec) {
        size_t nb = (size_t)B * a.lstm_units * sizeof(float);
        if (overlaps(h_out, nb, h_in, nb) || overlaps(h_out, nb, c_in, nb) || overlaps(c_out, nb, h_in, nb) ||
            overlaps(c_out, nb, c_in, nb) || overlaps(h_out, nb, c_out, nb))
            return fail(SEED_ERR_ALIASING, "h_out / c_out must not overlap h_in / c_in or each other");
    }
    int dev = -1;
    HIP_TRY(h, hipGetDevice(&dev));
    if (dev != h->device) return fail(SEED_ERR_INVALID_ARG, "current HIP device differs from the handle's device");

    hipStream_t s = (hipStream_t)hip_stream;
    if (!static_ws) {
        seed_status_t st = run_torso_fc(h, s, B, obs);
        if (st != SEED_OK) return st;
        return run_core_heads(h, s, 0, B, prev_action, prev_reward, h_in, c_in, done, h_out, c_out, uniforms, epsilon, explore_u,
                              action_out, logits_out, value_out, probs_out);
    }
    // The same kernels on a workspace laid out in the static array.  Only host-side pointers change hands: the
    // kernels receive theirs by value at launch, and a handle is used from one thread at a time.
    WorkspacePtrs ws;
    const size_t need = workspace_carve(h, B, nullptr, ws);
    if (need > (size_t)SEED_STATIC_SCRATCH_BYTES) {
        char msg[200];
        snprintf(msg, sizeof msg, "B = %d needs %zu bytes of workspace; the static workspace holds %u (use seed_infer_step)",
                 B, need, (unsigned)SEED_STATIC_SCRATCH_BYTES);
        h->err = msg;
        return SEED_ERR_BATCH_TOO_LARGE;
    }
    void* base = nullptr;
    HIP_TRY(h, scratch_address(dev, &base));
    workspace_carve(h, B, (char*)base, ws);
    if (h->bf) {
        // rows of the feature and linear-layer matrices are padded to whole K chunks; the dense kernels read the
        // padding (against zero weights), and the array keeps whatever the previous call left there
        const Bf16State* b = h->bf;
        if ((size_t)b->ldf != p.flat) {
            const size_t n16 = ((size_t)B * b->ldf * 2 + 15) / 16;
            hipLaunchKernelGGL(zero_fill16_kernel, dim3(blocks_for(n16)), dim3(256), 0, s, (uint4*)ws.feat, n16);
        }
        if (b->ldfc != a.fc_units) {
            const size_t n16 = ((size_t)B * b->ldfc * 2 + 15) / 16;
            hipLaunchKernelGGL(zero_fill16_kernel, dim3(blocks_for(n16)), dim3(256), 0, s, (uint4*)ws.fc_bf16, n16);
        }
    }
    const WorkspacePtrs own = workspace_get(h);
    workspace_set(h, ws);
    seed_status_t st = run_torso_fc(h, s, B, obs);
    if (st == SEED_OK)
        st = run_core_heads(h, s, 0, B, prev_action, prev_reward, h_in, c_in, done, h_out, c_out, uniforms, epsilon, explore_u,
                            action_out, logits_out, value_out, probs_out);
    workspace_set(h, own);
    return st;
}

extern "C" seed_status_t seed_infer_step_ext(seed_infer_t* h, int32_t B, const uint8_t* obs,
                                             const int32_t* prev_action, const float* prev_reward,
                                             const float* h_in, const float* c_in, const float* uniforms,
                                             const seed_step_ext_t* ext,
                                             int32_t* action_out, float* logits_out, float* value_out,
                                             float* h_out, float* c_out, float* probs_out, void* hip_stream)
{
    return step_impl(h, B, obs, prev_action, prev_reward, h_in, c_in, uniforms, ext, action_out, logits_out, value_out,
                     h_out, c_out, probs_out, hip_stream, false);
}

extern "C" seed_status_t seed_infer_step_static(seed_infer_t* h, int32_t B, const uint8_t* obs,
                                                const int32_t* prev_action, const float* prev_reward,
                                                const float* h_in, const float* c_in, const float* uniforms,
                                                const seed_step_ext_t* ext,
                                                int32_t* action_out, float* logits_out, float* value_out,
                                                float* h_out, float* c_out, float* probs_out, void* hip_stream)
{
    return step_impl(h, B, obs, prev_action, prev_reward, h_in, c_in, uniforms, ext, action_out, logits_out, value_out,
                     h_out, c_out, probs_out, hip_stream, true);
}

extern "C" seed_status_t seed_infer_unroll(seed_infer_t* h, int32_t T, int32_t B, const uint8_t* obs,
                                           const int32_t* prev_action, const float* prev_reward, const uint8_t* done,
                                           const float* h0, const float* c0, const float* uniforms,
                                           int32_t* action_out, float* logits_out, float* value_out,
                                           float* h_out, float* c_out, float* probs_out, void* hip_stream)
{
    if (!h) return SEED_ERR_INVALID_ARG;
    const Plan& p = h->plan;
    const seed_arch_t& a = p.arch;
    auto fail = [&](seed_status_t st, const char* m) { h->err = m; return st; };
    if (T < 0 || B < 0) return fail(SEED_ERR_INVALID_ARG, "T or B is negative");
    if ((long long)T * B > a.max_batch) return fail(SEED_ERR_BATCH_TOO_LARGE, "T * B exceeds max_batch");
    if (T == 0 || B == 0) return SEED_OK;
    if (!obs || !action_out || !logits_out || !value_out) return fail(SEED_ERR_INVALID_ARG, "obs, action_out, logits_out and value_out are required");
    const bool rec = a.lstm_units > 0;
    if (rec && (!prev_action || !prev_reward || !h0 || !c0 || !h_out || !c_out))
        return fail(SEED_ERR_INVALID_ARG, "a recurrent arch needs prev_action, prev_reward, h0, c0, h_out and c_out");
    if (!rec && (prev_action || prev_reward || done || h0 || c0 || h_out || c_out))
        return fail(SEED_ERR_INVALID_ARG, "a feed-forward arch takes no recurrent arguments (pass NULL)");
    if (a.select == SEED_SELECT_GUMBEL && !uniforms) return fail(SEED_ERR_INVALID_ARG, "Gumbel-max selection needs uniforms");
    if (a.select == SEED_SELECT_GREEDY && uniforms) return fail(SEED_ERR_INVALID_ARG, "greedy selection takes no uniforms (pass NULL)");
    if (misaligned16(obs, h0, c0, h_out, c_out))
        return fail(SEED_ERR_INVALID_ARG, "obs, h0, c0, h_out and c_out must be 16-byte aligned");
    if (rec) {
        size_t nb = (size_t)B * a.lstm_units * sizeof(float);
        if (overlaps(h_out, nb, h0, nb) || overlaps(h_out, nb, c0, nb) || overlaps(c_out, nb, h0, nb) ||
            overlaps(c_out, nb, c0, nb) || overlaps(h_out, nb, c_out, nb))
            return fail(SEED_ERR_ALIASING, "h_out / c_out must not overlap h0 / c0 or each other");
    }
    int dev = -1;
    HIP_TRY(h, hipGetDevice(&dev));
    if (dev != h->device) return fail(SEED_ERR_INVALID_ARG, "current HIP device differs from the handle's device");

    hipStream_t s = (hipStream_t)hip_stream;
    // the torso and the linear layer do not depend on time: one pass over all T * B frames
    seed_status_t st = run_torso_fc(h, s, T * B, obs);
    if (st != SEED_OK) return st;
    const size_t A = (size_t)a.num_actions, Hn = (size_t)a.lstm_units, mb = (size_t)a.max_batch;
    if (!rec) {
        // nothing depends on time: heads and selection over all T * B rows at once
        return run_core_heads(h, s, 0, T * B, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, uniforms, nullptr,
                              nullptr, action_out, logits_out, value_out, probs_out);
    }
    // Only the recurrent core is sequential.  Step t reads h_{t-1} from, and writes h_t to, rows t * B .. of one
    // [T * B, units] buffer (the first quarter of d_roll); c alternates between two [B, units] buffers behind it
    // and the last step writes the caller's.  The dueling hidden layers, the heads and the selection then run
    // once over all T * B rows of that buffer instead of T times over B.
    float* hseq = h->d_roll;
    float* cb[2] = {h->d_roll + mb * Hn, h->d_roll + 2 * mb * Hn};
    for (int t = 0; t < T; ++t) {
        const size_t r = (size_t)t * B;
        st = run_core_heads(h, s, (int)r, B, prev_action + r, prev_reward + r, t == 0 ? h0 : hseq + (r - B) * Hn,
                            t == 0 ? c0 : cb[(t - 1) & 1], done ? done + r : nullptr, hseq + r * Hn,
                            t == T - 1 ? c_out : cb[t & 1], nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, PHASE_CORE);
        if (st != SEED_OK) return st;
    }
    HIP_TRY(h, hipMemcpyAsync(h_out, hseq + (size_t)(T - 1) * B * Hn, (size_t)B * Hn * sizeof(float), hipMemcpyDeviceToDevice, s));
    return run_core_heads(h, s, 0, T * B, nullptr, nullptr, nullptr, nullptr, nullptr, hseq, nullptr, uniforms, nullptr, nullptr,
                          action_out, logits_out, value_out, probs_out, PHASE_HEADS);
}

extern "C" seed_status_t seed_infer_set_weights(seed_infer_t* h, const float* weights_host, size_t n_weights,
                                                void* hip_stream)
{
    if (!h) return SEED_ERR_INVALID_ARG;
    const Plan& p = h->plan;
    auto fail = [&](seed_status_t st, const char* m) { h->err = m; return st; };
    if (!weights_host) return fail(SEED_ERR_INVALID_ARG, "weights_host is NULL");
    if (n_weights != p.n_weights) return fail(SEED_ERR_INVALID_ARG, "n_weights does not match the handle's arch");
    int dev = -1;
    HIP_TRY(h, hipGetDevice(&dev));
    if (dev != h->device) return fail(SEED_ERR_INVALID_ARG, "current HIP device differs from the handle's device");
    hipStream_t s = (hipStream_t)hip_stream;
    // two staging buffers, used alternately: the upload of the update before the previous one may still be
    // reading this one
    const int sb = h->stage_next;
    HIP_TRY(h, hipEventSynchronize(h->staged[sb]));
    const int idle = 1 - h->active;
    const size_t wb = p.n_weights * sizeof(float);
    pool_memcpy(host_pool(h), h->staging[sb], weights_host, wb);
    // The update runs on the handle's own stream.  The idle copy was last read by the steps enqueued before the
    // PREVIOUS update made it idle (an event on the caller's stream marks that point), so the upload need not wait
    // for the steps enqueued since, which read the active copy: it runs beside them.
    hipStream_t up = h->up_stream;
    if (h->retired_set[idle]) HIP_TRY(h, hipStreamWaitEvent(up, h->retired[idle], 0));
    HIP_TRY(h, hipMemcpyAsync(h->d_w_set[idle], h->staging[sb], wb, hipMemcpyHostToDevice, up));
    HIP_TRY(h, hipEventRecord(h->staged[sb], up));
    h->stage_next = 1 - sb;
    if (h->bf) {
        // the matrix-core kernels' operand layouts are a fixed gather of the flat vector: packed on the device
        bf16_repack(h->bf, h->d_w_set[idle], idle, up);
        HIP_TRY(h, hipGetLastError());
    }
    HIP_TRY(h, hipEventRecord(h->uploaded[idle], up));
    // what the caller enqueues from here on waits for the update; the copy that was active until now retires here
    HIP_TRY(h, hipStreamWaitEvent(s, h->uploaded[idle], 0));
    HIP_TRY(h, hipEventRecord(h->retired[h->active], s));
    h->retired_set[h->active] = true;
    // every piece of the update is enqueued: steps enqueued from here on read the new set
    if (h->bf) h->bf->active = idle;
    h->active = idle;
    h->d_w = h->d_w_set[idle];
    return SEED_OK;
}

extern "C" seed_status_t seed_infer_read_intermediate(seed_infer_t* h, int32_t which, int32_t B, float* dst,
                                                      size_t capacity, void* hip_stream)
{
    if (!h) return SEED_ERR_INVALID_ARG;
    const Plan& p = h->plan;
    auto fail = [&](seed_status_t st, const char* m) { h->err = m; return st; };
    if (!dst || B <= 0 || B > p.arch.max_batch) return fail(SEED_ERR_INVALID_ARG, "bad dst or B");
    if (which != 0 && which != 1) return fail(SEED_ERR_INVALID_ARG, "which must be 0 or 1");
    size_t n = (size_t)B * (which == 0 ? p.flat : (size_t)p.arch.fc_units);
    if (capacity < n) return fail(SEED_ERR_INVALID_ARG, "dst too small");
    hipStream_t s = (hipStream_t)hip_stream;
    if (p.arch.precision == SEED_PRECISION_FP32) {
        const float* src = which == 0 ? h->feat_f32 : h->d_fc;
        if (!src) return fail(SEED_ERR_INVALID_ARG, "no step has run yet");
        hipLaunchKernelGGL(copy_f32_kernel, dim3(blocks_for(n)), dim3(256), 0, s, src, dst, n);
    } else {
        seed_status_t st = bf16_read_intermediate(h->bf, p, which, B, dst, s, h->err);
        if (st != SEED_OK) return st;
    }
    HIP_TRY(h, hipGetLastError());
    return SEED_OK;
}

extern "C" seed_status_t seed_infer_set_profiling(seed_infer_t* h, int32_t enable)
{
    if (!h) return SEED_ERR_INVALID_ARG;
    if (enable && h->ev.empty()) {
        h->ev.reserve(2 * SEED_PROFILE_SLOTS);
        for (int i = 0; i < 2 * SEED_PROFILE_SLOTS; ++i) {
            hipEvent_t e;
            HIP_TRY(h, hipEventCreate(&e));
            h->ev.push_back(e);
        }
    } else if (!enable) {
        for (hipEvent_t e : h->ev) (void)hipEventDestroy(e);
        h->ev.clear();
    }
    h->ev_used = 0;
    return SEED_OK;
}

extern "C" seed_status_t seed_infer_profile_read(seed_infer_t* h, float* torso_ms_sum, int32_t* n_steps)
{
    if (!h || !torso_ms_sum || !n_steps) return SEED_ERR_INVALID_ARG;
    float sum = 0.f;
    for (int i = 0; i < h->ev_used; ++i) {
        HIP_TRY(h, hipEventSynchronize(h->ev[2 * i + 1]));
        float ms = 0.f;
        HIP_TRY(h, hipEventElapsedTime(&ms, h->ev[2 * i], h->ev[2 * i + 1]));
        sum += ms;
    }
    *torso_ms_sum = sum;
    *n_steps = h->ev_used;
    h->ev_used = 0;
    return SEED_OK;
}
#include "batcher.h"
