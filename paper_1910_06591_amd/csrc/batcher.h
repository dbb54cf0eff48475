// Host batching front-end: staging, state gather/scatter and the pipelined
// round (copy stream + compute stream).  Included at the end of seedinf.hip.
#pragma once

namespace seedinf {

// rows of `table` picked by `idx` -> dense rows of `out` (one thread per element)
__global__ __launch_bounds__(256) void gather_rows_kernel(const float* __restrict__ table, const int32_t* __restrict__ idx,
                                                          float* __restrict__ out, int rows, int width)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (long)rows * width) return;
    const int r = (int)(i / width), c = (int)(i % width);
    out[i] = table[(size_t)idx[r] * width + c];
}

__global__ __launch_bounds__(256) void scatter_rows_kernel(const float* __restrict__ in, const int32_t* __restrict__ idx,
                                                           float* __restrict__ table, int rows, int width)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (long)rows * width) return;
    const int r = (int)(i / width), c = (int)(i % width);
    table[(size_t)idx[r] * width + c] = in[i];
}

__global__ __launch_bounds__(256) void gather_i32_kernel(const int32_t* __restrict__ table, const int32_t* __restrict__ idx,
                                                         int32_t* __restrict__ out, int rows)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < rows) out[i] = table[idx[i]];
}

__global__ __launch_bounds__(256) void scatter_i32_kernel(const int32_t* __restrict__ in, const int32_t* __restrict__ idx,
                                                          int32_t* __restrict__ table, int rows)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < rows) table[idx[i]] = in[i];
}

}  // namespace seedinf

struct seed_batcher {
    seed_infer* h = nullptr;
    int n_actors = 0, max_rows = 0, A = 0, Hn = 0;
    size_t frame = 0;
    hipStream_t copy_s = nullptr, comp_s = nullptr;
    // per-actor device state
    float* st_h = nullptr; float* st_c = nullptr; int32_t* st_action = nullptr;
    struct Set {
        // pinned host staging
        uint8_t* obs = nullptr; float* reward = nullptr; uint8_t* done = nullptr; int32_t* actor = nullptr;
        float* uniforms = nullptr; float* epsilon = nullptr; float* explore = nullptr; int32_t* actions = nullptr;
        // device mirrors and per-batch work buffers
        uint8_t* d_obs = nullptr; float* d_reward = nullptr; uint8_t* d_done = nullptr; int32_t* d_actor = nullptr;
        float* d_uniforms = nullptr; float* d_epsilon = nullptr; float* d_explore = nullptr;
        int32_t* d_prev_action = nullptr; int32_t* d_actions = nullptr;
        float* d_h_in = nullptr; float* d_c_in = nullptr; float* d_h_out = nullptr; float* d_c_out = nullptr;
        float* d_logits = nullptr; float* d_value = nullptr;
        hipEvent_t copied = nullptr, finished = nullptr;
        int rows = 0;                   // rows added to the batch being filled
        int result_rows = 0;            // rows of the submitted batch `ticket`
        int ticket = -1;
        bool in_flight = false;
    } set[2];
    int fill = 0;                       // staging set being filled
    int next_ticket = 0;
    std::vector<int32_t> seen;          // per actor: ticket of the batch it was last added to
    std::string err;
};

#define B_TRY(b, expr)                                                                \
    do {                                                                              \
        hipError_t e_ = (expr);                                                       \
        if (e_ != hipSuccess) {                                                       \
            (b)->err = std::string(#expr) + ": " + hipGetErrorString(e_);             \
            return e_ == hipErrorOutOfMemory ? SEED_ERR_OOM : SEED_ERR_DEVICE;        \
        }                                                                             \
    } while (0)

static void batcher_free(seed_batcher* b)
{
    if (!b) return;
    if (b->comp_s) (void)hipStreamSynchronize(b->comp_s);
    if (b->copy_s) (void)hipStreamSynchronize(b->copy_s);
    for (auto& s : b->set) {
        void* host[] = {s.obs, s.reward, s.done, s.actor, s.uniforms, s.epsilon, s.explore, s.actions};
        for (void* p : host) if (p) (void)hipHostFree(p);
        void* dev[] = {s.d_obs, s.d_reward, s.d_done, s.d_actor, s.d_uniforms, s.d_epsilon, s.d_explore, s.d_prev_action,
                       s.d_actions, s.d_h_in, s.d_c_in, s.d_h_out, s.d_c_out, s.d_logits, s.d_value};
        for (void* p : dev) if (p) (void)hipFree(p);
        if (s.copied) (void)hipEventDestroy(s.copied);
        if (s.finished) (void)hipEventDestroy(s.finished);
    }
    if (b->st_h) (void)hipFree(b->st_h);
    if (b->st_c) (void)hipFree(b->st_c);
    if (b->st_action) (void)hipFree(b->st_action);
    if (b->copy_s) (void)hipStreamDestroy(b->copy_s);
    if (b->comp_s) (void)hipStreamDestroy(b->comp_s);
    delete b;
}

static seed_status_t batcher_alloc(seed_batcher* b)
{
    const size_t R = (size_t)b->max_rows, A = (size_t)b->A, Hn = (size_t)b->Hn, N = (size_t)b->n_actors;
    B_TRY(b, hipStreamCreateWithFlags(&b->copy_s, hipStreamNonBlocking));
    B_TRY(b, hipStreamCreateWithFlags(&b->comp_s, hipStreamNonBlocking));
    B_TRY(b, hipMalloc(&b->st_action, N * sizeof(int32_t)));
    B_TRY(b, hipMemset(b->st_action, 0, N * sizeof(int32_t)));
    if (Hn) {
        B_TRY(b, hipMalloc(&b->st_h, N * Hn * sizeof(float)));
        B_TRY(b, hipMalloc(&b->st_c, N * Hn * sizeof(float)));
        B_TRY(b, hipMemset(b->st_h, 0, N * Hn * sizeof(float)));
        B_TRY(b, hipMemset(b->st_c, 0, N * Hn * sizeof(float)));
    }
    for (auto& s : b->set) {
        B_TRY(b, hipHostMalloc((void**)&s.obs, R * b->frame, hipHostMallocDefault));
        B_TRY(b, hipHostMalloc((void**)&s.reward, R * sizeof(float), hipHostMallocDefault));
        B_TRY(b, hipHostMalloc((void**)&s.done, R, hipHostMallocDefault));
        B_TRY(b, hipHostMalloc((void**)&s.actor, R * sizeof(int32_t), hipHostMallocDefault));
        B_TRY(b, hipHostMalloc((void**)&s.uniforms, R * A * sizeof(float), hipHostMallocDefault));
        B_TRY(b, hipHostMalloc((void**)&s.epsilon, R * sizeof(float), hipHostMallocDefault));
        B_TRY(b, hipHostMalloc((void**)&s.explore, R * 2 * sizeof(float), hipHostMallocDefault));
        B_TRY(b, hipHostMalloc((void**)&s.actions, R * sizeof(int32_t), hipHostMallocDefault));
        B_TRY(b, hipMalloc(&s.d_obs, R * b->frame));
        B_TRY(b, hipMalloc(&s.d_reward, R * sizeof(float)));
        B_TRY(b, hipMalloc(&s.d_done, R));
        B_TRY(b, hipMalloc(&s.d_actor, R * sizeof(int32_t)));
        B_TRY(b, hipMalloc(&s.d_uniforms, R * A * sizeof(float)));
        B_TRY(b, hipMalloc(&s.d_epsilon, R * sizeof(float)));
        B_TRY(b, hipMalloc(&s.d_explore, R * 2 * sizeof(float)));
        B_TRY(b, hipMalloc(&s.d_prev_action, R * sizeof(int32_t)));
        B_TRY(b, hipMalloc(&s.d_actions, R * sizeof(int32_t)));
        B_TRY(b, hipMalloc(&s.d_logits, R * A * sizeof(float)));
        B_TRY(b, hipMalloc(&s.d_value, R * sizeof(float)));
        if (Hn) {
            B_TRY(b, hipMalloc(&s.d_h_in, R * Hn * sizeof(float)));
            B_TRY(b, hipMalloc(&s.d_c_in, R * Hn * sizeof(float)));
            B_TRY(b, hipMalloc(&s.d_h_out, R * Hn * sizeof(float)));
            B_TRY(b, hipMalloc(&s.d_c_out, R * Hn * sizeof(float)));
        }
        B_TRY(b, hipEventCreateWithFlags(&s.copied, hipEventDisableTiming));
        B_TRY(b, hipEventCreateWithFlags(&s.finished, hipEventDisableTiming));
    }
    B_TRY(b, hipDeviceSynchronize());
    return SEED_OK;
}

extern "C" seed_status_t seed_batcher_create(seed_infer_t* h, int32_t n_actors, seed_batcher_t** out)
{
    g_create_err.clear();
    if (!h || !out) { g_create_err = "handle or out is NULL"; return SEED_ERR_INVALID_ARG; }
    if (n_actors <= 0 || n_actors > (1 << 24)) { g_create_err = "n_actors must be in 1..2^24"; return SEED_ERR_INVALID_ARG; }
    seed_batcher* b = new (std::nothrow) seed_batcher;
    if (!b) { g_create_err = "host allocation failed"; return SEED_ERR_OOM; }
    const seed_arch_t& a = h->plan.arch;
    b->h = h; b->n_actors = n_actors; b->max_rows = a.max_batch; b->A = a.num_actions; b->Hn = a.lstm_units;
    b->frame = (size_t)a.obs_h * a.obs_w * a.obs_c;
    b->seen.assign((size_t)n_actors, -1);
    seed_status_t st = batcher_alloc(b);
    if (st != SEED_OK) { g_create_err = b->err; batcher_free(b); return st; }
    *out = b;
    return SEED_OK;
}

extern "C" void seed_batcher_destroy(seed_batcher_t* b) { batcher_free(b); }
extern "C" const char* seed_batcher_last_error(const seed_batcher_t* b) { return b ? b->err.c_str() : g_create_err.c_str(); }
extern "C" void* seed_batcher_stream(seed_batcher_t* b) { return b ? (void*)b->comp_s : nullptr; }

extern "C" seed_status_t seed_batcher_reserve(seed_batcher_t* b, int32_t actor, float prev_reward, uint8_t done,
                                              uint8_t** obs_slot)
{
    if (!b) return SEED_ERR_INVALID_ARG;
    auto fail = [&](seed_status_t st, const char* m) { b->err = m; return st; };
    if (!obs_slot) return fail(SEED_ERR_INVALID_ARG, "obs_slot is NULL");
    if (actor < 0 || actor >= b->n_actors) return fail(SEED_ERR_INVALID_ARG, "actor out of range");
    seed_batcher::Set& s = b->set[b->fill];
    if (s.in_flight) {
        // this staging set's earlier batch must have left the host buffers before they are overwritten
        B_TRY(b, hipEventSynchronize(s.finished));
        s.in_flight = false;
        s.rows = 0;
        s.ticket = -1;                  // its results were never collected and are about to be overwritten
    }
    if (s.rows >= b->max_rows) return fail(SEED_ERR_BATCH_TOO_LARGE, "the batch already holds max_batch rows");
    if (b->seen[actor] == b->next_ticket) return fail(SEED_ERR_INVALID_ARG, "actor added twice to one batch");
    b->seen[actor] = b->next_ticket;
    const int r = s.rows++;
    s.reward[r] = prev_reward;
    s.done[r] = done;
    s.actor[r] = actor;
    *obs_slot = s.obs + (size_t)r * b->frame;
    return SEED_OK;
}

extern "C" seed_status_t seed_batcher_add(seed_batcher_t* b, int32_t actor, const uint8_t* obs_host, float prev_reward,
                                          uint8_t done)
{
    if (!b) return SEED_ERR_INVALID_ARG;
    if (!obs_host) { b->err = "obs_host is NULL"; return SEED_ERR_INVALID_ARG; }
    uint8_t* slot = nullptr;
    seed_status_t st = seed_batcher_reserve(b, actor, prev_reward, done, &slot);
    if (st == SEED_OK) memcpy(slot, obs_host, b->frame);
    return st;
}

extern "C" seed_status_t seed_batcher_add_many(seed_batcher_t* b, int32_t n, const int32_t* actors, const uint8_t* obs_host,
                                               const float* prev_rewards, const uint8_t* dones)
{
    if (!b) return SEED_ERR_INVALID_ARG;
    if (n < 0 || !actors || !obs_host || !prev_rewards || !dones) { b->err = "n is negative or a pointer is NULL"; return SEED_ERR_INVALID_ARG; }
    std::vector<uint8_t*> slot((size_t)n);
    int32_t ok = 0;
    seed_status_t st = SEED_OK;
    for (; ok < n; ++ok) {
        st = seed_batcher_reserve(b, actors[ok], prev_rewards[ok], dones[ok], &slot[ok]);
        if (st != SEED_OK) break;
    }
    // the frame copies are the expensive part: large batches go over the handle's persistent host threads, in
    // pieces of about a megabyte
    const int32_t per = (int32_t)std::max<size_t>(1, ((size_t)1 << 20) / b->frame);
    const int pieces = (ok + per - 1) / per;
    auto copy = [&](int t) {
        const int32_t i1 = std::min(ok, (t + 1) * per);
        for (int32_t i = t * per; i < i1; ++i) memcpy(slot[i], obs_host + (size_t)i * b->frame, b->frame);
    };
    HostPool* pool = pieces > 1 ? host_pool(b->h) : nullptr;
    if (pool) pool->run(pieces, copy);
    else for (int t = 0; t < pieces; ++t) copy(t);
    return st;
}

extern "C" seed_status_t seed_batcher_submit(seed_batcher_t* b, const float* uniforms_host, const float* epsilon_host,
                                             const float* explore_host, int32_t* ticket)
{
    if (!b || !ticket) return SEED_ERR_INVALID_ARG;
    auto fail = [&](seed_status_t st, const char* m) { b->err = m; return st; };
    seed_batcher::Set& s = b->set[b->fill];
    const seed_arch_t& a = b->h->plan.arch;
    const int R = s.rows;
    if (R == 0) return fail(SEED_ERR_INVALID_ARG, "the batch is empty");
    if (a.select == SEED_SELECT_GUMBEL && !uniforms_host) return fail(SEED_ERR_INVALID_ARG, "Gumbel-max selection needs uniforms");
    if (a.select == SEED_SELECT_GREEDY && uniforms_host) return fail(SEED_ERR_INVALID_ARG, "greedy selection takes no uniforms (pass NULL)");
    if ((epsilon_host == nullptr) != (explore_host == nullptr)) return fail(SEED_ERR_INVALID_ARG, "epsilon and explore_uniforms must be given together");
    const size_t A = (size_t)b->A, Hn = (size_t)b->Hn;
    if (uniforms_host) memcpy(s.uniforms, uniforms_host, R * A * sizeof(float));
    if (epsilon_host) {
        memcpy(s.epsilon, epsilon_host, R * sizeof(float));
        memcpy(s.explore, explore_host, R * 2 * sizeof(float));
    }
    // host -> device on the copy stream (overlaps the previous batch's compute)
    hipStream_t cs = b->copy_s, ks = b->comp_s;
    B_TRY(b, hipMemcpyAsync(s.d_obs, s.obs, R * b->frame, hipMemcpyHostToDevice, cs));
    B_TRY(b, hipMemcpyAsync(s.d_reward, s.reward, R * sizeof(float), hipMemcpyHostToDevice, cs));
    B_TRY(b, hipMemcpyAsync(s.d_done, s.done, R, hipMemcpyHostToDevice, cs));
    B_TRY(b, hipMemcpyAsync(s.d_actor, s.actor, R * sizeof(int32_t), hipMemcpyHostToDevice, cs));
    if (uniforms_host) B_TRY(b, hipMemcpyAsync(s.d_uniforms, s.uniforms, R * A * sizeof(float), hipMemcpyHostToDevice, cs));
    if (epsilon_host) {
        B_TRY(b, hipMemcpyAsync(s.d_epsilon, s.epsilon, R * sizeof(float), hipMemcpyHostToDevice, cs));
        B_TRY(b, hipMemcpyAsync(s.d_explore, s.explore, R * 2 * sizeof(float), hipMemcpyHostToDevice, cs));
    }
    B_TRY(b, hipEventRecord(s.copied, cs));
    B_TRY(b, hipStreamWaitEvent(ks, s.copied, 0));
    // compute stream: gather state, step, scatter state, actions back
    const bool rec = Hn > 0;
    if (rec) {
        const unsigned nb = (unsigned)((R * Hn + 255) / 256);
        hipLaunchKernelGGL(gather_rows_kernel, dim3(nb), dim3(256), 0, ks, b->st_h, s.d_actor, s.d_h_in, R, (int)Hn);
        hipLaunchKernelGGL(gather_rows_kernel, dim3(nb), dim3(256), 0, ks, b->st_c, s.d_actor, s.d_c_in, R, (int)Hn);
        hipLaunchKernelGGL(gather_i32_kernel, dim3((R + 255) / 256), dim3(256), 0, ks, b->st_action, s.d_actor, s.d_prev_action, R);
    }
    seed_step_ext_t ext{};
    ext.struct_size = sizeof(ext);
    ext.done = rec ? s.d_done : nullptr;
    ext.epsilon = epsilon_host ? s.d_epsilon : nullptr;
    ext.explore_uniforms = epsilon_host ? s.d_explore : nullptr;
    seed_status_t st = seed_infer_step_ext(b->h, R, s.d_obs, rec ? s.d_prev_action : nullptr, rec ? s.d_reward : nullptr,
                                           rec ? s.d_h_in : nullptr, rec ? s.d_c_in : nullptr,
                                           uniforms_host ? s.d_uniforms : nullptr, &ext, s.d_actions, s.d_logits, s.d_value,
                                           rec ? s.d_h_out : nullptr, rec ? s.d_c_out : nullptr, nullptr, ks);
    if (st != SEED_OK) { b->err = b->h->err; return st; }
    if (rec) {
        const unsigned nb = (unsigned)((R * Hn + 255) / 256);
        hipLaunchKernelGGL(scatter_rows_kernel, dim3(nb), dim3(256), 0, ks, s.d_h_out, s.d_actor, b->st_h, R, (int)Hn);
        hipLaunchKernelGGL(scatter_rows_kernel, dim3(nb), dim3(256), 0, ks, s.d_c_out, s.d_actor, b->st_c, R, (int)Hn);
    }
    hipLaunchKernelGGL(scatter_i32_kernel, dim3((R + 255) / 256), dim3(256), 0, ks, s.d_actions, s.d_actor, b->st_action, R);
    B_TRY(b, hipMemcpyAsync(s.actions, s.d_actions, R * sizeof(int32_t), hipMemcpyDeviceToHost, ks));
    B_TRY(b, hipEventRecord(s.finished, ks));
    B_TRY(b, hipGetLastError());
    s.ticket = b->next_ticket;
    s.result_rows = R;
    s.in_flight = true;
    *ticket = b->next_ticket++;
    b->fill ^= 1;
    // the set that is filled next starts empty; if its own batch is still in flight the first add waits for it
    seed_batcher::Set& n = b->set[b->fill];
    if (!n.in_flight) n.rows = 0;
    return SEED_OK;
}

extern "C" seed_status_t seed_batcher_wait(seed_batcher_t* b, int32_t ticket, int32_t* actions_out, int32_t capacity,
                                           int32_t* n_rows)
{
    if (!b || !actions_out || !n_rows) return SEED_ERR_INVALID_ARG;
    auto fail = [&](seed_status_t st, const char* m) { b->err = m; return st; };
    for (auto& s : b->set) {
        if (s.ticket != ticket) continue;
        if (capacity < s.result_rows) return fail(SEED_ERR_INVALID_ARG, "actions_out is too small");
        B_TRY(b, hipEventSynchronize(s.finished));
        memcpy(actions_out, s.actions, (size_t)s.result_rows * sizeof(int32_t));
        *n_rows = s.result_rows;
        if (s.in_flight) {              // finished: the set may be refilled
            s.in_flight = false;
            s.rows = 0;
        }
        return SEED_OK;
    }
    return fail(SEED_ERR_INVALID_ARG, "unknown ticket (only the two most recent batches can be waited for)");
}

extern "C" seed_status_t seed_batcher_read_state(seed_batcher_t* b, int32_t actor, float* h_host, float* c_host)
{
    if (!b || !h_host || !c_host) return SEED_ERR_INVALID_ARG;
    auto fail = [&](seed_status_t st, const char* m) { b->err = m; return st; };
    if (b->Hn == 0) return fail(SEED_ERR_INVALID_ARG, "a feed-forward arch has no recurrent state");
    if (actor < 0 || actor >= b->n_actors) return fail(SEED_ERR_INVALID_ARG, "actor out of range");
    B_TRY(b, hipStreamSynchronize(b->comp_s));
    const size_t nb = (size_t)b->Hn * sizeof(float);
    B_TRY(b, hipMemcpy(h_host, b->st_h + (size_t)actor * b->Hn, nb, hipMemcpyDeviceToHost));
    B_TRY(b, hipMemcpy(c_host, b->st_c + (size_t)actor * b->Hn, nb, hipMemcpyDeviceToHost));
    return SEED_OK;
}
