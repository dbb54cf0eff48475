/*
 * seedinf.h -- C ABI of libseedinf: SEED RL's central batched inference step
 * on one MI355X (gfx950).
 *
 * The operation (Section 3, "Detailed Learner architecture"): an inference
 * thread holds a batch of observations, previous rewards and per-actor
 * recurrent states gathered from many actors; one call runs the agent network
 * forward on the whole batch and returns the selected actions and the new
 * recurrent states.  Network families: the R2D2 conv stack + linear + LSTM +
 * dueling heads (Appendix A.3.1), and the deep ResNet torso the paper names
 * for DeepMind Lab (Section 4.1) and Football (Section 4.2) with a linear
 * layer, an optional LSTM core and policy/value heads.
 *
 * Conventions
 *   - "device" pointers are HIP device memory on the device that was current
 *     when the handle was created; "host" pointers are ordinary host memory.
 *   - All arrays are dense, row-major, C order.  Activations are NHWC;
 *     convolution kernels are [kh][kw][cin][cout]; dense matrices are
 *     [in][out].
 *   - Every function returns a seed_status_t (except where noted); nothing
 *     throws or aborts across this boundary.  On an error return no output
 *     array has been written.
 *   - The caller owns every pointer it passes.  The library owns the handle,
 *     its repacked copy of the weights and a workspace sized for max_batch.
 *   - One handle is used from one host thread and one stream at a time.
 */
#ifndef SEEDINF_H
#define SEEDINF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct seed_infer seed_infer_t; /* opaque */

typedef enum {
    SEED_OK = 0,
    SEED_ERR_INVALID_ARG = 1,      /* null pointer, bad size, bad field value */
    SEED_ERR_UNSUPPORTED_ARCH = 2, /* a network this build has no kernels for */
    SEED_ERR_BATCH_TOO_LARGE = 3,  /* B > max_batch given at creation */
    SEED_ERR_ALIASING = 4,         /* an output overlaps an input it must not */
    SEED_ERR_DEVICE = 5,           /* a HIP runtime call failed (see last_error) */
    SEED_ERR_OOM = 6               /* device or host allocation failed */
} seed_status_t;

enum { SEED_TORSO_CONV_STACK = 0, SEED_TORSO_RESNET = 1 };
enum { SEED_HEAD_POLICY_VALUE = 0, SEED_HEAD_DUELING_Q = 1 };
enum { SEED_SELECT_GREEDY = 0, SEED_SELECT_GUMBEL = 1 };
enum { SEED_PRECISION_FP32 = 0, SEED_PRECISION_BF16 = 1 };

#define SEED_MAX_LAYERS 4
#define SEED_MAX_ACTIONS 64

/*
 * Network description (plain data; set struct_size = sizeof(seed_arch_t)).
 *
 * torso == SEED_TORSO_CONV_STACK (Appendix A.3.1): n_conv layers of
 *   conv(conv_k[i] x conv_k[i], stride conv_stride[i], "valid" padding,
 *   conv_ch[i] filters) + ReLU; then flatten (h, w, c order), a linear layer of
 *   fc_units, ReLU.
 * torso == SEED_TORSO_RESNET (the model Sections 4.1 / 4.2 name): n_sections
 *   sections; section s is conv 3x3 SAME to section_ch[s] channels (no ReLU),
 *   max-pool 3x3 stride 2 SAME (window cells outside the image are ignored;
 *   odd total padding puts the extra cell after), then two residual blocks
 *   x + conv3x3(ReLU(conv3x3(ReLU(x)))); after the last section ReLU, flatten,
 *   linear fc_units, ReLU.
 * lstm_units > 0 (Appendix A.3.1): an LSTM step whose input is
 *   [linear output, one-hot(prev_action, num_actions), prev_reward];
 *   gate columns ordered input | forget | cell | output; no peepholes.
 * head == SEED_HEAD_POLICY_VALUE: logits[num_actions] and a scalar value, both
 *   linear in the core output.  head == SEED_HEAD_DUELING_Q (Section 3.2,
 *   Appendix A.3.1): value and advantage streams, each linear(head_hidden) +
 *   ReLU + linear; Q = V + Adv - mean(Adv).
 * select: greedy argmax (lowest index wins ties) or Gumbel-max sampling
 *   argmax_j(logit_j - log(-log(u_j))) with caller-supplied uniforms, which
 *   draws from softmax(logits) ("sampled actions", Section 3).
 * precision: SEED_PRECISION_FP32 computes everything in fp32.
 *   SEED_PRECISION_BF16 feeds bf16 operands to the matrix cores with fp32
 *   accumulation; the residual stream, LSTM gate math, cell state, heads and
 *   selection stay fp32.  Inputs and outputs have the same types in both.
 */
typedef struct {
    uint32_t struct_size;
    int32_t obs_h, obs_w, obs_c;
    int32_t torso;
    int32_t n_conv;
    int32_t conv_ch[SEED_MAX_LAYERS], conv_k[SEED_MAX_LAYERS], conv_stride[SEED_MAX_LAYERS];
    int32_t n_sections;
    int32_t section_ch[SEED_MAX_LAYERS];
    int32_t fc_units;
    int32_t lstm_units;   /* 0 = no recurrent core */
    int32_t num_actions;  /* 1 .. SEED_MAX_ACTIONS */
    int32_t head;
    int32_t head_hidden;  /* dueling hidden width; ignored for policy/value */
    int32_t select;
    int32_t precision;
    int32_t max_batch;    /* largest B seed_infer_step will be called with */
} seed_arch_t;

/*
 * Length of the canonical flat fp32 weight vector for `arch`, or 0 if the
 * arch is invalid.  Order: per conv W[kh][kw][cin][cout] then b[cout], layers
 * in forward order (ResNet section: conv0, block1.a, block1.b, block2.a,
 * block2.b); linear W[in][out], b; LSTM W[(fc_units+num_actions+1)+lstm_units]
 * [4*lstm_units] with rows [linear features | action rows | reward row | h rows]
 * and column blocks [i|f|g|o], then b[4*lstm_units]; heads: policy W[n][A], b[A],
 * value W[n][1], b[1]; or dueling value W1[n][hid], b1, W2[hid][1], b2, then
 * advantage W1[n][hid], b1, W2[hid][A], b2.  Host-only; touches no device.
 */
size_t seed_infer_weight_count(const seed_arch_t* arch);

/*
 * Validate `arch` without touching a device.  Returns SEED_OK,
 * SEED_ERR_INVALID_ARG (null, wrong struct_size, non-positive sizes, a conv
 * that does not fit its input, ...) or SEED_ERR_UNSUPPORTED_ARCH (valid in
 * principle but outside the shapes the kernels were written for).
 */
seed_status_t seed_infer_validate(const seed_arch_t* arch);

/*
 * Create a handle on the current HIP device.  weights_host: host pointer to
 * n_weights fp32 values in the canonical order; n_weights must equal
 * seed_infer_weight_count(arch).  The weights are copied and repacked (to
 * bf16 tiles in bf16 mode) before the call returns; the caller may free them.
 * Allocates the workspace for max_batch rows once.  *out is set only on
 * SEED_OK.  Validation errors are reported before any device call is made.
 */
seed_status_t seed_infer_create(const seed_arch_t* arch, const float* weights_host,
                                size_t n_weights, seed_infer_t** out);

/*
 * One inference step on B gathered rows (Section 3).  All array arguments are
 * device pointers.  The work is enqueued on `hip_stream` (a hipStream_t, NULL =
 * the default stream) and the call returns without synchronising; it allocates
 * nothing.
 *
 *   obs          [B, obs_h, obs_w, obs_c] uint8 frames (scaled by 1/255 inside)
 *   prev_action  [B] int32  } required iff lstm_units > 0, else must be NULL;
 *   prev_reward  [B] fp32   } an action outside [0, num_actions) gives an
 *   h_in, c_in   [B, lstm_units] fp32 } all-zero one-hot
 *   uniforms     [B, num_actions] fp32 in (0,1); required iff select is
 *                SEED_SELECT_GUMBEL, else must be NULL
 *   action_out   [B] int32
 *   logits_out   [B, num_actions] fp32: policy logits, or Q-values (dueling)
 *   value_out    [B] fp32: value head, or the dueling value stream
 *   h_out, c_out [B, lstm_units] fp32; required iff lstm_units > 0; must not
 *                overlap h_in / c_in (SEED_ERR_ALIASING): the caller ping-pongs
 *   probs_out    [B, num_actions] fp32 softmax(logits_out), or NULL to skip
 *
 * obs, h_in, c_in, h_out and c_out must be 16-byte aligned (any hipMalloc'ed
 * or framework-allocated buffer is; the kernels move frames and state 16 bytes
 * per lane), else SEED_ERR_INVALID_ARG.  B == 0 is a no-op returning SEED_OK.
 * B < 0 is SEED_ERR_INVALID_ARG, B > max_batch is SEED_ERR_BATCH_TOO_LARGE.
 */
seed_status_t seed_infer_step(seed_infer_t* handle, int32_t B,
                              const uint8_t* obs,
                              const int32_t* prev_action, const float* prev_reward,
                              const float* h_in, const float* c_in,
                              const float* uniforms,
                              int32_t* action_out, float* logits_out, float* value_out,
                              float* h_out, float* c_out, float* probs_out,
                              void* hip_stream);

/*
 * The step with episode boundaries and epsilon-greedy exploration.
 *
 * Section 3 ("Detailed Learner architecture"): the inference thread receives
 * episode termination flags with the observations; Appendix A.3.1 (agent
 * hyperparameters): training actor i of N acts epsilon-greedily with
 * epsilon_i = 0.4^(1 + 7 i / (N - 1)), evaluation uses 1e-3.  `ext` carries the
 * extra inputs, all device pointers, each optional (NULL = absent; ext == NULL
 * or all fields NULL makes this call identical to seed_infer_step):
 *
 *   done              [B] uint8; a non-zero flag means the row starts a new
 *                     episode: its recurrent core runs from the zero state and
 *                     h_in / c_in of that row are not read.  prev_action and
 *                     prev_reward are used as given.  Recurrent archs only
 *                     (SEED_ERR_INVALID_ARG otherwise).
 *   epsilon           [B] fp32 exploration rates, with
 *   explore_uniforms  [B, 2] fp32 uniforms in [0, 1): after the greedy /
 *                     Gumbel-max selection, a row with u0 < epsilon takes the
 *                     action min(floor(u1 * num_actions), num_actions - 1)
 *                     instead.  logits_out, value_out and probs_out are
 *                     unaffected.  The two must be given together.
 *
 * Set struct_size = sizeof(seed_step_ext_t).  Everything else (arguments,
 * stream behaviour, error returns) is as for seed_infer_step.
 */
typedef struct seed_step_ext {
    uint32_t struct_size;
    const uint8_t* done;
    const float* epsilon;
    const float* explore_uniforms;
} seed_step_ext_t;

seed_status_t seed_infer_step_ext(seed_infer_t* handle, int32_t B,
                                  const uint8_t* obs,
                                  const int32_t* prev_action, const float* prev_reward,
                                  const float* h_in, const float* c_in,
                                  const float* uniforms, const seed_step_ext_t* ext,
                                  int32_t* action_out, float* logits_out, float* value_out,
                                  float* h_out, float* c_out, float* probs_out,
                                  void* hip_stream);

/*
 * seed_infer_step_ext for callers that cannot allocate device memory or want
 * none allocated on their behalf at run time: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and same results as seed_infer_step_ext, but the activations between
 * the kernels (torso features, linear-layer rows, dueling hidden rows, the
 * layer-by-layer paths' maps) live in a static device array of
 * SEED_STATIC_SCRATCH_BYTES that is part of the library's code object (each
 * GPU the library runs on holds its own copy until the process ends), not in
 * the handle's workspace.  The call itself makes no hipMalloc / hipFree and no
 * allocating library call, records no memset, and does not synchronise.
 *
 *   - The rows must fit: a B whose workspace exceeds SEED_STATIC_SCRATCH_BYTES
 *     is rejected with SEED_ERR_BATCH_TOO_LARGE and a message that states the
 *     bytes needed (e.g. the DeepMind Lab agent in bf16 mode takes 8448 bytes
 *     per row: up to 1985 rows).  B > max_batch is rejected as usual.
 *   - All calls on one GPU, from any handle, share that GPU's array, and it
 *     keeps the previous call's contents (what has to start at zero is cleared
 *     by a fill kernel on the stream).  Calls that overlap in time on one GPU
 *     race: order them on one stream or with events.
 *   - seed_infer_read_intermediate reads the handle's own workspace, not this
 *     one.
 */
#define SEED_STATIC_SCRATCH_BYTES (16u << 20)
seed_status_t seed_infer_step_static(seed_infer_t* handle, int32_t B,
                                     const uint8_t* obs,
                                     const int32_t* prev_action, const float* prev_reward,
                                     const float* h_in, const float* c_in,
                                     const float* uniforms, const seed_step_ext_t* ext,
                                     int32_t* action_out, float* logits_out, float* value_out,
                                     float* h_out, float* c_out, float* probs_out,
                                     void* hip_stream);

/*
 * T-step unroll: the forward pass over stored trajectories, time-major
 * (Section 3: the learner unrolls trajectories step by step with the stored
 * recurrent state; Appendix A lists the unroll length, 32 for the V-trace
 * agents).  Step t is seed_infer_step on the t-th slice of every input with
 * the state step t-1 left; done[t] zeroes the state a row starts step t from.
 * The torso and the linear layer do not depend on time and run once over all
 * T * B frames; the recurrent core, the heads and the selection step through
 * time on the same kernels as seed_infer_step.
 *
 *   obs          [T, B, H, W, C] uint8      prev_action, prev_reward  [T, B]
 *   done         [T, B] uint8 or NULL       uniforms  [T, B, A] (iff Gumbel-max)
 *   h0, c0       [B, lstm_units] fp32: the state before step 0
 *   action_out   [T, B]   logits_out [T, B, A]   value_out [T, B]
 *   probs_out    [T, B, A] or NULL
 *   h_out, c_out [B, lstm_units]: the state after step T-1
 * All device pointers; recurrent arguments NULL iff the arch has no core (then
 * the call is one step over T * B rows).  T * B must not exceed max_batch
 * (SEED_ERR_BATCH_TOO_LARGE).  The states between steps live in the handle;
 * h_out / c_out must not overlap h0 / c0 or each other (SEED_ERR_ALIASING);
 * obs, h0, c0, h_out and c_out must be 16-byte aligned (SEED_ERR_INVALID_ARG).
 * Allocates nothing, enqueues on `hip_stream`, returns without synchronising;
 * on an error status nothing has been enqueued.
 */
seed_status_t seed_infer_unroll(seed_infer_t* handle, int32_t T, int32_t B,
                                const uint8_t* obs,
                                const int32_t* prev_action, const float* prev_reward,
                                const uint8_t* done,
                                const float* h0, const float* c0,
                                const float* uniforms,
                                int32_t* action_out, float* logits_out, float* value_out,
                                float* h_out, float* c_out, float* probs_out,
                                void* hip_stream);

/*
 * Replace the weights of a live handle (Section 3: the learner holds the only
 * copy of the model and the inference threads always use the latest one, so
 * every training step is followed by a weight refresh of the inference path).
 *
 *   weights_host  host pointer, the same flat layout and count as at creation;
 *                 copied into the handle's pinned staging buffer before the call
 *                 returns: the caller may reuse the buffer at once.
 *
 * The handle keeps two device copies of its weights.  The call enqueues, on a
 * stream the handle owns (default priority), the upload of the flat vector into
 * the idle copy and (bf16 mode) one kernel that packs it into the matrix-core
 * kernels' operand layouts, makes `hip_stream` wait for them, and makes that
 * copy the active one: steps enqueued on `hip_stream` afterwards use the new
 * weights, steps enqueued before keep the old ones and are not waited for - the
 * upload runs beside them.  The host's share is one copy of the flat vector
 * (spread over a few threads).  If an enqueue fails the active weights are
 * unchanged.  Steps and updates must be enqueued on the same stream (or be
 * ordered by the caller): the update after next overwrites the copy that steps
 * enqueued before this call are still reading, and waits only for what was
 * enqueued on `hip_stream` before the previous update.
 * The call waits only for the upload of the update BEFORE the previous one
 * (two staging buffers are used alternately).  Allocates no device or pinned
 * memory.
 * SEED_ERR_INVALID_ARG on a null pointer or a wrong count; the active weights
 * are then unchanged.
 */
seed_status_t seed_infer_set_weights(seed_infer_t* handle, const float* weights_host,
                                     size_t n_weights, void* hip_stream);

/* Number of features the torso feeds the linear layer (H*W*C), 0 if invalid. */
size_t seed_infer_torso_features(const seed_arch_t* arch);

/* Text of the most recent error on this handle ("" if none); never NULL.
 * With handle == NULL returns the text of the last failed seed_infer_create or
 * seed_infer_validate on the calling thread.  Owned by the library. */
const char* seed_infer_last_error(const seed_infer_t* handle);

/* Free the handle and everything it owns.  NULL is allowed.  The caller must
 * have synchronised every stream the handle was used on. */
void seed_infer_destroy(seed_infer_t* handle);

/* ------------------------------------------------------------------------
 * Host batching front-end (Section 3: a batching module gathers the actors'
 * inference calls into one batch; the inference thread holds the recurrent
 * states of all actors on the learner and returns only the actions).
 *
 * A batcher belongs to one seed_infer handle and one host thread.  It owns,
 * on the device, the recurrent state (h, c, zero at creation) and the last
 * action (0 at creation) of every actor, two pinned host staging sets and
 * their device mirrors, a copy stream and a compute stream (default
 * priority).  One round:
 *
 *   seed_batcher_add     once per actor call: copies the frame (host pointer,
 *                        obs_h*obs_w*obs_c bytes), the reward that followed the
 *                        actor's previous action and its episode flag into the
 *                        next row of the staging set being filled.  Errors:
 *                        actor out of [0, n_actors), the same actor twice in
 *                        one batch, more than max_batch rows.
 *   seed_batcher_submit  closes the batch (rows in the order they were added):
 *                        host->device copies on the copy stream, then on the
 *                        compute stream: gather the rows' states by actor,
 *                        seed_infer_step_ext (done flags reset states; epsilon
 *                        optional), scatter the new states and actions back,
 *                        copy the actions to pinned host memory.  Returns at
 *                        once with a ticket; the other staging set can be
 *                        filled while this batch is in flight (the call waits
 *                        only if that set's own earlier batch is unfinished).
 *                        uniforms [rows, num_actions] (host) is required iff
 *                        select is SEED_SELECT_GUMBEL; epsilon [rows] and
 *                        explore_uniforms [rows, 2] (host) are optional, given
 *                        together.  An empty batch is SEED_ERR_INVALID_ARG.
 *   seed_batcher_wait    blocks until the ticket's batch has finished and
 *                        copies its actions (row order) into actions_out
 *                        [capacity >= rows]; *n_rows receives the row count.
 *                        Only the two most recent tickets can be waited for.
 *
 * seed_batcher_read_state copies one actor's h and c ([lstm_units] each, host
 * pointers) after synchronising the compute stream (diagnostic).  Feed-forward
 * archs have no state: the call returns SEED_ERR_INVALID_ARG.
 * The handle must outlive the batcher; seed_infer_set_weights may be called
 * between rounds with the stream returned by seed_batcher_stream.
 */
typedef struct seed_batcher seed_batcher_t;

seed_status_t seed_batcher_create(seed_infer_t* handle, int32_t n_actors, seed_batcher_t** out);
seed_status_t seed_batcher_add(seed_batcher_t* b, int32_t actor, const uint8_t* obs_host,
                               float prev_reward, uint8_t done);
/* seed_batcher_add without the frame copy: *obs_slot receives the address of the row's frame in the pinned
 * staging set, for the caller (e.g. the RPC layer) to write obs_h*obs_w*obs_c bytes into before
 * seed_batcher_submit.  Same errors as seed_batcher_add. */
seed_status_t seed_batcher_reserve(seed_batcher_t* b, int32_t actor, float prev_reward, uint8_t done,
                                   uint8_t** obs_slot);
/* n calls of seed_batcher_add: actors [n], obs_host n contiguous frames, prev_rewards [n], dones [n] (host).
 * Stops at the first row that fails; the rows before it stay in the batch. */
seed_status_t seed_batcher_add_many(seed_batcher_t* b, int32_t n, const int32_t* actors,
                                    const uint8_t* obs_host, const float* prev_rewards,
                                    const uint8_t* dones);
seed_status_t seed_batcher_submit(seed_batcher_t* b, const float* uniforms_host,
                                  const float* epsilon_host, const float* explore_uniforms_host,
                                  int32_t* ticket);
seed_status_t seed_batcher_wait(seed_batcher_t* b, int32_t ticket, int32_t* actions_out,
                                int32_t capacity, int32_t* n_rows);
seed_status_t seed_batcher_read_state(seed_batcher_t* b, int32_t actor, float* h_host, float* c_host);
/* The compute stream (a hipStream_t) the batcher enqueues its steps on. */
void* seed_batcher_stream(seed_batcher_t* b);
/* Text of the batcher's most recent error; never NULL. */
const char* seed_batcher_last_error(const seed_batcher_t* b);
/* Waits for work in flight and frees the batcher.  NULL is allowed. */
void seed_batcher_destroy(seed_batcher_t* b);

/* ------------------------------------------------------------------------
 * Diagnostics.  Not part of the inference path: a tap for tests that compare
 * intermediates, and kernel timing for benchmarks.  A serving caller needs
 * neither.
 * ------------------------------------------------------------------------ */

/*
 * Test/diagnostic tap: copy an intermediate of the most recent step into a
 * device buffer as fp32 (converted from the internal storage type), enqueued
 * on `hip_stream` after the step's work.  which = 0: the rectified, flattened
 * torso output [B, torso_features]; which = 1: the linear layer's rectified
 * output [B, fc_units].  `capacity` is the number of floats `dst` can hold.
 */
seed_status_t seed_infer_read_intermediate(seed_infer_t* handle, int32_t which, int32_t B,
                                           float* dst, size_t capacity, void* hip_stream);

/*
 * Kernel timing for callers that measure (benchmarks, profilers).  With
 * profiling enabled, every seed_infer_step brackets its dominant kernel (the
 * torso: the fused ResNet kernel, or the conv-stack layers) with HIP events on
 * the step's stream, up to `SEED_PROFILE_SLOTS` steps between reads.
 * seed_infer_profile_read waits for the recorded events, returns the summed
 * torso time in milliseconds and the number of steps it covers, and starts a
 * new measurement.  Enabling allocates events (not allowed under graph
 * capture); disabled (the default) the step records nothing.
 */
#define SEED_PROFILE_SLOTS 4096
seed_status_t seed_infer_set_profiling(seed_infer_t* handle, int32_t enable);
seed_status_t seed_infer_profile_read(seed_infer_t* handle, float* torso_ms_sum, int32_t* n_steps);

#ifdef __cplusplus
}
#endif
#endif /* SEEDINF_H */
