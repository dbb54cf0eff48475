"""Seeded synthetic workloads for the central inference step.

This module holds configuration tables and random input generators only: no
layer arithmetic.  It is the one module both the CPU oracle's tests and the
HIP library's tests/bench draw inputs from, so both sides see the same bytes.

The five configurations have the shapes and value structure of the paper's
three workloads (DeepMind Lab 96x72 RGB frames, Section 2 footnote and
Section 4.1; Google Research Football minimap bitmaps, Section 4.2; Atari
84x84 grayscale with a frame stack of 4 and 18 actions, Appendix A.3) and
stand in for them: no environment frames are used anywhere.
"""
from __future__ import annotations

import numpy as np

# select: 0 greedy, 1 Gumbel-max; head: 0 policy+value, 1 dueling Q
CONFIGS = {
    "C1": dict(label="tiny feed-forward policy (Atari-shaped)",
               obs_h=84, obs_w=84, obs_c=4, torso=0, convs=[(16, 8, 4), (32, 4, 2)],
               fc_units=256, lstm_units=0, num_actions=6, head=0, head_hidden=0, select=1,
               precision="fp32", batch=8, obs_kind="uniform", index=1),
    "C2": dict(label="Atari R2D2 dueling-Q network",
               obs_h=84, obs_w=84, obs_c=4, torso=0, convs=[(32, 8, 4), (64, 4, 2), (64, 3, 1)],
               fc_units=512, lstm_units=512, num_actions=18, head=1, head_hidden=512, select=0,
               precision="bf16", batch=256, obs_kind="blobs", index=2),
    "C3": dict(label="DMLab IMPALA deep-ResNet + LSTM-256 agent",
               obs_h=72, obs_w=96, obs_c=3, torso=1, sections=[16, 32, 32],
               fc_units=256, lstm_units=256, num_actions=15, head=0, head_hidden=0, select=1,
               precision="bf16", batch=1024, obs_kind="uniform", index=3),
    "C4": dict(label="Football deep-ResNet policy on 16 minimap planes",
               obs_h=72, obs_w=96, obs_c=16, torso=1, sections=[16, 32, 32, 32],
               fc_units=256, lstm_units=0, num_actions=19, head=0, head_hidden=0, select=1,
               precision="bf16", batch=2048, obs_kind="sparse", index=4),
}
# C5 is the batch sweep of the C3 agent (one weight set for every batch size).
CONFIGS["C5"] = dict(CONFIGS["C3"], label="DMLab agent, batch sweep", batch=4096,
                     sweep=[64, 256, 1024, 4096, 8192], index=5)


def torso_out_shape(cfg):
    """(H, W, C) of the torso output (host-side shape bookkeeping only)."""
    h, w, c = cfg["obs_h"], cfg["obs_w"], cfg["obs_c"]
    if cfg["torso"] == 0:
        for ch, k, s in cfg["convs"]:
            h, w, c = (h - k) // s + 1, (w - k) // s + 1, ch
    else:
        for ch in cfg["sections"]:
            h, w, c = (h + 1) // 2, (w + 1) // 2, ch
    return h, w, c


def weight_layout(cfg):
    """Canonical flat order of the parameters as (name, shape, fan_in) with
    fan_in None for biases.  Conv kernels are [kh, kw, cin, cout]; dense
    matrices are [in, out]; the LSTM matrix has rows [features | one-hot
    action rows | reward row | h rows] and column blocks [i|f|g|o]."""
    out = []
    c = cfg["obs_c"]
    if cfg["torso"] == 0:
        for i, (ch, k, s) in enumerate(cfg["convs"]):
            out.append((f"conv{i}.w", (k, k, c, ch), k * k * c))
            out.append((f"conv{i}.b", (ch,), None))
            c = ch
    else:
        for s, ch in enumerate(cfg["sections"]):
            out.append((f"sec{s}.conv0.w", (3, 3, c, ch), 9 * c))
            out.append((f"sec{s}.conv0.b", (ch,), None))
            for blk in (1, 2):
                for ab in "ab":
                    out.append((f"sec{s}.block{blk}.{ab}.w", (3, 3, ch, ch), 9 * ch))
                    out.append((f"sec{s}.block{blk}.{ab}.b", (ch,), None))
            c = ch
    h, w, c = torso_out_shape(cfg)
    flat, fc = h * w * c, cfg["fc_units"]
    out.append(("fc.w", (flat, fc), flat))
    out.append(("fc.b", (fc,), None))
    core = fc
    A = cfg["num_actions"]
    if cfg["lstm_units"] > 0:
        hn = cfg["lstm_units"]
        rows = fc + A + 1 + hn
        out.append(("lstm.w", (rows, 4 * hn), rows))
        out.append(("lstm.b", (4 * hn,), None))
        core = hn
    if cfg["head"] == 0:
        out += [("policy.w", (core, A), core), ("policy.b", (A,), None),
                ("value.w", (core, 1), core), ("value.b", (1,), None)]
    else:
        hid = cfg["head_hidden"]
        out += [("v1.w", (core, hid), core), ("v1.b", (hid,), None),
                ("v2.w", (hid, 1), hid), ("v2.b", (1,), None),
                ("a1.w", (core, hid), core), ("a1.b", (hid,), None),
                ("a2.w", (hid, A), hid), ("a2.b", (A,), None)]
    return out


def weight_count(cfg) -> int:
    return int(sum(int(np.prod(s)) for _, s, _ in weight_layout(cfg)))


def weight_slices(cfg):
    """name -> (offset, shape) into the flat vector."""
    off, d = 0, {}
    for name, shape, _ in weight_layout(cfg):
        n = int(np.prod(shape))
        d[name] = (off, shape)
        off += n
    return d


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16-representable value (ties to
    even) and return them as fp32.  Part of the input recipe: in bf16 mode the
    generated weights are bf16-representable, so weight quantisation is not
    charged to the activation tolerance."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def make_weights(cfg, seed=None, bf16_representable=None) -> np.ndarray:
    """Weights ~ N(0, 1/fan_in), biases ~ U(-0.1, 0.1), flat fp32."""
    if seed is None:
        seed = 2000 + cfg["index"]
    if bf16_representable is None:
        bf16_representable = cfg["precision"] == "bf16"
    rng = np.random.default_rng(seed)
    parts = []
    for _, shape, fan_in in weight_layout(cfg):
        if fan_in is None:
            parts.append(rng.uniform(-0.1, 0.1, size=shape).astype(np.float32).ravel())
        else:
            parts.append((rng.standard_normal(size=shape) / np.sqrt(fan_in)).astype(np.float32).ravel())
    w = np.concatenate(parts)
    return round_to_bf16(w) if bf16_representable else w


def make_obs(cfg, batch=None, seed=None) -> np.ndarray:
    """uint8 [B, H, W, C] frames with the value structure of the config's
    workload: iid bytes (DMLab-like RGB), smooth moving blobs plus noise
    (Atari-like frame stack), or ~1 % set cells (Football minimap planes)."""
    B = cfg["batch"] if batch is None else batch
    if seed is None:
        seed = 1000 + cfg["index"]
    rng = np.random.default_rng(seed)
    H, W, Cc = cfg["obs_h"], cfg["obs_w"], cfg["obs_c"]
    kind = cfg["obs_kind"]
    if kind == "uniform":
        return rng.integers(0, 256, size=(B, H, W, Cc), dtype=np.uint8)
    if kind == "sparse":
        return np.where(rng.random(size=(B, H, W, Cc)) < 0.01, 255, 0).astype(np.uint8)
    if kind == "blobs":
        yy, xx = np.mgrid[0:H, 0:W].astype(np.float32)
        obs = np.empty((B, H, W, Cc), np.uint8)
        for b in range(B):
            nb = int(rng.integers(4, 9))
            cy, cx = rng.uniform(0, H, nb), rng.uniform(0, W, nb)
            sg, amp = rng.uniform(3, 12, nb), rng.uniform(64, 255, nb)
            dy, dx = rng.integers(-2, 3, nb), rng.integers(-2, 3, nb)
            for c in range(Cc):
                img = np.zeros((H, W), np.float32)
                for j in range(nb):
                    img += amp[j] * np.exp(-((yy - cy[j] - c * dy[j]) ** 2 + (xx - cx[j] - c * dx[j]) ** 2)
                                           / (2 * sg[j] ** 2))
                img += rng.integers(0, 16, size=(H, W))
                obs[b, :, :, c] = np.clip(np.rint(img), 0, 255).astype(np.uint8)
        return obs
    raise ValueError(kind)


def make_core_inputs(cfg, batch=None, seed=None):
    """prev_action int32 [B], prev_reward fp32 [B] ~ N(0,1), h and c fp32
    [B, lstm_units] ~ N(0, 0.5^2); None for each when there is no core."""
    if cfg["lstm_units"] == 0:
        return None, None, None, None
    B = cfg["batch"] if batch is None else batch
    if seed is None:
        seed = 1500 + cfg["index"]
    rng = np.random.default_rng(seed)
    pa = rng.integers(0, cfg["num_actions"], size=B, dtype=np.int32)
    pr = rng.standard_normal(B).astype(np.float32)
    h = (0.5 * rng.standard_normal((B, cfg["lstm_units"]))).astype(np.float32)
    c = (0.5 * rng.standard_normal((B, cfg["lstm_units"]))).astype(np.float32)
    return pa, pr, h, c


def make_uniforms(cfg, batch=None, seed=None):
    """fp32 [B, A] uniforms in (0,1) for Gumbel-max selection (None if greedy)."""
    if cfg["select"] == 0:
        return None
    B = cfg["batch"] if batch is None else batch
    if seed is None:
        seed = 3000 + cfg["index"]
    rng = np.random.default_rng(seed)
    u = rng.random((B, cfg["num_actions"]), dtype=np.float32)
    return np.clip(u, np.float32(1e-7), np.float32(1.0 - 6e-8))


def epsilon_schedule(n_actors: int) -> np.ndarray:
    """Exploration rate of each of N training actors (Appendix A.3.1, agent hyperparameter table):
    epsilon_i = 0.4 ** (1 + 7 i / (N - 1)); evaluation uses 1e-3."""
    i = np.arange(n_actors, dtype=np.float64)
    return (0.4 ** (1.0 + 7.0 * i / max(n_actors - 1, 1))).astype(np.float32)


def make_episode_inputs(cfg, batch=None, seed=None, done_rate=0.05):
    """Episode flags and exploration inputs of one step: done [B] uint8 (a row starts a new episode with
    probability done_rate), epsilon [B] (the training schedule over B actors) and explore_u [B, 2] uniforms.
    Seed 3500 + config index."""
    B = cfg["batch"] if batch is None else batch
    if seed is None:
        seed = 3500 + cfg["index"]
    rng = np.random.default_rng(seed)
    done = (rng.random(B) < done_rate).astype(np.uint8)
    eps = epsilon_schedule(B)
    u = rng.random((B, 2), dtype=np.float32)
    return done, eps, u


def make_batch(cfg, batch=None, seed_shift=0):
    """All step inputs for one batch as a dict of numpy arrays."""
    B = cfg["batch"] if batch is None else batch
    k = cfg["index"]
    pa, pr, h, c = make_core_inputs(cfg, B, 1500 + k + seed_shift)
    return dict(obs=make_obs(cfg, B, 1000 + k + seed_shift), prev_action=pa, prev_reward=pr,
                h_in=h, c_in=c, uniforms=make_uniforms(cfg, B, 3000 + k + seed_shift))


def make_trajectory(cfg, T, batch, done_rate=0.1):
    """Inputs of a T-step unroll over `batch` trajectories, time-major: obs [T, B, H, W, C], prev_action,
    prev_reward, done [T, B], uniforms [T, B, A] and the initial state h0, c0 [B, Hn].  Step t draws from the
    same recipes as a single step, with seeds shifted by 10 t (done: seed 3600 + 10 t + config index)."""
    steps = [make_batch(cfg, batch, seed_shift=10 * t) for t in range(T)]
    out = {k: (np.stack([s[k] for s in steps]) if steps[0][k] is not None else None)
           for k in ("obs", "prev_action", "prev_reward", "uniforms")}
    out["h0"], out["c0"] = steps[0]["h_in"], steps[0]["c_in"]
    out["done"] = None
    if cfg["lstm_units"]:
        out["done"] = np.stack([make_episode_inputs(cfg, batch, seed=3600 + 10 * t + cfg["index"], done_rate=done_rate)[0]
                                for t in range(T)])
    return out


def hbm_bytes_per_frame(cfg) -> int:
    """Bytes per frame that any implementation of the step must move to and from HBM: the frame, the row's
    other inputs (previous action and reward, recurrent state, uniforms) and its outputs (action, logits, value,
    probabilities, new state).  Weights (read once per step) are not per-frame traffic."""
    a, hn = cfg["num_actions"], cfg["lstm_units"]
    frame = cfg["obs_h"] * cfg["obs_w"] * cfg["obs_c"]
    core_in = (8 + 2 * hn * 4) if hn else 0
    core_out = 2 * hn * 4 if hn else 0
    uniforms = a * 4 if cfg["select"] == 1 else 0
    return frame + core_in + uniforms + core_out + 4 + a * 4 + 4 + a * 4


def macs_per_frame(cfg) -> int:
    """Useful multiply-accumulates per frame (no tile padding counted)."""
    h, w, c = cfg["obs_h"], cfg["obs_w"], cfg["obs_c"]
    macs = 0
    if cfg["torso"] == 0:
        for ch, k, s in cfg["convs"]:
            h, w = (h - k) // s + 1, (w - k) // s + 1
            macs += h * w * k * k * c * ch
            c = ch
    else:
        for ch in cfg["sections"]:
            macs += h * w * 9 * c * ch
            h, w, c = (h + 1) // 2, (w + 1) // 2, ch
            macs += 4 * h * w * 9 * c * c
    fc = cfg["fc_units"]
    macs += h * w * c * fc
    core, A = fc, cfg["num_actions"]
    if cfg["lstm_units"]:
        hn = cfg["lstm_units"]
        macs += (fc + A + 1 + hn) * 4 * hn
        core = hn
    if cfg["head"] == 0:
        macs += core * (A + 1)
    else:
        macs += 2 * core * cfg["head_hidden"] + cfg["head_hidden"] * (A + 1)
    return macs
