"""Whole-network pins for the oracle: re-composition from torch CPU fp64
library routines, invariants across batch rows, the paper's printed sizes,
the sampling law on 1e6 draws, and the f32 build against the f64 build."""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from paper_1910_06591_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")


def read_golden():
    d = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = (t.strip() for t in line.split("="))
            num = lambda t: int(t) if t.lstrip("-").isdigit() else float(t)
            d[k] = [num(t) for t in v.split(",")] if "," in v else num(v)
    return d


def test_paper_printed_sizes():
    g = read_golden()
    # DMLab frames: 96 x 72 x 3 bytes, 1e5 per second ~ 2 GB/s -> one byte per channel value
    c3 = wl.CONFIGS["C3"]
    assert (c3["obs_w"], c3["obs_h"], c3["obs_c"]) == (g["dmlab_obs_w"], g["dmlab_obs_h"], g["dmlab_obs_c"])
    frame = wl.make_obs(c3, 1)
    assert frame.dtype == np.uint8 and frame.nbytes == 96 * 72 * 3
    assert round(frame.nbytes * g["dmlab_obs_per_s"] / 1e9) == g["dmlab_obs_gb_per_s"]
    # Atari: 84x84 one-byte grayscale; 1e5 x 120 of them ~ 85 GB; stack of 4 at inference
    c2 = wl.CONFIGS["C2"]
    assert (c2["obs_h"], c2["obs_w"], c2["obs_c"]) == (g["atari_obs_h"], g["atari_obs_w"], g["atari_frame_stack"])
    assert round(84 * 84 * g["replay_sequences"] * g["replay_seq_len"] / 1e9) == g["replay_gb"]
    # R2D2 network
    assert [c[0] for c in c2["convs"]] == g["r2d2_filters"]
    assert [c[1] for c in c2["convs"]] == g["r2d2_kernels"]
    assert [c[2] for c in c2["convs"]] == g["r2d2_strides"]
    assert c2["fc_units"] == g["r2d2_linear"] and c2["lstm_units"] == g["r2d2_lstm"]
    assert c2["head_hidden"] == g["r2d2_dueling_hidden"] and c2["num_actions"] == g["atari_actions"]
    assert g["atari_inference_batch"] in wl.CONFIGS["C5"]["sweep"]


def test_weight_counts_agree(orc):
    # per-frame useful MACs of the five configurations
    assert wl.macs_per_frame(wl.CONFIGS["C1"]) == 2_967_296
    assert wl.macs_per_frame(wl.CONFIGS["C2"]) == 12_013_056
    assert wl.macs_per_frame(wl.CONFIGS["C3"]) == 52_191_232
    assert wl.macs_per_frame(wl.CONFIGS["C4"]) == 66_053_120
    # bytes per frame any implementation moves to and from HBM, written out by hand:
    # C3/C5: frame 72*96*3, prev action + reward 8, state in and out 4 * 256 * 4, uniforms 60, action 4, logits 60,
    # value 4, probabilities 60; C2: frame 84*84*4, 8, state 4 * 512 * 4, no uniforms, 4 + 72 + 4 + 72;
    # C4: frame 72*96*16, no core, uniforms 76, 4 + 76 + 4 + 76
    assert wl.hbm_bytes_per_frame(wl.CONFIGS["C5"]) == 20736 + 8 + 4096 + 60 + 4 + 60 + 4 + 60 == 25_028
    assert wl.hbm_bytes_per_frame(wl.CONFIGS["C2"]) == 28224 + 8 + 8192 + 4 + 72 + 4 + 72 == 36_576
    assert wl.hbm_bytes_per_frame(wl.CONFIGS["C4"]) == 110592 + 76 + 4 + 76 + 4 + 76 == 110_828
    for cfg in wl.CONFIGS.values():
        a = oracle.make_arch(cfg)
        assert orc.weight_count(a) == wl.weight_count(cfg)
        h, w, c = wl.torso_out_shape(cfg)
        assert orc.torso_features(a) == h * w * c


# ---- independent fp64 re-composition from torch library routines ----------

def torch_forward(cfg, weights, batch):
    W = {k: torch.from_numpy(np.asarray(weights[o:o + int(np.prod(s))], np.float64).reshape(s))
         for k, (o, s) in wl.weight_slices(cfg).items()}
    x = torch.from_numpy(batch["obs"].astype(np.float64) / 255.0).permute(0, 3, 1, 2)
    conv = lambda t, n, **kw: F.conv2d(t, W[n + ".w"].permute(3, 2, 0, 1), W[n + ".b"], **kw)

    def pool(t):
        H, Wd = t.shape[2:]
        th, tw = max((-(-H // 2) - 1) * 2 + 3 - H, 0), max((-(-Wd // 2) - 1) * 2 + 3 - Wd, 0)
        t = F.pad(t, (tw // 2, tw - tw // 2, th // 2, th - th // 2), value=float("-inf"))
        return F.max_pool2d(t, 3, 2)

    if cfg["torso"] == 0:
        for i, (ch, k, s) in enumerate(cfg["convs"]):
            x = F.relu(conv(x, f"conv{i}", stride=s))
    else:
        for s in range(len(cfg["sections"])):
            x = pool(conv(x, f"sec{s}.conv0", padding=1))
            for blk in (1, 2):
                y = conv(F.relu(x), f"sec{s}.block{blk}.a", padding=1)
                x = x + conv(F.relu(y), f"sec{s}.block{blk}.b", padding=1)
        x = F.relu(x)
    feat = x.permute(0, 2, 3, 1).reshape(x.shape[0], -1)       # (h, w, c) flatten order
    fc = F.relu(feat @ W["fc.w"] + W["fc.b"])
    out = {"torso_feat": feat.numpy(), "fc_act": fc.numpy()}
    core = fc
    A = cfg["num_actions"]
    if cfg["lstm_units"]:
        Hn = cfg["lstm_units"]
        z = torch.cat([fc, F.one_hot(torch.from_numpy(batch["prev_action"]).long(), A).double(),
                       torch.from_numpy(batch["prev_reward"].astype(np.float64))[:, None],
                       torch.from_numpy(batch["h_in"].astype(np.float64))], 1)
        g = z @ W["lstm.w"] + W["lstm.b"]
        i, f, gg, o = g.split(Hn, 1)
        c = torch.sigmoid(f) * torch.from_numpy(batch["c_in"].astype(np.float64)) + torch.sigmoid(i) * torch.tanh(gg)
        h = torch.sigmoid(o) * torch.tanh(c)
        out["h"], out["c"] = h.numpy(), c.numpy()
        core = h
    if cfg["head"] == 0:
        out["logits"] = (core @ W["policy.w"] + W["policy.b"]).numpy()
        out["value"] = (core @ W["value.w"] + W["value.b"])[:, 0].numpy()
    else:
        V = F.relu(core @ W["v1.w"] + W["v1.b"]) @ W["v2.w"] + W["v2.b"]
        Adv = F.relu(core @ W["a1.w"] + W["a1.b"]) @ W["a2.w"] + W["a2.b"]
        out["logits"] = (V + Adv - Adv.mean(1, keepdim=True)).numpy()
        out["value"] = V[:, 0].numpy()
    lg = out["logits"]
    if cfg["select"]:
        lg = lg - np.log(-np.log(batch["uniforms"].astype(np.float64)))
    out["action"] = lg.argmax(1)
    srt = np.sort(lg, 1)
    out["margin"] = srt[:, -1] - srt[:, -2]
    out["probs"] = torch.softmax(torch.from_numpy(out["logits"]), 1).numpy()
    return out


SMALL_B = {"C1": 3, "C2": 2, "C3": 2, "C4": 2}


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4"])
def test_forward_matches_torch_recomposition(orc, orc64, name):
    cfg = wl.CONFIGS[name]
    B = SMALL_B[name]
    w = wl.make_weights(cfg)
    batch = wl.make_batch(cfg, B)
    ref = torch_forward(cfg, w, batch)
    arch = oracle.make_arch(cfg)
    kw = {k: batch[k] for k in ("prev_action", "prev_reward", "h_in", "c_in", "uniforms")}
    o64 = orc64.forward(arch, w, batch["obs"], want_intermediates=True, **kw)
    o32 = orc.forward(arch, w, batch["obs"], want_intermediates=True, **kw)
    keys = ["torso_feat", "fc_act", "logits", "value", "probs"] + (["h", "c"] if cfg["lstm_units"] else [])
    for k in keys:
        scale = max(1.0, np.abs(ref[k]).max())
        assert np.abs(o64[k] - ref[k]).max() <= 1e-11 * scale, k
        # the f32 build stays within fp32 rounding of the fp64 truth
        assert np.abs(o32[k] - ref[k]).max() <= 2e-5 * scale, (k, np.abs(o32[k] - ref[k]).max())
    safe = ref["margin"] > 1e-4
    assert np.array_equal(o64["action"][safe], ref["action"][safe])
    assert np.array_equal(o32["action"][safe], ref["action"][safe])
    np.testing.assert_allclose(o64["margin"], ref["margin"], atol=1e-9)
    if cfg["head"] == 1:      # value_out of a Q agent is the dueling value stream = mean_a Q
        np.testing.assert_allclose(o64["logits"].mean(1), o64["value"], atol=1e-12)


def test_rows_are_independent(orc):
    cfg = wl.CONFIGS["C3"]
    arch = oracle.make_arch(cfg)
    w = wl.make_weights(cfg)
    b = wl.make_batch(cfg, 4)
    keys = ("prev_action", "prev_reward", "h_in", "c_in", "uniforms")
    full = orc.forward(arch, w, b["obs"], **{k: b[k] for k in keys})
    perm = np.array([2, 0, 3, 1])
    pr = orc.forward(arch, w, b["obs"][perm], **{k: b[k][perm] for k in keys})
    one = orc.forward(arch, w, b["obs"][1:2], **{k: b[k][1:2] for k in keys})
    for k in ("action", "logits", "value", "h", "c", "probs", "margin"):
        np.testing.assert_array_equal(pr[k], full[k][perm])
        np.testing.assert_array_equal(one[k][0], full[k][1])


def test_sampling_law_one_million_draws(orc):
    """1e6 rows through the whole forward pass of a degenerate network whose
    logits equal the policy bias: action frequencies follow softmax(logits)
    within 5 sigma (the law an inverse-CDF sampler has), and each row's
    uniforms are the ones used for that row."""
    logits = np.array([0.4, -1.1, 1.3, 0.0], np.float32)
    A = 4
    cfg = dict(obs_h=1, obs_w=1, obs_c=1, torso=0, convs=[(1, 1, 1)], fc_units=1, lstm_units=0,
               num_actions=A, head=0, head_hidden=0, select=1, index=9)
    arch = oracle.make_arch(cfg)
    w = np.zeros(wl.weight_count(cfg), np.float32)
    off, _ = wl.weight_slices(cfg)["policy.b"]
    w[off:off + A] = logits
    N = 1_000_000
    rng = np.random.default_rng(123)
    u = rng.random((N, A), dtype=np.float32)
    out = orc.forward(arch, w, np.zeros((N, 1, 1, 1), np.uint8), uniforms=u)
    np.testing.assert_array_equal(out["logits"], np.broadcast_to(logits, (N, A)))
    p = np.exp(logits.astype(np.float64) - logits.max()); p /= p.sum()
    freq = np.bincount(out["action"], minlength=A) / N
    assert np.all(np.abs(freq - p) < 5 * np.sqrt(p * (1 - p) / N)), (freq, p)
    # row alignment: recompute a few rows directly
    for i in (0, 17, N - 1):
        a, _, m = orc.select_gumbel(logits, u[i])
        assert a == out["action"][i] and m == out["margin"][i]
    np.testing.assert_allclose(out["probs"][5], p, rtol=1e-6)


def test_generators_are_seeded_and_shaped():
    for name, cfg in wl.CONFIGS.items():
        b1, b2 = wl.make_batch(cfg, 3), wl.make_batch(cfg, 3)
        for k in b1:
            if b1[k] is None:
                assert b2[k] is None
            else:
                np.testing.assert_array_equal(b1[k], b2[k])
        assert b1["obs"].shape == (3, cfg["obs_h"], cfg["obs_w"], cfg["obs_c"]) and b1["obs"].dtype == np.uint8
        w = wl.make_weights(cfg)
        assert w.dtype == np.float32 and w.size == wl.weight_count(cfg)
        if cfg["precision"] == "bf16":
            assert np.all((w.view(np.uint32) & 0xFFFF) == 0)
    sp = wl.make_obs(wl.CONFIGS["C4"], 4)
    assert set(np.unique(sp)) <= {0, 255} and 0.005 < (sp == 255).mean() < 0.015
    bl = wl.make_obs(wl.CONFIGS["C2"], 2)
    assert bl.max() > 64 and bl.std() > 5
    # bf16 rounding: ties to even
    x = np.array([1.0, 1.00390625, 1.01171875, -1.00390625], np.float32)   # 1, 1+2^-8, 1+3*2^-8, ...
    np.testing.assert_array_equal(wl.round_to_bf16(x), np.array([1.0, 1.0, 1.015625, -1.0], np.float32))
