"""GPU parity on the degenerate cases of action selection (Section 3, "sampled actions"; Appendix A.3.1,
epsilon-greedy) and on saturated frames.

The selection cases run a network whose weights are all zero except the biases of the output heads, so the
logits (or Q-values) are the same exact fp32 numbers on both sides and every decision below is forced by the
rule, not by rounding: uniforms of exactly 0 and 1 (the clamp to [FLT_MIN, 1 - 2^-24]), exact ties (lowest index
wins), u0 == epsilon (the comparison is strict), u1 at and next to 1 (the clamp to A - 1).  Actions must equal
the oracle's exactly.  Each case runs at three (input width, action count) pairs so that both heads kernels and
several lane-group widths see it."""
import numpy as np
import pytest

import oracle
from paper_1910_06591_amd import seedinf, workloads as wl
from tests.parity import check_against_oracle, to_device

pytestmark = pytest.mark.gpu
FLT_MIN = np.float32(np.finfo(np.float32).tiny)
BELOW_ONE = np.nextafter(np.float32(1), np.float32(0))


def head_only_net(A, width, select, head=0, hidden=0):
    """(cfg, zero weights): one pixel -> 1x1 conv -> linear `width` -> heads; every activation is zero."""
    cfg = dict(label=f"heads only A={A} n={width}", obs_h=1, obs_w=1, obs_c=1, torso=0, convs=[(1, 1, 1)], fc_units=width,
               lstm_units=0, num_actions=A, head=head, head_hidden=hidden, select=select, precision="fp32",
               obs_kind="uniform", index=130)
    return cfg, np.zeros(wl.weight_count(cfg), np.float32)


def set_bias(cfg, w, name, values):
    off, shape = wl.weight_slices(cfg)[name]
    n = int(np.prod(shape))
    assert n == len(values)
    w[off:off + n] = np.asarray(values, np.float32)


def run_both(orc, cfg, w, B, uniforms=None, epsilon=None, explore_u=None):
    import torch
    obs = np.zeros((B, 1, 1, 1), np.uint8)
    net = seedinf.SeedInfer(seedinf.make_arch(cfg, max_batch=B, precision="fp32"), w)
    kw = {}
    if epsilon is not None:
        kw = dict(epsilon=torch.from_numpy(epsilon).cuda(), explore_uniforms=torch.from_numpy(explore_u).cuda())
    out = net.step(torch.from_numpy(obs).cuda(), uniforms=None if uniforms is None else torch.from_numpy(uniforms).cuda(), **kw)
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in out.items()}
    net.close()
    ref = orc.forward(oracle.make_arch(cfg), w, obs, uniforms=uniforms, epsilon=epsilon, explore_u=explore_u)
    return got, ref


SHAPES = [(6, 1), (15, 256), (19, 64), (33, 50)]       # (actions, input width of the heads)


@pytest.mark.parametrize("A,width", SHAPES)
def test_gumbel_uniforms_at_zero_and_one_and_ties(orc, A, width):
    rng = np.random.default_rng(A)
    logits = rng.normal(0, 1, A).astype(np.float32)
    logits[A // 2] = logits.max() + np.float32(0.5)              # a unique best logit, in the middle
    cfg, w = head_only_net(A, width, select=1)
    set_bias(cfg, w, "policy.b", logits)
    rows = []
    u = np.full(A, 0.5, np.float32); u[2] = 1.0; rows.append(u)                    # u = 1: clamped, forces action 2
    u = np.full(A, 0.5, np.float32); u[A - 1] = BELOW_ONE; rows.append(u)          # largest value below 1: forces A - 1
    u = np.full(A, 1.0, np.float32); rows.append(u)                                # all 1: equal noise, best logit wins
    u = np.zeros(A, np.float32); rows.append(u)                                    # all 0: clamped to FLT_MIN, best logit wins
    u = np.full(A, 0.9, np.float32); u[A // 2] = 0.0; rows.append(u)               # the best logit gets the smallest noise
    u = np.full(A, FLT_MIN, np.float32); u[1] = np.float32(1e-45); rows.append(u)  # a denormal below the clamp
    u = np.full(A, 0.5, np.float32); u[0] = 0.0; u[1] = 1.0; rows.append(u)
    u = rng.random(A, dtype=np.float32); u[rng.integers(A)] = 1.0; rows.append(u)
    u = rng.random(A, dtype=np.float32); u[rng.integers(A)] = 0.0; rows.append(u)
    U = np.stack(rows)
    got, ref = run_both(orc, cfg, w, len(rows), uniforms=U)
    assert np.array_equal(got["logits"], np.broadcast_to(logits, (len(rows), A)))
    assert np.array_equal(ref["logits"], got["logits"])
    assert np.array_equal(got["action"], ref["action"]), (got["action"], ref["action"])
    assert got["action"][0] == 2 and got["action"][1] == A - 1 and got["action"][2] == A // 2 and got["action"][3] == A // 2
    assert np.isfinite(got["probs"]).all() and np.abs(got["probs"] - ref["probs"]).max() < 1e-6

    # equal logits and equal uniforms: an exact tie over all actions -> index 0; a tie between two -> the lower one
    set_bias(cfg, w, "policy.b", np.full(A, 0.25, np.float32))
    rows = [np.full(A, 0.5, np.float32), np.zeros(A, np.float32), np.ones(A, np.float32)]
    u = np.full(A, 0.3, np.float32); u[3] = u[A - 2] = 0.8; rows.append(u)         # two equal maxima: 3 wins
    u = np.full(A, 0.3, np.float32); u[A - 1] = u[1] = 1.0; rows.append(u)         # both clamped to the same value: 1 wins
    U = np.stack(rows)
    got, ref = run_both(orc, cfg, w, len(rows), uniforms=U)
    assert np.array_equal(got["action"], ref["action"]), (got["action"], ref["action"])
    assert list(got["action"]) == [0, 0, 0, 3, 1]
    assert np.array_equal(ref["margin"], np.zeros(len(rows), np.float32))          # the oracle saw exact ties too


@pytest.mark.parametrize("A,width", SHAPES)
def test_greedy_planted_ties(orc, A, width):
    q = np.linspace(-1, 1, A).astype(np.float32)
    q[1] = q[A - 2] = q[A // 2] = np.float32(1.5)                # three equal maxima: the lowest index wins
    cfg, w = head_only_net(A, width, select=0)
    set_bias(cfg, w, "policy.b", q)
    got, ref = run_both(orc, cfg, w, 5)
    assert np.array_equal(got["action"], ref["action"]) and (got["action"] == 1).all()
    assert np.array_equal(got["logits"], ref["logits"])
    # dueling heads: Q = V + Adv - mean(Adv) keeps equal advantages equal
    hidden = {1: 16, 256: 64, 64: 32, 50: 48}[width]
    cfg, w = head_only_net(A, width, select=0, head=1, hidden=hidden)
    set_bias(cfg, w, "a2.b", q)
    set_bias(cfg, w, "v2.b", [0.125])
    got, ref = run_both(orc, cfg, w, 5)
    assert np.array_equal(got["action"], ref["action"]) and (got["action"] == 1).all()
    assert np.abs(got["logits"] - ref["logits"]).max() <= 1e-6
    # all Q-values equal
    set_bias(cfg, w, "a2.b", np.full(A, -0.75, np.float32))
    got, ref = run_both(orc, cfg, w, 3)
    assert np.array_equal(got["action"], ref["action"]) and (got["action"] == 0).all()


@pytest.mark.parametrize("A,width", SHAPES)
def test_epsilon_greedy_boundaries(orc, A, width):
    q = np.linspace(1, -1, A).astype(np.float32)                 # greedy action 0
    cfg, w = head_only_net(A, width, select=0)
    set_bias(cfg, w, "policy.b", q)
    e = np.float32(0.37)
    below = np.nextafter(e, np.float32(0))
    cases = [                                                    # (epsilon, u0, u1, expected action)
        (e, e, 0.99, 0),                                         # u0 == epsilon: strict comparison, no exploration
        (e, below, 0.99, min(int(np.floor(0.99 * A)), A - 1)),   # one ulp below: explores
        (e, below, 1.0, A - 1),                                  # u1 = 1 is clamped to the last action
        (e, below, BELOW_ONE, A - 1),
        (e, below, 0.0, 0),
        (e, 0.0, 0.5, int(np.floor(0.5 * A))),
        (0.0, 0.0, 0.9, 0),                                      # epsilon = 0 never explores, even at u0 = 0
        (1.0, BELOW_ONE, 0.5, int(np.floor(0.5 * A))),           # epsilon = 1 always explores
        (1.0, 1.0, 0.5, 0),                                      # u0 = 1 (outside [0, 1)) does not
        (e, np.nextafter(e, np.float32(1)), 0.2, 0),
        (np.float32(1e-3), np.float32(9.99e-4), 0.75, int(np.floor(0.75 * A))),   # the evaluation epsilon
    ]
    eps = np.array([c[0] for c in cases], np.float32)
    eu = np.array([[c[1], c[2]] for c in cases], np.float32)
    want = np.array([c[3] for c in cases], np.int32)
    got, ref = run_both(orc, cfg, w, len(cases), epsilon=eps, explore_u=eu)
    assert np.array_equal(ref["action"], want), (ref["action"], want)
    assert np.array_equal(got["action"], ref["action"]), (got["action"], ref["action"])
    assert np.array_equal(got["logits"], ref["logits"])
    # the same after Gumbel-max selection
    cfg, w = head_only_net(A, width, select=1)
    set_bias(cfg, w, "policy.b", q)
    U = np.full((len(cases), A), 0.5, np.float32)
    got, ref = run_both(orc, cfg, w, len(cases), uniforms=U, epsilon=eps, explore_u=eu)
    assert np.array_equal(ref["action"], want) and np.array_equal(got["action"], ref["action"])


@pytest.mark.parametrize("name,precision", [("C3", "bf16"), ("C2", "bf16"), ("C3", "fp32"), ("C4", "bf16")])
def test_saturated_frames(orc, name, precision):
    """All-0 and all-255 frames (the ends of the uint8 range through the 1/255 scaling and, in bf16 mode, the
    exact-integer operand path), alone and next to ordinary frames."""
    import torch
    cfg = wl.CONFIGS[name]
    B = 6
    w = wl.make_weights(cfg, bf16_representable=(precision == "bf16"))
    batch = wl.make_batch(cfg, B)
    batch["obs"][0] = 0
    batch["obs"][1] = 255
    batch["obs"][3] = 255
    batch["obs"][4] = 0
    batch["obs"][4, ::2] = 255                                    # alternate rows saturated
    print(f"saturated frames {cfg['label']} {precision}", flush=True)
    net = seedinf.SeedInfer(seedinf.make_arch(cfg, max_batch=B, precision=precision), w)
    out = net.step(**to_device(batch))
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in out.items()}
    net.close()
    keys = ("prev_action", "prev_reward", "h_in", "c_in", "uniforms")
    ref = orc.forward(oracle.make_arch(cfg), w, batch["obs"], **{k: batch[k] for k in keys})
    rep = check_against_oracle(got, ref, 1e-4 if precision == "fp32" else 2e-2, batch["uniforms"])
    print("   ", rep, flush=True)
