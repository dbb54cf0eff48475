"""Pins for the oracle's episode-boundary and epsilon-greedy steps (Section 3: termination flags reach the
inference thread; Appendix A.3.1: epsilon-greedy actors)."""
import numpy as np
import pytest

import oracle
from paper_1910_06591_amd import workloads as wl
from tests.test_oracle_forward import read_golden


def test_epsilon_schedule_matches_the_printed_formula():
    g = read_golden()
    n = 256
    eps = wl.epsilon_schedule(n).astype(np.float64)
    # end points of the printed formula: actor 0 explores with 0.4, the last with 0.4^8
    assert eps[0] == pytest.approx(g["eps_base"], rel=1e-6)
    assert eps[-1] == pytest.approx(g["eps_base"] ** (1 + g["eps_exponent_span"]), rel=1e-6)
    assert eps[-1] == pytest.approx(0.00065536, rel=1e-6)
    # geometric in i: constant ratio between neighbours
    r = eps[1:] / eps[:-1]
    assert np.allclose(r, g["eps_base"] ** (g["eps_exponent_span"] / (n - 1)), rtol=1e-5)
    assert np.all(np.diff(eps) < 0)
    assert g["eps_eval"] == 0.001


def test_episode_state_is_zero_or_unchanged(orc64):
    rng = np.random.default_rng(5)
    h, c = rng.standard_normal(7), rng.standard_normal(7)
    h0, c0 = orc64.episode_state(0, h, c)
    assert np.array_equal(h0, h) and np.array_equal(c0, c)
    h0, c0 = orc64.episode_state(1, h, c)
    assert not h0.any() and not c0.any()
    h0, c0 = orc64.episode_state(255, h, c)          # any non-zero byte is a flag
    assert not h0.any() and not c0.any()


def test_epsilon_greedy_special_cases(orc, orc64):
    for o in (orc, orc64):
        A = 15
        assert o.epsilon_greedy(7, A, 0.0, 0.0, 0.5) == 7          # eps = 0 never explores, even at u0 = 0
        assert o.epsilon_greedy(7, A, 1.0, 0.999, 0.0) == 0         # eps = 1 always explores
        assert o.epsilon_greedy(7, A, 0.25, 0.25, 0.9) == 7         # strict: u0 == eps keeps the action
        assert o.epsilon_greedy(7, A, 0.25, 0.2499, 0.9) == 13      # floor(0.9 * 15)
        assert o.epsilon_greedy(7, A, 1.0, 0.0, 0.99999) == A - 1
        assert o.epsilon_greedy(7, A, 1.0, 0.0, 1.0) == A - 1       # clamped
        # every action is reachable and bins are the equal intervals [a/A, (a+1)/A)
        for a in range(A):
            assert o.epsilon_greedy(0, A, 1.0, 0.0, (a + 0.5) / A) == a


def test_epsilon_greedy_law(orc):
    # explored fraction ~ eps, explored actions uniform (chi-square), kept actions untouched
    rng = np.random.default_rng(11)
    n, A, eps = 200_000, 6, 0.3
    u = rng.random((n, 2), dtype=np.float32)
    sel = rng.integers(0, A, n)
    out = np.array([orc.epsilon_greedy(int(s), A, eps, float(a), float(b)) for s, a, b in zip(sel[:20000], u[:20000, 0], u[:20000, 1])])
    explored = u[:20000, 0] < np.float32(eps)
    assert abs(explored.mean() - eps) < 0.015
    assert np.array_equal(out[~explored], sel[:20000][~explored])
    counts = np.bincount(out[explored], minlength=A)
    expect = explored.sum() / A
    chi2 = ((counts - expect) ** 2 / expect).sum()
    assert chi2 < 25.0                                          # 5 degrees of freedom, p ~ 1e-4


@pytest.mark.parametrize("name", ["C1r", "C3"])
def test_forward_ext_equals_forward_on_prepared_inputs(orc, name):
    """The extended step is the plain step run on a state zeroed by hand, with the exploration rule
    applied afterwards by hand: pins where the flags and the rule enter the network."""
    if name == "C1r":
        cfg = dict(wl.CONFIGS["C1"], lstm_units=32, index=1)      # a small recurrent variant of C1
    else:
        cfg = wl.CONFIGS[name]
    arch = oracle.make_arch(cfg)
    B = 6
    w = wl.make_weights(cfg)
    b = wl.make_batch(cfg, B)
    done, _, eu = wl.make_episode_inputs(cfg, B, done_rate=0.5)
    done[0], done[1] = 1, 0
    eps = np.array([0.0, 1.0, 0.5, 0.5, 1.0, 0.0], np.float32)
    ext = orc.forward(arch, w, b["obs"], b["prev_action"], b["prev_reward"], b["h_in"], b["c_in"],
                      b["uniforms"], done=done, epsilon=eps, explore_u=eu)
    h0, c0 = b["h_in"].copy(), b["c_in"].copy()
    h0[done != 0] = 0
    c0[done != 0] = 0
    ref = orc.forward(arch, w, b["obs"], b["prev_action"], b["prev_reward"], h0, c0,
                      b["uniforms"])
    for k in ("logits", "value", "h", "c", "probs"):
        assert np.array_equal(ext[k], ref[k]), k
    A = cfg["num_actions"]
    want = ref["action"].copy()
    for i in range(B):
        if eu[i, 0] < eps[i]:
            want[i] = min(int(np.floor(float(eu[i, 1]) * A)), A - 1)
    assert np.array_equal(ext["action"], want)
    assert (ext["action"] != ref["action"]).any()       # the draw really explored somewhere
    # a flagged row really differs from the unflagged run (the state matters)
    plain = orc.forward(arch, w, b["obs"], b["prev_action"], b["prev_reward"], b["h_in"], b["c_in"],
                        b["uniforms"])
    assert not np.allclose(plain["h"][0], ext["h"][0])
    assert np.array_equal(plain["h"][1], ext["h"][1])
