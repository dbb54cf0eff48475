"""GPU parity for the T-step unroll (seed_infer_unroll) against the CPU oracle's unroll, and its error paths."""
import ctypes as C

import numpy as np
import pytest

import oracle
from paper_1910_06591_amd import seedinf, workloads as wl
from tests.parity import check_against_oracle, supported_random_arch

pytestmark = pytest.mark.gpu
TOL = {"fp32": 1e-4, "bf16": 2e-2}


def recurrent_c1():
    return dict(wl.CONFIGS["C1"], lstm_units=32, index=1, label="C1 with a 32-unit core")


def unroll_case(orc, cfg, T, B, precision, done_rate=0.2):
    import torch
    rec = cfg["lstm_units"] > 0
    w = wl.make_weights(cfg, bf16_representable=(precision == "bf16"))
    tr = wl.make_trajectory(cfg, T, B, done_rate=done_rate)
    print(f"unroll case {cfg['label']} T={T} B={B} {precision}", flush=True)
    net = seedinf.SeedInfer(seedinf.make_arch(cfg, max_batch=T * B, precision=precision), w)
    dev = {k: (None if v is None else torch.from_numpy(v).cuda()) for k, v in tr.items()}
    out = net.unroll(dev["obs"], dev["prev_action"], dev["prev_reward"], dev["h0"], dev["c0"], dev["uniforms"], dev["done"])
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in out.items()}
    ref = orc.unroll(oracle.make_arch(cfg), w, tr["obs"], tr["prev_action"], tr["prev_reward"], tr["h0"], tr["c0"],
                     tr["uniforms"], done=tr["done"])
    A = cfg["num_actions"]
    flat = lambda d: {"action": d["action"].reshape(T * B), "logits": d["logits"].reshape(T * B, A),
                      "value": d["value"].reshape(T * B), "probs": d["probs"].reshape(T * B, A)}
    g, r = flat(got), flat(ref)
    r["margin"] = ref["margin"].reshape(T * B)
    rep = check_against_oracle(g, r, TOL[precision], None if tr["uniforms"] is None else tr["uniforms"].reshape(T * B, A))
    if rec:
        for k in ("h", "c"):
            sc = np.maximum(1.0, np.abs(ref[k]).max(axis=1))
            err = (np.abs(got[k].astype(np.float64) - ref[k]).max(axis=1) / sc).max()
            assert err <= TOL[precision], (k, err)
            rep[k + "_err"] = float(err)
    print("   ", rep, flush=True)
    net.close()
    return got


@pytest.mark.parametrize("name,T,B", [("C1r", 5, 7), ("C3", 4, 6), ("C2", 3, 5), ("C4", 3, 4)])
def test_unroll_fp32(orc, name, T, B):
    unroll_case(orc, recurrent_c1() if name == "C1r" else wl.CONFIGS[name], T, B, "fp32")


@pytest.mark.parametrize("name,T,B", [("C3", 5, 40), ("C2", 3, 33), ("C4", 2, 20), ("C3", 1, 17), ("C2", 9, 250)])
def test_unroll_bf16(orc, name, T, B):
    """(C2 with T * B = 2250: the linear layer over all T * B rows takes the large-batch kernel, the per-step
    core the small-batch one.)"""
    unroll_case(orc, wl.CONFIGS[name], T, B, "bf16")


@pytest.mark.parametrize("seed,precision", [(s, p) for p in ("fp32", "bf16") for s in range(8)])
def test_unroll_random_architectures(orc, seed, precision):
    """The unroll on seeded random architectures (recurrent and feed-forward, both heads and selections), random T
    and B."""
    cfg = supported_random_arch(100 + seed, precision)
    st, msg = seedinf.validate(seedinf.make_arch(cfg, max_batch=64, precision=precision))
    assert st == 0, (cfg, msg)
    rng = np.random.default_rng(seed)
    unroll_case(orc, cfg, int(rng.integers(1, 7)), int(rng.integers(1, 10)), precision)


def test_unroll_without_flags_and_every_row_flagged(orc):
    cfg = wl.CONFIGS["C3"]
    unroll_case(orc, cfg, 3, 24, "bf16", done_rate=0.0)
    unroll_case(orc, cfg, 3, 24, "bf16", done_rate=1.0)


def test_unroll_equals_successive_steps_fp32():
    """fp32 mode: the unroll and T calls of the step run the same per-row kernels, so they agree bit for bit."""
    import torch
    cfg = recurrent_c1()
    T, B = 4, 9
    w = wl.make_weights(cfg)
    tr = wl.make_trajectory(cfg, T, B, done_rate=0.3)
    net = seedinf.SeedInfer(seedinf.make_arch(cfg, max_batch=T * B, precision="fp32"), w)
    dev = {k: (None if v is None else torch.from_numpy(v).cuda()) for k, v in tr.items()}
    u = net.unroll(dev["obs"], dev["prev_action"], dev["prev_reward"], dev["h0"], dev["c0"], dev["uniforms"], dev["done"])
    h, c = dev["h0"], dev["c0"]
    for t in range(T):
        o = net.step(dev["obs"][t], dev["prev_action"][t], dev["prev_reward"][t], h, c, dev["uniforms"][t], done=dev["done"][t])
        for k in ("action", "logits", "value", "probs"):
            assert torch.equal(o[k], u[k][t]), (t, k)
        h, c = o["h"], o["c"]
    assert torch.equal(h, u["h"]) and torch.equal(c, u["c"])
    net.close()


def test_unroll_error_paths():
    import torch
    cfg = wl.CONFIGS["C3"]
    T, B = 3, 4
    w = wl.make_weights(cfg, bf16_representable=True)
    net = seedinf.SeedInfer(seedinf.make_arch(cfg, max_batch=T * B, precision="bf16"), w)
    tr = wl.make_trajectory(cfg, T, B)
    dev = {k: (None if v is None else torch.from_numpy(v).cuda()) for k, v in tr.items()}
    A, Hn = cfg["num_actions"], cfg["lstm_units"]
    out = {"action": torch.full((T, B), -7, dtype=torch.int32, device="cuda"),
           "logits": torch.full((T, B, A), 3.0, device="cuda"), "value": torch.full((T, B), 3.0, device="cuda"),
           "h": torch.full((B, Hn), 3.0, device="cuda"), "c": torch.full((B, Hn), 3.0, device="cuda")}
    p = lambda t: None if t is None else C.c_void_p(t.data_ptr())

    def call(T_=T, B_=B, h_out=None, c_out=None, obs=dev["obs"], pa=dev["prev_action"]):
        return net.unroll_raw(T_, B_, p(obs), p(pa), p(dev["prev_reward"]), p(dev["done"]), p(dev["h0"]), p(dev["c0"]),
                              p(dev["uniforms"]), p(out["action"]), p(out["logits"]), p(out["value"]),
                              p(out["h"] if h_out is None else h_out), p(out["c"] if c_out is None else c_out), None)

    st, msg = call(T_=T + 1)
    assert st == seedinf.STATUS_BY_NAME["SEED_ERR_BATCH_TOO_LARGE"] and "max_batch" in msg
    st, msg = call(h_out=dev["h0"])
    assert st == seedinf.STATUS_BY_NAME["SEED_ERR_ALIASING"]
    st, msg = call(pa=None)
    assert st == seedinf.STATUS_BY_NAME["SEED_ERR_INVALID_ARG"]
    st, msg = call(T_=-1)
    assert st == seedinf.STATUS_BY_NAME["SEED_ERR_INVALID_ARG"]
    torch.cuda.synchronize()
    # nothing was written by the failed calls, and an empty unroll is a no-op
    st, msg = call(T_=0)
    assert st == 0
    torch.cuda.synchronize()
    assert (out["action"] == -7).all() and (out["logits"] == 3.0).all() and (out["h"] == 3.0).all()
    st, msg = call()
    assert st == 0, msg
    torch.cuda.synchronize()
    assert (out["action"] >= 0).all()
    net.close()
    # a feed-forward arch takes no recurrent arguments
    cfg4 = wl.CONFIGS["C4"]
    net4 = seedinf.SeedInfer(seedinf.make_arch(cfg4, max_batch=4, precision="bf16"), wl.make_weights(cfg4, bf16_representable=True))
    tr4 = wl.make_trajectory(cfg4, 2, 2)
    d4 = {k: (None if v is None else torch.from_numpy(v).cuda()) for k, v in tr4.items()}
    A4 = cfg4["num_actions"]
    o4 = {"action": torch.empty(2, 2, dtype=torch.int32, device="cuda"), "logits": torch.empty(2, 2, A4, device="cuda"),
          "value": torch.empty(2, 2, device="cuda")}
    st, msg = net4.unroll_raw(2, 2, p(d4["obs"]), None, None, p(dev["done"]), None, None, p(d4["uniforms"]), p(o4["action"]),
                              p(o4["logits"]), p(o4["value"]), None, None, None)
    assert st == seedinf.STATUS_BY_NAME["SEED_ERR_INVALID_ARG"]
    net4.close()
