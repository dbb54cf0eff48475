"""GPU tests of the host batching front-end (seed_batcher_*): rounds over random subsets of actors, pipelined two
deep, against the CPU oracle run on the same gathered rows with per-actor state kept in numpy."""
import numpy as np
import pytest

import oracle
from paper_1910_06591_amd import seedinf, workloads as wl

pytestmark = pytest.mark.gpu


def run_rounds(orc, cfg, precision, n_actors, max_rows, rounds, tol, use_eps):
    rng = np.random.default_rng(77)
    bf = precision == "bf16"
    w = wl.make_weights(cfg, bf16_representable=bf)
    net = seedinf.SeedInfer(seedinf.make_arch(cfg, max_batch=max_rows, precision=precision), w)
    bat = seedinf.Batcher(net, n_actors)
    arch = oracle.make_arch(cfg)
    A, Hn = cfg["num_actions"], cfg["lstm_units"]
    st_h = np.zeros((n_actors, Hn), np.float32)
    st_c = np.zeros((n_actors, Hn), np.float32)
    st_a = np.zeros(n_actors, np.int32)
    frames = wl.make_obs(cfg, n_actors * 2, seed=4242)
    pending = []                                    # (ticket, actors, oracle inputs)
    mismatches = 0

    def collect(item):
        nonlocal mismatches
        ticket, actors, obs, rew, done, un, eps, eu = item
        got = bat.wait(ticket)
        assert got.shape == (len(actors),)
        ref = orc.forward(arch, w, obs, st_a[actors], rew, st_h[actors], st_c[actors], un, done=done, epsilon=eps, explore_u=eu)
        # actions: identical unless the oracle's top two are within the usual margin
        scale = np.maximum(1.0, np.abs(ref["logits"]).max(axis=1))
        near = ref["margin"] <= 2 * tol * scale
        explored = (eu[:, 0] < eps) if eps is not None else np.zeros(len(actors), bool)
        differ = got != ref["action"]
        assert not (differ & ~near & ~explored).any(), (got, ref["action"])
        assert np.array_equal(got[explored], ref["action"][explored])
        mismatches += int(differ.sum())
        # the reference trajectory follows the device's own actions, so one near-tie does not fork the two
        st_a[actors] = got
        st_h[actors] = ref["h"]
        st_c[actors] = ref["c"]

    for k in range(rounds):
        n = int(rng.integers(1, max_rows + 1))
        actors = rng.choice(n_actors, size=n, replace=False).astype(np.int32)
        obs = frames[rng.integers(0, len(frames), n)]
        rew = rng.standard_normal(n).astype(np.float32)
        done = (rng.random(n) < 0.25).astype(np.uint8)
        un = wl.make_uniforms(cfg, n, seed=9000 + k)
        eps = eu = None
        if use_eps:
            eps = rng.random(n).astype(np.float32) * 0.5
            eu = rng.random((n, 2), dtype=np.float32)
        for i, a in enumerate(actors):
            bat.add(int(a), obs[i], float(rew[i]), bool(done[i]))
        t = bat.submit(un, eps, eu)
        pending.append((t, actors, obs, rew, done, un, eps, eu))
        if len(pending) == 2:                       # two batches in flight: collect the older one
            collect(pending.pop(0))
    while pending:
        collect(pending.pop(0))
    # final per-actor states on the device against the reference trajectory
    worst = 0.0
    for a in range(n_actors):
        h, c = bat.read_state(a)
        worst = max(worst, float(np.abs(h - st_h[a]).max()), float(np.abs(c - st_c[a]).max() / max(1.0, np.abs(st_c[a]).max())))
    print(f"batcher {cfg['label']} {precision}: rounds {rounds}, worst state error {worst:.3e}, action near-tie picks {mismatches}", flush=True)
    assert worst <= tol * rounds
    bat.close()
    net.close()


def test_batcher_fp32_small_recurrent(orc):
    cfg = dict(wl.CONFIGS["C1"], lstm_units=32, label="C1 + LSTM-32", index=51)
    run_rounds(orc, cfg, "fp32", n_actors=11, max_rows=6, rounds=9, tol=1e-4, use_eps=True)


def test_batcher_bf16_dmlab(orc):
    run_rounds(orc, dict(wl.CONFIGS["C3"], index=52), "bf16", n_actors=20, max_rows=12, rounds=6, tol=2e-2, use_eps=False)


def test_batcher_feed_forward_and_errors(orc):
    cfg = dict(wl.CONFIGS["C4"], index=53)          # no recurrent core
    w = wl.make_weights(cfg, bf16_representable=True)
    net = seedinf.SeedInfer(seedinf.make_arch(cfg, max_batch=4, precision="bf16"), w)
    bat = seedinf.Batcher(net, 5)
    frames = wl.make_obs(cfg, 5, seed=99)
    with pytest.raises(seedinf.SeedError):
        bat.submit(wl.make_uniforms(cfg, 1))                      # empty batch
    with pytest.raises(seedinf.SeedError):
        bat.add(5, frames[0])                                     # actor out of range
    bat.add(2, frames[0])
    with pytest.raises(seedinf.SeedError):
        bat.add(2, frames[1])                                     # twice in one batch
    bat.add(0, frames[0])
    bat.reserve(1)[...] = frames[1]                               # written straight into the pinned staging row
    bat.add_many(np.array([3]), frames[3:4], np.zeros(1, np.float32), np.zeros(1, np.uint8))
    with pytest.raises(seedinf.SeedError):
        bat.add(4, frames[4])                                     # a fifth row, max_batch is 4
    with pytest.raises(seedinf.SeedError):
        bat.submit(None)                                          # Gumbel-max needs uniforms
    un = wl.make_uniforms(cfg, 4, seed=5)
    t = bat.submit(un)
    got = bat.wait(t)
    obs = np.stack([frames[0], frames[0], frames[1], frames[3]])  # rows in the order they were added: actors 2, 0, 1, 3
    ref = orc.forward(oracle.make_arch(cfg), w, obs, uniforms=un)
    near = ref["margin"] <= 2 * 2e-2 * np.maximum(1.0, np.abs(ref["logits"]).max(axis=1))
    assert ((got == ref["action"]) | near).all()
    with pytest.raises(seedinf.SeedError):
        bat.read_state(0)                                         # feed-forward: no state
    with pytest.raises(seedinf.SeedError):
        bat.wait(t + 7)                                           # unknown ticket
    bat.close()
    net.close()
