"""ctypes front end of the CPU oracle (test infrastructure, not product code).

Only tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It never imports the HIP library or
its binding, and they never import it.

Two builds of ``seed_oracle.c`` are produced: ``f32`` (activations stored as
float, dot products accumulated in double) is the oracle the GPU is compared
with; ``f64`` stores everything in double and serves to bound the f32
build's own rounding in the pins.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "seed_oracle.c")


def _lib_path(kind: str) -> str:
    return os.path.join(_HERE, f"libseed_oracle_{kind}.so")


def build(force: bool = False) -> None:
    """Compile both oracle builds with gcc (-O2, OpenMP over batch rows)."""
    for kind, defs in (("f32", []), ("f64", ["-DORACLE_F64"])):
        out = _lib_path(kind)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-ffp-contract=off",
               *defs, _SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)


class Arch(C.Structure):
    _fields_ = [
        ("obs_h", C.c_int32), ("obs_w", C.c_int32), ("obs_c", C.c_int32),
        ("torso", C.c_int32),
        ("n_conv", C.c_int32),
        ("conv_ch", C.c_int32 * 4), ("conv_k", C.c_int32 * 4), ("conv_stride", C.c_int32 * 4),
        ("n_sections", C.c_int32),
        ("section_ch", C.c_int32 * 4),
        ("fc_units", C.c_int32), ("lstm_units", C.c_int32), ("num_actions", C.c_int32),
        ("head", C.c_int32), ("head_hidden", C.c_int32), ("select", C.c_int32),
    ]


def make_arch(cfg: dict) -> Arch:
    """Build the oracle's arch struct from a plain config dict (see
    paper_1910_06591_amd.workloads for the dict's keys)."""
    a = Arch()
    a.obs_h, a.obs_w, a.obs_c = cfg["obs_h"], cfg["obs_w"], cfg["obs_c"]
    a.torso = cfg["torso"]
    convs = cfg.get("convs", [])
    a.n_conv = len(convs)
    for i, (ch, k, s) in enumerate(convs):
        a.conv_ch[i], a.conv_k[i], a.conv_stride[i] = ch, k, s
    secs = cfg.get("sections", [])
    a.n_sections = len(secs)
    for i, ch in enumerate(secs):
        a.section_ch[i] = ch
    a.fc_units = cfg["fc_units"]
    a.lstm_units = cfg.get("lstm_units", 0)
    a.num_actions = cfg["num_actions"]
    a.head = cfg.get("head", 0)
    a.head_hidden = cfg.get("head_hidden", 0)
    a.select = cfg.get("select", 0)
    return a


class Oracle:
    """Thin typed wrapper; every method maps to one exported C function."""

    def __init__(self, kind: str = "f32"):
        assert kind in ("f32", "f64")
        path = _lib_path(kind)
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_SRC):
            build()
        self.lib = C.CDLL(path)
        self.kind = kind
        self.dtype = np.float32 if kind == "f32" else np.float64
        self._real = C.c_float if kind == "f32" else C.c_double
        assert self.lib.oracle_sizeof_real() == np.dtype(self.dtype).itemsize
        self.lib.oracle_weight_count.restype = C.c_int64
        self.lib.oracle_torso_features.restype = C.c_int64

    # -- helpers
    def _r(self, a):
        return np.ascontiguousarray(a, dtype=self.dtype)

    def _p(self, a):
        return a.ctypes.data_as(C.c_void_p) if a is not None else None

    # -- layers
    def normalise(self, obs):
        obs = np.ascontiguousarray(obs, dtype=np.uint8)
        y = np.empty(obs.shape, self.dtype)
        self.lib.oracle_normalise(self._p(obs), C.c_int64(obs.size), self._p(y))
        return y

    def out_size(self, n, k, stride, same):
        return self.lib.oracle_out_size(int(n), int(k), int(stride), int(same))

    def conv2d(self, x, w, b, stride, same):
        x, w = self._r(x), self._r(w)
        H, W, Cin = x.shape
        k, k2, cin2, Cout = w.shape
        assert k == k2 and cin2 == Cin
        b = self._r(b) if b is not None else None
        OH, OW = self.out_size(H, k, stride, same), self.out_size(W, k, stride, same)
        y = np.empty((OH, OW, Cout), self.dtype)
        self.lib.oracle_conv2d(self._p(x), H, W, Cin, self._p(w), self._p(b), k, stride,
                               int(same), Cout, self._p(y))
        return y

    def maxpool(self, x):
        x = self._r(x)
        H, W, Cc = x.shape
        y = np.empty((self.out_size(H, 3, 2, 1), self.out_size(W, 3, 2, 1), Cc), self.dtype)
        self.lib.oracle_maxpool_3x3_s2(self._p(x), H, W, Cc, self._p(y))
        return y

    def relu(self, x):
        x = self._r(x)
        y = np.empty_like(x)
        self.lib.oracle_relu(self._p(x), C.c_int64(x.size), self._p(y))
        return y

    def dense(self, x, w, b):
        x, w = self._r(x), self._r(w)
        b = self._r(b) if b is not None else None
        y = np.empty(w.shape[1], self.dtype)
        self.lib.oracle_dense(self._p(x), w.shape[0], self._p(w), self._p(b), w.shape[1], self._p(y))
        return y

    def residual_block(self, x, wflat):
        x, wflat = self._r(x), self._r(wflat)
        H, W, Cc = x.shape
        assert wflat.size == 2 * (9 * Cc * Cc + Cc)
        y = np.empty_like(x)
        self.lib.oracle_residual_block(self._p(x), H, W, Cc, self._p(wflat), self._p(y))
        return y

    def lstm_cell(self, feat, prev_action, A, prev_reward, h, c, w, b):
        feat, h, c, w, b = map(self._r, (feat, h, c, w, b))
        F, H = feat.size, h.size
        assert w.shape == (F + A + 1 + H, 4 * H) and b.size == 4 * H
        ho, co = np.empty(H, self.dtype), np.empty(H, self.dtype)
        self.lib.oracle_lstm_cell(self._p(feat), F, int(prev_action), int(A),
                                  self._real(float(prev_reward)), self._p(h), self._p(c), H,
                                  self._p(w), self._p(b), self._p(ho), self._p(co))
        return ho, co

    def head_policy_value(self, core, A, wflat):
        core, wflat = self._r(core), self._r(wflat)
        n = core.size
        assert wflat.size == n * A + A + n + 1
        logits, value = np.empty(A, self.dtype), np.empty(1, self.dtype)
        self.lib.oracle_head_policy_value(self._p(core), n, A, self._p(wflat), self._p(logits),
                                          self._p(value))
        return logits, value[0]

    def head_dueling(self, core, hid, A, wflat):
        core, wflat = self._r(core), self._r(wflat)
        n = core.size
        assert wflat.size == 2 * (n * hid + hid) + hid + 1 + hid * A + A
        q, value = np.empty(A, self.dtype), np.empty(1, self.dtype)
        self.lib.oracle_head_dueling(self._p(core), n, hid, A, self._p(wflat), self._p(q),
                                     self._p(value))
        return q, value[0]

    def softmax(self, logits):
        logits = self._r(logits)
        p = np.empty_like(logits)
        self.lib.oracle_softmax(self._p(logits), logits.size, self._p(p))
        return p

    def select_greedy(self, logits):
        logits = self._r(logits)
        m = np.zeros(1, self.dtype)
        a = self.lib.oracle_select_greedy(self._p(logits), logits.size, self._p(m))
        return a, m[0]

    def select_gumbel(self, logits, u):
        logits, u = self._r(logits), self._r(u)
        m = np.zeros(1, self.dtype)
        pert = np.empty_like(logits)
        a = self.lib.oracle_select_gumbel(self._p(logits), self._p(u), logits.size,
                                          self._p(pert), self._p(m))
        return a, pert, m[0]

    # -- whole network
    def weight_count(self, arch: Arch) -> int:
        return int(self.lib.oracle_weight_count(C.byref(arch)))

    def torso_features(self, arch: Arch) -> int:
        return int(self.lib.oracle_torso_features(C.byref(arch)))

    def episode_state(self, done, h_in, c_in):
        h_in, c_in = self._r(h_in), self._r(c_in)
        h0, c0 = np.empty_like(h_in), np.empty_like(c_in)
        self.lib.oracle_episode_state(int(done), self._p(h_in), self._p(c_in), h_in.size, self._p(h0), self._p(c0))
        return h0, c0

    def epsilon_greedy(self, selected, A, eps, u0, u1):
        r = self.dtype.type if hasattr(self.dtype, "type") else self.dtype
        ct = C.c_double if np.dtype(self.dtype) == np.float64 else C.c_float
        self.lib.oracle_epsilon_greedy.restype = C.c_int
        return int(self.lib.oracle_epsilon_greedy(int(selected), int(A), ct(float(r(eps))), ct(float(r(u0))), ct(float(r(u1)))))

    def forward(self, arch: Arch, weights, obs, prev_action=None, prev_reward=None,
                h_in=None, c_in=None, uniforms=None, want_intermediates=False,
                done=None, epsilon=None, explore_u=None):
        """Returns a dict of numpy arrays: action, logits, value, probs, margin
        and, with a recurrent core, h and c; plus torso_feat / fc_act on request.
        done [B] uint8, epsilon [B] and explore_u [B, 2] are optional (episode
        flags and epsilon-greedy exploration)."""
        obs = np.ascontiguousarray(obs, dtype=np.uint8)
        B = obs.shape[0]
        A, Hn = arch.num_actions, arch.lstm_units
        weights = self._r(weights)
        assert weights.size == self.weight_count(arch), (weights.size, self.weight_count(arch))
        assert obs.shape[1:] == (arch.obs_h, arch.obs_w, arch.obs_c)
        pa = pr = hi = ci = un = None
        if Hn > 0:
            pa = np.ascontiguousarray(prev_action, dtype=np.int32)
            pr, hi, ci = self._r(prev_reward), self._r(h_in), self._r(c_in)
            assert pa.shape == (B,) and pr.shape == (B,) and hi.shape == (B, Hn) and ci.shape == (B, Hn)
        if arch.select:
            un = self._r(uniforms)
            assert un.shape == (B, A)
        out = {
            "action": np.empty(B, np.int32),
            "logits": np.empty((B, A), self.dtype),
            "value": np.empty(B, self.dtype),
            "probs": np.empty((B, A), self.dtype),
            "margin": np.empty(B, self.dtype),
        }
        if Hn > 0:
            out["h"] = np.empty((B, Hn), self.dtype)
            out["c"] = np.empty((B, Hn), self.dtype)
        if want_intermediates:
            out["torso_feat"] = np.empty((B, self.torso_features(arch)), self.dtype)
            out["fc_act"] = np.empty((B, arch.fc_units), self.dtype)
        dn = ep = eu = None
        if done is not None:
            dn = np.ascontiguousarray(done, dtype=np.uint8)
            assert dn.shape == (B,) and Hn > 0
        if epsilon is not None:
            ep, eu = self._r(epsilon), self._r(explore_u)
            assert ep.shape == (B,) and eu.shape == (B, 2)
        rc = self.lib.oracle_forward_ext(
            C.byref(arch), self._p(weights), B, self._p(obs), self._p(pa), self._p(pr),
            self._p(hi), self._p(ci), self._p(un), self._p(dn), self._p(ep), self._p(eu),
            self._p(out["action"]), self._p(out["logits"]), self._p(out["value"]),
            self._p(out.get("h")), self._p(out.get("c")), self._p(out["probs"]),
            self._p(out["margin"]), self._p(out.get("torso_feat")), self._p(out.get("fc_act")))
        if rc != 0:
            raise ValueError("oracle_forward: unsupported arch")
        return out

    def unroll(self, arch: Arch, weights, obs, prev_action=None, prev_reward=None,
               h0=None, c0=None, uniforms=None, done=None):
        """Forward pass over stored trajectories, time-major (Section 3: a trajectory is
        unrolled step by step; Appendix A: unroll length): step t runs forward() on
        obs[t] with the recurrent state that step t-1 left, done[t] zeroing the state a
        row starts from.  obs [T, B, H, W, C]; prev_action, prev_reward, done [T, B];
        uniforms [T, B, A]; h0, c0 [B, Hn].  Returns action [T, B], logits [T, B, A],
        value [T, B], probs [T, B, A], margin [T, B] and the final h, c [B, Hn]."""
        obs = np.ascontiguousarray(obs, dtype=np.uint8)
        T = obs.shape[0]
        Hn = arch.lstm_units
        h, c = (self._r(h0), self._r(c0)) if Hn > 0 else (None, None)
        steps = []
        for t in range(T):
            o = self.forward(arch, weights, obs[t],
                             prev_action[t] if Hn > 0 else None, prev_reward[t] if Hn > 0 else None,
                             h, c, uniforms[t] if arch.select else None,
                             done=done[t] if done is not None else None)
            if Hn > 0:
                h, c = o["h"], o["c"]
            steps.append(o)
        out = {k: np.stack([o[k] for o in steps]) for k in ("action", "logits", "value", "probs", "margin")}
        if Hn > 0:
            out["h"], out["c"] = h, c
        return out

