"""ctypes binding over libseedinf's C ABI (include/seedinf.h).

Argument marshalling only: every step of the inference path runs in the HIP
library.  PyTorch supplies device memory and the stream.  There is no CPU
fallback: if the shared library is missing or a call fails, this raises.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
LIB_PATH = os.environ.get("SEEDINF_LIB", os.path.join(_PKG, "libseedinf.so"))
SOURCES = [os.path.join(_PKG, "csrc", f) for f in
           ("seedinf.hip", "plan.h", "kernels_fp32.h", "kernels_heads.h", "bf16_path.h", "bf16_common.h", "gemm_bf16.h", "gemm_bf16_lds.h",
            "conv_stack_bf16.h", "conv_stack_fused.h", "resnet_fused.h", "resnet_layerwise.h", "resnet_blockfused.h", "resnet_firstpool.h", "resnet_convpool.h", "resnet_convtile.h", "batcher.h", "host_pool.h")]
PROBE_SOURCE = os.path.join(_PKG, "csrc", "probe.hip")
PROBE_LIB_PATH = os.path.join(_PKG, "libseedprobe.so")
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]

STATUS = {0: "SEED_OK", 1: "SEED_ERR_INVALID_ARG", 2: "SEED_ERR_UNSUPPORTED_ARCH", 3: "SEED_ERR_BATCH_TOO_LARGE",
          4: "SEED_ERR_ALIASING", 5: "SEED_ERR_DEVICE", 6: "SEED_ERR_OOM"}
STATUS_BY_NAME = {v: k for k, v in STATUS.items()}
EXPORTS = ["seed_infer_weight_count", "seed_infer_validate", "seed_infer_create", "seed_infer_step",
           "seed_infer_step_ext", "seed_infer_step_static", "seed_infer_unroll", "seed_infer_set_weights",
           "seed_batcher_create", "seed_batcher_add", "seed_batcher_reserve", "seed_batcher_add_many", "seed_batcher_submit", "seed_batcher_wait",
           "seed_batcher_read_state", "seed_batcher_stream", "seed_batcher_last_error", "seed_batcher_destroy",
           "seed_infer_read_intermediate", "seed_infer_torso_features", "seed_infer_last_error",
           "seed_infer_destroy", "seed_infer_set_profiling", "seed_infer_profile_read"]


class SeedStepExt(C.Structure):
    """seed_step_ext_t: optional inputs of seed_infer_step_ext (device pointers, 0 = absent)."""
    _fields_ = [("struct_size", C.c_uint32), ("done", C.c_void_p), ("epsilon", C.c_void_p),
                ("explore_uniforms", C.c_void_p)]


class SeedError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS.get(status, status)}: {message}")
        self.status = status
        self.message = message


class SeedArch(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32),
        ("obs_h", C.c_int32), ("obs_w", C.c_int32), ("obs_c", C.c_int32),
        ("torso", C.c_int32),
        ("n_conv", C.c_int32),
        ("conv_ch", C.c_int32 * 4), ("conv_k", C.c_int32 * 4), ("conv_stride", C.c_int32 * 4),
        ("n_sections", C.c_int32),
        ("section_ch", C.c_int32 * 4),
        ("fc_units", C.c_int32), ("lstm_units", C.c_int32), ("num_actions", C.c_int32),
        ("head", C.c_int32), ("head_hidden", C.c_int32), ("select", C.c_int32),
        ("precision", C.c_int32), ("max_batch", C.c_int32),
    ]


def build_library(verbose: bool = False) -> str:
    """Compile csrc/ into libseedinf.so (and the measurement probes into
    libseedprobe.so) for gfx950 with hipcc (cross-compiles without a GPU)."""
    for src, out in ((SOURCES[0], LIB_PATH), (PROBE_SOURCE, PROBE_LIB_PATH)):
        cmd = ["hipcc", *HIPCC_FLAGS, src, "-o", out]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + r.stderr)
        if verbose:
            print(" ".join(cmd))
    return LIB_PATH


def load_probe_library():
    """libseedprobe.so: the MFMA-only loop and the streaming copy bench.py measures the chip's own peaks with."""
    import torch  # noqa: F401
    if not os.path.exists(PROBE_LIB_PATH):
        raise RuntimeError(f"{PROBE_LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = C.CDLL(PROBE_LIB_PATH)
    lib.seed_probe_mfma_bf16.restype = C.c_int
    lib.seed_probe_mfma_bf16.argtypes = [C.c_int, C.c_int, C.c_void_p, C.c_void_p]
    lib.seed_probe_mfma_flops.restype = C.c_double
    lib.seed_probe_mfma_flops.argtypes = [C.c_int, C.c_int]
    lib.seed_probe_copy.restype = C.c_int
    lib.seed_probe_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    return lib


_lib = None


def load_library():
    """Load libseedinf.so (torch first, so both share one HIP runtime)."""
    global _lib
    if _lib is not None:
        return _lib
    import torch  # noqa: F401  (loads the HIP runtime the library links against)
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = C.CDLL(LIB_PATH)
    lib.seed_infer_weight_count.restype = C.c_size_t
    lib.seed_infer_weight_count.argtypes = [C.POINTER(SeedArch)]
    lib.seed_infer_torso_features.restype = C.c_size_t
    lib.seed_infer_torso_features.argtypes = [C.POINTER(SeedArch)]
    lib.seed_infer_validate.restype = C.c_int
    lib.seed_infer_validate.argtypes = [C.POINTER(SeedArch)]
    lib.seed_infer_create.restype = C.c_int
    lib.seed_infer_create.argtypes = [C.POINTER(SeedArch), C.c_void_p, C.c_size_t, C.POINTER(C.c_void_p)]
    lib.seed_infer_step.restype = C.c_int
    lib.seed_infer_step.argtypes = [C.c_void_p, C.c_int32] + [C.c_void_p] * 13
    lib.seed_infer_read_intermediate.restype = C.c_int
    lib.seed_infer_step_ext.restype = C.c_int
    lib.seed_infer_step_ext.argtypes = [C.c_void_p, C.c_int32] + [C.c_void_p] * 6 + [C.POINTER(SeedStepExt)] + [C.c_void_p] * 7
    lib.seed_infer_step_static.restype = C.c_int
    lib.seed_infer_step_static.argtypes = lib.seed_infer_step_ext.argtypes
    lib.seed_infer_set_weights.restype = C.c_int
    lib.seed_infer_unroll.restype = C.c_int
    lib.seed_infer_unroll.argtypes = [C.c_void_p, C.c_int32, C.c_int32] + [C.c_void_p] * 14
    lib.seed_infer_set_weights.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.seed_batcher_create.restype = C.c_int
    lib.seed_batcher_create.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_void_p)]
    lib.seed_batcher_add.restype = C.c_int
    lib.seed_batcher_add.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_float, C.c_uint8]
    lib.seed_batcher_reserve.restype = C.c_int
    lib.seed_batcher_reserve.argtypes = [C.c_void_p, C.c_int32, C.c_float, C.c_uint8, C.POINTER(C.c_void_p)]
    lib.seed_batcher_add_many.restype = C.c_int
    lib.seed_batcher_add_many.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.seed_batcher_submit.restype = C.c_int
    lib.seed_batcher_submit.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_int32)]
    lib.seed_batcher_wait.restype = C.c_int
    lib.seed_batcher_wait.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.POINTER(C.c_int32)]
    lib.seed_batcher_read_state.restype = C.c_int
    lib.seed_batcher_read_state.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
    lib.seed_batcher_stream.restype = C.c_void_p
    lib.seed_batcher_stream.argtypes = [C.c_void_p]
    lib.seed_batcher_last_error.restype = C.c_char_p
    lib.seed_batcher_last_error.argtypes = [C.c_void_p]
    lib.seed_batcher_destroy.restype = None
    lib.seed_batcher_destroy.argtypes = [C.c_void_p]
    lib.seed_infer_read_intermediate.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.seed_infer_last_error.restype = C.c_char_p
    lib.seed_infer_last_error.argtypes = [C.c_void_p]
    lib.seed_infer_set_profiling.restype = C.c_int
    lib.seed_infer_set_profiling.argtypes = [C.c_void_p, C.c_int32]
    lib.seed_infer_profile_read.restype = C.c_int
    lib.seed_infer_profile_read.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.POINTER(C.c_int32)]
    lib.seed_infer_destroy.restype = None
    lib.seed_infer_destroy.argtypes = [C.c_void_p]
    _lib = lib
    return lib


def make_arch(cfg: dict, max_batch: int | None = None, precision: str | None = None) -> SeedArch:
    """seed_arch_t from a workload config dict (see workloads.CONFIGS)."""
    a = SeedArch()
    a.struct_size = C.sizeof(SeedArch)
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
    prec = precision if precision is not None else cfg.get("precision", "fp32")
    a.precision = {"fp32": 0, "bf16": 1}[prec]
    a.max_batch = max_batch if max_batch is not None else cfg.get("batch", 1)
    return a


def weight_count(arch: SeedArch) -> int:
    return int(load_library().seed_infer_weight_count(C.byref(arch)))


def torso_features(arch: SeedArch) -> int:
    return int(load_library().seed_infer_torso_features(C.byref(arch)))


def validate(arch: SeedArch) -> tuple[int, str]:
    lib = load_library()
    st = lib.seed_infer_validate(C.byref(arch))
    return st, lib.seed_infer_last_error(None).decode()


def _ptr(t, dtype, shape, name):
    import torch
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a CUDA tensor")
    if t.dtype != dtype or tuple(t.shape) != tuple(shape) or not t.is_contiguous():
        raise TypeError(f"{name} must be contiguous {dtype} of shape {tuple(shape)}, got {t.dtype} {tuple(t.shape)}")
    return C.c_void_p(t.data_ptr())


class SeedInfer:
    """Handle on one network instance (seed_infer_create ... seed_infer_destroy)."""

    def __init__(self, arch: SeedArch, weights: np.ndarray):
        self.lib = load_library()
        self.arch = arch
        w = np.ascontiguousarray(weights, dtype=np.float32)
        self._h = C.c_void_p()
        st = self.lib.seed_infer_create(C.byref(arch), w.ctypes.data_as(C.c_void_p), w.size, C.byref(self._h))
        if st != 0:
            self._h = None
            raise SeedError(st, self.lib.seed_infer_last_error(None).decode())
        self.A, self.Hn = arch.num_actions, arch.lstm_units

    def close(self):
        if getattr(self, "_h", None):
            self.lib.seed_infer_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def step_raw(self, B, obs, prev_action, prev_reward, h_in, c_in, uniforms, action, logits, value,
                 h_out, c_out, probs, stream=0):
        """Direct call with raw pointers/ints (used by the error-path tests)."""
        st = self.lib.seed_infer_step(self._h, B, obs, prev_action, prev_reward, h_in, c_in, uniforms, action,
                                      logits, value, h_out, c_out, probs, stream)
        return st, self.lib.seed_infer_last_error(self._h).decode()

    def step_ext_raw(self, B, obs, prev_action, prev_reward, h_in, c_in, uniforms, ext, action, logits, value,
                     h_out, c_out, probs, stream=0):
        """Direct call of seed_infer_step_ext with raw pointers/ints; `ext` is a SeedStepExt or None."""
        st = self.lib.seed_infer_step_ext(self._h, B, obs, prev_action, prev_reward, h_in, c_in, uniforms,
                                          C.byref(ext) if ext is not None else None, action, logits, value,
                                          h_out, c_out, probs, stream)
        return st, self.lib.seed_infer_last_error(self._h).decode()

    def set_weights(self, weights, stream=None):
        """Replace the handle's weights (host numpy array, same layout as at creation); steps enqueued
        afterwards on the same stream use them."""
        import torch
        w = np.ascontiguousarray(weights, dtype=np.float32)
        s = torch.cuda.current_stream().cuda_stream if stream is None else stream
        st = self.lib.seed_infer_set_weights(self._h, w.ctypes.data_as(C.c_void_p), w.size, C.c_void_p(s))
        if st != 0:
            raise SeedError(st, self.lib.seed_infer_last_error(self._h).decode())

    def step(self, obs, prev_action=None, prev_reward=None, h_in=None, c_in=None, uniforms=None,
             want_probs=True, out=None, stream=None, done=None, epsilon=None, explore_uniforms=None,
             static_workspace=False):
        """Run one inference step on device tensors; returns a dict of device
        tensors (allocated here with torch unless `out` supplies them).  done [B] uint8,
        epsilon [B] and explore_uniforms [B, 2] are the optional episode flags and
        epsilon-greedy inputs (seed_infer_step_ext).  static_workspace=True calls
        seed_infer_step_static (the library's static device workspace) instead."""
        import torch
        a = self.arch
        B = obs.shape[0]
        dev = obs.device
        if out is None:
            out = {"action": torch.empty(B, dtype=torch.int32, device=dev),
                   "logits": torch.empty(B, self.A, dtype=torch.float32, device=dev),
                   "value": torch.empty(B, dtype=torch.float32, device=dev)}
            if self.Hn:
                out["h"] = torch.empty(B, self.Hn, dtype=torch.float32, device=dev)
                out["c"] = torch.empty(B, self.Hn, dtype=torch.float32, device=dev)
            if want_probs:
                out["probs"] = torch.empty(B, self.A, dtype=torch.float32, device=dev)
        s = torch.cuda.current_stream(dev).cuda_stream if stream is None else stream
        ext = None
        if done is not None or epsilon is not None or explore_uniforms is not None:
            addr = lambda p_: None if p_ is None else p_.value
            ext = SeedStepExt(C.sizeof(SeedStepExt),
                              addr(_ptr(done, torch.uint8, (B,), "done")),
                              addr(_ptr(epsilon, torch.float32, (B,), "epsilon")),
                              addr(_ptr(explore_uniforms, torch.float32, (B, 2), "explore_uniforms")))
        entry = self.lib.seed_infer_step_static if static_workspace else self.lib.seed_infer_step_ext
        st = entry(
            self._h, B,
            _ptr(obs, torch.uint8, (B, a.obs_h, a.obs_w, a.obs_c), "obs"),
            _ptr(prev_action, torch.int32, (B,), "prev_action"),
            _ptr(prev_reward, torch.float32, (B,), "prev_reward"),
            _ptr(h_in, torch.float32, (B, self.Hn), "h_in"),
            _ptr(c_in, torch.float32, (B, self.Hn), "c_in"),
            _ptr(uniforms, torch.float32, (B, self.A), "uniforms"),
            C.byref(ext) if ext is not None else None,
            _ptr(out["action"], torch.int32, (B,), "action"),
            _ptr(out["logits"], torch.float32, (B, self.A), "logits"),
            _ptr(out["value"], torch.float32, (B,), "value"),
            _ptr(out.get("h"), torch.float32, (B, self.Hn), "h_out"),
            _ptr(out.get("c"), torch.float32, (B, self.Hn), "c_out"),
            _ptr(out.get("probs"), torch.float32, (B, self.A), "probs"),
            C.c_void_p(s))
        if st != 0:
            raise SeedError(st, self.lib.seed_infer_last_error(self._h).decode())
        return out

    def unroll(self, obs, prev_action=None, prev_reward=None, h0=None, c0=None, uniforms=None, done=None,
               want_probs=True, stream=None):
        """seed_infer_unroll on time-major device tensors: obs [T, B, H, W, C]; prev_action, prev_reward,
        done [T, B]; uniforms [T, B, A]; h0, c0 [B, Hn].  Returns action [T, B], logits [T, B, A],
        value [T, B], probs [T, B, A] and, with a core, the final h, c [B, Hn]."""
        import torch
        a = self.arch
        T, B = obs.shape[0], obs.shape[1]
        dev = obs.device
        out = {"action": torch.empty(T, B, dtype=torch.int32, device=dev),
               "logits": torch.empty(T, B, self.A, dtype=torch.float32, device=dev),
               "value": torch.empty(T, B, dtype=torch.float32, device=dev)}
        if self.Hn:
            out["h"] = torch.empty(B, self.Hn, dtype=torch.float32, device=dev)
            out["c"] = torch.empty(B, self.Hn, dtype=torch.float32, device=dev)
        if want_probs:
            out["probs"] = torch.empty(T, B, self.A, dtype=torch.float32, device=dev)
        s = torch.cuda.current_stream(dev).cuda_stream if stream is None else stream
        st = self.lib.seed_infer_unroll(
            self._h, T, B,
            _ptr(obs, torch.uint8, (T, B, a.obs_h, a.obs_w, a.obs_c), "obs"),
            _ptr(prev_action, torch.int32, (T, B), "prev_action"),
            _ptr(prev_reward, torch.float32, (T, B), "prev_reward"),
            _ptr(done, torch.uint8, (T, B), "done"),
            _ptr(h0, torch.float32, (B, self.Hn), "h0"),
            _ptr(c0, torch.float32, (B, self.Hn), "c0"),
            _ptr(uniforms, torch.float32, (T, B, self.A), "uniforms"),
            _ptr(out["action"], torch.int32, (T, B), "action"),
            _ptr(out["logits"], torch.float32, (T, B, self.A), "logits"),
            _ptr(out["value"], torch.float32, (T, B), "value"),
            _ptr(out.get("h"), torch.float32, (B, self.Hn), "h_out"),
            _ptr(out.get("c"), torch.float32, (B, self.Hn), "c_out"),
            _ptr(out.get("probs"), torch.float32, (T, B, self.A), "probs"),
            C.c_void_p(s))
        if st != 0:
            raise SeedError(st, self.lib.seed_infer_last_error(self._h).decode())
        return out

    def unroll_raw(self, T, B, obs, prev_action, prev_reward, done, h0, c0, uniforms, action, logits, value,
                   h_out, c_out, probs, stream=0):
        """Direct call of seed_infer_unroll with raw pointers/ints (error-path tests)."""
        st = self.lib.seed_infer_unroll(self._h, T, B, obs, prev_action, prev_reward, done, h0, c0, uniforms,
                                        action, logits, value, h_out, c_out, probs, stream)
        return st, self.lib.seed_infer_last_error(self._h).decode()

    def set_profiling(self, enable: bool):
        st = self.lib.seed_infer_set_profiling(self._h, int(enable))
        if st != 0:
            raise SeedError(st, self.lib.seed_infer_last_error(self._h).decode())

    def profile_read(self):
        """(summed torso-kernel milliseconds, number of steps covered) since the last read."""
        ms, n = C.c_float(), C.c_int32()
        st = self.lib.seed_infer_profile_read(self._h, C.byref(ms), C.byref(n))
        if st != 0:
            raise SeedError(st, self.lib.seed_infer_last_error(self._h).decode())
        return ms.value, n.value

    def read_intermediate(self, which: int, B: int, stream=None):
        """Diagnostic tap: 0 = torso features [B, H*W*C], 1 = linear output [B, fc_units] (fp32)."""
        import torch
        n = torso_features(self.arch) if which == 0 else self.arch.fc_units
        dst = torch.empty(B, n, dtype=torch.float32, device="cuda")
        s = torch.cuda.current_stream().cuda_stream if stream is None else stream
        st = self.lib.seed_infer_read_intermediate(self._h, which, B, C.c_void_p(dst.data_ptr()), dst.numel(),
                                                   C.c_void_p(s))
        if st != 0:
            raise SeedError(st, self.lib.seed_infer_last_error(self._h).decode())
        return dst


class Batcher:
    """Host batching front-end of one SeedInfer handle (seed_batcher_*): numpy in, numpy out."""

    def __init__(self, net: SeedInfer, n_actors: int):
        self.net, self.lib = net, net.lib
        self.A, self.Hn = net.A, net.Hn
        self.max_rows = net.arch.max_batch
        h = C.c_void_p()
        st = self.lib.seed_batcher_create(net._h, n_actors, C.byref(h))
        if st != 0:
            raise SeedError(st, self.lib.seed_batcher_last_error(None).decode())
        self._b = h

    def _check(self, st):
        if st != 0:
            raise SeedError(st, self.lib.seed_batcher_last_error(self._b).decode())

    def add(self, actor: int, obs: np.ndarray, prev_reward: float = 0.0, done: bool = False):
        obs = np.ascontiguousarray(obs, dtype=np.uint8)
        a = self.net.arch
        assert obs.shape == (a.obs_h, a.obs_w, a.obs_c), obs.shape
        self._check(self.lib.seed_batcher_add(self._b, actor, obs.ctypes.data_as(C.c_void_p), float(prev_reward), int(bool(done))))

    def reserve(self, actor: int, prev_reward: float = 0.0, done: bool = False) -> np.ndarray:
        """Adds a row and returns a writable uint8 view of its frame slot in the pinned staging memory."""
        slot = C.c_void_p()
        self._check(self.lib.seed_batcher_reserve(self._b, actor, float(prev_reward), int(bool(done)), C.byref(slot)))
        a = self.net.arch
        n = a.obs_h * a.obs_w * a.obs_c
        buf = (C.c_uint8 * n).from_address(slot.value)
        return np.frombuffer(buf, dtype=np.uint8).reshape(a.obs_h, a.obs_w, a.obs_c)

    def add_many(self, actors, obs, prev_rewards, dones):
        actors = np.ascontiguousarray(actors, dtype=np.int32)
        obs = np.ascontiguousarray(obs, dtype=np.uint8)
        rew = np.ascontiguousarray(prev_rewards, dtype=np.float32)
        dn = np.ascontiguousarray(dones, dtype=np.uint8)
        a = self.net.arch
        n = actors.size
        assert obs.shape == (n, a.obs_h, a.obs_w, a.obs_c) and rew.shape == (n,) and dn.shape == (n,)
        p = lambda x: x.ctypes.data_as(C.c_void_p)
        self._check(self.lib.seed_batcher_add_many(self._b, n, p(actors), p(obs), p(rew), p(dn)))

    def submit(self, uniforms=None, epsilon=None, explore_uniforms=None) -> int:
        keep = [None if x is None else np.ascontiguousarray(x, dtype=np.float32) for x in (uniforms, epsilon, explore_uniforms)]
        ptr = [None if x is None else x.ctypes.data_as(C.c_void_p) for x in keep]
        t = C.c_int32()
        self._check(self.lib.seed_batcher_submit(self._b, ptr[0], ptr[1], ptr[2], C.byref(t)))
        return t.value

    def wait(self, ticket: int) -> np.ndarray:
        out = np.empty(self.max_rows, np.int32)
        n = C.c_int32()
        self._check(self.lib.seed_batcher_wait(self._b, ticket, out.ctypes.data_as(C.c_void_p), out.size, C.byref(n)))
        return out[:n.value].copy()

    def read_state(self, actor: int):
        h, c = np.empty(self.Hn, np.float32), np.empty(self.Hn, np.float32)
        self._check(self.lib.seed_batcher_read_state(self._b, actor, h.ctypes.data_as(C.c_void_p), c.ctypes.data_as(C.c_void_p)))
        return h, c

    @property
    def stream(self) -> int:
        return self.lib.seed_batcher_stream(self._b) or 0

    def close(self):
        if getattr(self, "_b", None):
            self.lib.seed_batcher_destroy(self._b)
            self._b = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
