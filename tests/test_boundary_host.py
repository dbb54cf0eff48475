"""Host-only checks of the C ABI: the library loads, exports every declared
symbol, and validation / weight counting work without touching a device."""
import ctypes as C
import os
import re

import pytest

from paper_1910_06591_amd import seedinf, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(seedinf.LIB_PATH):
        seedinf.build_library()
    return seedinf.load_library()


def test_exports_match_header(lib):
    hdr = open(os.path.join(ROOT, "include", "seedinf.h")).read()
    declared = set(re.findall(r"\b(seed_(?:infer|batcher)_[a-z_]+)\s*\(", hdr))
    assert declared == set(seedinf.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_struct_layout_matches_header():
    # 3 + 1 + 1 + 12 + 1 + 4 + 8 int32 fields after struct_size
    assert C.sizeof(seedinf.SeedArch) == 4 * (1 + 3 + 1 + 1 + 12 + 1 + 4 + 8)


def test_weight_count_and_features(lib):
    for cfg in wl.CONFIGS.values():
        a = seedinf.make_arch(cfg, precision="fp32")
        assert seedinf.weight_count(a) == wl.weight_count(cfg)
        h, w, c = wl.torso_out_shape(cfg)
        assert seedinf.torso_features(a) == h * w * c
        st, msg = seedinf.validate(a)
        assert st == 0, msg


@pytest.mark.parametrize("field,value", [
    ("struct_size", 8), ("obs_h", 0), ("obs_c", -1), ("torso", 7), ("fc_units", 0), ("lstm_units", -2),
    ("num_actions", 0), ("num_actions", 65), ("head", 3), ("select", 2), ("precision", 5), ("max_batch", 0),
    ("n_conv", 0), ("n_conv", 5),
])
def test_validation_rejects_bad_fields(lib, field, value):
    a = seedinf.make_arch(wl.CONFIGS["C1"])
    setattr(a, field, value)
    st, msg = seedinf.validate(a)
    assert st == 1 and msg
    assert seedinf.weight_count(a) == 0
    # create reports the same error before any device call (there is no device here)
    h = C.c_void_p()
    assert lib.seed_infer_create(C.byref(a), None, 0, C.byref(h)) == 1
    assert not h.value


def test_validation_conv_geometry(lib):
    a = seedinf.make_arch(wl.CONFIGS["C1"])
    a.conv_k[1] = 40                       # larger than its 20x20 input
    assert seedinf.validate(a)[0] == 1
    a = seedinf.make_arch(wl.CONFIGS["C1"])
    a.conv_stride[0] = 0
    assert seedinf.validate(a)[0] == 1
    a = seedinf.make_arch(wl.CONFIGS["C2"], precision="fp32")
    a.head_hidden = 0
    assert seedinf.validate(a)[0] == 1
    a = seedinf.make_arch(wl.CONFIGS["C3"], precision="fp32")
    a.n_sections = 0
    assert seedinf.validate(a)[0] == 1


def test_create_rejects_null_and_wrong_count(lib):
    a = seedinf.make_arch(wl.CONFIGS["C1"])
    h = C.c_void_p()
    assert lib.seed_infer_create(C.byref(a), None, wl.weight_count(wl.CONFIGS["C1"]), C.byref(h)) == 1
    buf = (C.c_float * 4)()
    assert lib.seed_infer_create(C.byref(a), buf, 4, C.byref(h)) == 1
    assert b"n_weights" in lib.seed_infer_last_error(None)
    assert lib.seed_infer_create(C.byref(a), buf, 4, None) == 1
    assert lib.seed_infer_create(None, buf, 4, C.byref(h)) == 1
    # NULL handles are tolerated
    lib.seed_infer_destroy(None)
    assert lib.seed_infer_step(None, 1, *([None] * 13)) == 1


def test_probe_library_loads_and_exports():
    """bench.py's measurement probes (the MFMA-only loop and the streaming copy) live in their own library."""
    if not os.path.exists(seedinf.PROBE_LIB_PATH):
        seedinf.build_library()
    probe = seedinf.load_probe_library()
    for name in ("seed_probe_mfma_bf16", "seed_probe_mfma_flops", "seed_probe_copy"):
        assert hasattr(probe, name)
    # 1 block x 8 wavefronts x 1 iteration x 64 MFMAs of 16 x 16 x 32 multiply-adds
    assert probe.seed_probe_mfma_flops(1, 1) == 8 * 64 * 2 * 16 * 16 * 32


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU: any other --gpus value ends with a message and a non-zero status before anything
    touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
