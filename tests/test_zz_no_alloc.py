"""seed_infer_step_static (the step on the library's static device workspace) against seed_infer_step_ext.

Both entry points launch the same kernels; only where the activations between them live differs, so every
output must agree bit for bit.  Each case makes two calls in a row, the second with a smaller batch (the array
keeps the first call's contents), and a batch beyond the static workspace must be refused with no output
written."""
import numpy as np
import pytest

from paper_1910_06591_amd import seedinf, workloads as wl
from tests.parity import random_arch, to_device

pytestmark = pytest.mark.gpu


def both_ways(cfg, precision, batches):
    import torch
    w = wl.make_weights(cfg, bf16_representable=(precision == "bf16"))
    net = seedinf.SeedInfer(seedinf.make_arch(cfg, max_batch=max(batches), precision=precision), w)
    for B in batches:
        print(f"static workspace: {cfg['label']} {precision} B={B}", flush=True)
        dev = to_device(wl.make_batch(cfg, B))
        own = net.step(**dev)
        torch.cuda.synchronize()
        got = net.step(**dev, static_workspace=True)
        torch.cuda.synchronize()
        for k in own:
            a, b = own[k].cpu().numpy(), got[k].cpu().numpy()
            assert np.array_equal(a, b), f"{k} differs at B={B}: max abs diff {np.abs(a.astype(np.float64) - b).max()}"
    net.close()


@pytest.mark.parametrize("name,precision,batches", [
    ("C1", "fp32", (8, 3)),            # fp32 layer kernels: two activation buffers + linear rows
    ("C3", "bf16", (200, 67)),         # fused ResNet torso, LSTM core
    ("C2", "bf16", (64, 21)),          # fused conv stack, dueling hidden rows
    ("C4", "bf16", (48, 17)),          # Football torso, no core
])
def test_static_workspace_matches_own_workspace(name, precision, batches):
    both_ways(wl.CONFIGS[name], precision, batches)


def test_static_workspace_with_padded_rows_and_layerwise_paths():
    # widths that are not whole 32-value chunks (padding columns must be cleared) and the layer-by-layer kernels
    for seed in (0, 1, 2, 3, 5, 6):
        cfg = random_arch(seed, "bf16")
        st, _ = seedinf.validate(seedinf.make_arch(cfg, max_batch=40, precision="bf16"))
        if st != 0:
            continue
        both_ways(cfg, "bf16", (40, 9))


def test_static_workspace_rejects_what_does_not_fit():
    import torch
    cfg = wl.CONFIGS["C3"]
    B = 2048                                   # 8448 bytes per row: 17.3 MB > 16 MiB
    net = seedinf.SeedInfer(seedinf.make_arch(cfg, max_batch=B, precision="bf16"), wl.make_weights(cfg, bf16_representable=True))
    dev = to_device(wl.make_batch(cfg, B))
    out = {"action": torch.full((B,), -7, dtype=torch.int32, device="cuda"),
           "logits": torch.full((B, 15), -7.0, device="cuda"), "value": torch.full((B,), -7.0, device="cuda"),
           "h": torch.full((B, 256), -7.0, device="cuda"), "c": torch.full((B, 256), -7.0, device="cuda")}
    with pytest.raises(seedinf.SeedError) as e:
        net.step(**dev, out=out, want_probs=False, static_workspace=True)
    assert e.value.status == seedinf.STATUS_BY_NAME["SEED_ERR_BATCH_TOO_LARGE"] and "static workspace" in e.value.message
    torch.cuda.synchronize()
    assert all(bool((v == -7).all()) for v in out.values())
    # the largest batch that fits still runs
    Bok = (16 << 20) // 8448
    dev = to_device(wl.make_batch(cfg, Bok))
    a = net.step(**dev)
    b = net.step(**dev, static_workspace=True)
    torch.cuda.synchronize()
    assert all(torch.equal(a[k], b[k]) for k in a)
    net.close()
