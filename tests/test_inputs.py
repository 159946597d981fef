"""The synthetic workloads have the sizes the paper prints (Table 2; Sec. 3.4)."""
import os

import numpy as np
import torch

from paper_2512_17570_amd import inputs as I

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_model_shapes.txt")


def _gold():
    models, vals = {}, {}
    for line in open(GOLD):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "model":
            models[f[1]] = tuple(int(x) for x in f[2:])
        else:
            vals[f[0]] = float(f[1])
    return models, vals


def test_layer_numel_matches_paper_figures():
    models, vals = _gold()
    h65 = models["65B"][2]
    assert abs(I.layer_numel(h65) / vals["layer_params_65B"] - 1) < 2e-3      # paper: "approximately 8.05e8"
    assert abs(8 * 2048 * h65 / vals["checkpoint_elems_65B"] - 1) < 2e-3
    # layers x per-layer parameters is the bulk of the model size the table names
    for name, total in (("30B", 30e9), ("65B", 65e9), ("175B", 175e9)):
        layers, _, h = models[name]
        assert abs(layers * I.layer_numel(h) / total - 1) < 0.03
    assert I.WORKLOADS["gpt65b_layer_h8192_k16"].h == h65
    assert I.WORKLOADS["gpt175b_layer_h12288_k8_split"].h == models["175B"][2]
    assert I.WORKLOADS["gpt30b_layer_h7168_k16"].h == models["30B"][2]


def test_layer_numel_values_and_segments():
    assert I.layer_numel(1024) == 12_596_224
    assert I.layer_numel(4096) == 201_379_840
    assert I.layer_numel(8192) == 805_412_864
    assert I.layer_numel(12288) == 1_812_099_072
    assert I.WORKLOADS["gpt65b_8layers_streamed_k8"].n == 6_443_302_912
    for h in (64, 1024):
        assert sum(c for _, c in I.layer_segments(h)) == I.layer_numel(h) == 12 * h * h + 13 * h


def test_generators_are_seeded_and_distributed_as_stated():
    n = 1 << 18
    p, m, v = I.make_states(n, seed=0)
    p2, m2, v2 = I.make_states(n, seed=0)
    assert torch.equal(p, p2) and torch.equal(m, m2) and torch.equal(v, v2)
    p3, _, _ = I.make_states(n, seed=1)
    assert not torch.equal(p, p3)
    assert abs(float(p.std()) / 0.02 - 1) < 0.02 and abs(float(m.std()) / 1e-3 - 1) < 0.02
    assert float(v.min()) >= 0 and abs(float(v.mean()) / 1e-6 - 1) < 0.03
    g = I.make_grads(n, 3, 1e-3, seed=0)
    assert len(g) == 3 and g[0].dtype == torch.bfloat16 and not torch.equal(g[0], g[1])
    assert abs(float(g[0].float().std()) / 1e-3 - 1) < 0.02
    go = I.make_grads(n, 1, 1e-3, seed=0, outlier_frac=1e-3, outlier_scale=100.0)[0].float()
    frac = float((go.abs() > 0.02).float().mean())          # 20 sigma: only scaled entries get there
    assert 0.3e-3 < frac < 1.5e-3
    bits = I.bf16_bits(g[0])
    assert bits.dtype == np.uint16 and bits.shape == (n,)
