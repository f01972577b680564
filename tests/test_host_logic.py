"""Host-side logic that holds none of the method's arithmetic: the seeded input generators, the
grid of the numerical study, the benchmark's pass list and the argument checks of the Python
binding that run before anything touches a GPU."""
import numpy as np
import pytest
import torch

from paper_2605_08565_amd import study
from paper_2605_08565_amd import workloads as W


def test_study_grid_is_the_papers():
    """Numerical Study: 151 standard deviations evenly spaced in [0.0005, 0.05], block sizes
    4, 8, 16, 32, five recipes."""
    s = study.study_sigmas()
    assert len(s) == 151 and s[0] == 0.0005 and s[-1] == 0.05
    assert np.allclose(np.diff(s), (0.05 - 0.0005) / 150, rtol=1e-9)
    assert study.BLOCKS == (4, 8, 16, 32)
    assert sorted(study.RECIPES.values()) == [0, 1, 2, 3, 4]


def test_study_tensor_rows_follow_their_sigma():
    sig = study.study_sigmas(5)
    x = study.study_tensor(sig, 4000, 8)
    assert x.shape == (5 * 4000, 8) and x.dtype == np.float32
    assert (x == study.study_tensor(sig, 4000, 8)).all()              # seeded
    per = x.reshape(5, -1).std(axis=1)
    assert np.allclose(per, sig, rtol=0.02)
    assert abs(float(x.mean())) < 1e-3


def test_bf16_cast_is_round_to_nearest_even():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(200_000) * np.exp2(rng.uniform(-30, 30, 200_000))).astype(np.float32)
    ties = (np.arange(1, 4000, dtype=np.uint32) << np.uint32(16) | np.uint32(0x8000)).view(np.float32)   # exact ties
    x = np.concatenate([x, ties, -ties, np.float32([0.0, -0.0, 1.0, 3.0e38])])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = W.f32_to_bf16_bits(x)
    assert (got == want).all()
    assert (W.bf16_bits_to_f32(got).view(np.uint32) == (got.astype(np.uint32) << 16)).all()


def test_benchmark_tensors_shapes_seeds_and_prefix_stability():
    c1 = W.config1()
    assert c1.shape == (1024, 4096) and c1.dtype == np.float32
    assert abs(float(c1.std()) - 1.0) < 0.01
    a = W.config2(rows=64)
    assert a.shape == (64, 14336) and a.dtype == np.uint16
    assert (a[:16] == W.config2(rows=16)).all()                       # the first rows do not depend on the row count
    assert (a == W.config2(rows=64)).all()
    f = W.bf16_bits_to_f32(a).astype(np.float64)
    assert abs(f.std() / (0.02 * np.sqrt(2.0)) - 1.0) < 0.1           # 0.02 * Student-t(4): variance 2 * 0.02^2
    assert np.abs(f).max() > 0.2                                      # heavy tails


def test_activation_tensor_has_seeded_outlier_channels():
    x = W.bf16_bits_to_f32(W.config3(rows=512))
    assert x.shape == (512, 4096)
    assert (W.config3(rows=128) == W.config3(rows=512)[:128]).all()
    col_std = x.std(axis=0)
    out = col_std > 10.0
    assert out.sum() == 41                                            # 1 % of 4096 channels, times 50
    assert abs(float(col_std[~out].mean()) - 1.0) < 0.05 and abs(float(col_std[out].mean()) - 50.0) < 5.0


def test_model_layer_matrices():
    assert list(W.LAYER_SHAPES) == ["q", "k", "v", "o", "gate", "up", "down"] and W.N_LAYERS == 32
    assert sum(r * c for r, c in W.LAYER_SHAPES.values()) == 218_103_808
    k0, k1 = W.layer_matrix(0, "k", rows=8), W.layer_matrix(1, "k", rows=8)
    assert k0.shape == (8, 4096) and (k0 != k1).any()
    assert (W.layer_matrix(0, "k", rows=8) == k0).all()
    assert (W.layer_matrix(0, "v", rows=8) != k0).any()               # every matrix has its own seed


def test_benchmark_pass_list():
    import bench

    step = bench.step_passes()
    names = [p[1] for p in step]
    assert len(names) == len(set(names)) == 22
    quant = [p for p in step if p[0] == "quant"]
    assert len(quant) == 20 and sum(1 for p in quant if p[4] == bench.BRUTE) == 4
    assert sum(1 for p in step if p[0] == "absmax") == 1 and sum(1 for p in step if p[0] == "dequant") == 1
    # the brute-force passes come last, the issue-bound streaming passes right before them
    kinds = ["brute" if p[4] == bench.BRUTE and p[0] == "quant" else "other" for p in step]
    assert kinds[-4:] == ["brute"] * 4 and "brute" not in kinds[:-4]
    extra = [p[2] for p in bench.extra_passes()]
    assert len(extra) == len(set(extra))
    assert not set(extra) & set(names)


def test_binding_checks_arguments_before_any_launch():
    """Wrong devices, shapes and dtypes are refused by the binding itself."""
    from paper_2605_08565_amd import mxq

    x = torch.zeros((4, 32), dtype=torch.bfloat16)                    # on the CPU
    with pytest.raises(ValueError):
        mxq.quantize(x, 16, mxq.SCALE_E4M3, mxq.RECIPE_ABSMAX)
    with pytest.raises(ValueError):
        mxq.quantize_batch([x], 16, mxq.SCALE_E4M3, mxq.RECIPE_ABSMAX)
