"""The synthetic input recipe: seeded, shaped as the five configurations state."""
import numpy as np

from paper_2406_02540_amd import workloads as wl


def test_streams_are_reproducible_and_distinct():
    a = wl.rng(1, 0, 0, wl.T_X).standard_normal(8)
    b = wl.rng(1, 0, 0, wl.T_X).standard_normal(8)
    c = wl.rng(1, 0, 0, wl.T_W).standard_normal(8)
    assert np.array_equal(a, b) and not np.array_equal(a, c)


def test_config_shapes_and_ops():
    assert [(s.M, s.K, s.N, s.w_bits) for s in wl.config1()] == [(256, 1152, 1152, 8)]
    assert [(s.M, s.K, s.N, s.w_bits) for s in wl.config3()] == [(256, 1152, 1152, 4)]
    c2 = {s.name: (s.M, s.K, s.N) for s in wl.config2()}
    assert c2 == {"qkv": (8192, 1152, 3456), "proj": (8192, 1152, 1152),
                  "fc1": (8192, 1152, 4608), "fc2": (8192, 4608, 1152)}
    c4 = {s.name: (s.M, s.K, s.N) for s in wl.config4()}
    assert c4["ca_kv"] == (240, 4096, 2304) and c4["fc2"] == (32768, 4608, 1152)
    assert abs(sum(s.ops for s in wl.config4()) / 1e9 - 1048.2) < 0.1
    c5 = wl.config5()
    assert len(c5) == 168
    assert abs(sum(s.ops for s in c5[:6]) / 1e9 - 1135.2) < 0.1
    frac = np.mean([s.w_bits == 4 for s in c5])
    assert 0.2 < frac < 0.4
    assert wl.config5_step_scale(1) == 0.55 and wl.config5_step_scale(20) == 1.5


def test_config1_inputs():
    d = wl.draw_layer(wl.config1()[0])
    assert d.x.dtype == np.float16 and d.x.shape == (256, 1152)
    assert d.w.dtype == np.float32 and d.bias.dtype == np.float16 and d.chan_mul is None
    std = d.x.astype(np.float32).std(axis=0)
    assert (std > 15).sum() == 8                     # the 8 outlier channels, x30
    assert abs(np.median(std) - 1.0) < 0.1
    assert abs(d.w.std() - 0.02) < 1e-3 and abs(d.bias.astype(np.float32).std() - 0.01) < 2e-3
    again = wl.draw_layer(wl.config1()[0])
    assert np.array_equal(again.x, d.x) and np.array_equal(again.w, d.w)


def test_balanced_and_gelu_and_video_inputs():
    spec = wl.config2()[3]
    small = wl.LayerSpec(spec.name, 64, spec.K, 32, 8, cfg=2, layer=3, x_kind="gelu", balanced=True)
    d = wl.draw_layer(small)
    assert d.x.astype(np.float32).min() > -0.2       # GELU output is bounded below
    assert d.s.min() >= 0.25 and d.s.max() <= 4.0
    assert np.array_equal(d.chan_mul, np.float32(1) / d.s)
    v = wl.LayerSpec("qkv", 512, 1152, 16, 8, cfg=4, layer=0, x_kind="video")
    x = wl.draw_x(v).astype(np.float32)
    std = x.std(axis=0)
    assert np.isfinite(x).all() and (std > 10.5).sum() >= 5 and std.min() < 0.2 and np.abs(x).max() < 65504
