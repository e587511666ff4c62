"""GPU parity of the two comparison kernels (Sec. 5.3: FP16 layers, and the "naive" static W8A8
baseline) against the CPU oracle.

vq_quantize_static is integer work: bit-exact.  vq_gemm_f16 sums exact fp16 products in fp32
in the matrix cores' order, the oracle in fp64: an output may differ by the fp32 accumulation
error, at most K * 2^-24 * sum_k |x_k w_k| (every partial sum is bounded by that sum), plus one
rounding to fp16 on each side (half a step of the rounded value):
    |g - r| <= ulp16(g)/2 + ulp16(r)/2 + K * 2^-24 * sum_k |x_k w_k|.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vq():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2406_02540_amd as pkg
    from paper_2406_02540_amd import binding
    binding.lib()  # raises if the HIP library is missing: there is no fallback
    return pkg


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.cpu().numpy()


def say(msg):
    print(msg, flush=True)


def assert_f16_gemm_close(got, ref, x, w, K, b=None):
    """|g - r| <= ulp(g)/2 + ulp(r)/2 + K * 2^-24 * (sum_k |x_k w_k| + |b|): the two sides round to fp16 once
    each (half a step of their own result) and differ before that by the fp32 accumulation error only (K - 1
    additions of products and one of the bias, each within 2^-24 of a partial sum no larger than the sum of
    the magnitudes).  How many
    outputs end up more than one step apart depends on how strongly the products of an output cancel, so no
    count of such outputs is asserted: the bound above is per element and complete."""
    s_abs = np.abs(x.astype(np.float64)) @ np.abs(w.astype(np.float64)).T
    # the step of a value towards larger magnitudes: at a power of two it is the larger of the two steps next to it
    step = lambda a: np.spacing(np.abs(a.astype(np.float16))).astype(np.float64)  # noqa: E731
    if b is not None:
        s_abs = s_abs + np.abs(b.astype(np.float64))[None, :]
    bound = 0.5 * step(got) + 0.5 * step(ref) + K * 2.0 ** -24 * s_abs
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    assert np.all(err <= bound), f"worst excess {(err - bound).max():.3e}"


F16_SHAPES = [(1, 8, 8), (5, 7, 64), (300, 200, 384), (256, 256, 128), (257, 264, 72), (513, 520, 200),
              (64, 1152, 1152), (700, 1030, 1160), (1024, 512, 4608)]


@pytest.mark.parametrize("M,N,K", F16_SHAPES)
@pytest.mark.parametrize("with_bias", [False, True])
def test_gemm_f16(vq, oracle, M, N, K, with_bias):
    say(f"gemm_f16 M={M} N={N} K={K} bias={with_bias}")
    g = np.random.default_rng(500 + M + N + K)
    x = (g.standard_normal((M, K)) * g.uniform(0.1, 4, (M, 1))).astype(np.float16)
    w = (g.standard_normal((N, K)) * 0.05).astype(np.float16)
    b = (g.standard_normal(N) * 0.2).astype(np.float16) if with_bias else None
    ref = oracle.gemm_f16(x, w, b)
    y = vq.vq_gemm_f16(dev(x), dev(w), dev(b))
    torch.cuda.synchronize()
    assert_f16_gemm_close(host(y), ref, x, w, K, b)


def test_gemm_f16_exact_integers_and_identity(vq):
    g = np.random.default_rng(77)
    M, N, K = 300, 264, 136
    x = g.integers(-8, 9, (M, K)).astype(np.float16)
    w = g.integers(-4, 5, (N, K)).astype(np.float16)
    y = host(vq.vq_gemm_f16(dev(x), dev(w)))
    assert np.array_equal(y.astype(np.int64), x.astype(np.int64) @ w.astype(np.int64).T)
    x = g.standard_normal((70, 256)).astype(np.float16)
    y = host(vq.vq_gemm_f16(dev(x), dev(np.eye(256, dtype=np.float16))))
    assert np.array_equal(y.view(np.uint16), x.view(np.uint16))


def test_gemm_f16_full_size_sampled_rows(vq, oracle):
    M, N, K = 32768, 4608, 1152
    say(f"full size gemm_f16 {M}x{K}->{N}")
    g = np.random.default_rng(78)
    x = g.standard_normal((M, K), dtype=np.float32).astype(np.float16)
    w = (g.standard_normal((N, K), dtype=np.float32) * 0.02).astype(np.float16)
    b = (g.standard_normal(N) * 0.01).astype(np.float16)
    y = host(vq.vq_gemm_f16(dev(x), dev(w), dev(b)))
    rows = np.unique(np.concatenate([[0, M - 1], g.integers(0, M, 96)]))
    ref = oracle.gemm_f16(x[rows], w, b)
    assert_f16_gemm_close(y[rows], ref, x[rows], w, K, b)


@pytest.mark.parametrize("M,K", [(1, 8), (5, 64), (37, 1152), (9, 333), (3, 1), (130, 4608), (1000, 1152)])
@pytest.mark.parametrize("with_mul", [False, True])
def test_quantize_static_bit_exact(vq, oracle, M, K, with_mul):
    say(f"quantize_static M={M} K={K} mul={with_mul}")
    g = np.random.default_rng(600 + M + K)
    x = (g.standard_normal((M, K)) * g.uniform(0.05, 10, (M, 1))).astype(np.float16)
    cm = np.exp(g.uniform(np.log(0.25), np.log(4), K)).astype(np.float32) if with_mul else None
    for scale in (0.037, 0.5, 1e-3):
        ref = oracle.quantize_static(x, scale, cm)
        q = vq.vq_quantize_static(dev(x), scale, dev(cm))
        torch.cuda.synchronize()
        assert np.array_equal(host(q), ref)


def test_static_w8a8_layer_matches_the_oracle_pipeline(vq, oracle):
    from parity_util import assert_fp16_close
    g = np.random.default_rng(79)
    M, N, K = 600, 520, 1152
    x = (g.standard_normal((M, K)) * 2).astype(np.float16)
    w = (g.standard_normal((N, K)) * 0.02).astype(np.float32)
    b = (g.standard_normal(N) * 0.01).astype(np.float16)
    wq, ws = oracle.quantize_weight(w, None, 8)
    scale = np.float32(np.abs(x.astype(np.float32)).max() / 127.0)  # calibrated once, for the whole tensor
    xs = np.full(M, scale, np.float32)
    xq_ref = oracle.quantize_static(x, float(scale))
    acc_ref = oracle.gemm_i8(xq_ref, wq)
    y_ref = oracle.dequant(acc_ref, xs, ws, b)
    xq = vq.vq_quantize_static(dev(x), float(scale))
    y, acc = vq.vq_gemm_w8a8(xq, dev(xs), dev(wq), dev(ws), dev(b), return_acc=True)
    torch.cuda.synchronize()
    assert np.array_equal(host(xq), xq_ref) and np.array_equal(host(acc), acc_ref)
    assert_fp16_close(host(y), y_ref, acc_ref, xs, ws, b)


def test_comparison_calls_rejected_or_empty(vq):
    from paper_2406_02540_amd.binding import VqError
    x = torch.zeros((4, 12), dtype=torch.float16, device="cuda")  # K not a multiple of 8
    w = torch.zeros((8, 12), dtype=torch.float16, device="cuda")
    with pytest.raises(VqError) as e:
        vq.vq_gemm_f16(x, w)
    assert e.value.status == 2
    with pytest.raises(VqError):
        vq.vq_quantize_static(x, 0.0)
    empty = torch.zeros((0, 64), dtype=torch.float16, device="cuda")
    assert vq.vq_quantize_static(empty, 1.0).shape == (0, 64)
    assert vq.vq_gemm_f16(empty, torch.zeros((8, 64), dtype=torch.float16, device="cuda")).shape == (0, 8)


# ---- offline calibration of Eq. 3's mask (Sec. 4.2) -------------------------------------------

@pytest.mark.parametrize("R,K", [(1, 1), (37, 50), (300, 1152), (5000, 333), (240, 4096), (4099, 1160)])
def test_channel_absmax_bit_exact(vq, oracle, R, K):
    say(f"channel_absmax R={R} K={K}")
    g = np.random.default_rng(700 + R + K)
    x = (g.standard_normal((R, K)) * np.exp(g.uniform(-2, 3, (1, K)))).astype(np.float16)
    if K > 3:
        x[:, 3] = 0
    got = vq.vq_channel_absmax(dev(x))
    torch.cuda.synchronize()
    assert np.array_equal(host(got), oracle.channel_absmax(x))
    w = g.standard_normal((R, K)).astype(np.float32)
    assert np.array_equal(host(vq.vq_channel_absmax(dev(w))), oracle.channel_absmax(w))
    # the running maximum over two batches is the maximum over both
    x2 = (g.standard_normal((max(1, R // 2), K)) * 40).astype(np.float16)
    vq.vq_channel_absmax(dev(x2), got, accumulate=True)
    torch.cuda.synchronize()
    assert np.array_equal(host(got), oracle.channel_absmax(np.concatenate([x, x2])))


@pytest.mark.parametrize("alpha", [0.0, 0.3, 0.5, 1.0])
def test_balance_mask(vq, oracle, alpha):
    g = np.random.default_rng(800)
    K = 1152
    ax = np.exp(g.uniform(-3, 5, K)).astype(np.float32)
    aw = np.exp(g.uniform(-6, 0, K)).astype(np.float32)
    ax[5] = 0; aw[9] = 0; ax[11] = 0; aw[11] = 0
    s_ref, cm_ref = oracle.balance_mask(ax, aw, alpha)
    s, cm = vq.vq_balance_mask(dev(ax), dev(aw), alpha)
    torch.cuda.synchronize()
    s, cm = host(s), host(cm)
    # powf against the oracle's fp64 pow: a few fp32 ulps; the reciprocal is the exact IEEE one
    assert np.allclose(s, s_ref, rtol=2e-6, atol=0) and np.all((s >= 1e-5) & (s <= 1e5))
    assert np.array_equal(cm, (np.float32(1) / s).astype(np.float32))


def test_calibrated_layer_end_to_end(vq, oracle):
    """Statistics, mask, weight quantizer, activation quantizer and GEMM, all on the device, against the
    oracle's pipeline fed with the device's mask (the mask itself is compared above)."""
    from parity_util import assert_fp16_close
    g = np.random.default_rng(801)
    M, N, K = 520, 264, 1152
    x = (g.standard_normal((M, K)) * np.exp(g.uniform(-2, 2, (1, K)))).astype(np.float16)
    w = (g.standard_normal((N, K)) * 0.02).astype(np.float32)
    b = (g.standard_normal(N) * 0.01).astype(np.float16)
    xd, wd = dev(x), dev(w)
    s, cm = vq.vq_balance_mask(vq.vq_channel_absmax(xd), vq.vq_channel_absmax(wd), 0.5)
    wq, ws = vq.vq_quantize_weight(wd, s, 8)
    y = vq.vq_linear(xd, cm, wq, 8, ws, dev(b))
    torch.cuda.synchronize()
    wq_ref, ws_ref = oracle.quantize_weight(w, host(s), 8)
    ref = oracle.linear(x, host(cm), wq_ref, 8, ws_ref, b)
    assert np.array_equal(host(wq), wq_ref) and np.array_equal(host(ws), ws_ref)
    assert_fp16_close(host(y), ref["y"], ref["acc"], ref["x_scale"], ws_ref, b)
