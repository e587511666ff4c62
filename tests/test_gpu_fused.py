"""GPU parity of the quantizer fused behind its producer (vq_gelu_quantize,
vq_layernorm_quantize, vq_residual_quantize) against the CPU oracle.

The residual variant is fully determined in fp32 and is compared bit for bit (fp16 sum,
int8 codes, scales).  GELU and LayerNorm are evaluated by the oracle in fp64; the kernel
evaluates them in fp32 (its own order of summation, the device's exp and erf), so several
integer results are correct where a value sits next to a rounding boundary.  What is
unique is checked exactly, the rest for validity:

  * the kernel's fp32 value t~ of an element is within EPS_T * amax of the exact t
    (amax = largest magnitude of the token): a few fp32 ulps per operation, 1e-5 is ample;
  * hence the token scale agrees within EPS_T relative, and every code q satisfies
    |q * scale - t| <= scale / 2 * (1 + 2^-15) + EPS_T * amax   (Sec. 3.1: the rounding
    error of Eq. 2 is at most s/2; 2^-15 covers the single fp32 reciprocal);
  * every token that is not negligible (largest magnitude above 1e-10) holds a code of
    magnitude 127, no code exceeds it; a negligible token (GELU deep in its left tail, where
    the fp64 forms 1 + tanh u and 1 + erf z have themselves cancelled to nothing) only has to
    dequantize to less than that;
  * all but a small fraction of the codes equal the oracle's exactly.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

pytestmark = pytest.mark.gpu

EPS_T = 1e-5


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


TINY = 1e-10  # below this the fp64 forms have lost their own digits (1 + tanh u and 1 + erf z cancel)


def check_valid(q, s, t_f32, chan_mul, q_ref, s_ref, min_equal=0.995):
    t = t_f32.astype(np.float64)
    if chan_mul is not None:
        t = t * chan_mul.astype(np.float32).astype(np.float64)[None, :]
    amax = np.abs(t).max(axis=1)
    s64 = s.astype(np.float64)
    assert np.all(np.abs(s64 - s_ref.astype(np.float64)) <= 2 * EPS_T * s_ref.astype(np.float64) + TINY / 127)
    err = np.abs(q.astype(np.float64) * s64[:, None] - t)
    bound = 0.5 * s64[:, None] * (1 + 2.0 ** -15) + EPS_T * amax[:, None] + TINY
    assert np.all(err <= bound), f"worst excess {(err - bound).max():.3e}"
    assert np.abs(q.astype(np.int32)).max(initial=0) <= 127
    nz = amax > TINY
    assert np.all(np.abs(q[nz].astype(np.int32)).max(axis=1) == 127)
    equal = float((q[nz] == q_ref[nz]).mean()) if nz.any() else 1.0
    assert equal >= min_equal, f"only {equal:.4f} of the codes equal the oracle's"
    return equal


def rows(seed, M, K, spread=True):
    g = np.random.default_rng(seed)
    x = g.standard_normal((M, K))
    if spread:
        x = x * g.uniform(0.05, 20, (M, 1)) + g.uniform(-3, 3, (M, 1))
    return x.astype(np.float16), g


FUSED_SHAPES = [(1, 8), (5, 64), (37, 1152), (130, 4608), (7, 4096), (3, 8192), (9, 2048), (6, 520),
                (3, 3584), (1000, 1152), (2, 5000), (11, 384), (11, 1280), (11, 2304)]


@pytest.mark.parametrize("M,K", FUSED_SHAPES)
@pytest.mark.parametrize("approximate", [False, True])
@pytest.mark.parametrize("with_mul", [False, True])
def test_gelu_quantize(vq, oracle, M, K, approximate, with_mul):
    say(f"gelu_quantize M={M} K={K} approximate={approximate} mul={with_mul}")
    h, g = rows(100 + M + K, M, K, spread=False)
    h = (h.astype(np.float32) * 2.5).astype(np.float16)
    if M > 2:
        h[1] = 0
        h[2, :] = np.float16(-9.0)  # a token deep in the left tail: tiny negative values
    cm = np.exp(g.uniform(np.log(0.25), np.log(4), K)).astype(np.float32) if with_mul else None
    t, q_ref, s_ref = oracle.gelu_quantize(h, cm, approximate)
    q, s = vq.vq_gelu_quantize(dev(h), approximate, dev(cm))
    torch.cuda.synchronize()
    check_valid(host(q), host(s), t, cm, q_ref, s_ref)


@pytest.mark.parametrize("M,K", FUSED_SHAPES)
@pytest.mark.parametrize("mod", ["none", "scale_shift", "shift_mul"])
def test_layernorm_quantize(vq, oracle, M, K, mod):
    say(f"layernorm_quantize M={M} K={K} mod={mod}")
    x, g = rows(200 + M + K, M, K)
    if M > 2:
        x[1] = np.float16(3.0)  # a constant token: nothing to normalise
    T = max(1, M // 3)
    B = (M + T - 1) // T
    sc = (g.standard_normal((B, K)) * 0.3).astype(np.float32) if mod == "scale_shift" else None
    sh = (g.standard_normal((B, K)) * 0.5).astype(np.float32) if mod != "none" else None
    cm = np.exp(g.uniform(np.log(0.25), np.log(4), K)).astype(np.float32) if mod == "shift_mul" else None
    t, q_ref, s_ref = oracle.layernorm_quantize(x, sc, sh, T, 1e-6, cm)
    q, s = vq.vq_layernorm_quantize(dev(x), dev(sc), dev(sh), T, 1e-6, dev(cm))
    torch.cuda.synchronize()
    check_valid(host(q), host(s), t, cm, q_ref, s_ref)


@pytest.mark.parametrize("M,K", FUSED_SHAPES)
@pytest.mark.parametrize("with_gate", [False, True])
def test_residual_quantize_bit_exact(vq, oracle, M, K, with_gate):
    say(f"residual_quantize M={M} K={K} gate={with_gate}")
    x, g = rows(300 + M + K, M, K)
    y = (g.standard_normal((M, K)) * g.uniform(0.1, 5, (M, 1))).astype(np.float16)
    if M > 2:
        y[1] = (-x[1].astype(np.float32)).astype(np.float16)  # the sum of this token is zero
    T = max(1, M // 2)
    B = (M + T - 1) // T
    gate = g.standard_normal((B, K)).astype(np.float32) if with_gate else None
    if with_gate and M > 2:
        gate[(1 // T)] = 1.0
    cm = np.exp(g.uniform(np.log(0.25), np.log(4), K)).astype(np.float32) if with_gate else None
    r_ref, q_ref, s_ref = oracle.residual_quantize(x, y, gate, T, cm)
    r, q, s = vq.vq_residual_quantize(dev(x), dev(y), dev(gate), T, None, dev(cm))
    torch.cuda.synchronize()
    assert np.array_equal(host(r).view(np.uint16), r_ref.view(np.uint16))
    assert np.array_equal(host(q), q_ref)
    assert np.array_equal(host(s).view(np.uint32), s_ref.view(np.uint32))


def test_fused_calls_rejected_or_empty(vq):
    from paper_2406_02540_amd.binding import VqError
    x = torch.zeros((4, 12), dtype=torch.float16, device="cuda")  # K not a multiple of 8
    with pytest.raises(VqError) as e:
        vq.vq_gelu_quantize(x)
    assert e.value.status == 2
    big = torch.zeros((1, 8200), dtype=torch.float16, device="cuda")  # beyond the register-resident rows
    with pytest.raises(VqError):
        vq.vq_layernorm_quantize(big)
    empty = torch.zeros((0, 64), dtype=torch.float16, device="cuda")
    q, s = vq.vq_gelu_quantize(empty, True)
    assert q.shape == (0, 64) and s.shape == (0,)
    r, q, s = vq.vq_residual_quantize(empty, empty)
    assert r.shape == (0, 64)


# ---- at the sizes of the video-DiT linears (the shapes bench.py times) ---------------------

def test_full_size_gelu_feeds_fc2(vq, oracle):
    M, K = 32768, 4608
    say(f"full size gelu_quantize {M}x{K}")
    g = np.random.default_rng(4242)
    h = (g.standard_normal((M, K), dtype=np.float32) * 1.5).astype(np.float16)
    t, q_ref, s_ref = oracle.gelu_quantize(h, None, True)
    q, s = vq.vq_gelu_quantize(dev(h), True)
    torch.cuda.synchronize()
    check_valid(host(q), host(s), t, None, q_ref, s_ref, min_equal=0.999)


def test_full_size_layernorm_feeds_qkv_and_residual_feeds_it(vq, oracle):
    M, K, T = 32768, 1152, 16384
    say(f"full size residual + layernorm {M}x{K}")
    g = np.random.default_rng(4343)
    sigma = np.exp(g.uniform(np.log(0.1), np.log(10), K)).astype(np.float32)
    x = (g.standard_normal((M, K), dtype=np.float32) * sigma).astype(np.float16)
    y = (g.standard_normal((M, K), dtype=np.float32) * 0.5).astype(np.float16)
    gate = (g.standard_normal((2, K)) * 0.5).astype(np.float32)
    sc = (g.standard_normal((2, K)) * 0.3).astype(np.float32)
    sh = (g.standard_normal((2, K)) * 0.5).astype(np.float32)
    r_ref, q_ref, s_ref = oracle.residual_quantize(x, y, gate, T, None)
    r, q, s = vq.vq_residual_quantize(dev(x), dev(y), dev(gate), T)
    torch.cuda.synchronize()
    assert np.array_equal(host(r).view(np.uint16), r_ref.view(np.uint16))
    assert np.array_equal(host(q), q_ref) and np.array_equal(host(s).view(np.uint32), s_ref.view(np.uint32))
    t, q_ref, s_ref = oracle.layernorm_quantize(r_ref, sc, sh, T, 1e-6, None)
    q, s = vq.vq_layernorm_quantize(r, dev(sc), dev(sh), T, 1e-6)
    torch.cuda.synchronize()
    check_valid(host(q), host(s), t, None, q_ref, s_ref, min_equal=0.999)


# ---- rotation-based balancing: block Hadamard transform fused with the quantizer (Sec. 4.2) ----

HADAMARD_SHAPES = [(1, 128), (5, 256), (37, 1152), (130, 4608), (7, 4096), (3, 8192), (9, 2176), (1000, 1152),
                   (11, 384), (11, 1280), (11, 2304)]


@pytest.mark.parametrize("M,K", HADAMARD_SHAPES)
@pytest.mark.parametrize("with_mul", [False, True])
def test_hadamard_quantize(vq, oracle, M, K, with_mul):
    say(f"hadamard_quantize M={M} K={K} mul={with_mul}")
    x, g = rows(400 + M + K, M, K)
    x[:, g.integers(0, K, max(1, K // 100))] *= np.float16(30)  # outlier channels: what the rotation is for
    if M > 2:
        x[1] = 0
    cm = np.exp(g.uniform(np.log(0.25), np.log(4), K)).astype(np.float32) if with_mul else None
    t, q_ref, s_ref = oracle.hadamard_quantize(x, cm)
    q, s = vq.vq_hadamard_quantize(dev(x), dev(cm))
    torch.cuda.synchronize()
    check_valid(host(q), host(s), t, None, q_ref, s_ref)


def test_rotate_weight_and_rotated_layer(vq, oracle):
    g = np.random.default_rng(4545)
    M, N, K = 300, 264, 1152
    x = g.standard_normal((M, K)).astype(np.float32)
    x[:, g.integers(0, K, 12)] *= 50          # time-varying outlier channels
    x = x.astype(np.float16)
    w = (g.standard_normal((N, K)) * 0.02).astype(np.float32)
    s = np.exp(g.uniform(np.log(0.5), np.log(2), K)).astype(np.float32)
    cm = (np.float32(1) / s).astype(np.float32)
    b = (g.standard_normal(N) * 0.01).astype(np.float16)
    # weight side: the GPU rotation against the oracle's (fp32 butterflies against fp64 sums)
    w_rot_ref = oracle.rotate_weight(w, s)
    w_rot = vq.vq_rotate_weight(dev(w), dev(s))
    torch.cuda.synchronize()
    norm = np.sqrt((w_rot_ref.astype(np.float64) ** 2).reshape(N, K // 128, 128).sum(axis=2)).repeat(128, axis=1)
    assert np.all(np.abs(host(w_rot).astype(np.float64) - w_rot_ref) <= 1e-6 * norm + 1e-12)
    w_in_place = dev(w)
    vq.vq_rotate_weight(w_in_place, dev(s), out=w_in_place)  # input and output may be one buffer
    torch.cuda.synchronize()
    assert np.array_equal(host(w_in_place), host(w_rot))
    # the whole rotated W8A8 layer on the GPU ...
    wq, ws = vq.vq_quantize_weight(w_rot, None, 8)
    xq, xs = vq.vq_hadamard_quantize(dev(x), dev(cm))
    y = vq.vq_gemm_w8a8(xq, xs, wq, ws, dev(b))
    torch.cuda.synchronize()
    # ... stays within the rounding-error bound of Eq. 2 around the exact product (Sec. 4.2: the
    # rotation leaves X W^T unchanged), and is closer to it than the layer without rotation
    exact = x.astype(np.float64) @ w.astype(np.float64).T + b.astype(np.float64)
    xr = oracle.hadamard_rotate(x, cm).astype(np.float64)
    bound = (np.abs(xr) @ np.full((K, 1), 1.0)) * (host(ws).astype(np.float64)[None, :] / 2) \
        + host(xs).astype(np.float64)[:, None] / 2 * np.abs(w_rot_ref.astype(np.float64)).sum(axis=1)[None, :] \
        + K * host(xs).astype(np.float64)[:, None] * host(ws).astype(np.float64)[None, :] / 4
    err_rot = np.abs(host(y).astype(np.float64) - exact)
    assert np.all(err_rot <= bound + 2.0 ** -10 * np.abs(exact) + 1e-3)
    wq0, ws0 = vq.vq_quantize_weight(dev(w), dev(s), 8)
    xq0, xs0 = vq.vq_quantize_per_token(dev(x), dev(cm))
    y0 = vq.vq_gemm_w8a8(xq0, xs0, wq0, ws0, dev(b))
    torch.cuda.synchronize()
    err_plain = np.abs(host(y0).astype(np.float64) - exact)
    say(f"rms error with rotation {np.sqrt((err_rot ** 2).mean()):.4e}, without {np.sqrt((err_plain ** 2).mean()):.4e}")
    assert np.sqrt((err_rot ** 2).mean()) < np.sqrt((err_plain ** 2).mean())


def test_hadamard_calls_rejected(vq):
    from paper_2406_02540_amd.binding import VqError
    x = torch.zeros((4, 192), dtype=torch.float16, device="cuda")  # K not a multiple of 128
    with pytest.raises(VqError) as e:
        vq.vq_hadamard_quantize(x)
    assert e.value.status == 2
    with pytest.raises(VqError):
        vq.vq_rotate_weight(torch.zeros((4, 192), device="cuda"))


# ---- the layer behind a producer in one call: bit for bit the two separate calls -------------

LAYER_SHAPES = [(8, 300, 264, 1152), (4, 300, 264, 1152), (8, 517, 392, 640), (4, 130, 1160, 4608),
                (8, 2900, 2824, 1152), (8, 1, 8, 128)]


def _layer(seed, bits, M, N, K, oracle):
    g = np.random.default_rng(seed)
    x = (g.standard_normal((M, K)) * g.uniform(0.1, 8, (M, 1))).astype(np.float16)
    w = (g.standard_normal((N, K)) * 0.03).astype(np.float32)
    s = np.exp(g.uniform(np.log(0.5), np.log(2), K)).astype(np.float32)
    b = (g.standard_normal(N) * 0.05).astype(np.float16)
    return g, x, w, s, (np.float32(1) / s).astype(np.float32), b


@pytest.mark.parametrize("bits,M,N,K", LAYER_SHAPES)
def test_producer_linear_equals_the_two_calls(vq, oracle, bits, M, N, K):
    say(f"producer linear bits={bits} M={M} N={N} K={K}")
    g, x, w, s, cm, b = _layer(7000 + M + N + K + bits, bits, M, N, K, oracle)
    gemm = vq.vq_gemm_w8a8 if bits == 8 else vq.vq_gemm_w4a8
    wq, ws = vq.vq_quantize_weight(dev(w), dev(s), bits)
    T = max(1, M // 2)
    B = (M + T - 1) // T
    sc = (g.standard_normal((B, K)) * 0.3).astype(np.float32)
    sh = (g.standard_normal((B, K)) * 0.5).astype(np.float32)
    gate = g.standard_normal((B, K)).astype(np.float32)
    y_in = (g.standard_normal((M, K)) * 0.7).astype(np.float16)
    dx, dcm, db = dev(x), dev(cm), dev(b)

    q, xs = vq.vq_layernorm_quantize(dx, dev(sc), dev(sh), T, 1e-6, dcm)
    want = gemm(q, xs, wq, ws, db)
    got = vq.vq_layernorm_linear(dx, wq, bits, ws, dev(sc), dev(sh), T, 1e-6, dcm, db)
    torch.cuda.synchronize()
    assert torch.equal(got, want)

    for approximate in (False, True):
        q, xs = vq.vq_gelu_quantize(dx, approximate, dcm)
        want = gemm(q, xs, wq, ws, db)
        got = vq.vq_gelu_linear(dx, wq, bits, ws, approximate, dcm, db)
        torch.cuda.synchronize()
        assert torch.equal(got, want)

    r_want, q, xs = vq.vq_residual_quantize(dx, dev(y_in), dev(gate), T, None, dcm)
    want = gemm(q, xs, wq, ws, db)
    r_got, got = vq.vq_residual_linear(dx, dev(y_in), wq, bits, ws, dev(gate), T, None, dcm, db)
    torch.cuda.synchronize()
    assert torch.equal(r_got, r_want) and torch.equal(got, want)
    # this producer is fully determined: the oracle's layer on the oracle's residual stream
    r_ref, _, _ = oracle.residual_quantize(x, y_in, gate, T, cm)
    assert np.array_equal(host(r_got).view(np.uint16), r_ref.view(np.uint16))
    rows_ = np.unique(np.concatenate([[0, M - 1], g.integers(0, M, 24)]))
    wq_ref, ws_ref = oracle.quantize_weight(w, s, bits)
    assert np.array_equal(host(ws).view(np.uint32), ws_ref.view(np.uint32))
    ref = oracle.linear(r_ref[rows_], cm, wq_ref if bits == 8 else oracle.pack_int4(wq_ref), bits, ws_ref, b)
    from parity_util import assert_fp16_close
    assert_fp16_close(host(got)[rows_], ref["y"], ref["acc"], ref["x_scale"], ws_ref, b)

    if K % 128 == 0:
        w_rot = vq.vq_rotate_weight(dev(w), dev(s))
        wq_r, ws_r = vq.vq_quantize_weight(w_rot, None, bits)
        q, xs = vq.vq_hadamard_quantize(dx, dcm)
        want = gemm(q, xs, wq_r, ws_r, db)
        got = vq.vq_hadamard_linear(dx, dcm, wq_r, bits, ws_r, db)
        torch.cuda.synchronize()
        assert torch.equal(got, want)


def test_producer_linear_rejected_or_empty(vq):
    from paper_2406_02540_amd.binding import VqError
    w = torch.zeros((8, 192), dtype=torch.int8, device="cuda")
    ws = torch.ones((8,), dtype=torch.float32, device="cuda")
    x = torch.zeros((4, 192), dtype=torch.float16, device="cuda")
    with pytest.raises(VqError) as e:
        vq.vq_hadamard_linear(x, None, w, 8, ws)       # K not whole blocks of 128
    assert e.value.status == 2
    with pytest.raises(VqError) as e:
        vq.vq_gelu_linear(x, w, 8, ws, workspace=torch.zeros((64,), dtype=torch.uint8, device="cuda"))
    assert e.value.status == 4
    empty = torch.zeros((0, 192), dtype=torch.float16, device="cuda")
    assert vq.vq_layernorm_linear(empty, w, 8, ws).shape == (0, 8)
    r, y = vq.vq_residual_linear(empty, empty, w, 8, ws)
    assert r.shape == (0, 192) and y.shape == (0, 8)
