"""Pins the oracle's producer functions (GELU, LayerNorm + modulation, residual add:
the operations the quantizer is fused into, Sec. 5.1 "Hardware Implementation
Settings") to things other than themselves: library routines that compute the same
textbook function by another route (scipy's normal distribution function, torch's
float64 gelu and layer_norm, numpy's float32/float16 arithmetic), closed forms,
symmetries and hand-worked roundings.  Further down, in the same way: the block Hadamard
rotation (Sec. 4.2), the mask of Eq. 3 from absmax statistics, and the two comparison points of
Sec. 5.3 (FP16 layer, static quantizer).
"""
import numpy as np
import pytest
import torch
from scipy.special import ndtr


def _f16_grid():
    """Every finite fp16 value of magnitude at most 12 (GELU is x or 0 beyond)."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    v = bits.view(np.float16)
    keep = np.isfinite(v) & (np.abs(v.astype(np.float32)) <= 12.0)
    return v[keep].reshape(1, -1)


# ---- GELU -------------------------------------------------------------------------

def test_gelu_exact_is_x_times_normal_cdf(oracle):
    x = _f16_grid()
    want = x.astype(np.float64) * ndtr(x.astype(np.float64))  # scipy's Phi, not erf
    got = oracle.gelu(x, approximate=False).astype(np.float64)
    assert np.all(np.abs(got - want) <= 1e-7 * np.abs(want) + 1e-12 + np.abs(np.spacing(want.astype(np.float32))))


def test_gelu_known_values(oracle):
    # Phi(1) = 0.841344746068543, Phi(2) = 0.977249868051821 (standard normal table)
    x = np.array([[0.0, 1.0, -1.0, 2.0, -2.0]], np.float16)
    got = oracle.gelu(x, approximate=False)[0].astype(np.float64)
    want = np.array([0.0, 0.841344746068543, -0.158655253931457, 1.954499736103642, -0.045500263896358])
    assert np.allclose(got, want, rtol=2e-7, atol=1e-9)


def test_gelu_tanh_form_against_torch(oracle):
    x = _f16_grid()
    want = torch.nn.functional.gelu(torch.from_numpy(x.astype(np.float64)), approximate="tanh").numpy()
    got = oracle.gelu(x, approximate=True).astype(np.float64)
    assert np.all(np.abs(got - want) <= np.abs(np.spacing(want.astype(np.float32))) + 1e-12)
    # and the two forms differ by what the approximation is known for (< 5e-4 absolute), not more
    exact = oracle.gelu(x, approximate=False).astype(np.float64)
    d = np.abs(got - exact).max()
    assert 1e-5 < d < 5e-4


@pytest.mark.parametrize("approximate", [False, True])
def test_gelu_odd_part_is_half_x(oracle, approximate):
    # x Phi(x) - (-x) Phi(-x) = x (Phi(x) + Phi(-x)) = x, for both forms (tanh is odd)
    x = _f16_grid()
    pos = oracle.gelu(x, approximate).astype(np.float64)
    neg = oracle.gelu((-x).astype(np.float16), approximate).astype(np.float64)
    xf = x.astype(np.float64)
    assert np.all(np.abs((pos - neg) - xf) <= 2.5e-7 * np.abs(xf) + 1e-12)


@pytest.mark.parametrize("approximate", [False, True])
def test_gelu_tails(oracle, approximate):
    x = np.array([[8.0, 10.0, 100.0, 60000.0, -8.0, -10.0, -100.0, -60000.0]], np.float16)
    got = oracle.gelu(x, approximate)[0]
    assert np.array_equal(got[:4], x[0, :4].astype(np.float32))
    assert np.all(np.abs(got[4:]) < 1e-13) and not np.isnan(got).any()


# ---- LayerNorm + modulation -------------------------------------------------------

def test_layernorm_against_torch_float64(oracle):
    g = np.random.default_rng(11)
    for K in (8, 100, 1152):
        x = (g.standard_normal((9, K)) * g.uniform(0.1, 30, (9, 1)) + g.uniform(-5, 5, (9, 1))).astype(np.float16)
        want = torch.nn.functional.layer_norm(torch.from_numpy(x.astype(np.float64)), (K,), eps=1e-6).numpy()
        got = oracle.layernorm_modulate(x, eps=1e-6).astype(np.float64)
        assert np.all(np.abs(got - want) <= np.abs(np.spacing(want.astype(np.float32))) + 1e-12)


def test_layernorm_closed_forms(oracle):
    K = 64
    # +-a alternating: mean 0, variance a^2
    a = 3.0
    x = np.tile(np.array([a, -a], np.float16), K // 2)[None, :]
    got = oracle.layernorm_modulate(x, eps=1e-6)[0].astype(np.float64)
    assert np.allclose(got, x[0].astype(np.float64) / np.sqrt(a * a + 1e-6), rtol=1e-7)
    # 0, 1, ..., K-1: mean (K-1)/2, variance (K^2-1)/12
    x = np.arange(K, dtype=np.float16)[None, :]
    got = oracle.layernorm_modulate(x, eps=0.0)[0].astype(np.float64)
    want = (np.arange(K) - (K - 1) / 2) / np.sqrt((K * K - 1) / 12)
    assert np.allclose(got, want, rtol=1e-7, atol=1e-9)
    # a constant token has nothing to normalise: zeros, and the shift alone after modulation
    x = np.full((1, K), 7.0, np.float16)
    assert np.array_equal(oracle.layernorm_modulate(x, eps=1e-6), np.zeros((1, K), np.float32))
    sh = np.linspace(-1, 1, K, dtype=np.float32)[None, :]
    assert np.array_equal(oracle.layernorm_modulate(x, shift=sh, eps=1e-6), sh)


def test_layernorm_invariances(oracle):
    g = np.random.default_rng(12)
    x = g.integers(-40, 40, (5, 96)).astype(np.float16)
    base = oracle.layernorm_modulate(x, eps=0.0)
    # a shift of the whole token and a positive scaling leave it unchanged (eps = 0);
    # integers keep the fp16 inputs exact
    assert np.allclose(oracle.layernorm_modulate((x + 17).astype(np.float16), eps=0.0), base, rtol=0, atol=1e-6)
    assert np.allclose(oracle.layernorm_modulate((x * 4).astype(np.float16), eps=0.0), base, rtol=0, atol=1e-6)
    assert np.allclose(oracle.layernorm_modulate((-x).astype(np.float16), eps=0.0), -base, rtol=0, atol=1e-6)
    # what it returns has mean 0 and mean square var / (var + eps)
    t = oracle.layernorm_modulate(x, eps=1e-2).astype(np.float64)
    var = x.astype(np.float64).var(axis=1)
    assert np.allclose(t.mean(axis=1), 0, atol=1e-7)
    assert np.allclose((t * t).mean(axis=1), var / (var + 1e-2), rtol=1e-6)


def test_modulation_uses_the_sample_of_the_token(oracle):
    g = np.random.default_rng(13)
    M, K, T = 7, 32, 3  # samples of 3, 3 and 1 tokens
    x = g.standard_normal((M, K)).astype(np.float16)
    sc = g.standard_normal((3, K)).astype(np.float32)
    sh = g.standard_normal((3, K)).astype(np.float32)
    y = oracle.layernorm_modulate(x, eps=1e-6).astype(np.float64)
    got = oracle.layernorm_modulate(x, sc, sh, tokens_per_sample=T, eps=1e-6).astype(np.float64)
    b = np.arange(M) // T
    want = y * (1.0 + sc[b].astype(np.float64)) + sh[b].astype(np.float64)
    assert np.allclose(got, want, rtol=3e-7, atol=3e-7)
    # scale = -1 removes the token: the shift alone is left, exactly
    got = oracle.layernorm_modulate(x, -np.ones((3, K), np.float32), sh, tokens_per_sample=T)
    assert np.array_equal(got, sh[b])
    with pytest.raises(ValueError):
        oracle.layernorm_modulate(x, sc[:2], sh, tokens_per_sample=T)


# ---- residual add ------------------------------------------------------------------

def test_residual_hand_roundings(oracle):
    # fp16 has steps of 2 from 2048 on: 2049 -> 2048 (down), 2051 is a tie -> 2052 (even), 2053 -> 2052
    x = np.array([[2048, 2048, 2048, 1.0, 1.0]], np.float16)
    y = np.array([[1, 3, 5, 0.5, 3.0]], np.float16)
    assert oracle.residual(x, y)[0].tolist() == [2048.0, 2052.0, 2052.0, 1.5, 4.0]
    # gate 0.5: 1 + 0.25 = 1.25; gate fl(1/3) * 3 rounds to exactly 1 in fp32, so 1 + 1 = 2
    gate = np.array([[0.5, 0.5, 0.5, 0.5, np.float32(1.0) / np.float32(3.0)]], np.float32)
    got = oracle.residual(x, y, gate)[0].tolist()
    assert got == [2048.0, 2050.0, 2050.0, 1.25, 2.0]  # 2049.5 -> 2050, 2050.5 -> 2050


def test_residual_against_numpy_float32(oracle):
    g = np.random.default_rng(14)
    M, K, T = 10, 200, 4
    x = (g.standard_normal((M, K)) * 50).astype(np.float16)
    y = (g.standard_normal((M, K)) * 3).astype(np.float16)
    gate = g.standard_normal((3, K)).astype(np.float32)
    b = np.arange(M) // T
    want = (x.astype(np.float32) + gate[b] * y.astype(np.float32)).astype(np.float16)  # numpy rounds each step
    assert np.array_equal(oracle.residual(x, y, gate, tokens_per_sample=T).view(np.uint16), want.view(np.uint16))
    want = (x.astype(np.float32) + y.astype(np.float32)).astype(np.float16)
    assert np.array_equal(oracle.residual(x, y).view(np.uint16), want.view(np.uint16))


# ---- the quantizer on fp32 rows, and the three fused front ends --------------------

def test_quantize_rows_f32_reduces_to_the_fp16_quantizer(oracle):
    g = np.random.default_rng(15)
    x = (g.standard_normal((12, 160)) * g.uniform(0.01, 100, (12, 1))).astype(np.float16)
    x[3] = 0
    cm = np.exp(g.uniform(np.log(0.25), np.log(4), 160)).astype(np.float32)
    for mul in (None, cm):
        q16, s16 = oracle.quantize_per_token(x, mul)
        q32, s32 = oracle.quantize_rows_f32(x.astype(np.float32), mul)
        assert np.array_equal(q16, q32) and np.array_equal(s16.view(np.uint32), s32.view(np.uint32))


def test_quantize_rows_f32_error_bound_on_fp32_rows(oracle):
    g = np.random.default_rng(16)
    t = (g.standard_normal((20, 333)) * g.uniform(1e-3, 1e3, (20, 1))).astype(np.float32)
    q, s = oracle.quantize_rows_f32(t)
    err = np.abs(q.astype(np.float64) * s[:, None].astype(np.float64) - t.astype(np.float64))
    assert np.all(err <= 0.5 * s[:, None].astype(np.float64) * (1 + 2.0 ** -15))
    assert np.all(np.abs(q).max(axis=1) == 127)


def test_fused_front_ends_compose_the_pinned_parts(oracle):
    g = np.random.default_rng(17)
    M, K, T = 6, 64, 3
    x = g.standard_normal((M, K)).astype(np.float16)
    y = g.standard_normal((M, K)).astype(np.float16)
    cm = np.exp(g.uniform(-1, 1, K)).astype(np.float32)
    sc = g.standard_normal((2, K)).astype(np.float32)
    t, q, s = oracle.gelu_quantize(x, cm, approximate=True)
    assert np.array_equal(t, oracle.gelu(x, True))
    q2, s2 = oracle.quantize_rows_f32(t, cm)
    assert np.array_equal(q, q2) and np.array_equal(s, s2)
    t, q, s = oracle.layernorm_quantize(x, sc, None, T, 1e-6, cm)
    assert np.array_equal(t, oracle.layernorm_modulate(x, sc, None, T, 1e-6))
    r, q, s = oracle.residual_quantize(x, y, sc, T, cm)
    assert np.array_equal(r.view(np.uint16), oracle.residual(x, y, sc, T).view(np.uint16))
    q2, s2 = oracle.quantize_per_token(r, cm)
    assert np.array_equal(q, q2) and np.array_equal(s, s2)


# ---- comparison points: FP16 linear layer, static quantizer (Sec. 5.3) ----------------

def test_gemm_f16_against_numpy_float64(oracle):
    g = np.random.default_rng(21)
    for M, N, K in ((3, 5, 7), (17, 9, 300), (4, 33, 1152)):
        x = g.standard_normal((M, K)).astype(np.float16)
        w = (g.standard_normal((N, K)) * 0.05).astype(np.float16)
        b = (g.standard_normal(N) * 0.1).astype(np.float16)
        want = (x.astype(np.float64) @ w.astype(np.float64).T + b.astype(np.float64)).astype(np.float32).astype(np.float16)
        got = oracle.gemm_f16(x, w, b)
        assert np.array_equal(got.view(np.uint16), want.view(np.uint16))
        want = (x.astype(np.float64) @ w.astype(np.float64).T).astype(np.float32).astype(np.float16)
        assert np.array_equal(oracle.gemm_f16(x, w).view(np.uint16), want.view(np.uint16))


def test_gemm_f16_exact_cases(oracle):
    # small integers: every product and sum is exact, so the result is the integer matmul
    g = np.random.default_rng(22)
    x = g.integers(-8, 9, (6, 40)).astype(np.float16)
    w = g.integers(-4, 5, (10, 40)).astype(np.float16)
    want = x.astype(np.int64) @ w.astype(np.int64).T
    assert np.array_equal(oracle.gemm_f16(x, w).astype(np.int64), want)
    # identity weights select the activations; a transposed operand would not
    x = g.standard_normal((5, 8)).astype(np.float16)
    assert np.array_equal(oracle.gemm_f16(x, np.eye(8, dtype=np.float16)).view(np.uint16), x.view(np.uint16))
    w = np.zeros((3, 8), np.float16)
    w[0, 1] = 1; w[1, 5] = 2; w[2, 7] = -1
    got = oracle.gemm_f16(x, w)
    assert np.array_equal(got[:, 0], x[:, 1]) and np.array_equal(got[:, 1], (2 * x[:, 5].astype(np.float32)).astype(np.float16))
    assert np.array_equal(got[:, 2], -x[:, 7])


def test_quantize_static_hand_examples_and_clipping(oracle):
    # scale 0.5 (inv = 2 exactly): 0.25 -> 0.5 -> 0 (tie to even), 0.75 -> 1.5 -> 2, 1.25 -> 2.5 -> 2
    x = np.array([[0.25, 0.75, 1.25, -0.25, -0.75, 63.5, 63.75, 100.0, -100.0, 0.0]], np.float16)
    assert oracle.quantize_static(x, 0.5)[0].tolist() == [0, 2, 2, 0, -2, 127, 127, 127, -127, 0]
    # the balancing factor comes first
    cm = np.full(10, 0.5, np.float32)
    assert oracle.quantize_static(x, 0.5, cm)[0].tolist() == [0, 1, 1, 0, -1, 64, 64, 100, -100, 0]
    with pytest.raises(oracle.OracleError):
        oracle.quantize_static(x, 0.0)


def test_quantize_static_against_numpy_and_error_bound(oracle):
    g = np.random.default_rng(23)
    x = (g.standard_normal((9, 257)) * 3).astype(np.float16)
    cm = np.exp(g.uniform(-1, 1, 257)).astype(np.float32)
    scale = np.float32(0.037)
    inv = np.float32(1.0) / scale
    want = np.clip(np.rint((x.astype(np.float32) * cm) * inv), -127, 127).astype(np.int8)
    got = oracle.quantize_static(x, float(scale), cm)
    assert np.array_equal(got, want)
    t = x.astype(np.float64) * cm.astype(np.float64)
    inside = np.abs(t) <= 127 * float(scale)
    err = np.abs(got.astype(np.float64) * float(scale) - t)
    assert np.all(err[inside] <= 0.5 * float(scale) * (1 + 2.0 ** -15))
    assert np.all(np.abs(got[~inside]) == 127)


# ---- rotation-based balancing: block-diagonal Hadamard matrix (Sec. 4.2) ----------------

def _q_matrix(K, B):
    from scipy.linalg import hadamard  # Sylvester construction, natural order
    q = np.zeros((K, K))
    for b0 in range(0, K, B):
        q[b0:b0 + B, b0:b0 + B] = hadamard(B) / np.sqrt(B)
    return q


@pytest.mark.parametrize("K,B", [(128, 128), (384, 128), (64, 16), (96, 32)])
def test_hadamard_rotate_against_scipy_matrix(oracle, K, B):
    g = np.random.default_rng(31)
    x = (g.standard_normal((5, K)) * 3).astype(np.float16)
    cm = np.exp(g.uniform(-1, 1, K)).astype(np.float32)
    q = _q_matrix(K, B)
    for mul in (None, cm):
        xs = x.astype(np.float64) * (1.0 if mul is None else mul.astype(np.float64))
        want = xs @ q
        got = oracle.hadamard_rotate(x, mul, B).astype(np.float64)
        assert np.all(np.abs(got - want) <= np.abs(np.spacing(want.astype(np.float32))) + 1e-12)


def test_hadamard_rotate_closed_forms(oracle):
    B = 128
    # a unit pulse at channel k becomes row k of H / sqrt(B): all magnitudes equal, signs (-1)^popcount(k & c)
    x = np.zeros((3, 2 * B), np.float16)
    x[0, 0] = 1; x[1, 1] = 1; x[2, B + 5] = 2
    t = oracle.hadamard_rotate(x, None, B).astype(np.float64)
    r = 1 / np.sqrt(B)
    assert np.allclose(t[0, :B], r) and not t[0, B:].any()
    assert np.allclose(t[1, :B], r * np.where(np.arange(B) & 1, -1, 1))
    signs = np.array([(-1) ** bin(5 & c).count("1") for c in range(B)])
    assert np.allclose(t[2, B:], 2 * r * signs) and not t[2, :B].any()
    # a constant block has only its first (mean) component: sqrt(B) times the constant
    x = np.full((1, B), 0.5, np.float16)
    t = oracle.hadamard_rotate(x, None, B)[0]
    assert np.isclose(t[0], 0.5 * np.sqrt(B)) and np.allclose(t[1:], 0, atol=1e-7)


def test_hadamard_is_orthogonal_and_its_own_inverse(oracle):
    g = np.random.default_rng(32)
    K = 256
    w = g.standard_normal((7, K)).astype(np.float32)
    r1 = oracle.rotate_weight(w, None, 128)
    assert np.allclose((r1.astype(np.float64) ** 2).sum(axis=1), (w.astype(np.float64) ** 2).sum(axis=1), rtol=1e-6)
    r2 = oracle.rotate_weight(r1, None, 128)   # H is symmetric and H H = B I
    assert np.allclose(r2, w, rtol=0, atol=3e-6)


def test_rotation_leaves_the_product_unchanged(oracle):
    # Sec. 4.2: Y = X W^T = (X Q)(W Q)^T, here together with the scaling of Eq. 3
    g = np.random.default_rng(33)
    M, N, K = 6, 9, 384
    x = g.standard_normal((M, K)).astype(np.float16)
    w = (g.standard_normal((N, K)) * 0.05).astype(np.float32)
    s = np.exp(g.uniform(np.log(0.25), np.log(4), K)).astype(np.float32)
    cm = (np.float32(1.0) / s).astype(np.float32)
    xr = oracle.hadamard_rotate(x, cm, 128).astype(np.float64)
    wr = oracle.rotate_weight(w, s, 128).astype(np.float64)
    want = (x.astype(np.float64) * cm.astype(np.float64)) @ (w.astype(np.float64) * s.astype(np.float64)).T
    assert np.allclose(xr @ wr.T, want, rtol=0, atol=2e-5 * np.abs(want).max())


def test_rotation_spreads_an_outlier_channel(oracle):
    # what the rotation is for: one channel 100 times larger than the rest becomes a flat block
    g = np.random.default_rng(34)
    x = g.standard_normal((4, 128)).astype(np.float32)
    x[:, 17] *= 100
    x = x.astype(np.float16)
    t = oracle.hadamard_rotate(x, None, 128)
    before = np.abs(x.astype(np.float32)).max(axis=1) / np.sqrt((x.astype(np.float32) ** 2).mean(axis=1))
    after = np.abs(t).max(axis=1) / np.sqrt((t ** 2).mean(axis=1))
    assert np.all(before > 8) and np.all(after < 2)
    _, q, s = oracle.hadamard_quantize(x, None, 128)
    assert np.all(np.abs(q).max(axis=1) == 127)
    with pytest.raises(oracle.OracleError):
        oracle.hadamard_rotate(x, None, 96)


# ---- Eq. 3: the balancing mask from absmax statistics (Sec. 4.2) ------------------------

def test_channel_absmax_against_numpy(oracle):
    g = np.random.default_rng(41)
    x = (g.standard_normal((37, 50)) * g.uniform(0.1, 30, (1, 50))).astype(np.float16)
    x[:, 7] = 0
    assert np.array_equal(oracle.channel_absmax(x), np.abs(x.astype(np.float32)).max(axis=0))
    w = g.standard_normal((19, 50)).astype(np.float32)
    assert np.array_equal(oracle.channel_absmax(w), np.abs(w).max(axis=0))


def test_balance_mask_closed_forms(oracle):
    ax = np.array([4.0, 9.0, 1.0, 16.0, 0.0, 2.0], np.float32)
    aw = np.array([1.0, 4.0, 1.0, 0.25, 3.0, 0.0], np.float32)
    s, cm = oracle.balance_mask(ax, aw, 0.5)
    # sqrt(ax / aw); all-zero statistics are raised to 1e-5
    assert np.allclose(s[:4], [2.0, 1.5, 1.0, 8.0], rtol=1e-7)
    assert np.isclose(s[4], np.sqrt(1e-5 / 3.0), rtol=1e-6) and np.isclose(s[5], np.sqrt(2.0 / 1e-5), rtol=1e-6)
    assert np.array_equal(cm, (np.float32(1) / s).astype(np.float32))
    # alpha = 1 moves all of the difficulty to the weights (s = max|X|), alpha = 0 the other way
    assert np.allclose(oracle.balance_mask(ax[:4], aw[:4], 1.0)[0], ax[:4], rtol=1e-7)
    assert np.allclose(oracle.balance_mask(ax[:4], aw[:4], 0.0)[0], 1 / aw[:4], rtol=1e-7)
    with pytest.raises(oracle.OracleError):
        oracle.balance_mask(ax, aw, 1.5)


def test_balance_mask_equalises_the_two_sides_at_half(oracle):
    # with alpha = 1/2 the scaled activations and the scaled weights get the same per-channel
    # maximum sqrt(max|X_i| max|W_i|): the difficulty is shared evenly (Sec. 4.2)
    g = np.random.default_rng(42)
    x = (g.standard_normal((200, 64)) * np.exp(g.uniform(-2, 3, (1, 64)))).astype(np.float16)
    w = (g.standard_normal((48, 64)) * 0.05).astype(np.float32)
    ax, aw = oracle.channel_absmax(x), oracle.channel_absmax(w)
    s, cm = oracle.balance_mask(ax, aw, 0.5)
    xa = np.abs(x.astype(np.float64) * cm.astype(np.float64)).max(axis=0)
    wa = np.abs(w.astype(np.float64) * s.astype(np.float64)).max(axis=0)
    assert np.allclose(xa, wa, rtol=1e-6) and np.allclose(xa, np.sqrt(ax.astype(np.float64) * aw), rtol=1e-6)
    # and the product is unchanged (Eq. 3)
    want = x.astype(np.float64) @ w.astype(np.float64).T
    got = (x.astype(np.float64) * cm) @ (w.astype(np.float64) * s).T
    assert np.allclose(got, want, rtol=0, atol=1e-6 * np.abs(want).max())
