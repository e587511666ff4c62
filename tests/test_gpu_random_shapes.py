"""A seeded sweep of random in-range shapes through the parity checks of the other GPU test files:
ragged M, N and K, every lane group of the row kernels, both GEMM kernels and their store paths."""
import random

import pytest

torch = pytest.importorskip("torch")

pytestmark = pytest.mark.gpu

import test_gpu_compare as tc  # noqa: E402  (the comparison rules and case bodies live there)
import test_gpu_fused as tf    # noqa: E402
import test_gpu_parity as tp   # noqa: E402


@pytest.fixture(scope="module")
def vq():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2406_02540_amd as pkg
    from paper_2406_02540_amd import binding
    binding.lib()  # raises if the HIP library is missing: there is no fallback
    return pkg


def _k8(rnd, lo, hi):
    return 8 * rnd.randint(lo // 8, hi // 8)


@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_random_shapes(vq, oracle, seed):
    rnd = random.Random(20240602 + seed)
    for case in range(60):
        c = rnd.randrange(9)
        if c == 0:
            tp.test_quantize_per_token_bit_exact(vq, oracle, rnd.randint(1, 300),
                                                 rnd.choice([_k8(rnd, 8, 8192), rnd.randint(1, 9000)]), rnd.random() < 0.5)
        elif c == 1:
            bits = rnd.choice([8, 4])
            big = rnd.random() < 0.3  # enough tiles for the persistent kernel
            K = (16 if bits == 8 else 32) * rnd.randint(1, 10 if big else 75)
            M = rnd.randint(2300, 4200) if big else rnd.randint(1, 700)
            N = rnd.randint(2300, 3200) if big else rnd.randint(1, 700)
            print(f"gemm w{bits}a8 M={M} N={N} K={K}", flush=True)
            tp._gemm_case(vq, oracle, M, N, K, bits, seed=rnd.randrange(1 << 30), bias=rnd.random() < 0.8)
        elif c == 2:
            tf.test_gelu_quantize(vq, oracle, rnd.randint(1, 200), _k8(rnd, 8, 8192), rnd.random() < 0.5, rnd.random() < 0.5)
        elif c == 3:
            tf.test_layernorm_quantize(vq, oracle, rnd.randint(1, 200), _k8(rnd, 8, 8192),
                                       rnd.choice(["none", "scale_shift", "shift_mul"]))
        elif c == 4:
            tf.test_residual_quantize_bit_exact(vq, oracle, rnd.randint(1, 200), _k8(rnd, 8, 8192), rnd.random() < 0.5)
        elif c == 5:
            tf.test_hadamard_quantize(vq, oracle, rnd.randint(1, 200), 128 * rnd.randint(1, 64), rnd.random() < 0.5)
        elif c == 6:
            big = rnd.random() < 0.3
            M = rnd.randint(2300, 3000) if big else rnd.randint(1, 600)
            N = rnd.randint(2300, 3000) if big else rnd.randint(1, 640)
            tc.test_gemm_f16(vq, oracle, M, N, 8 * rnd.randint(1, 20 if big else 200), rnd.random() < 0.5)
        elif c == 7:
            tc.test_quantize_static_bit_exact(vq, oracle, rnd.randint(1, 400),
                                              rnd.choice([_k8(rnd, 8, 8192), rnd.randint(1, 5000)]), rnd.random() < 0.5)
        else:
            tc.test_channel_absmax_bit_exact(vq, oracle, rnd.randint(1, 3000), rnd.randint(1, 3000))
