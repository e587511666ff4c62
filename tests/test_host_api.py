"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol include/vq.h declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "vq.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2406_02540_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2406_02540_amd import build
        build.build(verbose=False)
    return binding.lib()


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vq_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_entry_points():
    names = _declared()
    for n in ("vq_quantize_per_token", "vq_gemm_w8a8", "vq_gemm_w4a8", "vq_linear",
              "vq_linear_workspace_bytes", "vq_quantize_weight", "vq_status_string"):
        assert n in names


def test_library_exports_every_declared_symbol(lib):
    from paper_2406_02540_amd import binding
    for n in _declared():
        assert hasattr(lib, n), n
        assert n in binding.SIGNATURES, f"binding has no signature for {n}"
    assert sorted(binding.SIGNATURES) == _declared()


def test_binding_exposes_the_same_names():
    import paper_2406_02540_amd as pkg
    for n in _declared():
        if n == "vq_status_string":
            continue
        assert callable(getattr(pkg, n)), n


def test_status_strings(lib):
    seen = set()
    for code in range(8):
        s = lib.vq_status_string(code).decode()
        assert s and s not in seen
        seen.add(s)
    assert lib.vq_status_string(99).decode() == "unknown status"


def test_workspace_bytes(lib):
    f = lib.vq_linear_workspace_bytes
    assert f(32768, 4608, 1152, 8) == 32768 * 1152 + 4 * 32768
    assert f(240, 2304, 4096, 4) == 240 * 4096 + 4 * 240
    assert f(3, 8, 16, 8) == 48 + 16          # both parts rounded up to 16 bytes
    assert f(0, 8, 16, 8) == 0
    assert f(-1, 8, 16, 8) == 0 and f(1, 8, 0, 8) == 0 and f(1, 8, 16, 5) == 0


A = 0x10000  # a made-up, 16-byte aligned, non-NULL address; never dereferenced by validation
P = ctypes.c_void_p


def test_quantize_argument_errors(lib):
    q = lib.vq_quantize_per_token
    assert q(P(A), None, P(A), P(A), -1, 64, None) == 2
    assert q(P(A), None, P(A), P(A), 4, 0, None) == 2
    assert q(P(A), None, P(A), P(A), 4, 131073, None) == 2
    assert q(None, None, P(A), P(A), 4, 64, None) == 1
    assert q(P(A), None, None, P(A), 4, 64, None) == 1
    assert q(P(A), None, P(A), None, 4, 64, None) == 1
    assert q(P(A + 2), None, P(A), P(A), 4, 64, None) == 3
    assert q(P(A), P(A + 4), P(A), P(A), 4, 64, None) == 3
    assert q(None, None, None, None, 0, 64, None) == 0  # empty: nothing to do


def test_fused_quantizer_argument_errors(lib):
    ge, ln, rs = lib.vq_gelu_quantize, lib.vq_layernorm_quantize, lib.vq_residual_quantize
    F = ctypes.c_float
    # the token must fit the registers: whole 16-byte chunks, K <= 8192
    assert ge(P(A), 1, None, P(A), P(A), 4, 12, None) == 2
    assert ge(P(A), 1, None, P(A), P(A), 4, 8200, None) == 2
    assert ge(P(A), 2, None, P(A), P(A), 4, 64, None) == 2
    assert ge(None, 1, None, P(A), P(A), 4, 64, None) == 1
    assert ge(P(A + 8), 1, None, P(A), P(A), 4, 64, None) == 3
    assert ge(None, 0, None, None, None, 0, 64, None) == 0
    assert ln(P(A), None, None, 0, F(1e-6), None, P(A), P(A), 4, 64, None) == 2
    assert ln(P(A), None, None, 2, F(-1.0), None, P(A), P(A), 4, 64, None) == 2
    assert ln(P(A), P(A + 4), None, 2, F(1e-6), None, P(A), P(A), 4, 64, None) == 3
    assert ln(P(A), None, None, 2, F(1e-6), None, P(A), None, 4, 64, None) == 1
    assert rs(P(A), None, None, 2, P(A), None, P(A), P(A), 4, 64, None) == 1
    assert rs(P(A), P(A), None, 2, None, None, P(A), P(A), 4, 64, None) == 1
    assert rs(P(A), P(A), P(A + 4), 2, P(A), None, P(A), P(A), 4, 64, None) == 3
    assert rs(P(A), P(A), None, 0, P(A), None, P(A), P(A), 4, 64, None) == 2
    # valid arguments reach the device check: no gfx950 here
    assert ge(P(A), 1, None, P(A), P(A), 4, 64, None) == 6
    assert ln(P(A), None, None, 2, F(1e-6), None, P(A), P(A), 4, 64, None) == 6
    assert rs(P(A), P(A), None, 2, P(A), None, P(A), P(A), 4, 64, None) == 6


def test_rotation_and_comparison_argument_errors(lib):
    hq, rw, gf, qs = lib.vq_hadamard_quantize, lib.vq_rotate_weight, lib.vq_gemm_f16, lib.vq_quantize_static
    F = ctypes.c_float
    assert hq(P(A), None, P(A), P(A), 4, 192, None) == 2       # K must be whole blocks of 128
    assert hq(P(A), None, P(A), P(A), 4, 8320, None) == 2      # and fit the registers
    assert hq(None, None, P(A), P(A), 4, 256, None) == 1
    assert hq(P(A), P(A + 4), P(A), P(A), 4, 256, None) == 3
    assert hq(P(A), None, P(A), P(A), 4, 256, None) == 6
    assert rw(P(A), None, P(A), 4, 200, None) == 2
    assert rw(None, None, P(A), 4, 256, None) == 1
    assert rw(P(A), None, P(A + 8), 4, 256, None) == 3
    assert rw(None, None, None, 0, 256, None) == 0
    assert gf(P(A), P(A), None, P(A), 4, 8, 12, None) == 2     # K % 8
    assert gf(P(A), None, None, P(A), 4, 8, 16, None) == 1
    assert gf(P(A), P(A), P(A + 2), P(A), 4, 8, 16, None) == 3
    assert gf(None, None, None, None, 0, 8, 16, None) == 0
    assert gf(P(A), P(A), None, P(A), 4, 8, 16, None) == 6
    assert qs(P(A), None, F(0.0), P(A), 4, 64, None) == 2
    assert qs(P(A), None, F(-1.0), P(A), 4, 64, None) == 2
    assert qs(P(A), None, F(0.5), None, 4, 64, None) == 1
    assert qs(P(A), None, F(0.5), P(A), 4, 64, None) == 6
    ca, bm = lib.vq_channel_absmax, lib.vq_balance_mask
    assert ca(P(A), 2, P(A), 4, 64, 0, None) == 2
    assert ca(P(A), 0, None, 4, 64, 0, None) == 1
    assert ca(None, 0, P(A), 4, 64, 0, None) == 1
    assert ca(P(A + 2), 0, P(A), 4, 64, 0, None) == 3
    assert ca(None, 0, P(A), 0, 64, 1, None) == 0
    assert ca(P(A), 1, P(A), 4, 64, 0, None) == 6
    assert bm(P(A), P(A), F(1.5), P(A), P(A), 64, None) == 2
    assert bm(P(A), None, F(0.5), P(A), P(A), 64, None) == 1
    assert bm(P(A), P(A), F(0.5), P(A), P(A), 64, None) == 6


def test_gemm_argument_errors(lib):
    for g, kmult in ((lib.vq_gemm_w8a8, 16), (lib.vq_gemm_w4a8, 32)):
        ok = [P(A), P(A), P(A), P(A), None, P(A), None]
        assert g(*ok, 4, 8, kmult - 8, None) == 2      # K not a multiple of what the path needs
        assert g(*ok, 4, 8, 0, None) == 2
        assert g(*ok, 4, -8, kmult, None) == 2
        assert g(*ok, 4, 8, 131072 + kmult, None) == 2  # beyond the int32-safe K
        for i in (0, 1, 2, 3, 5):
            bad = list(ok)
            bad[i] = None
            assert g(*bad, 4, 8, kmult, None) == 1
            bad[i] = P(A + 8)
            assert g(*bad, 4, 8, kmult, None) == 3
        bad = list(ok)
        bad[4] = P(A + 2)
        assert g(*bad, 4, 8, kmult, None) == 3
        assert g(None, None, None, None, None, None, None, 0, 8, kmult, None) == 0
        assert g(None, None, None, None, None, None, None, 4, 0, kmult, None) == 0


def test_linear_argument_errors(lib):
    f = lib.vq_linear
    need = lib.vq_linear_workspace_bytes(4, 8, 64, 8)
    base = dict(x=P(A), cm=None, w=P(A), bits=8, ws=P(A), b=None, y=P(A), wk=P(A), wb=need, M=4, N=8, K=64)

    def call(**kw):
        a = dict(base, **kw)
        return f(a["x"], a["cm"], a["w"], a["bits"], a["ws"], a["b"], a["y"], a["wk"], a["wb"],
                 a["M"], a["N"], a["K"], None)

    assert call(bits=5) == 7
    assert call(K=24) == 2
    assert call(bits=4, K=48) == 2
    assert call(wk=None) == 1
    assert call(wk=P(A + 4)) == 3
    assert call(wb=need - 1) == 4
    assert call(x=None) == 1 and call(w=None) == 1 and call(ws=None) == 1 and call(y=None) == 1
    assert call(M=0) == 0


def test_producer_linear_argument_errors(lib):
    """The layer behind a producer: the producer's checks, then those of vq_linear."""
    F = ctypes.c_float
    need = lib.vq_linear_workspace_bytes(4, 8, 256, 8)
    tail = dict(cm=None, w=P(A), bits=8, ws=P(A), b=None, y=P(A), wk=P(A), wb=need, M=4, N=8, K=256)

    def tail_args(a):
        return (a["cm"], a["w"], a["bits"], a["ws"], a["b"], a["y"], a["wk"], a["wb"], a["M"], a["N"], a["K"], None)

    def ln(x=P(A), sc=None, sh=None, T=2, eps=1e-6, **kw):
        return lib.vq_layernorm_linear(x, sc, sh, T, F(eps), *tail_args(dict(tail, **kw)))

    def ge(h=P(A), approx=1, **kw):
        return lib.vq_gelu_linear(h, approx, *tail_args(dict(tail, **kw)))

    def rs(x=P(A), yin=P(A), gate=None, T=2, r=P(A), **kw):
        return lib.vq_residual_linear(x, yin, gate, T, r, *tail_args(dict(tail, **kw)))

    def hd(x=P(A), **kw):
        return lib.vq_hadamard_linear(x, *tail_args(dict(tail, **kw)))

    for f in (ln, ge, rs, hd):
        assert f(bits=5) == 7
        assert f(K=24) == 2 and f(bits=4, K=48) == 2
        assert f(K=8192 + 128) == 2                      # the fused quantizers hold the token in registers
        assert f(wk=None) == 1 and f(wk=P(A + 4)) == 3 and f(wb=need - 1) == 4
        assert f(w=None) == 1 and f(ws=None) == 1 and f(y=None) == 1
        assert f(b=P(A + 2)) == 3 and f(cm=P(A + 4)) == 3
        assert f(M=0) == 0 and f(N=0) == 0
        assert f() == 6                                  # valid arguments reach the device check
    assert ln(x=None) == 1 and ge(h=None) == 1 and rs(x=None) == 1 and hd(x=None) == 1
    assert ln(T=0) == 2 and ln(eps=-1.0) == 2 and ln(sc=P(A + 4)) == 3 and ln(sh=P(A + 8)) == 3
    assert ge(approx=2) == 2
    assert rs(T=0) == 2 and rs(yin=None) == 1 and rs(r=None) == 1 and rs(gate=P(A + 4)) == 3 and rs(r=P(A + 2)) == 3
    assert hd(K=192) == 2                                # whole blocks of 128 channels
    assert ge(K=64, wb=lib.vq_linear_workspace_bytes(4, 8, 64, 8)) == 6


def test_quantize_weight_argument_errors(lib):
    f = lib.vq_quantize_weight
    assert f(P(A), None, 3, P(A), P(A), 4, 64, None) == 7
    assert f(P(A), None, 4, P(A), P(A), 4, 63, None) == 2
    assert f(None, None, 8, P(A), P(A), 4, 64, None) == 1
    assert f(P(A), P(A + 4), 8, P(A), P(A), 4, 64, None) == 3
    assert f(None, None, 8, None, None, 0, 64, None) == 0


def test_no_gfx950_device_is_an_error_not_a_launch(lib):
    torch = pytest.importorskip("torch")
    if torch.cuda.is_available():
        pytest.skip("a GPU is present; made-up pointers must not reach a kernel")
    assert lib.vq_quantize_per_token(P(A), None, P(A), P(A), 4, 64, None) == 6
    assert lib.vq_gemm_w8a8(P(A), P(A), P(A), P(A), None, P(A), None, 4, 8, 64, None) == 6


def test_binding_refuses_host_tensors():
    torch = pytest.importorskip("torch")
    import paper_2406_02540_amd as pkg
    with pytest.raises(TypeError):
        pkg.vq_quantize_per_token(torch.zeros((2, 8), dtype=torch.float16))


def test_lane_group_choice(tmp_path):
    """vq_lanes.h (plain C++): how many lanes share a token whose row is held in fp32 registers."""
    import subprocess
    src = tmp_path / "lanes.cpp"
    src.write_text('#include <cstdio>\n#include "vq_lanes.h"\n'
                   'int main() { for (int k8 = 1; k8 <= 1024; ++k8) std::printf("%d %d\\n", k8, vq::lanes_for_row(k8)); }\n')
    exe = tmp_path / "lanes"
    subprocess.run(["g++", "-O1", "-I", os.path.join(ROOT, "paper_2406_02540_amd", "csrc"), str(src), "-o", str(exe)],
                   check=True)
    got = dict(map(int, line.split()) for line in subprocess.run([str(exe)], check=True, capture_output=True,
                                                                 text=True).stdout.splitlines())
    # the shapes of the workloads: K = 1152 -> 32 lanes x 5 chunks, K = 4608 / 4096 -> a whole wavefront
    assert got[144] == 32 and got[576] == 64 and got[512] == 64 and got[1024] == 64
    # short rows that only a narrow group divides well
    assert got[48] == 16 and got[16] == 16 and got[1] == 16 and got[160] == 32
    for k8, lanes in got.items():
        assert lanes in (16, 32, 64)
        nch = -(-k8 // lanes)
        assert nch <= 16, (k8, lanes)                      # the kernels are instantiated for 1..16 chunks per lane
        idle = nch * lanes - k8
        for wider in (l for l in (32, 64) if l > lanes):   # a wider group was passed over only for its idle lanes
            n2 = -(-k8 // wider)
            assert n2 > 16 or (n2 * wider - k8) * 100 > 15 * n2 * wider
        if idle * 100 > 15 * nch * lanes:                  # nothing met the bar: the fewest idle lanes won
            assert all(-(-k8 // l) > 16 or (-(-k8 // l)) * l - k8 >= idle for l in (16, 32, 64))
