"""The library's calls under HIP graph capture: they only enqueue kernels on the stream they are given
(no allocation, no synchronisation, no memset), so a captured layer replays to the bits of the eager one."""
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


@pytest.mark.parametrize("bits", [8, 4])
def test_captured_layer_replays_bit_exactly(vq, oracle, bits):
    print(f"graph replay of vq_linear, {bits}-bit weights", flush=True)
    g = np.random.default_rng(900 + bits)
    M, N, K = 700, 520, 1152
    w = g.normal(0, 0.02, (N, K)).astype(np.float32)
    wq_h, ws_h = oracle.quantize_weight(w, None, bits)
    wq = torch.from_numpy(wq_h if bits == 8 else oracle.pack_int4(wq_h)).cuda()
    ws = torch.from_numpy(ws_h).cuda()
    bias = torch.from_numpy(g.normal(0, 0.01, N).astype(np.float16)).cuda()
    cm = torch.from_numpy(np.exp(g.uniform(-1, 1, K)).astype(np.float32)).cuda()
    x = torch.zeros((M, K), dtype=torch.float16, device="cuda")       # the graph's input buffer
    y = torch.empty((M, N), dtype=torch.float16, device="cuda")       # and its outputs
    xq = torch.empty((M, K), dtype=torch.int8, device="cuda")
    xs = torch.empty((M,), dtype=torch.float32, device="cuda")
    work = torch.empty((vq.vq_linear_workspace_bytes(M, N, K, bits),), dtype=torch.uint8, device="cuda")
    y2 = torch.empty_like(y)
    gemm = vq.vq_gemm_w8a8 if bits == 8 else vq.vq_gemm_w4a8

    def layer(out_linear, out_two):
        vq.vq_linear(x, cm, wq, bits, ws, bias, y=out_linear, workspace=work)
        vq.vq_quantize_per_token(x, cm, xq=xq, x_scale=xs)
        gemm(xq, xs, wq, ws, bias, y=out_two)

    layer(y, y2)  # eager once: the library's per-device set-up happens outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            layer(y, y2)
    torch.cuda.synchronize()

    for rep in range(4):
        xin = torch.from_numpy((g.standard_normal((M, K)) * (rep + 1)).astype(np.float16)).cuda()
        x.copy_(xin)
        y.zero_(); y2.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got, got2 = y.clone(), y2.clone()
        # the program's own eager work and synchronisation between the replays
        ref, ref2 = torch.empty_like(y), torch.empty_like(y)
        layer(ref, ref2)
        torch.cuda.synchronize()
        assert torch.equal(got, ref) and torch.equal(got2, ref2), f"replay {rep} differs from the eager run"
        assert torch.equal(got, got2)
    # and the eager result is the oracle's (sampled rows)
    rows = [0, 1, M - 1]
    o = oracle.linear(x.cpu().numpy()[rows], cm.cpu().numpy(), wq_h if bits == 8 else oracle.pack_int4(wq_h), bits, ws_h,
                      bias.cpu().numpy())
    from parity_util import assert_fp16_close
    assert_fp16_close(ref.cpu().numpy()[rows], o["y"], o["acc"], o["x_scale"], ws_h, bias.cpu().numpy())
