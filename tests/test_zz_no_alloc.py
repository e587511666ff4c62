"""vq_linear_static (the entry point that allocates nothing: its int8 activations and token scales live in
the library's built-in scratch array) against vq_linear on the same inputs, through the C-ABI: bit for bit,
on two calls in a row, the second with a smaller input, and the refusal of a layer beyond the scratch."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

pytestmark = pytest.mark.gpu


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("bits", [8, 4])
def test_static_scratch_entry_matches_vq_linear_twice(oracle, bits):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2406_02540_amd as vq
    from paper_2406_02540_amd import binding
    lib = binding.lib()
    g = np.random.default_rng(900 + bits)
    # the first call is large (persistent large-tile GEMM), the second smaller in M, N and K
    for call, (M, N, K) in enumerate([(3000, 2312, 1152), (517, 392, 608)]):
        print(f"vq_linear_static w{bits}a8 call {call}: M={M} N={N} K={K}", flush=True)
        x = (g.standard_normal((M, K)) * np.exp(g.uniform(-2, 2, (M, 1)))).astype(np.float16)
        cm = np.exp(g.uniform(np.log(0.25), np.log(4.0), K)).astype(np.float32)
        w = g.normal(0, 0.02, (N, K)).astype(np.float32)
        wq, ws = oracle.quantize_weight(w, (1.0 / cm).astype(np.float32), bits)
        wdev = wq if bits == 8 else oracle.pack_int4(wq)
        b = g.normal(0, 0.01, N).astype(np.float16)
        dx, dcm, dw, dws, db = dev(x), dev(cm), dev(wdev), dev(ws), dev(b)
        y_ref = vq.vq_linear(dx, dcm, dw, bits, dws, db)
        y = torch.full((M, N), 7.0, dtype=torch.float16, device="cuda")
        torch.cuda.synchronize()
        # straight through the C-ABI: device pointers and sizes, no workspace
        rc = lib.vq_linear_static(dx.data_ptr(), dcm.data_ptr(), dw.data_ptr(), bits, dws.data_ptr(), db.data_ptr(),
                                  y.data_ptr(), M, N, K, torch.cuda.current_stream().cuda_stream)
        assert rc == 0, binding.status_string(rc)
        torch.cuda.synchronize()
        assert torch.equal(y, y_ref), f"call {call}: {(y != y_ref).sum().item()} outputs differ from vq_linear"
        # and the oracle's result on sampled rows, to the rule of the other parity tests
        from parity_util import assert_fp16_close
        rows = np.unique(np.concatenate([[0, M - 1], g.integers(0, M, 40)]))
        ref = oracle.linear(x[rows], cm, wdev, bits, ws, b)
        assert_fp16_close(y.cpu().numpy()[rows], ref["y"], ref["acc"], ref["x_scale"], ws, b)


def test_static_scratch_entry_refuses_what_does_not_fit():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2406_02540_amd as vq
    from paper_2406_02540_amd import binding
    M, N, K = 32768, 8, 4608   # 151 MB of int8 activations: beyond the 40 MiB scratch
    assert vq.vq_linear_workspace_bytes(M, N, K, 8) > binding.LINEAR_STATIC_SCRATCH_BYTES
    x = torch.zeros((M, K), dtype=torch.float16, device="cuda")
    w = torch.zeros((N, K), dtype=torch.int8, device="cuda")
    y = torch.full((M, N), 7.0, dtype=torch.float16, device="cuda")
    with pytest.raises(vq.VqError) as e:
        vq.vq_linear_static(x, None, w, 8, torch.ones(N, device="cuda"), None, y=y)
    assert e.value.status == 4
    torch.cuda.synchronize()
    assert (y == 7.0).all()   # nothing was enqueued
