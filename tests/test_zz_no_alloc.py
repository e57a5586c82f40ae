"""patch_gemm_static (the entry point that allocates nothing: split-K partials go to a scratch array inside the
library's device image) against patch_gemm_ex with a caller workspace of the same size: bit-equal, on two calls in
a row, the second with a smaller input; and against the oracle.  Sizes whose schedule wants more scratch than the
array holds are refused with PATCH_ERR_SIZE."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2509_23410_amd import binding as B, synth

pytestmark = pytest.mark.gpu


def _dev_bf16(bits, dev):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)


def test_static_scratch_entry_point_matches_caller_workspace():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    dev = torch.device("cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    N, K, t = 768, 2048, 128
    c = synth.make_case("static", N, K, 300, t, 0.5, seed=51)
    W_hat_o = oracle.apply_mask(c.W, c.tile_map, c.mask24, t)
    vals_o, meta_o = oracle.pack(W_hat_o, c.tile_map, t)
    W_hat = _dev_bf16(W_hat_o, dev)
    P = B.patch_pack(W_hat, N, K, c.tile_map, t, st)
    X = _dev_bf16(c.X, dev)
    ws = torch.empty(B.STATIC_SCRATCH_BYTES // 4, device=dev, dtype=torch.float32)
    # 300 rows: the prefill kernel with K split over workgroups; 40 rows: a batched-decode pass with K chunks; both keep
    # their partial sums in the scratch.  Larger first, then smaller (stale partials of the first call stay behind).
    for M in (300, 40, 300, 1):
        need = B.patch_gemm_workspace_bytes(M, P)
        print(f"static scratch: M={M} schedule wants {need} bytes", flush=True)
        assert need <= B.STATIC_SCRATCH_BYTES and (need > 0 or M == 1)
        Y = torch.full((M, N), float("nan"), device=dev, dtype=torch.float32)
        B.patch_gemm_static(X, M, P, Y, st)
        ws.fill_(float("nan"))
        E = torch.full((M, N), float("nan"), device=dev, dtype=torch.float32)
        B.patch_gemm(X, M, P, E, st, workspace=ws)
        torch.cuda.synchronize()
        assert torch.isfinite(Y).all(), "unwritten outputs"
        assert torch.equal(Y, E), f"M={M}: static scratch and caller workspace disagree"
        Yo = oracle.gemm(c.X[:M], vals_o, meta_o, N, K, c.tile_map, t)
        Yh = Y.cpu().numpy().astype(np.float64)
        assert float(np.linalg.norm(Yh - Yo) / np.linalg.norm(Yo)) <= 2e-5
    P.close()


def test_static_scratch_refuses_oversized_schedules():
    dev = torch.device("cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    N = K = 5120
    M = 1024
    c = synth.make_case("static_big", N, K, M, 128, 0.0, seed=52, with_mask=False)
    P = B.patch_pack(_dev_bf16(c.W, dev), N, K, np.ones_like(c.tile_map), 128, st)
    X = _dev_bf16(c.X, dev)
    assert B.patch_gemm_workspace_bytes(M, P) > B.STATIC_SCRATCH_BYTES
    Y = torch.full((M, N), 3.0, device=dev, dtype=torch.float32)
    with pytest.raises(B.PatchError) as e:
        B.patch_gemm_static(X, M, P, Y, st)
    assert e.value.status == B.ERR_SIZE
    torch.cuda.synchronize()
    assert bool((Y == 3.0).all()), "a refused call must not launch anything"
    B.patch_gemm_static(X, 1, P, Y, st)      # decode: no scratch needed, runs
    torch.cuda.synchronize()
    assert torch.isfinite(Y[:1]).all()
    P.close()
