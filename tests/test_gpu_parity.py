"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element, on the same
seeded inputs.  Packing / mask merge / unpack: bit-exact.  Product: relative Frobenius error <= 1e-3
against the fp64 oracle (the stated tolerance; fp32 accumulation of exact bf16 products lands near 1e-6,
so a tighter internal bound of 2e-5 is asserted as well to catch dropped K-steps or tiles), and every
compared element within  ELEM_C * sqrt(K) * 2^-24 * |x_m| * |w_n|  of the oracle's (the products are exact in
fp32, so the only error is the rounding of K fp32 additions whose partial sums never exceed |x_m| |w_n|).
Split-K workspaces are filled with NaN before every call: a partial sum that is read without having been
written by the same call shows up as a NaN in Y."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2509_23410_amd import binding as B, synth

pytestmark = pytest.mark.gpu

TOL = 1e-3
TIGHT = 2e-5
ELEM_C = 2.0
U32 = 2.0 ** -24


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    B.lib()
    return torch.device("cuda:0")


def to_dev_bf16(bits, dev):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)


def bits_of(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def stream():
    return torch.cuda.current_stream().cuda_stream


def relF(a, b):
    return float(np.linalg.norm(a.astype(np.float64) - b) / max(np.linalg.norm(b), 1e-300))


def row_norms(bits):
    """Euclidean norm of every row of a bf16 matrix (fp64), in blocks so that large matrices stay cheap."""
    out = np.empty(bits.shape[0], np.float64)
    for i in range(0, bits.shape[0], 1024):
        a = synth.bf16_bits_to_f64(bits[i:i + 1024])
        out[i:i + 1024] = np.sqrt((a * a).sum(axis=1))
    return out


def elem_bound(xn, wn, K):
    """Element-wise error bound matrix (or vector, for paired norms): ELEM_C sqrt(K) 2^-24 |x_m| |w_n|."""
    return ELEM_C * np.sqrt(K) * U32 * xn * wn


def check_elements(Y, Yo, xn, wn, K, what=""):
    """relF within both bars and every element within its bound; prints the three error figures."""
    Y = np.asarray(Y, dtype=np.float64)
    assert np.isfinite(Y).all(), f"unwritten or non-finite outputs {what}"
    d = np.abs(Y - Yo)
    bound = elem_bound(xn[:, None], wn[None, :], K)
    r = float(np.linalg.norm(Y - Yo) / max(np.linalg.norm(Yo), 1e-300))
    big = np.abs(Yo) >= 1e-2 * np.sqrt((Yo * Yo).mean() + 1e-300)
    max_rel = float((d[big] / np.abs(Yo[big])).max()) if big.any() else 0.0
    print(f"  parity {what}: relF={r:.2e} max_abs={float(d.max()):.2e} max_rel(|y|>=1% rms)={max_rel:.2e} "
          f"max err/bound={float((d / np.maximum(bound, 1e-300)).max()):.3f}", flush=True)
    assert r <= TOL and r <= TIGHT, (what, r)
    worst = np.unravel_index(np.argmax(d - bound), d.shape)
    assert (d <= bound).all(), f"{what}: element {worst} off by {d[worst]:.3e}, bound {bound[worst]:.3e}"
    return r


class Prepared:
    """One case taken through both sides: oracle (W_hat, canonical pack) and GPU (W_hat, packed handle)."""

    def __init__(self, c, dev):
        self.c, self.dev = c, dev
        self.W_hat_o = oracle.apply_mask(c.W, c.tile_map, c.mask24, c.tile)
        self.vals_o, self.meta_o = oracle.pack(self.W_hat_o, c.tile_map, c.tile)
        W = to_dev_bf16(c.W, dev)
        m24 = torch.from_numpy(c.mask24).to(dev)
        self.W_hat = torch.empty_like(W)
        B.patch_apply_mask(W, m24, c.tile_map, c.N, c.K, c.tile, self.W_hat, stream())
        self.P = B.patch_pack(self.W_hat, c.N, c.K, c.tile_map, c.tile, stream())
        self._wn = None

    @property
    def wn(self):
        if self._wn is None:
            self._wn = row_norms(self.W_hat_o)
        return self._wn

    def gemm(self, X_bits, **kw):
        M = X_bits.shape[0]
        X = to_dev_bf16(X_bits, self.dev)
        Y = torch.full((M, self.c.N), float("nan"), device=self.dev, dtype=torch.float32)
        if kw.get("workspace") is not None:
            kw["workspace"].fill_(float("nan"))     # poisoned: every partial the launch reads it must have written
        B.patch_gemm(X, M, self.P, Y, stream(), **kw)
        torch.cuda.synchronize()
        return Y.cpu().numpy()

    def gemm_bf16(self, X_bits, **kw):
        """The same product with a bf16 Y (patch_gemm_opts.y_bf16): bit patterns, uint16."""
        M = X_bits.shape[0]
        X = to_dev_bf16(X_bits, self.dev)
        Y = torch.full((M, self.c.N), float("nan"), device=self.dev, dtype=torch.bfloat16)
        if kw.get("workspace") is not None:
            kw["workspace"].fill_(float("nan"))
        B.patch_gemm(X, M, self.P, Y, stream(), y_bf16=True, **kw)
        torch.cuda.synchronize()
        return bits_of(Y)

    def check(self, X_bits, Y, Yo=None, what=""):
        """Full-output comparison with the oracle: relF and every element."""
        if Yo is None:
            Yo = self.oracle_gemm(X_bits)
        return check_elements(Y, Yo, row_norms(X_bits), self.wn, self.c.K, what)

    def oracle_gemm(self, X_bits):
        c = self.c
        return oracle.gemm(X_bits, self.vals_o, self.meta_o, c.N, c.K, c.tile_map, c.tile)


PACK_CASES = [
    ("tiny", 512, 512, 64, 0.5),
    ("t64_ragged_tiles", 192, 320, 64, 0.4),
    ("t128_small", 256, 384, 128, 0.5),
    ("qwen_896", 896, 896, 128, 0.5),
    ("qwen_up_all24", 4864, 896, 128, 1.0),
    ("qwen_down_dense", 896, 4864, 128, 0.0),
]


@pytest.mark.parametrize("name,N,K,t,f", PACK_CASES)
def test_mask_merge_pack_unpack_bit_exact(dev, name, N, K, t, f):
    print(f"case {name} N={N} K={K} tile={t} f={f}", flush=True)
    c = synth.make_case(name, N, K, 1, t, f, seed=1)
    p = Prepared(c, dev)
    assert np.array_equal(bits_of(p.W_hat), p.W_hat_o)
    vals, meta = B.patch_export_canonical(p.P)
    assert np.array_equal(vals, p.vals_o)
    assert np.array_equal(meta, p.meta_o)
    assert p.P.nbytes == 2 * vals.size + meta.size
    ns = int((c.tile_map == 0).sum())
    assert p.P.nbytes * 16 * c.tile_map.size == 2 * N * K * (16 * c.tile_map.size - 7 * ns)   # closed form
    assert p.P.dims() == (N, K, t, ns)
    assert np.array_equal(p.P.tile_map(), c.tile_map)
    out = torch.empty_like(p.W_hat)
    B.patch_unpack(p.P, out, stream())
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(out), oracle.unpack(p.vals_o, p.meta_o, N, K, c.tile_map, t))
    p.P.close()


@pytest.mark.parametrize("N,K,t", [(128, 256, 64), (384, 640, 128), (64, 64, 64)])
def test_hard_masks_bit_exact_and_feed_the_pipeline(dev, N, K, t):
    """patch_hard_masks against the oracle, byte for byte, on logits with planted ties, zeros and NaNs; then the whole
    front end on both sides: logits -> hard masks -> mask merge -> pack, compared in canonical form."""
    pt, p24 = synth.mask_logits(5, N, K, t)
    tm_o, m24_o = oracle.hard_masks(pt, p24, N, K, t)
    m24 = torch.full((N, K), 7, device=dev, dtype=torch.uint8)
    tm = B.patch_hard_masks(pt, torch.from_numpy(p24).to(dev), N, K, t, m24, stream())
    torch.cuda.synchronize()
    assert np.array_equal(tm, tm_o)
    assert np.array_equal(m24.cpu().numpy(), m24_o)
    c = synth.make_case("hardmask", N, K, 4, t, 0.5, seed=5)
    W = to_dev_bf16(c.W, dev)
    W_hat = torch.empty_like(W)
    B.patch_apply_mask(W, m24, tm, N, K, t, W_hat, stream())
    P = B.patch_pack(W_hat, N, K, tm, t, stream())
    vals, meta = B.patch_export_canonical(P)
    vo, mo = oracle.pack(oracle.apply_mask(c.W, tm_o, m24_o, t), tm_o, t)
    assert np.array_equal(vals, vo) and np.array_equal(meta[: mo.size], mo)
    P.close()


def test_pack_special_values_and_padding_rule(dev):
    """Zeros, negative zeros, NaN, Inf, denormals; groups with 0 or 1 nonzeros exercise the padding rule."""
    c = synth.make_case("special", 256, 256, 1, 64, 0.6, seed=2)
    rng = np.random.default_rng(5)
    W = c.W.copy().reshape(-1)
    idx = rng.choice(W.size, size=W.size // 3, replace=False)
    specials = np.array([0x0000, 0x8000, 0x7FC0, 0x7F80, 0xFF80, 0x0001, 0x8001], np.uint16)
    W[idx] = specials[rng.integers(0, len(specials), size=idx.size)]
    c.W = W.reshape(256, 256)
    c.mask24 = synth.mask24_magnitude(c.W)
    p = Prepared(c, dev)
    assert np.array_equal(bits_of(p.W_hat), p.W_hat_o)
    vals, meta = B.patch_export_canonical(p.P)
    assert np.array_equal(vals, p.vals_o) and np.array_equal(meta, p.meta_o)
    p.P.close()


def test_pack_rejects_non_24(dev):
    c = synth.make_case("reject", 128, 128, 1, 64, 0.5, seed=3)
    W = to_dev_bf16(c.W, dev)   # not masked
    with pytest.raises(B.PatchError) as e:
        B.patch_pack(W, 128, 128, c.tile_map, 64, stream())
    assert e.value.status == B.ERR_NOT_24
    P = B.patch_pack(W, 128, 128, np.ones_like(c.tile_map), 64, stream())   # all dense is always fine
    P.close()


GEMM_CASES = [
    # name, N, K, tile, f, list of M
    ("tiny", 512, 512, 64, 0.5, [16, 1, 5]),
    ("t64_odd", 192, 320, 64, 0.4, [3, 16, 33, 130]),
    ("t128_mixed", 384, 640, 128, 0.5, [1, 16, 64, 200]),
    ("qwen_896_f0", 896, 896, 128, 0.0, [1, 64]),
    ("qwen_896_f05", 896, 896, 128, 0.5, [1, 64]),
    ("qwen_896_f1", 896, 896, 128, 1.0, [1, 64]),
    ("qwen_up", 4864, 896, 128, 0.5, [1, 64]),
    ("qwen_down", 896, 4864, 128, 0.5, [1, 64]),
]


@pytest.mark.parametrize("name,N,K,t,f,Ms", GEMM_CASES)
def test_gemm_matches_oracle(dev, name, N, K, t, f, Ms):
    c = synth.make_case(name, N, K, max(Ms), t, f, seed=4)
    p = Prepared(c, dev)
    for M in Ms:
        Xb = c.X[:M]
        Yo = p.oracle_gemm(Xb)
        paths = [B.PATH_AUTO, B.PATH_DECODE, B.PATH_PREFILL]
        for path in paths:
            print(f"case {name} N={N} K={K} tile={t} f={f} M={M} path={path}", flush=True)
            Y = p.gemm(Xb, path=path)
            p.check(Xb, Y, Yo, f"{name} M={M} path={path}")
    p.P.close()


@pytest.mark.parametrize("split_k", [1, 2, 3, 5, 8])
def test_decode_split_k_is_deterministic_and_exact_enough(dev, split_k):
    c = synth.make_case("splitk", 256, 1024, 16, 128, 0.5, seed=5)
    p = Prepared(c, dev)
    Yo = p.oracle_gemm(c.X)
    print(f"split_k={split_k}", flush=True)
    Y1 = p.gemm(c.X, path=B.PATH_DECODE, split_k=split_k)
    Y2 = p.gemm(c.X, path=B.PATH_DECODE, split_k=split_k)
    p.check(c.X, Y1, Yo, f"decode split_k={split_k}")
    assert np.array_equal(Y1, Y2), "split-K reduction must be bit-reproducible"
    # smaller M right after a larger one: stale workspace rows must not leak
    Y3 = p.gemm(c.X[:2], path=B.PATH_DECODE, split_k=split_k)
    assert np.array_equal(Y3, Y1[:2])
    p.P.close()


@pytest.mark.parametrize("t", [64, 128])
def test_one_hot_weight_positions(dev, t):
    """W_hat = one nonzero per (row, column-in-tile) pattern; X rows = distinct powers of two per column
    block.  Any error in the register layout or in the position bits moves an output."""
    N, K = 2 * t, 2 * t
    rng = np.random.default_rng(11)
    for tile_kind in (0, 1):
        tm = np.full((2, 2), tile_kind, np.uint8)
        W = np.zeros((N, K), np.float32)
        # every row gets nonzeros at columns congruent to a row-dependent residue: covers all (row%t, col%t)
        # classes over the sweep below while staying 2:4 (one nonzero per group of 4)
        for shift in range(4):
            W[:] = 0
            for n in range(N):
                ks = (np.arange(K // 4) * 4 + (n + shift) % 4)
                W[n, ks] = 1.0 + (n % 7)
            Wb = synth.f32_to_bf16_bits(W)
            Xf = rng.integers(-3, 4, size=(16, K)).astype(np.float32)
            Xb = synth.f32_to_bf16_bits(Xf)
            Wd = to_dev_bf16(Wb, dev)
            P = B.patch_pack(Wd, N, K, tm, t, stream())
            expect = Xf.astype(np.float64) @ W.astype(np.float64).T      # exact small integers
            for path in (B.PATH_DECODE, B.PATH_PREFILL):
                print(f"one-hot tile={t} kind={tile_kind} shift={shift} path={path}", flush=True)
                X = to_dev_bf16(Xb, dev)
                Y = torch.full((16, N), float("nan"), device=dev)
                B.patch_gemm(X, 16, P, Y, stream(), path=path)
                torch.cuda.synchronize()
                assert np.array_equal(Y.cpu().numpy().astype(np.float64), expect)
            P.close()


def test_full_size_decode_sampled(dev):
    """7B attention projection at full size (4096 x 4096, tile 128): all five 2:4 fractions, M in {1, 4, 16},
    checked on the full output against the oracle for M = 16 at f = 0.5 and on sampled outputs otherwise."""
    N = K = 4096
    for f in (0.0, 0.25, 0.5, 0.75, 1.0):
        c = synth.make_case("attn", N, K, 16, 128, f, seed=6)
        p = Prepared(c, dev)
        vals, meta = B.patch_export_canonical(p.P)
        assert np.array_equal(vals, p.vals_o) and np.array_equal(meta, p.meta_o)
        rng = np.random.default_rng(1)
        for M in (1, 4, 16):
            print(f"attn decode f={f} M={M}", flush=True)
            Y = p.gemm(c.X[:M])
            assert np.isfinite(Y).all()
            if f == 0.5 and M == 16:
                p.check(c.X[:M], Y, None, f"attn f={f} M={M}")
            mn = np.stack([rng.integers(0, M, 512), rng.integers(0, N, 512)], axis=1)
            ref = oracle.gemm_points(c.X[:M], p.W_hat_o, mn)
            got = Y[mn[:, 0], mn[:, 1]].astype(np.float64)
            assert float(np.linalg.norm(got - ref) / np.linalg.norm(ref)) <= TIGHT
            assert (np.abs(got - ref) <= elem_bound(row_norms(c.X[:M])[mn[:, 0]], p.wn[mn[:, 1]], K)).all()
        p.P.close()


def _sampled_checks(p, c, Xb, Y, rng, n_points=2048, n_rows=32, what=""):
    """Checks at sizes where the full fp64 product is too slow on a CPU: (1) sampled outputs computed one by
    one from the definition, (2) a seeded sample of whole rows - both element by element against the bound -,
    (3) two Freivalds projections over the full output, one on each side: r^T Y = (r^T X) W_hat^T for a random sign
    vector r over the rows and Y s = X (W_hat^T s) for one over the features.  A projection sums M (or N) independent
    element errors, so it is held to the root of the sum of their squared bounds: one wrong element of ordinary
    size (about sqrt(K) sigma_x sigma_w) in a column or row exceeds that at every size tested here."""
    M = Xb.shape[0]
    assert np.isfinite(Y).all(), "unwritten outputs"
    xn, wn = row_norms(Xb), p.wn
    mn = np.stack([rng.integers(0, M, n_points), rng.integers(0, c.N, n_points)], axis=1)
    ref = oracle.gemm_points(Xb, p.W_hat_o, mn)
    got = Y[mn[:, 0], mn[:, 1]].astype(np.float64)
    assert float(np.linalg.norm(got - ref) / np.linalg.norm(ref)) <= TIGHT
    assert (np.abs(got - ref) <= elem_bound(xn[mn[:, 0]], wn[mn[:, 1]], c.K)).all(), "a sampled output is off"
    rows = np.sort(rng.choice(M, size=min(n_rows, M), replace=False))
    Yo = oracle.gemm(np.ascontiguousarray(Xb[rows]), p.vals_o, p.meta_o, c.N, c.K, c.tile_map, c.tile)
    check_elements(Y[rows], Yo, xn[rows], wn, c.K, f"{what} {len(rows)} sampled rows")
    Xf, Wf = synth.bf16_bits_to_f64(Xb), synth.bf16_bits_to_f64(p.W_hat_o)
    Y64 = Y.astype(np.float64)
    r = rng.choice(np.array([-1.0, 1.0]), size=M)
    dn = np.abs(r @ Y64 - (r @ Xf) @ Wf.T)
    bound_n = elem_bound(np.sqrt((xn * xn).sum()), wn, c.K)          # per feature: root of the sum over rows of bound^2
    s = rng.choice(np.array([-1.0, 1.0]), size=c.N)
    dm = np.abs(Y64 @ s - Xf @ (Wf.T @ s))
    bound_m = elem_bound(xn, np.sqrt((wn * wn).sum()), c.K)
    print(f"  parity {what}: projections max err/bound over rows {float((dn / bound_n).max()):.3f} "
          f"over features {float((dm / bound_m).max()):.3f}", flush=True)
    assert (dn <= bound_n).all(), f"row-side projection: feature {int(np.argmax(dn - bound_n))}"
    assert (dm <= bound_m).all(), f"feature-side projection: row {int(np.argmax(dm - bound_m))}"


@pytest.mark.parametrize("N,K,M", [(11008, 4096, 4096), (4096, 11008, 2048), (4096, 11008, 4096), (11008, 4096, 2048)])
def test_full_size_prefill_sampled(dev, N, K, M):
    """7B MLP prefill at full size, in the launch configuration the benchmark times (tile 128, 60 % 2:4 tiles): both
    projections at both row counts of the configuration."""
    print(f"prefill N={N} K={K} M={M}", flush=True)
    c = synth.make_case("mlp_prefill", N, K, M, 128, 0.6, seed=7)
    p = Prepared(c, dev)
    vals, meta = B.patch_export_canonical(p.P)
    assert np.array_equal(vals, p.vals_o) and np.array_equal(meta, p.meta_o)
    Y = p.gemm(c.X)
    _sampled_checks(p, c, c.X, Y, np.random.default_rng(2), what=f"mlp {N}x{K} M={M}")
    # ragged M on the same weights: last row block partly empty
    Mr = M - 77
    Yr = p.gemm(c.X[:Mr])
    assert np.array_equal(Yr, Y[:Mr]), "rows must not depend on how many rows follow them"
    p.P.close()


def test_13b_layer_shapes_sampled(dev):
    """One decoder layer of the 13B stack (q/k/v/o 5120^2, gate/up 13824 x 5120, down 5120 x 13824) with the
    layer's 2:4 fraction drawn U[0,1), at M = 1, a batched-decode M = 16 and 48 (the wide-wavefront kernel on the
    13824-feature weight, alone and with K-chunks over a workspace on the others) and M = 512."""
    ws = torch.empty(8 * 512 * 13824, device=dev, dtype=torch.float32)
    fr = synth.layer_fractions(0, 40)
    for li, (N, K) in [(3, (5120, 5120)), (17, (13824, 5120)), (29, (5120, 13824))]:
        f = float(fr[li])
        print(f"13B layer {li} N={N} K={K} f={f:.3f}", flush=True)
        c = synth.make_case(f"l13b_{li}", N, K, 512, 128, f, seed=8)
        p = Prepared(c, dev)
        rng = np.random.default_rng(li)
        for M in (1, 512):
            Y = p.gemm(c.X[:M])
            _sampled_checks(p, c, c.X[:M], Y, rng, n_points=1024, n_rows=8, what=f"13B {N}x{K} M={M}")
        for M, kw in ((16, dict()), (48, dict()), (48, dict(workspace=ws)), (512, dict(workspace=ws))):
            Y = p.gemm(c.X[:M], **kw)
            _sampled_checks(p, c, c.X[:M], Y, rng, n_points=1024, n_rows=8, what=f"13B {N}x{K} M={M} ws={'workspace' in kw}")
        p.P.close()


@pytest.mark.parametrize("li,N,K", [(5, 5120, 5120), (21, 13824, 5120), (34, 5120, 13824)])
def test_13b_layer_shapes_prefill_4096(dev, li, N, K):
    """The 13B stack's three weight shapes at M = 4096 (320-, 864- and 320-tile launches, K of 40 and 108 tiles) with
    the 2:4 fraction drawn for decoder layer li, as patch_gemm runs them with and without a workspace (with one, a
    part-filled last round is split in K)."""
    M = 4096
    f = float(synth.layer_fractions(0, 40)[li])
    print(f"13B layer {li} N={N} K={K} M={M} f={f:.3f}", flush=True)
    c = synth.make_case(f"l13b_pf_{li}", N, K, M, 128, f, seed=9)
    p = Prepared(c, dev)
    vals, meta = B.patch_export_canonical(p.P)
    assert np.array_equal(vals, p.vals_o) and np.array_equal(meta, p.meta_o)
    del vals, meta
    need = B.patch_gemm_workspace_bytes(M, p.P)
    ws = torch.empty(max(need, 1 << 20) // 4, device=dev, dtype=torch.float32)
    rng = np.random.default_rng(li)
    for label, kw in (("plain", dict()), (f"workspace {need >> 20} MB", dict(workspace=ws))):
        print(f"  13B layer {li}: {label}", flush=True)
        Y = p.gemm(c.X, **kw)
        _sampled_checks(p, c, c.X, Y, rng, n_points=2048, n_rows=16, what=f"13B {N}x{K} M={M} {label}")
        del Y
    p.P.close()


def test_13b_fused_qkv_with_per_matrix_fractions(dev):
    """The allocation the paper reports inside a block (Section 5, "Sparsity allocation": key / value dense, query
    pruned the most of the attention matrices) on the 13B attention shapes: q / k / v of a middle layer with the
    fractions of synth.matrix_fractions, sharing X in one launch per pass, at M = 1, 16 and 512."""
    H, F = 5120, 13824
    fr = synth.matrix_fractions(40, [H * H] * 4 + [F * H] * 3, 0.5)[15]
    assert fr[0] > 0.5 and fr[1] == 0 and fr[2] == 0
    cases = [synth.make_case(f"alloc_{n}", H, H, 512, 128, float(fr[i]), seed=31) for i, n in enumerate(("q", "k", "v"))]
    X = cases[0].X
    preps = [Prepared(c, dev) for c in cases]
    Xd = to_dev_bf16(X, dev)
    ws = torch.empty(8 * 512 * H, device=dev, dtype=torch.float32)
    rng = np.random.default_rng(15)
    for M, kw in ((1, dict()), (16, dict()), (512, dict()), (512, dict(workspace=ws))):
        print(f"13B q/k/v fused f={[round(float(v), 2) for v in fr[:3]]} M={M} workspace={'workspace' in kw}", flush=True)
        if "workspace" in kw:
            ws.fill_(float("nan"))
        Ys = [torch.full((M, H), float("nan"), device=dev, dtype=torch.float32) for _ in cases]
        B.patch_gemm_many(Xd, M, [p.P for p in preps], Ys, stream(), **kw)
        torch.cuda.synchronize()
        for p, c, Y in zip(preps, cases, Ys):
            _sampled_checks(p, c, X[:M], Y.cpu().numpy(), rng, n_points=1024, n_rows=8, what=f"13B fused {c.name} M={M}")
    for p in preps:
        p.P.close()


@pytest.mark.parametrize("N,K,M,f", [(2112, 1088, 700, 0.6), (320, 2048, 257, 1.0), (576, 64, 300, 0.5), (1024, 1024, 512, 0.0)])
def test_tile64_prefill(dev, N, K, M, f):
    """Mask tile 64 on the 256 x 256 prefill kernel: every K-step a new tile, two tile rows per wavefront, feature counts
    that leave one to three tile rows in the last block, a single K-step, ragged M; the small kernel beside it, the bf16
    output, and repeated launches bit-equal (a spilled accumulator once made a few outputs differ from run to run)."""
    print(f"tile 64 prefill N={N} K={K} M={M} f={f}", flush=True)
    c = synth.make_case("t64_prefill", N, K, M, 64, f, seed=12)
    p = Prepared(c, dev)
    Yo = p.oracle_gemm(c.X)
    Y = p.gemm(c.X, path=B.PATH_PREFILL)
    p.check(c.X, Y, Yo, f"tile 64 {N}x{K} M={M}")
    for rep in range(3):
        assert np.array_equal(p.gemm(c.X, path=B.PATH_PREFILL), Y), "launches of one configuration must be bit-equal"
    p.check(c.X, p.gemm(c.X, path=B.PATH_PREFILL, variant=1), Yo, "tile 64, small kernel")
    Mr = M - 70
    assert np.array_equal(p.gemm(c.X[:Mr], path=B.PATH_PREFILL), Y[:Mr]), "rows must not depend on how many rows follow them"
    check_bf16(p.gemm_bf16(c.X, path=B.PATH_PREFILL), Yo, row_norms(c.X), p.wn, K, "tile 64 bf16 output")
    # K split over workgroups (partial products in a poisoned caller workspace, summed in slice order)
    ws = torch.empty(8 * M * N, device=dev, dtype=torch.float32)
    need = B.patch_gemm_workspace_bytes(M, p.P, path=B.PATH_PREFILL)
    print(f"  tile 64: automatic split wants {need} workspace bytes", flush=True)
    for kw in (dict(workspace=ws), dict(workspace=ws, split_k=3), dict(workspace=ws, split_k=8)):
        if kw.get("split_k", 0) > K // 64:
            continue
        Ys = p.gemm(c.X, path=B.PATH_PREFILL, **kw)
        p.check(c.X, Ys, Yo, f"tile 64 split_k={kw.get('split_k', 0)}")
        assert np.array_equal(p.gemm(c.X, path=B.PATH_PREFILL, **kw), Ys)
    p.P.close()


@pytest.mark.parametrize("t,N,K,M,f", [(64, 2112, 1088, 700, 0.6), (64, 320, 2048, 257, 1.0), (64, 576, 64, 130, 0.5),
                                       (128, 2176, 1152, 700, 0.6), (128, 384, 2048, 100, 1.0), (128, 1024, 1024, 512, 0.0),
                                       (128, 640, 128, 129, 0.5)])
def test_prefill_blocks_of_128_rows(dev, t, N, K, M, f):
    _blocks_of_128_rows(dev, t, N, K, M, f, 4)


@pytest.mark.parametrize("variant,t,N,K,M,f", [
    (5, 128, 2176, 1152, 700, 0.6), (5, 128, 384, 2048, 100, 1.0), (5, 128, 1024, 1024, 512, 0.0), (5, 128, 640, 128, 129, 0.5),
    (5, 128, 4224, 512, 300, 0.3),
    (5, 64, 2112, 1088, 700, 0.6), (5, 64, 320, 2048, 257, 1.0), (5, 64, 576, 64, 130, 0.5), (5, 64, 1024, 1024, 512, 0.0), (5, 64, 192, 448, 100, 0.5),
    (6, 64, 2112, 1088, 700, 0.6), (6, 64, 320, 2048, 257, 1.0), (6, 64, 576, 64, 130, 0.5), (6, 64, 1024, 1024, 512, 0.0), (6, 64, 192, 448, 100, 0.5)])
def test_prefill_weights_in_registers(dev, variant, t, N, K, M, f):
    """prefill_kernel_areg - weight fragments loaded straight into registers, X through LDS: blocks of 128 rows (variant 5)
    on both mask tiles and of 256 rows (variant 6) on mask tile 64; the cases and checks of the LDS-staged kernel, a
    weight of 33 tile rows, odd and even tile counts along K (mask tile 64 takes its steps in pairs)."""
    _blocks_of_128_rows(dev, t, N, K, M, f, variant)


def _blocks_of_128_rows(dev, t, N, K, M, f, variant):
    """The LDS-staged prefill kernel with blocks of 128 rows of X (a wavefront = 64 features x 64 rows): both mask tiles,
    feature counts that leave part of the last block empty, ragged M, one K-step, K split over a poisoned workspace,
    bf16 output, repeated launches bit-equal, rows independent of the rows behind them."""
    print(f"128-row blocks variant={variant} tile={t} N={N} K={K} M={M} f={f}", flush=True)
    c = synth.make_case("pf128", N, K, M, t, f, seed=14)
    p = Prepared(c, dev)
    Yo = p.oracle_gemm(c.X)
    kw = dict(path=B.PATH_PREFILL, variant=variant)
    Y = p.gemm(c.X, **kw)
    p.check(c.X, Y, Yo, f"128-row blocks tile {t} {N}x{K} M={M}")
    for rep in range(3):
        assert np.array_equal(p.gemm(c.X, **kw), Y), "launches of one configuration must be bit-equal"
    Mr = M - 70
    assert np.array_equal(p.gemm(c.X[:Mr], **kw), Y[:Mr]), "rows must not depend on how many rows follow them"
    check_bf16(p.gemm_bf16(c.X, **kw), Yo, row_norms(c.X), p.wn, K, "128-row blocks, bf16 output")
    ws = torch.empty(8 * M * N, device=dev, dtype=torch.float32)
    for more in (dict(workspace=ws), dict(workspace=ws, split_k=3), dict(workspace=ws, split_k=8)):
        if more.get("split_k", 0) > K // t:
            continue
        ws.fill_(float("nan"))
        Ys = p.gemm(c.X, **kw, **more)
        p.check(c.X, Ys, Yo, f"128-row blocks split_k={more.get('split_k', 0)}")
        assert np.array_equal(p.gemm(c.X, **kw, **more), Ys)
    p.P.close()


@pytest.mark.parametrize("t,N,K,f", [(128, 640, 512, 0.5), (64, 320, 448, 0.4), (128, 384, 256, 1.0)])
def test_saved_weight_round_trip(dev, t, N, K, f):
    """patch_serialize -> patch_deserialize: the loaded handle has the saved one's dimensions, tile map, launch order
    and canonical export (bit-equal to the oracle's pack), multiplies bit-identically on the decode and the prefill
    path, and the oracle confirms the product; a buffer with one payload bit flipped is refused."""
    c = synth.make_case("saved", N, K, 300, t, f, seed=77)
    p = Prepared(c, dev)
    buf = p.P.serialize(stream())
    assert buf.size == 64 + -(-c.tile_map.size // 64) * 64 + p.P.nbytes
    Ys = {M: p.gemm(c.X[:M]) for M in (1, 16, 40, 300)}
    order, dims = p.P.row_order(), p.P.dims()
    p.P.close()                                    # the saved bytes are all that is left
    p.P = B.patch_deserialize(buf, stream())
    assert p.P.dims() == dims and np.array_equal(p.P.tile_map(), c.tile_map) and np.array_equal(p.P.row_order(), order)
    vals, meta = B.patch_export_canonical(p.P)
    assert np.array_equal(vals, p.vals_o) and np.array_equal(meta, p.meta_o)
    for M, Y in Ys.items():
        assert np.array_equal(p.gemm(c.X[:M]), Y), f"M={M}: the loaded weight multiplies differently"
    p.check(c.X, p.gemm(c.X), None, "loaded weight")
    again = p.P.serialize(stream())
    assert np.array_equal(again, buf), "saving the loaded weight gives other bytes"
    bad = buf.copy()
    bad[buf.size // 2] ^= 4
    with pytest.raises(B.PatchError) as e:
        B.patch_deserialize(bad, stream())
    assert e.value.status == B.ERR_ARG
    with pytest.raises(B.PatchError) as e:
        B.patch_deserialize(buf[:-1], stream())
    assert e.value.status == B.ERR_SIZE
    p.P.close()


def test_x_of_four_gigabytes(dev):
    """The largest X the hand-scheduled prefill kernel takes (its lane offsets into X are 32 bits wide: M K 2 < 4 GB)
    and the first size beyond, which must go to a kernel with 64-bit addresses.  X is a 4099-row block repeated (4099
    does not divide the 262144 rows after which a 32-bit byte offset wraps, so a wrapped address reads another row):
    every row of Y must be bit-equal to the row of the first period with the same X, and rows sampled at both ends, at
    the wrap and at random are compared with the oracle."""
    N, K, t, period = 256, 8192, 128, 4099
    c = synth.make_case("x4g", N, K, period, t, 0.5, seed=61)
    p = Prepared(c, dev)
    Xs = to_dev_bf16(c.X, dev)
    rng = np.random.default_rng(8)
    for M, kw in ((262143, dict(path=B.PATH_PREFILL, variant=3)), (262145, dict(path=B.PATH_PREFILL, variant=3)), (262145, dict())):
        print(f"X of {M * K * 2 / 2 ** 30:.3f} GiB, M={M} {kw}", flush=True)
        idx = torch.arange(M, device=dev) % period
        X = Xs[idx]
        Y = torch.full((M, N), float("nan"), device=dev, dtype=torch.float32)
        B.patch_gemm(X, M, p.P, Y, stream(), **kw)
        torch.cuda.synchronize()
        del X
        assert torch.equal(Y, Y[:period][idx]), "rows with equal X differ: an address wrapped or a block was skipped"
        rows = np.unique(np.concatenate([np.arange(0, 130), np.arange(M - 130, M), np.arange(131072 - 4, 131072 + 4),
                                         np.arange(262144 - 300, min(M, 262144 + 4)), rng.integers(0, M, 100)]))
        rows = rows[rows < M]
        Yr = Y[torch.from_numpy(rows).to(dev)].cpu().numpy()
        Xr = np.ascontiguousarray(c.X[rows % period])
        check_elements(Yr, p.oracle_gemm(Xr), row_norms(Xr), p.wn, K, f"M={M} sampled rows")
        del Y
    p.P.close()


@pytest.mark.parametrize("K", [16384, 16512])
def test_longest_k_of_the_hand_scheduled_kernel(dev, K):
    """K = 16384 is the longest the hand-scheduled prefill kernel takes (128 tiles along K: two table registers per
    lane); K = 16512 must go to another kernel.  Full output against the oracle on every prefill variant, with and
    without a K split, and on the decode path."""
    N, M, t = 384, 300, 128
    c = synth.make_case("longk", N, K, M, t, 0.5, seed=62)
    p = Prepared(c, dev)
    Yo = p.oracle_gemm(c.X)
    ws = torch.empty(8 * M * N, device=dev, dtype=torch.float32)
    for kw in (dict(), dict(workspace=ws), dict(path=B.PATH_PREFILL, variant=3), dict(path=B.PATH_PREFILL, variant=3, workspace=ws),
               dict(path=B.PATH_PREFILL, variant=3, workspace=ws, split_k=7), dict(path=B.PATH_PREFILL, variant=5),
               dict(path=B.PATH_PREFILL, variant=2), dict(path=B.PATH_DECODE), dict(path=B.PATH_DECODE, workspace=ws)):
        print(f"K={K} " + str({k: v for k, v in kw.items() if k != 'workspace'}) + (" +workspace" if "workspace" in kw else ""), flush=True)
        p.check(c.X, p.gemm(c.X, **kw), Yo, f"K={K}")
    p.P.close()


def test_payload_beyond_four_gigabytes(dev):
    """A packed weight whose payload is larger than 4 GB (tile offsets are stored in 256-byte granules, kernel addresses
    are 64 bits wide): 2304 tile rows x 65 tile columns, a fifth of the tiles 2:4, 4.5 GB.  The weight is a block of
    33 tile rows repeated (33 tile rows are not a divisor of 2^32 bytes, so a wrapped offset reads another row): every
    column of Y must be bit-equal to the column of the first period with the same weight row, and sampled columns from
    both ends, around the 4 GB mark and at random are compared with the oracle - on the decode kernel, the batched
    decode kernel, the prefill kernels and after unpacking."""
    t, Tn, Tk, per = 128, 2304, 65, 33
    N, K, M = Tn * t, Tk * t, 300
    c = synth.make_case("big_payload", per * t, K, M, t, 0.2, seed=63)
    W_hat_s = oracle.apply_mask(c.W, c.tile_map, c.mask24, t)
    vals_s, meta_s = oracle.pack(W_hat_s, c.tile_map, t)
    ridx = torch.arange(N, device=dev) % (per * t)
    W_hat = to_dev_bf16(W_hat_s, dev)[ridx]
    tile_map = np.ascontiguousarray(c.tile_map[np.arange(Tn) % per])
    P = B.patch_pack(W_hat, N, K, tile_map, t, stream())
    assert P.nbytes > 2 ** 32, P.nbytes
    back = torch.full((N, K), -1, device=dev, dtype=torch.int16).view(torch.bfloat16)
    B.patch_unpack(P, back, stream())
    torch.cuda.synchronize()
    assert torch.equal(back.view(torch.int16), W_hat.view(torch.int16)), "unpack differs from what was packed"
    del back, W_hat
    X = to_dev_bf16(c.X, dev)
    rng = np.random.default_rng(9)
    row_bytes = np.where(tile_map == 1, 2 * t * t, t * t + t * t // 8).sum(axis=1)
    first_beyond = int(np.searchsorted(np.cumsum(row_bytes), 2 ** 32)) * t     # first feature whose tiles end past 4 GB
    assert 0 < first_beyond < N - 130
    cols = np.unique(np.concatenate([np.arange(0, 140), np.arange(N - 140, N), np.arange(first_beyond - 130, first_beyond + 130),
                                     rng.integers(0, N, 200)]))
    xn, wn = row_norms(c.X), row_norms(W_hat_s)
    ws = torch.empty(2 * M * N, device=dev, dtype=torch.float32)
    for rows, kw in ((1, dict()), (16, dict()), (48, dict()), (64, dict(workspace=ws)), (M, dict()), (M, dict(workspace=ws)),
                     (M, dict(path=B.PATH_PREFILL, variant=5)), (M, dict(path=B.PATH_PREFILL, variant=2))):
        print(f"payload {P.nbytes / 2 ** 30:.2f} GiB, M={rows} " + str({k: v for k, v in kw.items() if k != 'workspace'})
              + (" +workspace" if "workspace" in kw else ""), flush=True)
        Y = torch.full((rows, N), float("nan"), device=dev, dtype=torch.float32)
        if "workspace" in kw:
            ws.fill_(float("nan"))
        B.patch_gemm(X, rows, P, Y, stream(), **kw)
        torch.cuda.synchronize()
        assert torch.equal(Y, Y[:, : per * t][:, ridx]), "columns with equal weight rows differ: an offset wrapped"
        Yc = Y[:, torch.from_numpy(cols).to(dev)].cpu().numpy()
        Yo = oracle.gemm(np.ascontiguousarray(c.X[:rows]), vals_s, meta_s, per * t, K, c.tile_map, t)[:, cols % (per * t)]
        check_elements(Yc, Yo, xn[:rows], wn[cols % (per * t)], K, f"M={rows} sampled columns")
        del Y
    P.close()


def test_workspace_of_any_size_is_respected(dev):
    """Whatever size the caller's workspace has - what patch_gemm_workspace_bytes asks for, 16 bytes less, half, one
    slice, a page, 16 bytes - a launch writes nothing behind it (a guard region keeps its pattern) and the result is
    the oracle's: a launch that cannot use the workspace as it is splits less or not at all."""
    guard = 1 << 18
    pattern = 0x7FC0BEEF
    rng = np.random.default_rng(12)
    for t, N, K, M, f in ((128, 640, 2048, 300, 0.5), (64, 448, 1600, 513, 0.5), (128, 1152, 768, 64, 1.0), (128, 256, 4096, 130, 0.0)):
        c = synth.make_case("anyws", N, K, M, t, f, seed=71)
        p = Prepared(c, dev)
        Yo = p.oracle_gemm(c.X)
        X = to_dev_bf16(c.X, dev)
        xn = row_norms(c.X)
        big = torch.empty(8 * M * N + guard, device=dev, dtype=torch.int32)
        scheds = [dict(), dict(path=B.PATH_DECODE), dict(path=B.PATH_PREFILL), dict(path=B.PATH_PREFILL, variant=2, split_k=5),
                  dict(path=B.PATH_PREFILL, variant=3, split_k=int(rng.integers(2, 9))), dict(path=B.PATH_PREFILL, variant=5, split_k=4),
                  dict(path=B.PATH_PREFILL, variant=4), dict(path=B.PATH_PREFILL, variant=6, split_k=3), dict(path=B.PATH_DECODE, variant=4)]
        for kw in scheds:
            need = B.patch_gemm_workspace_bytes(M, p.P, **kw)
            for nbytes in sorted({need, need - 16, need // 32 * 16, 8 * M * N * 4, 2 * M * N * 4, M * N * 4, 4096, 16}):
                if nbytes <= 0:
                    continue
                n = nbytes // 4
                big.fill_(pattern)
                Y = torch.full((M, N), float("nan"), device=dev, dtype=torch.float32)
                what = f"tile {t} {N}x{K} M={M} {kw} workspace of {nbytes} bytes (asked for: {need})"
                B.patch_gemm(X, M, p.P, Y, stream(), workspace=big[:n].view(torch.float32), **kw)
                torch.cuda.synchronize()
                assert bool((big[n:] == pattern).all()), what + ": wrote behind the workspace"
                check_elements(Y.cpu().numpy(), Yo, xn, p.wn, K, what)
        p.P.close()


def test_nothing_is_written_outside_y(dev):
    """Y lies between two guard regions: with ragged M, a feature count that leaves part of the last block empty, fp32
    and bf16 output, on every path and kernel variant, with and without a workspace, both guards keep their pattern
    (a bf16 Y is half as large: a kernel that stored fp32 into it would run over its end)."""
    guard, pattern = 1 << 16, 0x7FC0BEEF
    ws = torch.empty(8 * 300 * 1152, device=dev, dtype=torch.float32)
    for t, N, K, M in ((128, 1152, 512, 300), (64, 320, 448, 131), (128, 384, 1024, 49), (64, 64, 64, 1), (128, 128, 128, 257)):
        c = synth.make_case("yguard", N, K, M, t, 0.5, seed=73)
        p = Prepared(c, dev)
        X = to_dev_bf16(c.X, dev)
        Yo = p.oracle_gemm(c.X)
        xn = row_norms(c.X)
        scheds = [dict(), dict(workspace=ws), dict(path=B.PATH_DECODE), dict(path=B.PATH_DECODE, workspace=ws), dict(path=B.PATH_DECODE, variant=4)]
        for v in range(0, 7):
            scheds += [dict(path=B.PATH_PREFILL, variant=v), dict(path=B.PATH_PREFILL, variant=v, workspace=ws)]
        for kw in scheds:
            for bf16 in (False, True):
                words = M * N // 2 if bf16 else M * N          # M N is even in every case but the single row of 64
                if bf16 and (M * N) % 2:
                    continue
                buf = torch.full((guard + words + guard,), pattern, device=dev, dtype=torch.int32)
                Y = buf[guard: guard + words].view(torch.bfloat16 if bf16 else torch.float32).view(M, N)
                what = f"tile {t} {N}x{K} M={M} bf16={bf16} " + str({k: v for k, v in kw.items() if k != 'workspace'}) + (" +workspace" if "workspace" in kw else "")
                B.patch_gemm(X, M, p.P, Y, stream(), y_bf16=bf16, **kw)
                torch.cuda.synchronize()
                assert bool((buf[:guard] == pattern).all()) and bool((buf[guard + words:] == pattern).all()), what + ": wrote outside Y"
                if bf16:
                    check_bf16(bits_of(Y), Yo, xn, p.wn, K, what)
                else:
                    check_elements(Y.cpu().numpy(), Yo, xn, p.wn, K, what)
        p.P.close()


@pytest.mark.parametrize("t,N,K", [(128, 384, 640), (64, 192, 320), (64, 128, 64), (128, 256, 2176)])
def test_decode_x_load_schedules(dev, t, N, K):
    """Up to 8 rows the strip kernel loads X either with two instructions per step (variant 5) or with one instruction
    for 8, 2 or 1 steps (variant 6: the operands of 1, up to 4, up to 8 rows side by side in the 16 operand columns,
    rotated into place per step).  Both against the oracle and bit-equal to each other (the same products summed in the
    same order), on all-dense, mixed and all-2:4 maps, K-step counts that leave the last pass of a wavefront part empty,
    forced wavefront counts, bf16 output, and weights sharing X in one launch."""
    for f in (0.0, 0.5, 1.0):
        c = synth.make_case("xsched", N, K, 8, t, f, seed=81)
        p = Prepared(c, dev)
        for M in range(1, 9):
            Yo = p.oracle_gemm(c.X[:M])
            print(f"tile {t} {N}x{K} f={f} M={M}", flush=True)
            Y5 = p.gemm(c.X[:M], path=B.PATH_DECODE, variant=5)
            Y6 = p.gemm(c.X[:M], path=B.PATH_DECODE, variant=6)
            p.check(c.X[:M], Y6, Yo, f"one X load for several steps, M={M}")
            assert np.array_equal(Y5, Y6), "the two X-load schedules differ"
            assert np.array_equal(p.gemm(c.X[:M]), Y6), "the default schedule differs"
            for kw in (1, 3, 16):
                Yk = p.gemm(c.X[:M], path=B.PATH_DECODE, variant=6, split_k=kw)
                p.check(c.X[:M], Yk, Yo, f"M={M}, {kw} wavefronts")
                assert np.array_equal(Yk, p.gemm(c.X[:M], path=B.PATH_DECODE, variant=5, split_k=kw))
            check_bf16(p.gemm_bf16(c.X[:M], path=B.PATH_DECODE, variant=6), Yo, row_norms(c.X[:M]), p.wn, K, f"bf16 M={M}")
        p.P.close()
    # two weights sharing X (different fractions: the set's overall share decides the default schedule)
    cases = [synth.make_case(f"xsched_set{i}", N, K, 8, t, f, seed=82 + i) for i, f in enumerate((0.2, 0.9))]
    preps = [Prepared(c, dev) for c in cases]
    X = cases[0].X
    Xd = to_dev_bf16(X, dev)
    for M in (1, 3, 8):
        for v in (0, 5, 6):
            Ys = [torch.full((M, N), float("nan"), device=dev, dtype=torch.float32) for _ in cases]
            B.patch_gemm_many(Xd, M, [p.P for p in preps], Ys, stream(), path=B.PATH_DECODE, variant=v)
            torch.cuda.synchronize()
            for p, Y in zip(preps, Ys):
                p.check(X[:M], Y.cpu().numpy(), None, f"set, M={M}, variant {v}")
    for p in preps:
        p.P.close()


def test_mid_m_paths_agree(dev):
    """M around the decode / prefill crossover: both paths must give the oracle's result."""
    c = synth.make_case("mid", 1024, 768, 300, 128, 0.5, seed=9)
    p = Prepared(c, dev)
    for M in (17, 31, 32, 33, 48, 64, 65, 100, 128, 129, 256, 257, 300):
        Yo = p.oracle_gemm(c.X[:M])
        for path in (B.PATH_AUTO, B.PATH_DECODE, B.PATH_PREFILL):
            print(f"mid M={M} path={path}", flush=True)
            p.check(c.X[:M], p.gemm(c.X[:M], path=path), Yo, f"mid M={M} path={path}")
    # the 64-features-per-wavefront kernel for 17 .. 64 rows per pass, unsplit and with K-chunks over a workspace
    ws = torch.empty(8 * 64 * 1024, device=dev, dtype=torch.float32)
    for M in (1, 7, 16, 17, 32, 33, 48, 64, 65, 100, 130):
        Yo = p.oracle_gemm(c.X[:M])
        for kw in (dict(), dict(workspace=ws), dict(workspace=ws, split_k=3), dict(workspace=ws, split_k=6)):
            print(f"mid kernel M={M} split_k={kw.get('split_k')} workspace={'workspace' in kw}", flush=True)
            p.check(c.X[:M], p.gemm(c.X[:M], path=B.PATH_DECODE, variant=4, **kw), Yo, f"mid kernel M={M}")
    p.P.close()
    # decode passes of up to 64 rows (1, 2 or 4 blocks of 16) on tile 64 and with forced wavefront counts
    c = synth.make_case("mid64", 192, 640, 70, 64, 0.5, seed=9)
    p = Prepared(c, dev)
    for M in (20, 40, 64, 70):
        Yo = p.oracle_gemm(c.X[:M])
        for sk in (0, 1, 3, 8):
            p.check(c.X[:M], p.gemm(c.X[:M], path=B.PATH_DECODE, split_k=sk), Yo, f"tile 64 M={M} split_k={sk}")
        for kw in (dict(), dict(workspace=ws), dict(workspace=ws, split_k=4)):
            p.check(c.X[:M], p.gemm(c.X[:M], path=B.PATH_DECODE, variant=4, **kw), Yo, f"tile 64 mid kernel M={M}")
    p.P.close()


def test_gemm_many_matches_single_calls(dev):
    """patch_gemm_many: several weights sharing X (different N, different maps) in one decode launch per 16 rows,
    bit-equal to the single calls and within tolerance of the oracle; prefill path: one launch per weight."""
    K, t = 1024, 128
    cases = [synth.make_case(f"many{i}", N, K, 300, t, f, seed=20) for i, (N, f) in enumerate([(512, 0.5), (128, 1.0), (384, 0.0)])]
    X = cases[0].X                       # shared input
    preps = [Prepared(c, dev) for c in cases]
    Xd = to_dev_bf16(X, dev)
    for M, path, variant in [(1, B.PATH_AUTO, 0), (16, B.PATH_DECODE, 0), (40, B.PATH_DECODE, 0), (40, B.PATH_PREFILL, 0),
                             (300, B.PATH_AUTO, 0), (24, B.PATH_DECODE, 4), (100, B.PATH_DECODE, 4)]:
        print(f"many M={M} path={path} variant={variant}", flush=True)
        Ys = [torch.full((M, c.N), float("nan"), device=dev, dtype=torch.float32) for c in cases]
        B.patch_gemm_many(Xd, M, [p.P for p in preps], Ys, stream(), path=path, variant=variant)
        for p, Y in zip(preps, Ys):
            single = torch.empty_like(Y)
            B.patch_gemm(Xd, M, p.P, single, stream(), path=path, variant=variant)
            torch.cuda.synchronize()
            assert torch.equal(Y, single), "fused launch differs from the single call"
            p.check(X[:M], Y.cpu().numpy(), None, f"many M={M}")
    # with a workspace the few output tiles of this set are split in K: one launch over the set, slices in the
    # (poisoned) workspace, one reduction launch; repeated launches bit-equal
    for M in (40, 300):
        ws = torch.full((8 * M * 1024,), float("nan"), device=dev, dtype=torch.float32)
        Ys = [torch.full((M, c.N), float("nan"), device=dev, dtype=torch.float32) for c in cases]
        B.patch_gemm_many(Xd, M, [p.P for p in preps], Ys, stream(), path=B.PATH_PREFILL, workspace=ws)
        torch.cuda.synchronize()
        first = [Y.clone() for Y in Ys]
        for p, Y in zip(preps, Ys):
            p.check(X[:M], Y.cpu().numpy(), None, f"many, K slices over the set, M={M}")
        ws.fill_(float("nan"))
        B.patch_gemm_many(Xd, M, [p.P for p in preps], Ys, stream(), path=B.PATH_PREFILL, workspace=ws)
        torch.cuda.synchronize()
        assert all(torch.equal(a_, b_) for a_, b_ in zip(first, Ys))
    # a workspace too small for two slices of the set: the unsplit launch
    ws = torch.full((300 * 1024,), float("nan"), device=dev, dtype=torch.float32)
    Ys = [torch.full((300, c.N), float("nan"), device=dev, dtype=torch.float32) for c in cases]
    B.patch_gemm_many(Xd, 300, [p.P for p in preps], Ys, stream(), path=B.PATH_PREFILL, workspace=ws)
    torch.cuda.synchronize()
    for p, Y in zip(preps, Ys):
        p.check(X[:300], Y.cpu().numpy(), None, "many, small workspace")
    other = Prepared(synth.make_case("manyk", 128, 512, 4, t, 0.5, seed=21), dev)
    with pytest.raises(B.PatchError):   # K differs
        B.patch_gemm_many(Xd, 1, [preps[0].P, other.P],
                          [torch.empty((1, 512), device=dev), torch.empty((1, 128), device=dev)], stream())
    other.P.close()
    for p in preps:
        p.P.close()


def test_prefill_split_k(dev):
    """Prefill with K split over workgroups (partial products in a caller workspace, summed in slice order): every
    slice count, slices that do not divide the tile count, ragged M, an odd tile-row count; auto picks a split for
    this small grid; a workspace that is too small or absent degrades to fewer slices / no split; reproducible."""
    c = synth.make_case("splitk", 384, 2048, 300, 128, 0.5, seed=13)
    p = Prepared(c, dev)
    ws = torch.empty(16 * 300 * 384, device=dev, dtype=torch.float32)
    for M in (300, 40):
        Yo = p.oracle_gemm(c.X[:M])
        need = B.patch_gemm_workspace_bytes(M, p.P, path=B.PATH_PREFILL)
        assert need > 0 and need % (M * 384 * 4) == 0, "auto must split this 2- or 4-tile grid"
        for sk in (0, 1, 2, 3, 5, 16):
            print(f"prefill split_k={sk} M={M}", flush=True)
            Y = p.gemm(c.X[:M], path=B.PATH_PREFILL, split_k=sk, workspace=ws)
            p.check(c.X[:M], Y, Yo, f"prefill split_k={sk} M={M}")
            assert np.array_equal(Y, p.gemm(c.X[:M], path=B.PATH_PREFILL, split_k=sk, workspace=ws)), "not reproducible"
        small = ws[: 2 * M * 384 + 5]            # room for two slices only
        assert relF(p.gemm(c.X[:M], path=B.PATH_PREFILL, split_k=5, workspace=small), Yo) <= TIGHT
        assert relF(p.gemm(c.X[:M], path=B.PATH_PREFILL, split_k=5), Yo) <= TIGHT   # none: unsplit
    assert B.patch_gemm_workspace_bytes(1, p.P) == 0            # decode path
    need40 = B.patch_gemm_workspace_bytes(40, p.P)              # auto: a decode pass of 40 rows, K in chunks
    assert need40 > 0 and need40 % (40 * 384 * 4) == 0
    assert relF(p.gemm(c.X[:40], workspace=ws), p.oracle_gemm(c.X[:40])) <= TIGHT
    assert B.patch_gemm_workspace_bytes(100, p.P) > 0           # auto: prefill, split, once a workspace is there
    assert relF(p.gemm(c.X[:100], workspace=ws), p.oracle_gemm(c.X[:100])) <= TIGHT
    p.P.close()


def test_tune_returns_a_valid_fast_schedule(dev):
    """patch_tune: the schedule it returns reproduces the oracle result, with and without a workspace, for a decode
    and a mid-M shape (times are printed, not asserted: they depend on the box)."""
    c = synth.make_case("tune", 512, 2048, 200, 128, 0.5, seed=14)
    p = Prepared(c, dev)
    ws = torch.empty(8 * 200 * 512, device=dev, dtype=torch.float32)
    for M, w in [(4, None), (200, None), (200, ws), (48, ws)]:
        X = to_dev_bf16(c.X[:M], dev)
        Y = torch.full((M, c.N), float("nan"), device=dev, dtype=torch.float32)
        opts, us = B.patch_tune(X, M, p.P, Y, workspace=w, stream=stream(), reps=5)
        print(f"tune M={M} workspace={w is not None}: {opts} {us:.1f} us", flush=True)
        assert us > 0 and opts["path"] in (B.PATH_DECODE, B.PATH_PREFILL)
        torch.cuda.synchronize()
        Yo = p.oracle_gemm(c.X[:M])
        p.check(c.X[:M], Y.cpu().numpy(), Yo, f"tuned M={M}")    # Y holds the chosen schedule's product
        if w is not None:
            w.fill_(float("nan"))
        Y2 = torch.full_like(Y, float("nan"))
        B.run_tuned(X, M, p.P, Y2, opts, workspace=w, stream=stream())
        torch.cuda.synchronize()
        assert torch.equal(Y, Y2), "run_tuned must run the schedule that was timed"
    p.P.close()
    c64 = synth.make_case("tune64", 256, 512, 150, 64, 0.5, seed=15)   # tile 64: decode passes or the simple prefill kernel
    p64 = Prepared(c64, dev)
    X = to_dev_bf16(c64.X, dev)
    Y = torch.empty((150, 256), device=dev, dtype=torch.float32)
    opts, us = B.patch_tune(X, 150, p64.P, Y, stream=stream(), reps=3)
    torch.cuda.synchronize()
    assert opts["path"] in (B.PATH_DECODE, B.PATH_PREFILL) and relF(Y.cpu().numpy(), p64.oracle_gemm(c64.X)) <= TIGHT
    p64.P.close()


def test_tune_report_table_and_small_execution_tile(dev):
    """patch_tune_all reports every candidate; the small 128 x 128 execution tile must not beat the 256 x 256 default
    on a compute-bound shape (the paper's Appendix O finds small execution tiles under-use the matrix units; times are
    printed, only their order is asserted).  patch_tune_layer tunes the decode input first, then the prefill input,
    and both stored schedules reproduce the oracle's result."""
    N, K, Mp = 2048, 2048, 2048
    c = synth.make_case("tune_layer", N, K, Mp, 128, 0.5, seed=16)
    p = Prepared(c, dev)
    X = to_dev_bf16(c.X, dev)
    Y = torch.full((Mp, N), float("nan"), device=dev, dtype=torch.float32)
    ws = torch.full((8 << 20,), float("nan"), device=dev, dtype=torch.float32)
    rep = B.patch_tune_all(X, Mp, p.P, Y, workspace=ws, stream=stream(), reps=5)
    for sch, us in rep:
        print(f"  candidate {sch}: {us:.1f} us", flush=True)
    pre = {sch["variant"]: us for sch, us in rep if sch["path"] == B.PATH_PREFILL and sch["split_k"] == 1}
    assert set(pre) == {0, 1, 2, 4, 5}, "every execution tile of the prefill path must be timed"
    assert pre[1] > pre[0], f"128 x 128 execution tile {pre[1]:.1f} us is not slower than 256 x 256 {pre[0]:.1f} us"
    assert all(sch["path"] == B.PATH_PREFILL for sch, _ in rep), "decode passes are no contenders at M = 2048"
    rep1 = B.patch_tune_all(X, 1, p.P, Y, stream=stream(), reps=5)
    assert len({(s_["split_k"], s_["variant"]) for s_, _ in rep1 if s_["path"] == B.PATH_DECODE}) >= 8, "wavefront counts not swept"
    tab = B.TuneTable()
    tab.tune_layer(X, 4, X, Mp, p.P, Y, workspace=ws, stream=stream(), reps=5)
    assert len(tab) == 2
    for M in (4, 3, Mp, Mp - 500):                      # 3 shares the decode bucket, Mp - 500 the prefill bucket
        sch = tab.get_for(M, p.P, workspace=ws)
        print(f"  stored for M={M}: {sch}", flush=True)
        assert sch is not None and sch["path"] == (B.PATH_DECODE if M <= 4 else B.PATH_PREFILL)
        Y2 = torch.full((M, N), float("nan"), device=dev, dtype=torch.float32)
        ws.fill_(float("nan"))
        B.run_tuned(X, M, p.P, Y2, sch, workspace=ws, stream=stream())
        torch.cuda.synchronize()
        p.check(c.X[:M], Y2.cpu().numpy(), None, f"stored schedule M={M}")
    assert tab.get_for(64, p.P, workspace=ws) is None   # nothing tuned for that bucket
    tab.close()
    p.P.close()


def test_prefill_long_k(dev):
    """K beyond the weights-in-registers kernel's limit (256 tiles): the default choice must fall back."""
    c = synth.make_case("longk", 128, 258 * 128, 40, 128, 0.5, seed=12)
    p = Prepared(c, dev)
    for variant in (0, 3):
        print(f"long K variant={variant}", flush=True)
        assert relF(p.gemm(c.X, path=B.PATH_PREFILL, variant=variant), p.oracle_gemm(c.X)) <= TIGHT
    p.P.close()


@pytest.mark.parametrize("variant", [0, 1, 2, 3, 4, 5, 6])
def test_prefill_kernel_variants(dev, variant):
    """Every prefill kernel variant (patch_gemm_opts.variant) against the oracle: odd tile-row count (N % 256 = 128),
    ragged M, K of several tiles, all-dense / mixed / all-2:4 maps."""
    for N, K, f in [(384, 640, 0.5), (512, 1024, 0.0), (256, 512, 1.0), (640, 384, 0.3), (128, 128, 0.5), (256, 256, 0.5)]:
        c = synth.make_case("variants", N, K, 300, 128, f, seed=10)
        p = Prepared(c, dev)
        for M in (300, 256, 17):
            print(f"variant={variant} N={N} K={K} f={f} M={M}", flush=True)
            Y = p.gemm(c.X[:M], path=B.PATH_PREFILL, variant=variant)
            p.check(c.X[:M], Y, None, f"variant={variant} N={N} K={K} f={f} M={M}")
        p.P.close()


def test_random_shapes_and_schedules(dev):
    """Seeded sweep: random (N, K, M, tile, f) within the ABI's limits, every path and kernel variant, with and
    without a workspace and a forced K split; every result against the oracle."""
    rng = np.random.default_rng(2024)
    ws = torch.empty(16 << 20, device=dev, dtype=torch.float32)
    for case in range(24):
        t = int(rng.choice([64, 128]))
        N = t * int(rng.integers(1, 7))
        K = t * int(rng.integers(1, 9))
        M = int(rng.choice([1, 2, 15, 16, 17, 63, 64, 65, 130, 255, 256, 257, 400]))
        f = float(rng.choice([0.0, 0.3, 0.5, 1.0]))
        c = synth.make_case("rnd%d" % case, N, K, M, t, f, seed=100 + case)
        p = Prepared(c, dev)
        Yo = p.oracle_gemm(c.X)
        scheds = [dict(), dict(path=B.PATH_DECODE), dict(path=B.PATH_PREFILL), dict(path=B.PATH_PREFILL, variant=1 if t == 64 else 2),
                  dict(path=B.PATH_PREFILL, variant=4), dict(path=B.PATH_PREFILL, variant=5, workspace=ws),
                  dict(workspace=ws), dict(path=B.PATH_PREFILL, workspace=ws, split_k=int(rng.integers(2, 5))),
                  dict(path=B.PATH_DECODE, split_k=int(rng.integers(1, 9)))]
        for kw in scheds:
            print(f"random case {case}: N={N} K={K} M={M} tile={t} f={f} " + str({k: v for k, v in kw.items() if k != 'workspace'})
                  + (" +workspace" if "workspace" in kw else ""), flush=True)
            Y = p.gemm(c.X, **kw)
            p.check(c.X, Y, Yo, f"random case {case}")
        p.P.close()


def _bf16_order(bits):
    """bf16 bit patterns -> integers whose difference counts representable values between two numbers."""
    b = bits.astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7FFF), b)


def check_bf16(bits, Yo, xn, wn, K, what=""):
    """bf16 output against the oracle's exact product rounded once (round_bf16): every element within one unit in
    the last place of it - or, where the product nearly cancels and an ulp of the result is smaller than the
    accumulation error allowed to the fp32 output, within that bound plus one ulp."""
    want = oracle.round_bf16(Yo)
    assert not ((bits & 0x7FFF) > 0x7F80).any(), f"{what}: NaN in the output (unwritten?)"
    dist = np.abs(_bf16_order(bits) - _bf16_order(want))
    got = synth.bf16_bits_to_f64(bits)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(Yo), 2.0 ** -126))) - 7)
    bound = elem_bound(xn[:, None], wn[None, :], K) + ulp
    ok = (dist <= 1) | (np.abs(got - Yo) <= bound)
    print(f"  bf16 parity {what}: exact {float((dist == 0).mean()):.4f}, one ulp off {float((dist == 1).mean()):.4f}, "
          f"by the absolute bound {int(((dist > 1) & ok).sum())} of {dist.size}", flush=True)
    assert ok.all(), f"{what}: element {np.unravel_index(np.argmax(~ok), ok.shape)} is more than one ulp off"
    assert (dist == 0).mean() > 0.98, "double rounding can cost an ulp only rarely"


def test_bf16_output_is_the_rounded_product(dev):
    """patch_gemm_opts.y_bf16 on every kernel and schedule that writes Y: within one ulp of the oracle's product
    rounded once, and bit-equal to the fp32 output of the same schedule rounded to nearest even (the same
    accumulator goes through the same rounding)."""
    ws = torch.empty(16 << 20, device=dev, dtype=torch.float32)
    for name, N, K, t, f, M in [("b128", 384, 1024, 128, 0.5, 300), ("b64", 192, 320, 64, 0.4, 130)]:
        c = synth.make_case("bf16out_" + name, N, K, M, t, f, seed=61)
        p = Prepared(c, dev)
        scheds = [(1, dict()), (16, dict(path=B.PATH_DECODE)), (40, dict(path=B.PATH_DECODE)), (40, dict(path=B.PATH_DECODE, variant=4)),
                  (40, dict(path=B.PATH_DECODE, variant=4, workspace=ws, split_k=2)), (M, dict(path=B.PATH_PREFILL)),
                  (M - 33, dict(path=B.PATH_PREFILL, variant=1 if t == 64 else 2)), (M, dict(workspace=ws))]
        if t == 128:
            scheds += [(M, dict(path=B.PATH_PREFILL, workspace=ws, split_k=3)), (70, dict(path=B.PATH_DECODE))]
        for Mi, kw in scheds:
            what = f"{name} M={Mi} " + str({k: v for k, v in kw.items() if k != "workspace"}) + (" +workspace" if "workspace" in kw else "")
            print("bf16 out: " + what, flush=True)
            Xb = c.X[:Mi]
            bits = p.gemm_bf16(Xb, **kw)
            Y32 = p.gemm(Xb, **kw)
            assert np.array_equal(bits, synth.f32_to_bf16_bits(Y32)), what + ": not the fp32 output rounded to nearest even"
            check_bf16(bits, p.oracle_gemm(Xb), row_norms(Xb), p.wn, K, what)
        p.P.close()
    # a set of weights sharing X, decode and prefill launches
    cases = [synth.make_case(f"bf16many{i}", N, 1024, 300, 128, f, seed=62) for i, (N, f) in enumerate([(512, 0.5), (256, 1.0)])]
    preps = [Prepared(c, dev) for c in cases]
    Xd = to_dev_bf16(cases[0].X, dev)
    for M in (1, 300):
        Ys = [torch.full((M, c.N), float("nan"), device=dev, dtype=torch.bfloat16) for c in cases]
        B.patch_gemm_many(Xd, M, [p.P for p in preps], Ys, stream(), y_bf16=True)
        torch.cuda.synchronize()
        for p, Y in zip(preps, Ys):
            check_bf16(bits_of(Y), p.oracle_gemm(cases[0].X[:M]), row_norms(cases[0].X[:M]), p.wn, 1024, f"set M={M}")
    for p in preps:
        p.P.close()


def test_bf16_output_full_size_prefill_sampled(dev):
    """The headline gate projection (11008 x 4096, M = 4096, 60 % 2:4 tiles) with a bf16 Y: a seeded sample of rows
    against the oracle's rounded product, and bit-equal to the rounded fp32 output everywhere."""
    N, K, M = 11008, 4096, 4096
    c = synth.make_case("mlp_prefill", N, K, M, 128, 0.6, seed=7)
    p = Prepared(c, dev)
    bits = p.gemm_bf16(c.X)
    assert np.array_equal(bits, synth.f32_to_bf16_bits(p.gemm(c.X)))
    rows = np.sort(np.random.default_rng(3).choice(M, size=16, replace=False))
    Xr = np.ascontiguousarray(c.X[rows])
    check_bf16(bits[rows], p.oracle_gemm(Xr), row_norms(Xr), p.wn, K, "gate projection, 16 sampled rows")
    p.P.close()


def test_empty_batch_is_a_no_op(dev):
    """M = 0: PATCH_OK, nothing launched, Y untouched; a negative M is an argument error."""
    c = synth.make_case("empty", 256, 256, 4, 128, 0.5, seed=3)
    p = Prepared(c, dev)
    X = to_dev_bf16(c.X, dev)
    Y = torch.full((4, c.N), 7.0, device=dev, dtype=torch.float32)
    for path in (B.PATH_AUTO, B.PATH_DECODE, B.PATH_PREFILL):
        B.patch_gemm(X, 0, p.P, Y, stream(), path=path)
    B.patch_gemm_many(X, 0, [p.P, p.P], [Y, Y], stream())
    torch.cuda.synchronize()
    assert bool((Y == 7.0).all())
    with pytest.raises(B.PatchError):
        B.patch_gemm(X, -1, p.P, Y, stream())
    p.P.close()


@pytest.mark.parametrize("pattern", ["row_bands", "alternating_rows", "columns", "one_sparse_row"])
def test_prefill_structured_tile_maps(dev, pattern):
    """Tile maps with structure (whole tile rows of one type, bands, columns): the packer pairs tile rows by pattern
    and reorders the feature blocks; every tile row must still be multiplied exactly once.  Odd tile-row count."""
    N, K, M, t = 1664, 768, 300, 128       # 13 tile rows x 6 tile columns
    c = synth.make_case("structured", N, K, M, t, 0.5, seed=17)
    Tn, Tk = N // t, K // t
    tm = np.ones((Tn, Tk), np.uint8)
    if pattern == "row_bands":
        tm[: Tn // 2] = 0
    elif pattern == "alternating_rows":
        tm[::2] = 0
    elif pattern == "columns":
        tm[:, : Tk // 2] = 0
    else:
        tm[Tn - 1] = 0
    W_hat_o = oracle.apply_mask(c.W, tm, c.mask24, t)
    vals_o, meta_o = oracle.pack(W_hat_o, tm, t)
    W = to_dev_bf16(c.W, dev)
    W_hat = torch.empty_like(W)
    B.patch_apply_mask(W, torch.from_numpy(c.mask24).to(dev), tm, N, K, t, W_hat, stream())
    P = B.patch_pack(W_hat, N, K, tm, t, stream())
    X = to_dev_bf16(c.X, dev)
    Yo = oracle.gemm(c.X, vals_o, meta_o, N, K, tm, t)
    ws = torch.empty(4 * M * N, device=dev, dtype=torch.float32)
    for kw in (dict(path=B.PATH_PREFILL), dict(path=B.PATH_PREFILL, workspace=ws, split_k=3), dict(path=B.PATH_PREFILL, variant=2)):
        Y = torch.full((M, N), float("nan"), device=dev, dtype=torch.float32)
        ws.fill_(float("nan"))
        B.patch_gemm(X, M, P, Y, stream(), **kw)
        torch.cuda.synchronize()
        Yh = Y.cpu().numpy()
        assert np.isfinite(Yh).all(), "a tile row was not written"
        check_elements(Yh, Yo, row_norms(c.X), row_norms(W_hat_o), K, f"structured {pattern}")
    P.close()


def test_row_order_is_a_permutation_and_pairs_common_24_steps(dev):
    """The prefill launch order the packer derives from the tile map: every tile row exactly once, -1 only as the
    partner of the one unpaired row of an odd count; on a random map the chosen pairs share more 2:4 steps than
    adjacent rows do; on a banded map every pair is of one kind."""
    t = 128
    for N, K, f in [(1664, 1024, 0.6), (1536, 4096, 0.5), (128, 256, 0.5)]:
        c = synth.make_case("order", N, K, 1, t, f, seed=23)
        p = Prepared(c, dev)
        order = p.P.row_order()
        Tn = N // t
        assert order.shape == ((Tn + 1) // 2, 2)
        rows = order[order >= 0]
        assert sorted(rows.tolist()) == list(range(Tn))
        assert int((order < 0).sum()) == Tn % 2 and (order[:, 0] >= 0).all()
        sp = c.tile_map == 0
        both = lambda a, b: int((sp[a] & sp[b]).sum())
        chosen = sum(both(a, b) for a, b in order if b >= 0)
        adjacent = sum(both(2 * i, 2 * i + 1) for i in range(Tn // 2))
        print(f"row order N={N} K={K}: common 2:4 steps chosen {chosen} adjacent {adjacent}", flush=True)
        assert chosen >= adjacent
        p.P.close()
    tm = np.ones((12, 8), np.uint8)
    tm[[0, 3, 4, 7, 9, 10]] = 0                      # six tile rows all 2:4, six all dense, interleaved
    c = synth.make_case("order_bands", 12 * t, 8 * t, 1, t, 0.5, seed=24)
    W = to_dev_bf16(c.W, dev)
    W_hat = torch.empty_like(W)
    B.patch_apply_mask(W, torch.from_numpy(c.mask24).to(dev), tm, 12 * t, 8 * t, t, W_hat, stream())
    P = B.patch_pack(W_hat, 12 * t, 8 * t, tm, t, stream())
    for a, b in P.row_order():
        assert tm[a, 0] == tm[b, 0], "a 2:4 row was paired with a dense one although an equal partner existed"
    P.close()
    c64 = synth.make_case("order64", 256, 256, 1, 64, 0.5, seed=25)
    p64 = Prepared(c64, dev)
    assert p64.P.row_order().size == 0                # tile 64: no prefill row order
    p64.P.close()


def test_prefill_part_filled_last_round_is_split(dev):
    """270 output tiles on 256 compute units: with a workspace the last 14 tiles are cut into K slices of their own
    (partial tiles in workspace slots, summed by a third launch).  Sampled checks against the oracle, with and
    without the workspace; rows outside the tail tiles are bit-equal between the two."""
    N, K, M, t = 2560, 4096, 6912 - 40, 128       # 10 feature blocks x 27 row blocks (the last one ragged)
    c = synth.make_case("tail", N, K, M, t, 0.5, seed=31)
    p = Prepared(c, dev)
    need = B.patch_gemm_workspace_bytes(M, p.P, path=B.PATH_PREFILL)
    print(f"tail split workspace: {need} bytes", flush=True)
    assert need > 0 and need % (256 * 256 * 4) == 0
    ws = torch.empty(need // 4, device=dev, dtype=torch.float32)
    Y0 = p.gemm(c.X, path=B.PATH_PREFILL)
    Y1 = p.gemm(c.X, path=B.PATH_PREFILL, workspace=ws)
    rng = np.random.default_rng(5)
    _sampled_checks(p, c, c.X, Y0, rng, n_points=1024, n_rows=8)
    _sampled_checks(p, c, c.X, Y1, rng, n_points=1024, n_rows=8)
    same = (Y0 == Y1).all(axis=1)
    assert same.mean() > 0.5 and relF(Y1, Y0.astype(np.float64)) <= TIGHT
    assert np.array_equal(Y1, p.gemm(c.X, path=B.PATH_PREFILL, workspace=ws)), "not reproducible"
    small = ws[: (need // 4) // 2 + 3]           # room for fewer slices: still correct
    assert relF(p.gemm(c.X, path=B.PATH_PREFILL, workspace=small), Y0.astype(np.float64)) <= TIGHT
    p.P.close()


def test_prefill_set_with_split_last_round(dev):
    """Two weights sharing X in one prefill launch whose 270 tiles end in a part-filled round: with a workspace the
    last tiles (of both weights) are split in K; every output against the oracle on samples, and equal to the
    unsplit set launch within rounding."""
    K, M, t = 4096, 6912 - 40, 128
    cases = [synth.make_case(f"tailset{i}", N, K, M, t, f, seed=33) for i, (N, f) in enumerate([(1280, 0.5), (1280, 0.8)])]
    X = cases[0].X
    preps = [Prepared(c, dev) for c in cases]
    Xd = to_dev_bf16(X, dev)
    ws = torch.full((8 * 16 * 256 * 256,), float("nan"), device=dev, dtype=torch.float32)
    outs = {}
    for label, kw in (("plain", dict()), ("workspace", dict(workspace=ws))):
        Ys = [torch.full((M, c.N), float("nan"), device=dev, dtype=torch.float32) for c in cases]
        B.patch_gemm_many(Xd, M, [p.P for p in preps], Ys, stream(), path=B.PATH_PREFILL, **kw)
        torch.cuda.synchronize()
        outs[label] = [Y.cpu().numpy() for Y in Ys]
    rng = np.random.default_rng(6)
    for i, (p, c) in enumerate(zip(preps, cases)):
        _sampled_checks(p, c, X, outs["workspace"][i], rng, n_points=1024, n_rows=8)
        assert relF(outs["workspace"][i], outs["plain"][i].astype(np.float64)) <= TIGHT
    # the last tiles of the launch order belong to the second weight: its sums were formed in a different order
    assert any(not np.array_equal(a_, b_) for a_, b_ in zip(outs["workspace"], outs["plain"])), "the last round was not split"
    for p in preps:
        p.P.close()


def test_hip_graph_replay_matches_eager(dev):
    """The product calls allocate nothing, never synchronise and record no memset: a HIP graph captured over a decode
    launch, a batched-decode pass with K chunks (two launches), a split prefill launch (two launches) and a plain one
    replays bit-equal to the eager results, several times, with eager work between the replays."""
    c = synth.make_case("graph", 768, 1024, 300, 128, 0.5, seed=41)
    p = Prepared(c, dev)
    X = to_dev_bf16(c.X, dev)
    ws = torch.full((8 * 300 * 768,), float("nan"), device=dev, dtype=torch.float32)
    jobs = [(1, dict()), (40, dict(path=B.PATH_DECODE, workspace=ws)), (300, dict(path=B.PATH_PREFILL, workspace=ws)),
            (300, dict(path=B.PATH_PREFILL))]
    eager = []
    for M, kw in jobs:                         # also the warm-up every kernel needs before a capture
        Y = torch.full((M, c.N), float("nan"), device=dev, dtype=torch.float32)
        B.patch_gemm(X, M, p.P, Y, stream(), **kw)
        eager.append(Y)
    torch.cuda.synchronize()
    outs = [torch.full_like(Y, float("nan")) for Y in eager]
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for (M, kw), Y in zip(jobs, outs):
                B.patch_gemm(X, M, p.P, Y, side.cuda_stream, **kw)
    for rep in range(3):
        for Y in outs:
            Y.fill_(float("nan"))
        ws.fill_(float("nan"))
        scratch = p.gemm(c.X[:7])               # eager work (and a synchronisation) between the replays
        assert np.isfinite(scratch).all()
        graph.replay()
        torch.cuda.synchronize()
        for (M, kw), Y, E in zip(jobs, outs, eager):
            assert torch.equal(Y, E), f"replay {rep}: M={M} differs from the eager launch"
    p.check(c.X, outs[2].cpu().numpy(), None, "graph replay, split prefill")
    p.P.close()


def test_store_probe_stays_inside_its_matrix(dev):
    """patch_probe_store_tiles (the output stage's stores on their own, timed by bench.py's ceilings section) writes
    every element of its M x N matrix and nothing outside it, in both store patterns and both element sizes."""
    M, N = 512, 768
    for bf16 in (False, True):
        dt = torch.bfloat16 if bf16 else torch.float32
        guard = 4096
        for pattern in (0, 1):
            buf = torch.full((guard + M * N + guard,), -7.0, device=dev, dtype=dt)   # the probe writes values >= 0 only
            Y = buf[guard:guard + M * N]
            B.patch_probe_store_tiles(pattern, bf16, Y, M, N, stream())
            torch.cuda.synchronize()
            assert bool((buf[:guard] == -7.0).all()) and bool((buf[guard + M * N:] == -7.0).all()), "wrote outside Y"
            assert bool((Y >= 0).all()), f"pattern {pattern}, bf16 {bf16}: elements left unwritten"


def test_lds_read_probe_runs(dev):
    """patch_probe_lds_read (bench.py's ceilings section): every lane sums the first float of its eight 16-byte pieces per
    pass over a buffer filled with buf[i] = i, so its result is known exactly."""
    wgs, iters = 8, 3
    out = torch.full((wgs * 256,), -1.0, device=dev, dtype=torch.float32)
    B.patch_probe_lds_read(wgs, iters, out, stream())
    torch.cuda.synchronize()
    lane = torch.arange(256, device=dev) % 64
    wave = torch.arange(256, device=dev) // 64
    first = (lane * 16 + wave * 8192) // 4                       # float index of the lane's first piece
    per_pass = sum((first + o // 4).float() for o in range(0, 8192, 1024))
    expect = (per_pass * iters).repeat(wgs)
    assert torch.equal(out, expect)
