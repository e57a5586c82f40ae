"""The seeded input recipes (no method arithmetic): tile maps with exact counts and the per-matrix allocation
stand-in used by the 13B stack benchmark."""
import numpy as np

from paper_2509_23410_amd import synth


def test_tile_map_has_the_exact_number_of_24_tiles():
    for T, f in ((64, 0.5), (49, 0.5), (2752, 0.6), (1024, 0.25), (10, 0.0), (10, 1.0)):
        tm = synth.tile_map(3, T, 1, f, "count")
        assert tm.shape == (T, 1) and int((tm == 0).sum()) == int(np.floor(f * T + 0.5))
    a, b = synth.tile_map(1, 8, 8, 0.5, "x"), synth.tile_map(2, 8, 8, 0.5, "x")
    assert not np.array_equal(a, b) and np.array_equal(a, synth.tile_map(1, 8, 8, 0.5, "x"))


def test_matrix_fractions_follow_the_reported_ordering():
    """Section 5, "Sparsity allocation": key / value never pruned, output moderate, query the most of the attention
    matrices, the MLP matrices the most; middle blocks more than the first, the deepest blocks least; global target met."""
    H, F = 5120, 13824
    params = [H * H] * 4 + [F * H] * 3
    for target in (0.3, 0.5, 0.7):
        fr = synth.matrix_fractions(40, params, target)
        assert fr.shape == (40, 7) and fr.min() >= 0.0 and fr.max() <= 1.0
        w = np.array(params, float)
        assert abs((fr * w).sum() / (w.sum() * 40) - target) < 1e-9
        q, k, v, o, gate, up, down = fr.T
        assert (k == 0).all() and (v == 0).all()
        assert (o <= q).all() and (q <= gate).all() and np.array_equal(gate, up) and np.array_equal(gate, down)
        assert (o[5:35] < q[5:35]).all()
        per_layer = fr @ w / w.sum()
        assert per_layer[39] < per_layer[0] < per_layer[15] and per_layer.argmax() in range(8, 24)
