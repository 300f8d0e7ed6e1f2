"""Pins for the reference's randomized quantizer (appendix "Additional details on gradient
quantization", Eqs. (rand_q), (xi)) and its Philox stream."""
import os

import numpy as np

import oracle
import synth_inputs as syn

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_philox_known_answers():
    for line in open(os.path.join(GOLD, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(t, 16) for t in line.split()]
        assert list(oracle.philox4x32_10(w[0:4], w[4:6])) == w[6:10]


def test_uniform_stream_statistics_and_indexing():
    u = oracle.uniform(0, 1 << 18, 77, 0)
    assert u.min() >= 0 and u.max() < 1
    assert np.array_equal(u * 2 ** 24, np.floor(u * 2 ** 24))      # 24-bit grid
    n = u.size
    assert abs(u.mean() - 0.5) < 4 / np.sqrt(12 * n)
    assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 4 / np.sqrt(n)
    hist = np.histogram(u, 64, (0, 1))[0]
    chi2 = ((hist - n / 64) ** 2 / (n / 64)).sum()
    assert chi2 < 130                                              # 63 dof, p ~ 1e-6
    # counter-by-index: any window of the stream can be generated on its own
    assert np.array_equal(oracle.uniform(1003, 50, 77, 0), u[1003:1053])
    assert not np.array_equal(oracle.uniform(0, 64, 77, 1), u[:64])   # streams differ
    assert not np.array_equal(oracle.uniform(0, 64, 78, 0), u[:64])   # seeds differ


def _one_tensor(g):
    return np.array([0, g.size], np.int64)


def test_values_on_grid_error_bound_and_extremes():
    rng = np.random.default_rng(0)
    for bits in (8, 4, 2):
        S = oracle.levels(bits)
        g = rng.standard_normal(5001).astype(np.float32)
        off = _one_tensor(g)
        codes, scales = oracle.quantize(g, off, S, seed=5)
        assert scales[0] == np.abs(g).max()
        assert codes.min() >= -S and codes.max() <= S
        gq = oracle.dequantize(codes, scales, off, S)
        step = scales[0] / S
        assert np.abs(gq - g).max() < step * (1 + 1e-6)             # |Q(g_i) - g_i| < scale/S
        i = np.abs(g).argmax()
        assert abs(codes[i]) == S and gq[i] == g[i]                   # absmax element is exact
        assert np.all(np.sign(codes[codes != 0]) == np.sign(g[codes != 0]))
        lo = np.floor(np.abs(g.astype(np.float64)) * S / float(scales[0]))
        assert np.all((np.abs(codes) == lo) | (np.abs(codes) == lo + 1) | (np.abs(codes) == np.minimum(lo, S)))


def test_unbiased_with_two_point_variance():
    # E[Q(g_i)] = g_i; Var = (scale/S)^2 p(1-p) with p the fractional part of |g_i| S/scale
    rng = np.random.default_rng(1)
    g = rng.standard_normal(400).astype(np.float32)
    off = _one_tensor(g)
    for bits in (8, 4):
        S = oracle.levels(bits)
        n_draws = 4000
        acc = np.zeros(g.size); acc2 = np.zeros(g.size)
        for s in range(n_draws):
            c, sc = oracle.quantize(g, off, S, seed=1000 + s)
            v = oracle.dequantize(c, sc, off, S).astype(np.float64)
            acc += v; acc2 += v * v
        mean = acc / n_draws
        var = acc2 / n_draws - mean ** 2
        step = float(np.abs(g).max()) / S
        r = np.abs(g.astype(np.float64)) / step
        p = r - np.floor(r)
        want_var = step ** 2 * p * (1 - p)
        assert np.abs(mean - g).max() < 5 * step * 0.5 / np.sqrt(n_draws)
        assert np.abs(var - want_var).max() < 0.05 * step ** 2
        # aggregate: mean over draws of ||Q(g)-g||^2 equals the sum of the closed-form variances
        assert abs(var.sum() - want_var.sum()) < 0.03 * want_var.sum()


def test_l2_scale_variant_obeys_qsgd_variance_bound():
    # paper-literal scale ||g||_2 with s levels: E||Q(g)-g||^2 <= min(d/s^2, sqrt(d)/s) ||g||^2
    rng = np.random.default_rng(2)
    d, s = 256, 16
    g = rng.standard_normal(d).astype(np.float32)
    off = _one_tensor(g)
    err = 0.0
    for seed in range(300):
        c, sc = oracle.quantize(g, off, s, seed, use_l2=True)
        assert abs(sc[0] - np.linalg.norm(g)) < 1e-5 * sc[0]
        err += ((oracle.dequantize(c, sc, off, s) - g) ** 2).sum()
    assert err / 300 <= min(d / s ** 2, np.sqrt(d) / s) * (g ** 2).sum()


def test_degenerate_tensors_and_per_tensor_scales():
    off = syn.ragged_offsets(3, 9, 700)
    g = syn.stress_gradient(3, off)
    S = oracle.levels(8)
    codes, scales = oracle.quantize(g, off, S, seed=11)
    for t in range(len(off) - 1):
        seg = g[off[t]:off[t + 1]]
        assert scales[t] == (np.abs(seg).max() if seg.size else 0)
    assert scales[1] == 0 and not codes[off[1]:off[2]].any()          # all-zero tensor
    seg = codes[off[2]:off[3]]                                        # one huge outlier
    assert np.abs(seg).max() == S and (np.abs(seg) <= 1).sum() == seg.size - 1
    # per-tensor streams use the global flat index: quantizing a tensor alone at its own
    # offset is not the same call, but the whole-vector call is reproducible
    c2, s2 = oracle.quantize(g, off, S, seed=11)
    assert np.array_equal(c2, codes) and np.array_equal(s2, scales)


def test_wire_format_sizes_and_roundtrip():
    # b bits per element including the sign (Table 4: bytes transmitted scale as b/32)
    rng = np.random.default_rng(3)
    for bits, d in ((8, 1001), (4, 1001), (4, 1000)):
        S = oracle.levels(bits)
        codes = rng.integers(-S, S + 1, size=d).astype(np.int32)
        q = oracle.pack(codes, bits)
        assert q.size == (d * bits + 7) // 8
        assert np.array_equal(oracle.unpack(q, d, bits), codes)
    q = oracle.pack(np.array([-7, 3, 1], np.int32), 4)
    assert list(q) == [0x39, 0x01]                                     # element 2j in the low nibble
    assert list(oracle.pack(np.array([-127, 5], np.int32), 8)) == [0x81, 0x05]
