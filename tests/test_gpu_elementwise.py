"""GPU parity (through the C ABI) of the HBM-streaming kernels against the CPU reference:
Philox stream, quantizer codes / scales / decoded values bit for bit, PGD init and update bit
for bit."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as syn

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dat():
    import paper_2206_06257_amd as dat
    return dat


def _cuda(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def test_philox_stream_word_for_word(dat):
    for start, n, seed, stream in [(0, 4099, 77, 0), (12345678901, 1000, (5 << 32) + 3, 1), (3, 17, 0, 0)]:
        got = dat.philox_uniform(start, n, seed, stream).cpu().numpy()
        assert np.array_equal(got, oracle.uniform(start, n, seed, stream))


@pytest.mark.parametrize("bits", [8, 4, 2, 16])
def test_quantizer_bit_exact_ragged_stress(dat, bits):
    off = syn.ragged_offsets(20 + bits, 37, 5000)
    g = syn.stress_gradient(20 + bits, off)
    d = g.size
    S = oracle.levels(bits)
    seed = syn.seed_for(3, "quantizer")
    codes, scales = oracle.quantize(g, off, S, seed)
    q, sc = dat.quantize(_cuda(g), _cuda(off), bits, seed)
    torch.cuda.synchronize()
    assert q.numel() == dat.quantized_bytes(d, bits) == (d * bits + 7) // 8
    assert np.array_equal(sc.cpu().numpy(), scales)
    assert np.array_equal(q.cpu().numpy(), oracle.pack(codes, bits))
    out = dat.dequantize(q, sc, _cuda(off), d, bits).cpu().numpy()
    assert np.array_equal(out, oracle.dequantize(codes, scales, off, S))


@pytest.mark.parametrize("d", [1, 3, 4, 5, 63, 64, 65, 1023, 8193])
def test_quantizer_tails(dat, d):
    rng = np.random.default_rng(d)
    g = rng.standard_normal(d).astype(np.float32)
    off = np.array([0, d], np.int64)
    for bits in (8, 4):
        S = oracle.levels(bits)
        codes, scales = oracle.quantize(g, off, S, 9)
        # guard bytes after the packed buffer must stay untouched
        nbytes = dat.quantized_bytes(d, bits)
        q = torch.full((nbytes + 8,), 0xAB, dtype=torch.uint8, device="cuda")
        dat.quantize(_cuda(g), _cuda(off), bits, 9, q=q)
        qh = q.cpu().numpy()
        assert np.array_equal(qh[:nbytes], oracle.pack(codes, bits))
        assert (qh[nbytes:] == 0xAB).all()


def test_quantizer_large_single_and_many_tensors(dat):
    # sizes that span many workgroups and a ragged tail; per-tensor and whole-vector scaling
    rng = np.random.default_rng(0)
    d = 3 * 8192 * 7 + 13
    g = (rng.standard_normal(d) * 10.0 ** rng.uniform(-4, 0, d)).astype(np.float32)
    lens = rng.integers(1, 3000, size=200)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    off = off[off < d]
    off = np.concatenate([off, [d]]).astype(np.int64)
    for offsets in (off, np.array([0, d], np.int64)):
        for bits in (8, 4):
            S = oracle.levels(bits)
            codes, scales = oracle.quantize(g, offsets, S, 1234)
            q, sc = dat.quantize(_cuda(g), _cuda(offsets), bits, 1234)
            assert np.array_equal(sc.cpu().numpy(), scales)
            assert np.array_equal(q.cpu().numpy(), oracle.pack(codes, bits))


def test_quantizer_nonfinite_scale_is_reported_not_encoded(dat):
    g = np.ones(300, np.float32)
    g[150] = np.inf
    g[250] = np.nan
    off = np.array([0, 100, 200, 300], np.int64)
    q, sc = dat.quantize(_cuda(g), _cuda(off), 8, 1)
    sc = sc.cpu().numpy(); q = q.cpu().numpy().view(np.int8)
    assert sc[0] == 1.0 and np.isinf(sc[1]) and np.isnan(sc[2])
    assert (q[:100] == 127).all() and not q[100:].any()


def test_unbiasedness_on_device(dat):
    # mean over seeds of decoded values -> g (Eq. E[Q(g)] = g); aggregation of M workers is this mean
    rng = np.random.default_rng(5)
    g = rng.standard_normal(4096).astype(np.float32)
    off = _cuda(np.array([0, 1000, 4096], np.int64))
    gd = _cuda(g)
    acc = torch.zeros(4096, dtype=torch.float64, device="cuda")
    n = 400
    for s in range(n):
        q, sc = dat.quantize(gd, off, 4, 500 + s)
        acc += dat.dequantize(q, sc, off, 4096, 4).double()
    step = np.abs(g).max() / 7
    assert np.abs(acc.cpu().numpy() / n - g).max() < 5 * step * 0.5 / np.sqrt(n)


@pytest.mark.parametrize("shape", [(2, 5, 7, 3), (3, 32, 32, 3), (1, 1, 1, 3), (2, 224, 224, 3)])
def test_pgd_init_and_update_bit_exact(dat, shape):
    eps, alpha = 8 / 255, 2 / 255
    x = syn.images(sum(shape), *shape[:3])
    x.reshape(-1)[::17] = 0.0
    x.reshape(-1)[5::19] = 1.0
    xd = _cuda(x)
    for mode, seed in ((oracle.INIT_ZERO, 0), (oracle.INIT_UNIFORM, syn.seed_for(2, "attack_init"))):
        want = oracle.init_delta(x, eps, mode, seed)
        got = dat.pgd_init(xd, eps, mode, seed).cpu().numpy()
        assert np.array_equal(got, want)
    given = ((syn.images(99, *shape[:3]) - 0.5) * 0.2).astype(np.float32)
    got = dat.pgd_init(xd, eps, oracle.INIT_GIVEN, 0, delta0=_cuda(given)).cpu().numpy()
    assert np.array_equal(got, oracle.init_delta(x, eps, oracle.INIT_GIVEN, 0, given))
    rng = np.random.default_rng(1)
    delta = oracle.init_delta(x, eps, oracle.INIT_UNIFORM, 7)
    for _ in range(3):
        G = rng.standard_normal(shape).astype(np.float32)
        G.reshape(-1)[::11] = 0.0
        G.reshape(-1)[3::13] = -0.0
        want = oracle.pgd_update(x, G, delta, eps, alpha)
        got = dat.pgd_update(xd, _cuda(G), _cuda(delta), eps, alpha).cpu().numpy()
        assert np.array_equal(got, want)
        assert np.abs(got).max() <= np.float32(eps) and (x + got).min() >= 0 and (x + got).max() <= 1
        delta = want
    # the batch handed to the outer step: clip(x + delta, 0, 1), also for perturbations that leave the box
    for d in (delta, (4.0 * delta).astype(np.float32)):
        xa = dat.make_xadv(xd, _cuda(d)).cpu().numpy()
        assert np.array_equal(xa, oracle.make_xadv(x, d)) and xa.min() >= 0 and xa.max() <= 1
    with pytest.raises(dat.DatError):
        dat.make_xadv(torch.zeros(4, device="cuda"), torch.zeros(4, device="cuda"))      # not whole pixels
