"""Pins for the CPU oracle: each test ties it to something other than itself.

Closed forms and printed numbers of the paper, invariants that must hold for
any correct implementation, special cases that reduce to scipy / numpy
routines, and brute force on tiny inputs.  No GPU.
"""
import os
import struct

import numpy as np
import pytest
import scipy.special
import scipy.stats

from oracle import pcc_oracle as po
from paper_2212_01185_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

# neighbour offsets as the workload text states them: rows r-2 and r-1 at
# columns c-2..c+1, row r at columns c-2 and c-1 (raster order)
OFFSETS = [(-2, -2), (-2, -1), (-2, 0), (-2, 1), (-1, -2), (-1, -1), (-1, 0), (-1, 1), (0, -2), (0, -1)]


def bf16(x):
    return synth.round_to_bf16(np.asarray(x, dtype=np.float32)).astype(np.float64)


# ----------------------------------------------------------------- closed forms

def test_config_network_size(blob):
    # 30*160+160 + 160*160+160 + 160*128+128 + 128*60+60
    assert synth.param_count(synth.DEFAULT_DIMS) == 59068
    assert sum(i * o for i, o in zip(synth.DEFAULT_DIMS[:-1], synth.DEFAULT_DIMS[1:])) == 58560
    assert len(blob) == 64 + 4 * 59068


def test_paper_parameter_counts():
    """The paper's seven printed counts follow from a 12-pixel causal mask
    (36 inputs), C-wide hidden layers and 12 outputs per mixture component,
    plus one stray scalar: printed = fc_count([36, C*(L-1).., 12K]) + 1."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "paper_param_counts.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 7
    for k, c, nl, printed in (map(int, r) for r in rows):
        dims = [36] + [c] * (nl - 1) + [12 * k]
        assert synth.param_count(dims) + 1 == printed
        assert tuple(dims) == synth.ablation_dims(k, c, nl)
    assert synth.ablation_dims(3, 128, 5) == synth.PAPER_DIMS
    assert 58917 + (75 - 36) * 128 == 63909      # Table I's "63.9 K"


def test_wavefront_pass_count_formula():
    # Eq. (6): T = D + (D-1)(h+1); 5x5 kernel has h = 2 -> 4D - 3
    for d in (64, 128, 256, 512):
        assert po.wavefront_steps(d, d, 3) == 4 * d - 3
    # right reach of one column (this build's neighbourhood) -> delay 2
    assert po.wavefront_steps(512, 768, 2) == 1790
    assert po.wavefront_steps(64, 64, 2) == 190
    assert po.wavefront_steps(1365, 2048, 2) == 4776
    assert po.wavefront_steps(2160, 4096, 2) == 8414


@pytest.mark.parametrize("h,w", [(1, 1), (1, 7), (7, 1), (2, 2), (5, 3), (6, 9)])
def test_schedule_is_causal(h, w):
    """Every in-image neighbour of (r, c) has a strictly smaller step 2r + c,
    the last step is W + 2(H-1) - 1, and raster order is causal too."""
    steps = set()
    for r in range(h):
        for c in range(w):
            t = 2 * r + c
            steps.add(t)
            for dr, dc in OFFSETS:
                rr, cc = r + dr, c + dc
                if 0 <= rr < h and 0 <= cc < w:
                    assert 2 * rr + cc < t
                    assert rr * w + cc < r * w + c
    # last pass index + 1 is the pass count (for W = 1 the odd passes are empty)
    assert max(steps) + 1 == po.wavefront_steps(h, w, 2)
    if w >= 2:
        assert steps == set(range(po.wavefront_steps(h, w, 2)))


# ----------------------------------------------------------------- network

def test_gather_matches_zero_padded_indexing(orc):
    rng = np.random.default_rng(1)
    img = rng.integers(0, 256, size=(5, 6, 3), dtype=np.uint8)
    pad = np.zeros((5 + 2, 6 + 4, 3), dtype=np.float64)   # 2 rows above, 2 columns each side
    pad[2:, 2:-2] = img / 256.0
    for r in range(5):
        for c in range(6):
            want = np.concatenate([pad[r + 2 + dr, c + 2 + dc] for dr, dc in OFFSETS])
            np.testing.assert_array_equal(orc.gather(img, r, c), want)


def _layers(blob):
    arr = np.frombuffer(blob[64:], dtype="<f4")
    out, pos = [], 0
    dims = synth.DEFAULT_DIMS
    for i, o in zip(dims[:-1], dims[1:]):
        w = arr[pos:pos + i * o].reshape(o, i).astype(np.float64)
        pos += i * o
        b = arr[pos:pos + o].astype(np.float64)
        pos += o
        out.append((w, b))
    assert pos == arr.size
    return out


def test_mlp_matches_float64_matmul(orc, blob):
    rng = np.random.default_rng(2)
    layers = _layers(blob)
    for _ in range(20):
        u = rng.integers(0, 256, 30) / 256.0
        a = u
        for i, (w, b) in enumerate(layers):
            a = w @ a + b
            if i < 3:
                a = np.maximum(a, 0.0)
        got = orc.mlp(u, po.MODE_EXACT)
        np.testing.assert_allclose(got, a, rtol=0, atol=1e-12)


def test_mlp_split_activation_mode(orc, blob):
    """Hidden activations rounded to hi + lo, hi = bf16(a), lo = bf16(a - hi)
    (numpy bit-trick rounding as the independent statement of the rounding)."""
    rng = np.random.default_rng(3)
    layers = _layers(blob)
    for _ in range(20):
        u = rng.integers(0, 256, 30) / 256.0
        a = u
        for i, (w, b) in enumerate(layers):
            a = w @ a + b
            if i < 3:
                a = np.maximum(a, 0.0)
                hi = bf16(a)
                a = hi + bf16(a - hi)
        got = orc.mlp(u, po.MODE_SPLIT)
        # the float32 pre-rounding of the numpy path can move a lo part by one unit (2^-17 relative)
        assert np.abs(got - a).max() < 1e-5
        # about 16 significant bits: close to the exact network, but not equal to it
        d = np.abs(got - orc.mlp(u, po.MODE_EXACT)).max()
        assert 1e-9 < d < 2e-4


def test_bf16_weights_are_exact(blob):
    for w, _ in _layers(blob):
        np.testing.assert_array_equal(bf16(w), w)


# ----------------------------------------------------------------- mixture, Eq. (1)-(4)

def _random_head(rng, scale=1.0):
    return rng.normal(0, scale, 60)


def test_mixture_parameterisation(orc):
    rng = np.random.default_rng(4)
    for _ in range(10):
        o = _random_head(rng, 3.0)
        for ch in range(3):
            pi, mu, sg = orc.mixture(o, ch, r=77, g=201)
            np.testing.assert_allclose(pi, scipy.special.softmax(o[15 * ch:15 * ch + 5]), atol=1e-15)
            np.testing.assert_allclose(sg, np.exp(np.clip(o[15 * ch + 10:15 * ch + 15], -8, 4)), rtol=1e-15)
            base = o[15 * ch + 5:15 * ch + 10]
            if ch == 0:
                want = base
            elif ch == 1:
                want = base + o[45:50] * 77 / 256
            else:
                want = base + o[50:55] * 77 / 256 + o[55:60] * 201 / 256
            np.testing.assert_allclose(mu, want, atol=1e-15)


def test_coupling_is_mean_only_and_ordered(orc):
    """Eq. (2)-(4): R depends on neither r nor g; G on r only; B on both; and
    only the means move (a shift of mu by alpha*r/256 reproduces the table)."""
    rng = np.random.default_rng(5)
    o = _random_head(rng)
    np.testing.assert_array_equal(orc.cdf_table(o, 0, 0, 0), orc.cdf_table(o, 0, 200, 100))
    np.testing.assert_array_equal(orc.cdf_table(o, 1, 50, 0), orc.cdf_table(o, 1, 50, 255))
    assert (orc.cdf_table(o, 1, 50, 0) != orc.cdf_table(o, 1, 51, 0)).any()
    assert (orc.cdf_table(o, 2, 50, 10) != orc.cdf_table(o, 2, 50, 11)).any()
    assert (orc.cdf_table(o, 2, 50, 10) != orc.cdf_table(o, 2, 51, 10)).any()
    # zero coupling coefficients: conditionally independent channels
    o0 = o.copy()
    o0[45:60] = 0
    np.testing.assert_array_equal(orc.cdf_table(o0, 1, 0, 0), orc.cdf_table(o0, 1, 255, 0))
    np.testing.assert_array_equal(orc.cdf_table(o0, 2, 0, 0), orc.cdf_table(o0, 2, 255, 255))
    # mean-only: folding alpha*r/256 into the means by hand gives the same table
    o1 = o.copy()
    o1[20:25] += o[45:50] * 50 / 256
    o1[45:50] = 0
    a, b = orc.cdf_table(o, 1, 50, 0).astype(int), orc.cdf_table(o1, 1, 50, 0).astype(int)
    assert np.abs(a - b).max() <= 1          # one rounding of mu apart


def test_tables_sum_and_min_frequency(orc):
    rng = np.random.default_rng(6)
    heads = [_random_head(rng, s) for s in (0.1, 1.0, 3.0, 10.0) for _ in range(10)]
    # extremes: tiny sigma on a bin centre / on a bin edge / far outside; huge sigma
    for mu in (0.0, 0.5, 100.2 / 256, 100.5 / 256, 255 / 256, -3.0, 4.0):
        for ls in (-20.0, -8.0, 0.0, 4.0, 20.0):
            o = np.zeros(60)
            o[5:10] = mu
            o[10:15] = ls
            heads.append(o)
    for o in heads:
        for ch in range(3):
            cq = orc.cdf_table(o, ch, 13, 240).astype(np.int64)
            assert cq[0] == 0 and cq[256] == 65536
            freq = np.diff(cq)
            assert freq.min() >= 1 and freq.sum() == 65536
            p = orc.pmf(o, ch, 13, 240)
            assert abs(p.sum() - 1.0) < 1e-12 and p.min() >= 0
            # quantisation: freq(x) = 1 + floor-difference of 65280*F, within one count of 1 + 65280 p(x)
            assert np.abs(freq - 1 - 65280 * p).max() < 1 + 1e-6


def test_single_component_reduces_to_scipy_normal(orc):
    """One component carrying all the weight: Cq(e) = e + floor(65280 Phi(z)),
    and the pmf is Eq. (1) in grey-level units with mu = 256 mu_hat, s = 256 sigma_hat."""
    rng = np.random.default_rng(7)
    for _ in range(20):
        mu_hat, ls = rng.uniform(-0.2, 1.2), rng.uniform(-6, 1)
        o = np.zeros(60)
        o[0:5] = [60.0, -60, -60, -60, -60]
        o[5] = mu_hat
        o[10] = ls
        o[6:10] = rng.uniform(0, 1, 4)          # ignored components
        e = np.arange(1, 256)
        z = ((e - 0.5) / 256 - mu_hat) / np.exp(ls)
        want = e + np.floor(65280 * scipy.special.ndtr(z)).astype(np.int64)
        got = orc.cdf_table(o, 0).astype(np.int64)
        assert np.abs(got[1:256] - want).max() <= 1
        assert (got[1:256] != want).mean() < 0.01
        x = np.arange(256)
        mu, s = 256 * mu_hat, 256 * np.exp(ls)
        p = scipy.stats.norm.cdf((x + 0.5 - mu) / s) - scipy.stats.norm.cdf((x - 0.5 - mu) / s)
        got_p = orc.pmf(o, 0)
        np.testing.assert_allclose(got_p[1:255], p[1:255], atol=1e-13)
        # open tails: the end bins take everything beyond the range
        assert abs(got_p[0] - scipy.stats.norm.cdf((0.5 - mu) / s)) < 1e-13
        assert abs(got_p[255] - scipy.stats.norm.sf((254.5 - mu) / s)) < 1e-13


def test_two_component_mixture_against_scipy(orc):
    o = np.zeros(60)
    o[15:20] = [np.log(0.25), np.log(0.75), -80, -80, -80]      # channel G
    o[20:22] = [0.25, 0.625]
    o[25:27] = [np.log(0.05), np.log(0.02)]
    o[45:47] = [0.5, -0.25]                                     # alpha
    r = 64
    mu = np.array([0.25 + 0.5 * r / 256, 0.625 - 0.25 * r / 256]) * 256
    s = np.array([0.05, 0.02]) * 256
    x = np.arange(1, 255)
    p = sum(w * (scipy.stats.norm.cdf((x + 0.5 - m) / sd) - scipy.stats.norm.cdf((x - 0.5 - m) / sd))
            for w, m, sd in zip((0.25, 0.75), mu, s))
    np.testing.assert_allclose(orc.pmf(o, 1, r=r)[1:255], p, atol=1e-13)


def test_degenerate_sigmas(orc):
    o = np.zeros(60)
    o[0:5] = [60.0, -60, -60, -60, -60]
    o[5] = 100.2 / 256
    o[10] = -30.0                # clamped to exp(-8): 0.086 grey levels
    f = np.diff(orc.cdf_table(o, 0).astype(np.int64))
    assert f.argmax() == 100 and f[100] > 65000
    o[10] = 30.0                 # clamped to exp(4): flat inside, half the mass in each end bin
    f = np.diff(orc.cdf_table(o, 0).astype(np.int64))
    assert f[0] > 30000 and f[255] > 30000 and f[1:255].max() <= 3


# ----------------------------------------------------------------- logistic mixture, Eq. (8)

def test_logistic_single_component_against_scipy(orc_logistic):
    """Eq. (8): F(x; mu, s) = 1 / (1 + exp(-(x - mu)/s)), in grey-level units mu = 256 mu_hat, s = 256 sigma_hat."""
    rng = np.random.default_rng(17)
    for _ in range(20):
        mu_hat, ls = rng.uniform(-0.2, 1.2), rng.uniform(-6, 0)
        o = np.zeros(60)
        o[30:35] = [60.0, -60, -60, -60, -60]       # channel B, first component only
        o[35] = mu_hat
        o[40] = ls
        mu, s = 256 * mu_hat, 256 * np.exp(ls)
        x = np.arange(256)
        p = scipy.stats.logistic.cdf(x + 0.5, loc=mu, scale=s) - scipy.stats.logistic.cdf(x - 0.5, loc=mu, scale=s)
        got = orc_logistic.pmf(o, 2)
        np.testing.assert_allclose(got[1:255], p[1:255], atol=1e-13)
        assert abs(got[0] - scipy.stats.logistic.cdf(0.5, loc=mu, scale=s)) < 1e-13
        assert abs(got[255] - scipy.stats.logistic.sf(254.5, loc=mu, scale=s)) < 1e-13
        e = np.arange(1, 256)
        want = e + np.floor(65280 * scipy.special.expit(((e - 0.5) / 256 - mu_hat) / np.exp(ls))).astype(np.int64)
        cq = orc_logistic.cdf_table(o, 2).astype(np.int64)
        assert np.abs(cq[1:256] - want).max() <= 1 and (cq[1:256] != want).mean() < 0.01
        f = np.diff(cq)
        assert f.min() >= 1 and f.sum() == 65536


def test_logistic_differs_from_gaussian_and_roundtrips(orc, orc_logistic):
    rng = np.random.default_rng(18)
    o = rng.normal(0, 1, 60)
    assert (orc.cdf_table(o, 0) != orc_logistic.cdf_table(o, 0)).any()
    imgs = synth.make_image(6, synth.ImageSpec(13, 9, 3, 2.0, 5.0))[None]
    stream, bits = orc_logistic.encode(imgs)
    np.testing.assert_array_equal(orc_logistic.decode(stream, 1, 9, 13, order=po.ORDER_WAVEFRONT), imgs)
    np.testing.assert_array_equal(orc_logistic.decode(stream, 1, 9, 13, order=po.ORDER_RASTER), imgs)
    # a Gaussian-mixture model must refuse a logistic-mixture stream
    with pytest.raises(po.OracleError):
        orc.decode(stream, 1, 9, 13)


# ----------------------------------------------------------------- the paper's own network shape

OFFSETS12 = [(-2, -2), (-2, -1), (-2, 0), (-2, 1), (-2, 2), (-1, -2), (-1, -1), (-1, 0), (-1, 1), (-1, 2),
             (0, -2), (0, -1)]


def test_paper_network_blob(paper_blob, orc_paper):
    # the printed 58,917 of the reference setting (K=3, C=128, L=5) is this fully connected count plus one
    assert synth.param_count(synth.PAPER_DIMS) + 1 == 58917
    assert len(paper_blob) == 64 + 4 * 58916
    assert orc_paper.dims == list(synth.PAPER_DIMS) and orc_paper.K == 3


@pytest.mark.parametrize("h,w", [(1, 1), (1, 7), (7, 1), (3, 2), (5, 9)])
def test_paper_neighbourhood_schedules(h, w):
    """Wavefront with delay 3 (Eq. (6), h = 2) is causal for the 12-pixel neighbourhood; the diagonal
    order r + c (Eq. (7)) leaves exactly the three upper-right pixels undecoded (Sec. III-C)."""
    for r in range(h):
        for c in range(w):
            for dr, dc in OFFSETS12:
                if 0 <= r + dr < h and 0 <= c + dc < w:
                    assert 3 * (r + dr) + (c + dc) < 3 * r + c
    late = [(dr, dc) for dr, dc in OFFSETS12 if dr + dc >= 0]
    assert sorted(late) == [(-2, 2), (-1, 1), (-1, 2)]
    assert po.wavefront_steps(h, w, 3) == w + 3 * (h - 1)
    d = 512
    assert po.wavefront_steps(d, d, 3) == 4 * d - 3 and 2 * d - 1 == 1023


def test_paper_gather_and_leaky_mlp(orc_paper, paper_blob):
    rng = np.random.default_rng(21)
    img = rng.integers(0, 256, size=(5, 6, 3), dtype=np.uint8)
    pad = np.zeros((5 + 2, 6 + 4, 3), dtype=np.float64)
    pad[2:, 2:-2] = img / 256.0
    for r in range(5):
        for c in range(6):
            want = np.concatenate([pad[r + 2 + dr, c + 2 + dc] for dr, dc in OFFSETS12])
            np.testing.assert_array_equal(orc_paper.gather(img, r, c), want)
    arr = np.frombuffer(paper_blob[64:], dtype="<f4")
    layers, pos = [], 0
    for i, o in zip(synth.PAPER_DIMS[:-1], synth.PAPER_DIMS[1:]):
        w = arr[pos:pos + i * o].reshape(o, i).astype(np.float64); pos += i * o
        b = arr[pos:pos + o].astype(np.float64); pos += o
        layers.append((w, b))
    for _ in range(10):
        u = rng.integers(0, 256, 36) / 256.0
        a = u
        for i, (w, b) in enumerate(layers):
            a = w @ a + b
            if i < 4:
                a = np.where(a > 0, a, 0.01 * a)
        np.testing.assert_allclose(orc_paper.mlp(u), a, rtol=0, atol=1e-12)
        assert (orc_paper.mlp(u) != 0).all()


def test_paper_network_roundtrip(orc_paper):
    rng = np.random.default_rng(22)
    for imgs in (rng.integers(0, 256, (1, 1, 1, 3), dtype=np.uint8), rng.integers(0, 256, (2, 4, 7, 3), dtype=np.uint8),
                 np.zeros((1, 5, 5, 3), dtype=np.uint8), synth.make_image(7, synth.ImageSpec(17, 9, 3, 2.0, 6.0))[None]):
        n, h, w, _ = imgs.shape
        stream, bits = orc_paper.encode(imgs)
        np.testing.assert_array_equal(orc_paper.decode(stream, n, h, w, order=po.ORDER_RASTER), imgs)
        np.testing.assert_array_equal(orc_paper.decode(stream, n, h, w, order=po.ORDER_WAVEFRONT), imgs)
        for ch in range(3):
            o = orc_paper.params_at(imgs[0], h - 1, w - 1)
            f = np.diff(orc_paper.cdf_table(o, ch, 3, 200).astype(np.int64))
            assert f.min() >= 1 and f.sum() == 65536


# ----------------------------------------------------------------- hand-structured weights with a closed form

def test_plane_predictor_weights_have_closed_form_outputs(orc_predictor):
    """With the plane-predictor weights every mean is exactly (left + up - upleft)/256 of its channel (zero
    padding outside), every log-sigma log(6/256), every logit and coupling coefficient 0: pins the
    neighbour order of the gather, the chaining of the four layers and the head layout at once."""
    rng = np.random.default_rng(51)
    img = rng.integers(0, 256, size=(7, 9, 3), dtype=np.uint8)
    pad = np.zeros((8, 10, 3), dtype=np.int64)
    pad[1:, 1:] = img
    for r in range(7):
        for c in range(9):
            o = orc_predictor.params_at(img, r, c)
            pred = (pad[r + 1, c] + pad[r, c + 1] - pad[r, c]) / 256.0      # left + up - upleft
            for ch in range(3):
                np.testing.assert_array_equal(o[15 * ch:15 * ch + 5], 0.0)
                np.testing.assert_allclose(o[15 * ch + 5:15 * ch + 10], pred[ch], rtol=0, atol=1e-15)
                np.testing.assert_allclose(o[15 * ch + 10:15 * ch + 15], np.log(np.float32(6.0 / 256.0)), rtol=0, atol=1e-12)
            np.testing.assert_array_equal(o[45:], 0.0)
    # and the pmf is the single discretised Gaussian of Eq. (1) around the prediction
    from scipy.stats import norm
    o = orc_predictor.params_at(img, 3, 4)
    pmf = orc_predictor.pmf(o, 1, 0, 0)
    mu = 256.0 * o[15 + 5]
    sig = 256.0 * np.exp(o[15 + 10])
    edges = np.concatenate([[-np.inf], np.arange(1, 256) - 0.5, [np.inf]])
    np.testing.assert_allclose(pmf, np.diff(norm.cdf((edges - mu) / sig)), rtol=0, atol=1e-12)


def test_plane_predictor_weights_compress_smooth_images(orc_predictor, orc):
    imgs = synth.make_image(3, synth.ImageSpec(48, 32, 4, 6.0, 20.0))[None]
    stream, bits = orc_predictor.encode(imgs)
    np.testing.assert_array_equal(orc_predictor.decode(stream, 1, 32, 48, order=po.ORDER_WAVEFRONT), imgs)
    bpsp = bits.sum() / imgs.size
    _, bits_random = orc.encode(imgs)
    assert bpsp < 5.5 < bits_random.sum() / imgs.size      # noise of sigma 3 under a 4-tap predictor: about 4.7 bits


def _probe_expected(img, r, c, diagonal):
    """Means [3 channels][3 components] of the tap-probe weights at (r, c): the probed neighbours' values / 256."""
    h, w, _ = img.shape
    out = np.zeros((3, 3))
    for k, tap in enumerate(synth.PROBE_TAPS):
        dr, dc = OFFSETS12[tap]
        if diagonal and dr + dc >= 0:
            dr, dc = -1, 0
        rr, cc = r + dr, c + dc
        if 0 <= rr < h and 0 <= cc < w:
            out[:, k] = img[rr, cc] / 256.0
    return out


@pytest.mark.parametrize("delay", [3, 1])
def test_tap_probe_weights_have_closed_form_outputs(delay):
    orc_probe = po.Oracle(synth.make_tap_probe_blob(delay))
    rng = np.random.default_rng(52)
    img = rng.integers(1, 256, size=(6, 8, 3), dtype=np.uint8)
    for r in range(6):
        for c in range(8):
            o = orc_probe.params_at(img, r, c)
            want = _probe_expected(img, r, c, delay == 1)
            for ch in range(3):
                np.testing.assert_array_equal(o[9 * ch:9 * ch + 3], 0.0)
                np.testing.assert_array_equal(o[9 * ch + 3:9 * ch + 6], want[ch])
            np.testing.assert_array_equal(o[27:], 0.0)


# ----------------------------------------------------------------- diagonal decoding order (Sec. III-C, Eq. (7))

def test_diagonal_pass_count_is_eq7():
    for d in (1, 2, 64, 128, 256, 512):
        assert po.wavefront_steps(d, d, 1) == 2 * d - 1          # Eq. (7): T = 2D - 1
    assert po.wavefront_steps(512, 768, 1) == 768 + 512 - 1


@pytest.mark.parametrize("h,w", [(1, 1), (1, 7), (7, 1), (3, 2), (5, 9), (9, 5)])
def test_diagonal_sources_are_decoded_before_the_pass(orc_diagonal, orc_paper, h, w):
    """Every position the diagonal model reads lies on an earlier anti-diagonal (or outside the image);
    exactly the three neighbours the paper names are replaced, all by the pixel straight above; the
    wavefront model of the same shape replaces none."""
    for r in range(h):
        for c in range(w):
            replaced = []
            for j, (dr, dc) in enumerate(OFFSETS12):
                rr, cc = orc_diagonal.tap_source(r, c, j)
                if 0 <= rr < h and 0 <= cc < w:
                    assert rr + cc < r + c                       # decoded in an earlier pass
                    assert rr * w + cc < r * w + c               # and earlier in raster order, too
                if (rr, cc) != (r + dr, c + dc):
                    replaced.append((dr, dc))
                    assert (rr, cc) == (r - 1, c)
                assert orc_paper.tap_source(r, c, j) == (r + dr, c + dc)
            assert sorted(replaced) == [(-2, 2), (-1, 1), (-1, 2)]
    # the pixels of one pass are exactly one anti-diagonal
    steps = {r + c for r in range(h) for c in range(w)}
    assert steps == set(range(po.wavefront_steps(h, w, 1)))


def test_diagonal_gather_copies_on_the_padded_patch(orc_diagonal, orc_paper):
    rng = np.random.default_rng(41)
    img = rng.integers(1, 256, size=(6, 7, 3), dtype=np.uint8)      # no zeros: padding is recognisable
    pad = np.zeros((6 + 2, 7 + 4, 3), dtype=np.float64)
    pad[2:, 2:-2] = img / 256.0
    for r in range(6):
        for c in range(7):
            patch = {(dr, dc): pad[r + 2 + dr, c + 2 + dc].copy() for dr, dc in OFFSETS12}
            above = pad[r + 2 - 1, c + 2]
            for key in ((-2, 2), (-1, 1), (-1, 2)):
                patch[key] = above
            want = np.concatenate([patch[o] for o in OFFSETS12])
            np.testing.assert_array_equal(orc_diagonal.gather(img, r, c), want)
    # a constant image: the copies equal what they replace where all three replaced positions lie in the
    # image, and in the first row, where the pixel above is padding like they are
    flat = np.full((5, 9, 3), 77, dtype=np.uint8)
    for r in range(5):
        for c in range(9):
            same = np.array_equal(orc_diagonal.gather(flat, r, c), orc_paper.gather(flat, r, c))
            assert same == (r == 0 or (r >= 2 and c + 2 < 9))


def test_diagonal_roundtrip_raster_equals_diagonal_order(orc_diagonal, orc_paper):
    rng = np.random.default_rng(42)
    cases = [rng.integers(0, 256, (1, 1, 1, 3), dtype=np.uint8), rng.integers(0, 256, (1, 1, 9, 3), dtype=np.uint8),
             rng.integers(0, 256, (1, 9, 1, 3), dtype=np.uint8), rng.integers(0, 256, (2, 6, 7, 3), dtype=np.uint8),
             np.zeros((1, 5, 5, 3), dtype=np.uint8), synth.make_image(8, synth.ImageSpec(19, 11, 3, 2.0, 6.0))[None]]
    for imgs in cases:
        n, h, w, _ = imgs.shape
        stream, bits = orc_diagonal.encode(imgs)
        np.testing.assert_array_equal(orc_diagonal.decode(stream, n, h, w, order=po.ORDER_RASTER), imgs)
        np.testing.assert_array_equal(orc_diagonal.decode(stream, n, h, w, order=po.ORDER_WAVEFRONT), imgs)
    # the stream says which order it was made for: the wavefront model of the same shape refuses it
    imgs = cases[3]
    stream, _ = orc_diagonal.encode(imgs)
    with pytest.raises(Exception):
        orc_paper.decode(stream, 2, 6, 7)


# ----------------------------------------------------------------- rANS

def _random_tables(rng, nsym):
    tabs = np.zeros((nsym, 257), dtype=np.uint32)
    for i in range(nsym):
        kind = rng.integers(0, 4)
        if kind == 0:      # everything but 255 counts on one symbol
            f = np.ones(256, dtype=np.int64)
            f[rng.integers(0, 256)] += 65536 - 256
        elif kind == 1:    # flat
            f = np.full(256, 256, dtype=np.int64)
        else:
            w = rng.dirichlet(np.full(256, 0.05))
            f = 1 + np.floor(w * (65536 - 256)).astype(np.int64)
            f[rng.integers(0, 256)] += 65536 - f.sum()
        assert f.sum() == 65536 and f.min() >= 1
        tabs[i, 1:] = np.cumsum(f)
    return tabs


@pytest.mark.parametrize("nsym", [0, 1, 2, 3, 17, 300, 5000])
def test_rans_roundtrip_and_length(nsym):
    rng = np.random.default_rng(100 + nsym)
    tabs = _random_tables(rng, nsym)
    # draw symbols with a bias towards the rare ones (frequency 1) and the common ones
    sym = rng.integers(0, 256, nsym)
    common = tabs[:, 1:].astype(np.int64) - tabs[:, :-1].astype(np.int64)
    pick = rng.random(nsym) < 0.5
    sym = np.where(pick, common.argmax(axis=1), sym)
    idx = np.arange(nsym)
    start = tabs[idx, sym]
    freq = tabs[idx, sym + 1] - start
    payload = po.rans_encode(start, freq)
    assert len(payload) % 4 == 0 and len(payload) <= 16 + 4 * (nsym // 2 + 2)
    rc, got = po.rans_decode_tables(payload, tabs)
    assert rc == po.OK
    np.testing.assert_array_equal(got, sym.astype(np.uint8))
    ideal = float(-np.log2(freq / 65536.0).sum())
    bits = 8 * len(payload)
    # two states of 64 bits, each carrying between 0 and 32 bits of the message: 64 to 128 bits over the ideal length
    # (plus at most 2^-14 bit per symbol)
    assert ideal + 64 - 1e-6 <= bits <= ideal + 128 + nsym * 2.0 ** -14 + 1e-6
    if nsym:
        rc, _ = po.rans_decode_tables(payload[:-4] if len(payload) > 16 else payload[:12], tabs)
        assert rc == po.E_STREAM
        rc, _ = po.rans_decode_tables(payload + b"\0\0\0\0", tabs)
        assert rc == po.E_STREAM


def test_rans_states_alternate_by_symbol():
    """Symbol i of a row is coded on state i mod 2, the payload holds state 0 then state 1: hand-computed cases.
    A symbol with the whole range (start 0, frequency 2^16) leaves its state at 2^31; one with start 0 and frequency
    2^15 turns 2^31 into ((2^31 / 2^15) << 16) = 2^32; neither makes a word."""
    full, half = (0, 65536), (0, 32768)
    for syms, want in (([full, full, full], (1 << 31, 1 << 31)), ([half, full, full], (1 << 32, 1 << 31)),
                       ([full, half, full], (1 << 31, 1 << 32)), ([full, full, half], (1 << 32, 1 << 31)),
                       ([half, half], (1 << 32, 1 << 32)), ([half, full, half], (1 << 33, 1 << 31))):
        start = np.array([s for s, _ in syms], dtype=np.uint32)
        freq = np.array([f for _, f in syms], dtype=np.uint32)
        assert po.rans_encode(start, freq) == struct.pack("<QQ", *want), syms
    # the words are shared: a decoder written here from the format's description (two states, one word sequence)
    rng = np.random.default_rng(7)
    tabs = _random_tables(rng, 400)
    sym = rng.integers(0, 256, 400)
    idx = np.arange(400)
    start = tabs[idx, sym]
    freq = tabs[idx, sym + 1] - start
    payload = po.rans_encode(start, freq)
    x = list(struct.unpack("<QQ", payload[:16]))
    words = list(struct.unpack("<%dI" % ((len(payload) - 16) // 4), payload[16:]))
    got = []
    for i in range(400):
        k = i & 1
        slot = x[k] & 0xFFFF
        v = int(np.searchsorted(tabs[i], slot, side="right")) - 1
        got.append(v)
        x[k] = (int(tabs[i, v + 1]) - int(tabs[i, v])) * (x[k] >> 16) + slot - int(tabs[i, v])
        if x[k] < (1 << 31):
            x[k] = (x[k] << 32) | words.pop(0)
    assert got == list(sym) and not words and x == [1 << 31, 1 << 31]


# ----------------------------------------------------------------- codec

def _images(rng):
    yield "1x1", rng.integers(0, 256, (1, 1, 1, 3), dtype=np.uint8)
    yield "1x9", rng.integers(0, 256, (1, 1, 9, 3), dtype=np.uint8)
    yield "9x1", rng.integers(0, 256, (1, 9, 1, 3), dtype=np.uint8)
    yield "2x2", rng.integers(0, 256, (1, 2, 2, 3), dtype=np.uint8)
    yield "3x5", rng.integers(0, 256, (2, 3, 5, 3), dtype=np.uint8)
    yield "zeros", np.zeros((1, 6, 7, 3), dtype=np.uint8)
    yield "ones", np.full((1, 6, 7, 3), 255, dtype=np.uint8)
    yield "blobs", synth.make_image(3, synth.ImageSpec(19, 11, 3, 2.0, 6.0))[None]


@pytest.mark.parametrize("mode", [po.MODE_EXACT, po.MODE_SPLIT])
@pytest.mark.parametrize("which", ["default", "sharp"])
def test_roundtrip_edge_shapes_raster_equals_wavefront(orc, orc_sharp, mode, which):
    o = orc if which == "default" else orc_sharp
    rng = np.random.default_rng(8)
    for name, imgs in _images(rng):
        n, h, w, _ = imgs.shape
        stream, bits = o.encode(imgs, mode)
        assert len(stream) <= po.stream_bound(n, h, w)
        ras = o.decode(stream, n, h, w, mode, po.ORDER_RASTER)
        wav = o.decode(stream, n, h, w, mode, po.ORDER_WAVEFRONT)
        np.testing.assert_array_equal(ras, imgs, err_msg=name)
        np.testing.assert_array_equal(wav, imgs, err_msg=name)
        # total code length = sum of -log2 p plus a bounded overhead (header, offsets, flush per row)
        rows = n * h
        over = 8 * len(stream) - bits.sum()
        lo = 8 * (32 + 8 * (rows + 1)) + rows * 64
        hi = 8 * (32 + 8 * (rows + 1)) + rows * 128 + 3 * n * h * w * 2.0 ** -14
        assert lo - 1e-6 <= over <= hi + 1e-6, name


def test_config0_roundtrip_and_bpsp(orc):
    imgs = synth.make_batch(0)
    stream, bits = orc.encode(imgs, po.MODE_SPLIT)
    out = orc.decode(stream, 1, 64, 64, po.MODE_SPLIT, po.ORDER_WAVEFRONT)
    np.testing.assert_array_equal(out, imgs)
    bpsp = bits.sum() / imgs.size
    assert 1.0 < bpsp < 16.0
    # exact network and split-bf16-activation network code almost equally well
    _, bits_exact = orc.encode(imgs, po.MODE_EXACT)
    assert abs(bits_exact.sum() / bits.sum() - 1) < 1e-3


def test_decoder_rejects_damaged_streams(orc):
    imgs = synth.make_image(5, synth.ImageSpec(12, 6, 2, 2.0, 5.0))[None]
    stream, _ = orc.encode(imgs)
    n, h, w = 1, 6, 12
    with pytest.raises(po.OracleError):
        orc.decode(stream[:-4], n, h, w)
    with pytest.raises(po.OracleError):
        orc.decode(stream, n, h, w + 1)
    bad = bytearray(stream)
    bad[0] ^= 1
    with pytest.raises(po.OracleError):
        orc.decode(bytes(bad), n, h, w)
    # a flipped payload bit must never be accepted silently: either an error or a different image
    rng = np.random.default_rng(9)
    table_end = 32 + 8 * (h + 1)
    for _ in range(10):
        bad = bytearray(stream)
        bad[rng.integers(table_end, len(stream))] ^= 1 << int(rng.integers(0, 8))
        try:
            out = orc.decode(bytes(bad), n, h, w)
        except po.OracleError:
            continue
        assert (out != imgs).any()


def test_delta_weights_reach_the_extreme_frequencies():
    """The test-only delta weights (all mass of a channel in one or two bins, sigma at its lower clamp): the
    oracle's tables are checked against the mixture written out with scipy's normal CDF in grey-level units
    (Eq. (1) with the open tails and the integer rule), they hold one bin of (nearly) the whole mass and
    frequency 1 (or 2 right next to the mass) everywhere else, and images made of such runs round-trip with
    the code length the frequencies give (a frequency-1 symbol costs exactly 16 bits)."""
    orc_d = po.Oracle(synth.make_delta_blob())
    img = synth.make_delta_image(5, 1, 6, 40)
    o = orc_d.params_at(img[0], 3, 7, po.MODE_EXACT)
    np.testing.assert_array_equal(o, orc_d.params_at(img[0], 0, 0, po.MODE_EXACT))     # weights are zero: biases only
    s_levels = 256.0 * np.exp(-8.0)
    means = {0: [synth.DELTA_R_LEVEL] * 5, 1: [synth.DELTA_G_LEVELS[0]] * 3 + [synth.DELTA_G_LEVELS[1]] * 2, 2: [768.0] * 5}
    tables = {}
    for ch in range(3):
        cq = orc_d.cdf_table(o, ch, 17, 201).astype(np.int64)
        edges = np.arange(1, 256) - 0.5
        F = sum(0.2 * scipy.stats.norm.cdf((edges - m) / s_levels) for m in means[ch])
        want = np.concatenate([[0], np.arange(1, 256) + np.minimum(np.floor(65280.0 * F), 65280).astype(np.int64), [65536]])
        np.testing.assert_array_equal(cq, want)
        freq = np.diff(cq)
        assert freq.sum() == 65536 and freq.min() == 1
        tables[ch] = freq
    assert tables[0][synth.DELTA_R_LEVEL] == 65280 and (tables[0] == 1).sum() == 254       # one neighbour bin holds 2
    assert tables[2][synth.DELTA_B_LEVEL] == 65281 and (tables[2] == 1).sum() == 255       # the open upper tail
    assert tables[1][synth.DELTA_G_LEVELS[0]] + tables[1][synth.DELTA_G_LEVELS[1]] == 65280 and (tables[1] == 1).sum() == 252
    stream, bits = orc_d.encode(img, po.MODE_EXACT)
    for order in (po.ORDER_RASTER, po.ORDER_WAVEFRONT):
        np.testing.assert_array_equal(orc_d.decode(stream, 1, 6, 40, po.MODE_EXACT, order), img)
    want_bits = sum(-np.log2(tables[ch][int(v)] / 65536.0) for px in img.reshape(-1, 3) for ch, v in enumerate(px))
    assert abs(bits.sum() - want_bits) < 1e-6
    assert (tables[0][img[..., 0].reshape(-1)] == 1).sum() > 50 and (tables[0][img[..., 0].reshape(-1)] == 65280).sum() > 50
    payload = len(stream) - (32 + 8 * 7)
    assert 6 * 64 <= 8 * payload - bits.sum() <= 6 * 128 + 3 * 240 * 2.0 ** -14


def test_blob_validation():
    blob = synth.make_blob(0)
    for bad in (blob[:-4], b"\0" * len(blob), blob + b"\0\0\0\0"):
        with pytest.raises(po.OracleError):
            po.Oracle(bad)
