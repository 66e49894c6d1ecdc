"""Pins for the CPU oracle: every oracle function is checked against something
other than itself -- closed forms, brute force written differently (numpy
vectorised, float64), library routines (numpy float16, scikit-learn Lloyd,
torch scaled_dot_product_attention), and the invariants the paper states
(App. C half-step bound and w(x-c) <= 2||x-c||_inf; Sec. 2.1 law of total
variance; Sec. 3.1 K-means objective; App. H memory ratios)."""
import os

import numpy as np
import pytest

from paper_2510_05176_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def f16(a):
    return np.asarray(a, np.float16)


def u16(a):
    return f16(a).view(np.uint16)


# ---------------------------------------------------------------- fp16 helpers

def test_half_to_float_all_bit_patterns(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle.half_to_float(int(b)) for b in bits], np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))


def test_float_to_half_rne_matches_numpy(oracle):
    rng = np.random.default_rng(1)
    vals = np.concatenate([
        rng.standard_normal(4000).astype(np.float32) * 10,
        rng.standard_normal(2000).astype(np.float32) * 1e-5,          # subnormal range
        np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e6, -1e6, 2.0 ** -24, 2.0 ** -25, 3 * 2.0 ** -25], np.float32),
        # exact halfway points between neighbouring halves
        (np.arange(1, 2000, dtype=np.float32) + 0.5) * np.float32(2.0 ** -10) + 1.0,
    ])
    with np.errstate(over="ignore"):
        ref = vals.astype(np.float16).view(np.uint16)
    got = np.array([oracle.float_to_half(float(v), "rne") for v in vals], np.uint16)
    assert np.array_equal(got, ref)


def test_float_to_half_directed(oracle):
    rng = np.random.default_rng(2)
    vals = np.concatenate([rng.standard_normal(5000).astype(np.float32) * 4,
                           rng.standard_normal(2000).astype(np.float32) * 3e-5,
                           f16(rng.standard_normal(500)).astype(np.float32)])  # exactly representable
    for v in vals:
        lo = np.array([oracle.float_to_half(float(v), "down")], np.uint16).view(np.float16)[0]
        hi = np.array([oracle.float_to_half(float(v), "up")], np.uint16).view(np.float16)[0]
        assert float(lo) <= float(v) <= float(hi)
        if float(f16(v)) == float(v):          # representable: both must return it
            assert float(lo) == float(v) == float(hi)
        else:                                   # neighbours: nothing representable in between
            assert np.nextafter(lo, f16(np.inf)) == hi


# ---------------------------------------------------------------- assignment

def _data(seed, T=200, d=128, P=9):
    rng = np.random.default_rng(seed)
    x = f16(rng.standard_normal((T, d)) * 2)
    M = f16(rng.standard_normal((P, d)) * 2)
    return x, M


def test_assign_l2_bruteforce(oracle):
    x, M = _data(3)
    idx, best, second = oracle.assign(x.view(np.uint16), M.view(np.uint16), oracle.METRIC_L2)
    X, MM = x.astype(np.float64), M.astype(np.float64)
    D = ((X[:, None, :] - MM[None, :, :]) ** 2).sum(-1)
    assert np.array_equal(idx, D.argmin(1))
    srt = np.sort(D, axis=1)
    assert np.allclose(best, srt[:, 0], rtol=1e-12) and np.allclose(second, srt[:, 1], rtol=1e-12)
    # expanded form ||x||^2 + ||m||^2 - 2 x.m in float64 selects the same pattern
    E = (X ** 2).sum(1)[:, None] + (MM ** 2).sum(1)[None, :] - 2 * X @ MM.T
    assert np.array_equal(idx, E.argmin(1))


def test_assign_minmax_definition_and_invariants(oracle):
    x, M = _data(4)
    idx, best, _ = oracle.assign(x.view(np.uint16), M.view(np.uint16), oracle.METRIC_MINMAX)
    diff = x.astype(np.float32)[:, None, :] - M.astype(np.float32)[None, :, :]
    D = diff.max(-1) - diff.min(-1)
    assert np.array_equal(idx, D.argmin(1))
    assert np.array_equal(best.astype(np.float32), D.min(1))
    # App. C: w(x - c) <= 2 ||x - c||_inf
    assert np.all(D <= 2 * np.abs(diff).max(-1) + 1e-6)
    # shift invariance: adding a constant (exactly representable) to a pattern leaves d_mm unchanged
    xs = f16(np.round(x.astype(np.float32) * 4) / 4)
    Ms = f16(np.round(M.astype(np.float32) * 4) / 4)
    _, b0, _ = oracle.assign(xs.view(np.uint16), Ms.view(np.uint16), oracle.METRIC_MINMAX)
    _, b1, _ = oracle.assign(xs.view(np.uint16), f16(Ms.astype(np.float32) + 0.75).view(np.uint16), oracle.METRIC_MINMAX)
    assert np.array_equal(b0, b1)


@pytest.mark.parametrize("metric", [0, 1])
def test_assign_special_cases(oracle, metric):
    x, M = _data(5, T=50, P=1)
    idx, _, _ = oracle.assign(x.view(np.uint16), M.view(np.uint16), metric)
    assert np.all(idx == 0)
    # patterns that are copies of tokens: those tokens are at distance exactly 0
    x, _ = _data(6, T=64)
    M = x[[7, 20, 33]]
    idx, best, _ = oracle.assign(x.view(np.uint16), M.view(np.uint16), metric)
    assert list(idx[[7, 20, 33]]) == [0, 1, 2] and np.all(best[[7, 20, 33]] == 0)
    # exact tie goes to the lowest index
    M2 = np.concatenate([M[:1], M[:1]])
    idx, _, _ = oracle.assign(x.view(np.uint16), M2.view(np.uint16), metric)
    assert np.all(idx == 0)


def test_dmm_worked_example(oracle):
    # tests/golden/dmm_example.txt : hand-evaluated d_mm of Sec. 3.2
    rows = [l.split() for l in open(os.path.join(GOLDEN, "dmm_example.txt")) if l.strip() and not l.startswith("#")]
    x = f16([float(v) for v in rows[0]])[None, :]
    pats = f16([[float(v) for v in r] for r in rows[1:4]])
    want = [float(v) for v in rows[4]]
    for p in range(3):
        _, best, _ = oracle.assign(x.view(np.uint16), pats[p:p + 1].view(np.uint16), oracle.METRIC_MINMAX)
        assert best[0] == want[p]
    idx, _, _ = oracle.assign(x.view(np.uint16), pats.view(np.uint16), oracle.METRIC_MINMAX)
    assert idx[0] == int(rows[5][0])


# ---------------------------------------------------------------- mining

def _mixture(seed, n_c=6, T=1200, d=16, sigma=0.05):
    rng = np.random.default_rng(seed)
    centres = rng.standard_normal((n_c, d)) * 3
    u = np.concatenate([np.arange(n_c), rng.integers(0, n_c, T - n_c)])   # one seed token per cluster first
    x = f16(centres[u] + sigma * rng.standard_normal((T, d)))
    return x, centres, u


def test_mine_recovers_separated_mixture(oracle):
    x, centres, u = _mixture(7)
    M, a, J, cnt = oracle.mine(x.view(np.uint16)[None], 6, 8)
    assert np.array_equal(a[0], u)
    assert np.array_equal(cnt[0], np.bincount(u, minlength=6))
    Mf = M[0].view(np.float16).astype(np.float64)
    n_p = np.bincount(u)
    assert np.all(np.abs(Mf - centres) < 5 * 0.05 / np.sqrt(n_p)[:, None] + 4e-3)
    # centroid = fp16(mean of members)
    for p in range(6):
        mean = x[u == p].astype(np.float64).mean(0)
        assert np.array_equal(M[0, p], f16(mean.astype(np.float32)).view(np.uint16))


def test_mine_matches_sklearn_lloyd(oracle):
    from sklearn.cluster import KMeans
    rng = np.random.default_rng(8)
    centres = rng.standard_normal((8, 32)) * 1.0
    x = f16(centres[rng.integers(0, 8, 900)] + 0.6 * rng.standard_normal((900, 32)))   # overlapping clusters
    P, iters = 8, 5
    M, a, J, _ = oracle.mine(x.view(np.uint16)[None], P, iters)
    # one Lloyd iteration at a time with the library, feeding it the oracle's fp16-rounded
    # centroids, so that both see the same centroids at every step
    cur = x[:P].astype(np.float64)
    for it in range(iters):
        km = KMeans(n_clusters=P, init=cur, n_init=1, algorithm="lloyd", max_iter=1, tol=0.0).fit(x.astype(np.float64))
        lab = ((x.astype(np.float64)[:, None] - cur[None]) ** 2).sum(-1).argmin(1)
        assert np.isclose(J[0, it], ((x.astype(np.float64) - cur[lab]) ** 2).sum(), rtol=1e-10)
        new = km.cluster_centers_
        cur = f16(new.astype(np.float32)).astype(np.float64)
    assert np.array_equal(M[0], f16(cur).view(np.uint16))


def test_mine_objective_and_total_variance(oracle):
    rng = np.random.default_rng(9)
    x = f16(rng.standard_normal((1500, 24)) + rng.integers(0, 4, (1500, 1)) * 1.5)
    M, a, J, cnt = oracle.mine(x.view(np.uint16)[None], 12, 12)
    J = J[0]
    # Sec. 3.1: Lloyd never increases the K-means objective (slack for the fp16 rounding of centroids)
    assert np.all(J[1:] <= J[:-1] * (1 + 1e-4))
    assert J[-1] < 0.8 * J[0]
    # Sec. 2.1 Eq. 2: Var(Z) = E[Var(Z|M)] + Var(E[Z|M]) for the partition of the last assignment
    X = x.astype(np.float64)
    lab = a[0]
    tot = ((X - X.mean(0)) ** 2).sum()
    intra = sum(((X[lab == p] - X[lab == p].mean(0)) ** 2).sum() for p in range(12) if np.any(lab == p))
    inter = sum((lab == p).sum() * ((X[lab == p].mean(0) - X.mean(0)) ** 2).sum() for p in range(12) if np.any(lab == p))
    assert np.isclose(tot, intra + inter, rtol=1e-10)
    # intra-pattern variance around the members' means lower-bounds the inertia seen by that assignment
    assert intra <= J[-1] * (1 + 1e-12)


def test_mine_empty_cluster_keeps_centroid(oracle):
    rng = np.random.default_rng(20)
    x = f16(1.0 + 0.1 * rng.standard_normal((40, 8)))
    init = f16(np.stack([np.ones(8), np.full(8, 100.0)]))[None]        # nothing is ever nearest to pattern 1
    M, a, J, cnt = oracle.mine(x.view(np.uint16)[None], 2, 3, init=init.view(np.uint16))
    assert cnt[0].tolist() == [40, 0] and np.all(a == 0)
    assert np.array_equal(M[0, 1], init[0, 1].view(np.uint16))
    assert np.array_equal(M[0, 0], f16(x.astype(np.float64).mean(0).astype(np.float32)).view(np.uint16))


# ---------------------------------------------------------------- quantization

def _numpy_asym_quant(r, bits, axis):
    """Textbook Eq. 1 with the stored-parameter reading: z = fp16 floor of min, s = fp16 ceil of (max - z)/(2^b-1)."""
    qmax = 2 ** bits - 1
    mn = r.min(axis=axis, keepdims=True)
    mx = r.max(axis=axis, keepdims=True)
    z = mn.astype(np.float16)
    z = np.where(z.astype(np.float32) > mn, np.nextafter(z, f16(-np.inf)), z)
    s32 = ((mx - z.astype(np.float32)) / np.float32(qmax)).astype(np.float32)
    s = s32.astype(np.float16)
    s = np.where(s.astype(np.float32) < s32, np.nextafter(s, f16(np.inf)), s)
    sf, zf = s.astype(np.float32), z.astype(np.float32)
    with np.errstate(divide="ignore", invalid="ignore"):
        q = np.rint((r - zf) * (np.float32(1) / sf))
    q = np.where(sf == 0, 0, np.clip(q, 0, qmax)).astype(np.uint8)
    return q, s, z


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("G", [32, 64, 128])
def test_quantize_reduces_to_textbook_with_zero_pattern(oracle, bits, G):
    rng = np.random.default_rng(10 + bits + G)
    n, d = 256, 128
    x = f16(rng.standard_normal((1, n, d)) * np.exp(rng.standard_normal((1, 1, d))))
    M = np.zeros((1, 1, d), np.uint16)
    set_of = np.zeros(1, np.int32)
    rk = oracle.quantize_streams(x.view(np.uint16), set_of, M, 0, bits, G, 0, want_codes=True)
    rv = oracle.quantize_streams(x.view(np.uint16), set_of, M, 0, bits, G, 1, want_codes=True)
    r = x[0].astype(np.float32)
    qk, sk, zk = _numpy_asym_quant(r.reshape(n // G, G, d), bits, axis=1)
    assert np.array_equal(rk["codes"][0], qk.reshape(n, d))
    assert np.array_equal(rk["scale"][0], sk.reshape(n // G, d).view(np.uint16))
    assert np.array_equal(rk["zero"][0], zk.reshape(n // G, d).view(np.uint16))
    Gc = min(G, d)
    qv, sv, zv = _numpy_asym_quant(r.reshape(n, d // Gc, Gc), bits, axis=2)
    assert np.array_equal(rv["codes"][0], qv.reshape(n, d))
    assert np.array_equal(oracle.v_params_by_token(rv["scale"][0]), sv.reshape(n, d // Gc).view(np.uint16))
    assert np.array_equal(oracle.v_params_by_token(rv["zero"][0]), zv.reshape(n, d // Gc).view(np.uint16))


@pytest.mark.parametrize("side", [0, 1])
@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("metric", [0, 1])
def test_quantize_invariants(oracle, side, bits, metric):
    spec = synth.KVSpec(1, 1, 2, 2, 256, 128, 8)
    K, V = synth.make_kv(11, spec)
    x = (K if side == 0 else V)[0]
    G = 64
    M = x[:, :12].copy()
    set_of = np.arange(2, dtype=np.int32)
    res = oracle.quantize_streams(x.view(np.uint16), set_of, M.view(np.uint16), metric, bits, G, side, want_codes=True)
    qmax = 2 ** bits - 1
    codes = res["codes"]
    assert codes.max() <= qmax
    for s in range(2):
        resid = x[s].astype(np.float32) - M[s][res["idx"][s]].astype(np.float32)
        sc, ze = res["scale"][s], res["zero"][s]
        if side == 1:
            sc, ze = oracle.v_params_by_token(sc), oracle.v_params_by_token(ze)
        sc = sc.view(np.float16).astype(np.float32)
        ze = ze.view(np.float16).astype(np.float32)
        if side == 0:
            sc_e, ze_e = np.repeat(sc, G, axis=0), np.repeat(ze, G, axis=0)
            grp = codes[s].reshape(-1, G, 128)
            gmin, gmax = grp.min(1), grp.max(1)
        else:
            sc_e, ze_e = np.repeat(sc, G, axis=1), np.repeat(ze, G, axis=1)
            grp = codes[s].reshape(256, -1, G)
            gmin, gmax = grp.min(2), grp.max(2)
        deq = sc_e * codes[s] + ze_e
        # App. C per-element form: error at most half a step of the stored scale
        assert np.all(np.abs(deq - resid) <= sc_e * 0.5 * (1 + 1e-5) + 1e-7)
        # every group uses its lowest level, and (nearly) its highest
        assert np.all(gmin == 0)
        assert np.all(gmax[sc > 0] >= qmax - 1)
        # first 12 tokens are patterns themselves: zero residual, exact reconstruction
        out = oracle.dequant(side, codes[s], res["scale"][s], res["zero"][s], res["idx"][s], M[s].view(np.uint16), G)
        assert np.all(np.abs(out - x[s].astype(np.float32)) <= sc_e * 0.5 * (1 + 1e-5) + 1e-6)


# ------------------------------------------------------------------ adaptive threshold on V (Sec. 3.3)

def test_rho_star_solves_the_criterion(oracle):
    from scipy.stats import norm
    for d, alpha in [(96, 0.05), (128, 0.05), (128, 0.01), (256, 0.1), (128, 0.3)]:
        rho = oracle.rho_star(d, alpha)
        c = 2.0 * norm.ppf(1.0 - alpha) / np.sqrt(5.0 * d)
        f = lambda r: (1.0 - r * r) - c * np.sqrt(1.0 + r ** 4)     # Sec. 3.3: keep iff f(rho) >= 0
        assert 0.0 < rho < 1.0 and abs(f(rho)) < 1e-12
        assert f(rho - 1e-6) > 0 > f(rho + 1e-6)                    # f decreases through its only root in (0, 1)
        grid = np.linspace(0.0, 1.0, 2001)
        assert np.all((f(grid) >= 0) == (grid <= rho))
    # a stricter test (smaller alpha) or a shorter vector keeps fewer ratios
    assert oracle.rho_star(128, 0.01) < oracle.rho_star(128, 0.05) < oracle.rho_star(256, 0.05)
    assert abs(oracle.rho_star(128, 0.05) - 0.9116) < 1e-4


@pytest.mark.parametrize("bits,G,metric", [(2, 64, 0), (4, 32, 0), (2, 128, 1)])
def test_v_threshold_decision_and_raw_fallback(oracle, bits, G, metric):
    spec = synth.KVSpec(1, 1, 2, 2, 256, 128, 8)
    _, V = synth.make_kv(21, spec)
    x = V[0].copy()
    x[0, 20] = np.float16(1.25)                     # a constant vector: R_raw = 0, rejected unless the residual is flat too
    x[1, 30] = x[1, 3]                              # a vector equal to a pattern: R_flat = 0, always kept
    M = x[:, :7].copy()
    set_of = np.arange(2, dtype=np.int32)
    rho = 0.8
    base = oracle.quantize_streams(x.view(np.uint16), set_of, M.view(np.uint16), metric, bits, G, 1, want_codes=True)
    thr = oracle.quantize_streams(x.view(np.uint16), set_of, M.view(np.uint16), metric, bits, G, 1, want_codes=True, v_rho=rho)
    zeroM = np.zeros_like(M)
    rawq = oracle.quantize_streams(x.view(np.uint16), set_of, zeroM.view(np.uint16), metric, bits, G, 1, want_codes=True)
    n_raw = 0
    for s in range(2):
        xf = x[s].astype(np.float32)
        resid = xf - M[s][base["idx"][s]].astype(np.float32)
        r_flat = resid.max(1) - resid.min(1)
        r_raw = xf.max(1) - xf.min(1)
        raw = ~(r_flat <= np.float32(rho) * r_raw)
        assert np.array_equal(thr["idx"][s] == oracle.NO_PATTERN, raw)
        assert np.array_equal(thr["idx"][s][~raw], base["idx"][s][~raw])
        # kept tokens: exactly the unthresholded result; rejected tokens: exactly the quantization of the vector itself
        pt = oracle.v_params_by_token
        for name in ("codes",):
            assert np.array_equal(thr[name][s][~raw], base[name][s][~raw])
            assert np.array_equal(thr[name][s][raw], rawq[name][s][raw])
        for name in ("scale", "zero"):
            assert np.array_equal(pt(thr[name][s])[~raw], pt(base[name][s])[~raw])
            assert np.array_equal(pt(thr[name][s])[raw], pt(rawq[name][s])[raw])
        # reconstruction never adds a pattern to a rejected token, and stays within half a step everywhere
        out = oracle.dequant(1, thr["codes"][s], thr["scale"][s], thr["zero"][s], thr["idx"][s], M[s].view(np.uint16), G,
                             thresholded=True)
        Gc = min(G, 128)
        sc = np.repeat(pt(thr["scale"][s]).view(np.float16).astype(np.float32), Gc, axis=1)
        assert np.all(np.abs(out - xf) <= sc * 0.5 * (1 + 1e-5) + 1e-6)
        n_raw += int(raw.sum())
    assert thr["idx"][0][20] == oracle.NO_PATTERN and np.all(thr["codes"][0][20] == 0)   # constant vector: raw, flat group
    assert thr["idx"][1][30] == 3                                                       # pattern itself: kept
    assert 0 < n_raw < 2 * 256
    # rho = 0 switches the test off; a looser rho keeps at least as many tokens
    off = oracle.quantize_streams(x.view(np.uint16), set_of, M.view(np.uint16), metric, bits, G, 1, want_codes=True, v_rho=0.0)
    assert all(np.array_equal(off[k], base[k]) for k in ("idx", "codes", "scale", "zero", "packed"))
    loose = oracle.quantize_streams(x.view(np.uint16), set_of, M.view(np.uint16), metric, bits, G, 1, v_rho=0.95)
    assert (loose["idx"] == oracle.NO_PATTERN).sum() <= n_raw


def test_v_threshold_minmax_range_is_dmm(oracle):
    # with the min-max metric the flat range of the chosen pattern is d_mm itself (Sec. 3.2), so a token is
    # rejected exactly when min_p d_mm(x, M_p) > rho * (max x - min x)
    rng = np.random.default_rng(31)
    x = f16(rng.standard_normal((1, 64, 128)))
    M = f16(rng.standard_normal((1, 6, 128)) * 0.5)
    rho = 0.9
    res = oracle.quantize_streams(x.view(np.uint16), np.zeros(1, np.int32), M.view(np.uint16), 1, 2, 64, 1, v_rho=rho)
    diff = x[0].astype(np.float32)[:, None, :] - M[0].astype(np.float32)[None]
    dmm = (diff.max(2) - diff.min(2)).min(1)
    xr = x[0].astype(np.float32)
    assert np.array_equal(res["idx"][0] == oracle.NO_PATTERN, ~(dmm <= np.float32(rho) * (xr.max(1) - xr.min(1))))


# ------------------------------------------------------------------ decode-stage patterns (Sec. 3.1 Eq. 5)

def test_window_pattern_is_the_per_channel_chebyshev_centre(oracle):
    rng = np.random.default_rng(41)
    x = f16(rng.standard_normal((3, 128, 128)) * np.exp(rng.standard_normal((3, 1, 128))))
    m = oracle.window_pattern(x.view(np.uint16)).view(np.float16)
    xf = x.astype(np.float64)
    mid = (xf.min(1) + xf.max(1)) / 2                              # Eq. 5 in exact arithmetic
    assert np.array_equal(m, mid.astype(np.float16))               # one rounding to fp16, ties to even
    # Chebyshev centre: no other fp16 value has a smaller worst deviation from the window, per channel
    dev = np.abs(xf - m.astype(np.float64)[:, None, :]).max(1)
    for other in (np.nextafter(m, np.float16(np.inf)), np.nextafter(m, np.float16(-np.inf)), xf.mean(1).astype(np.float16)):
        assert np.all(dev <= np.abs(xf - other.astype(np.float64)[:, None, :]).max(1) + 1e-12)
    # it halves the range a raw quantizer would see: residuals of the window lie in [-R/2, R/2] (+ fp16 rounding of m)
    R = xf.max(1) - xf.min(1)
    assert np.all(dev <= R / 2 + np.abs(m.astype(np.float64)) * 2.0 ** -11 + 1e-12)
    # a window of one vector is that vector; a constant channel stays exact
    assert np.array_equal(oracle.window_pattern(x[:, :1].view(np.uint16)), x[:, 0].view(np.uint16))


def test_zero_residual_reconstructs_exactly(oracle):
    rng = np.random.default_rng(12)
    M = f16(rng.standard_normal((1, 5, 128)))
    pick = rng.integers(0, 5, 64)
    x = M[0][pick][None]
    for side in (0, 1):
        res = oracle.quantize_streams(x.view(np.uint16), np.zeros(1, np.int32), M.view(np.uint16), 0, 2, 32, side, want_codes=True)
        assert np.all(res["codes"] == 0) and np.all(res["scale"] == 0)
        out = oracle.dequant(side, res["codes"][0], res["scale"][0], res["zero"][0], res["idx"][0], M[0].view(np.uint16), 32)
        assert np.array_equal(out, x[0].astype(np.float32))


def test_minmax_choice_minimises_v_scale(oracle):
    # Sec. 3.2: d_mm is the quantization range of the residual; with one channel group per V token
    # the chosen pattern gives the smallest stored scale among all patterns
    rng = np.random.default_rng(13)
    x = f16(rng.standard_normal((1, 64, 128)) * 2)
    M = f16(rng.standard_normal((1, 7, 128)) * 2)
    res = oracle.quantize_streams(x.view(np.uint16), np.zeros(1, np.int32), M.view(np.uint16), 1, 2, 128, 1)
    diff = x[0].astype(np.float32)[:, None] - M[0].astype(np.float32)[None]
    dmm = diff.max(-1) - diff.min(-1)
    s = oracle.v_params_by_token(res["scale"][0]).view(np.float16).astype(np.float64)[:, 0]
    assert np.all(s >= dmm.min(1) / 3 * (1 - 1e-6))
    assert np.all(s <= dmm.min(1) / 3 * (1 + 2.0 ** -9))


@pytest.mark.parametrize("bits", [2, 4])
def test_pack_roundtrip_and_format(oracle, bits):
    rng = np.random.default_rng(14)
    n, d = 96, 128
    codes = rng.integers(0, 2 ** bits, (n, d)).astype(np.uint8)
    wk = oracle.pack_k(codes, bits)
    assert np.array_equal(oracle.unpack_k(wk, n, d, bits), codes)
    bv = oracle.pack_v(codes, bits)
    assert np.array_equal(oracle.unpack_v(bv, n, d, bits), codes)
    assert wk.nbytes == bv.nbytes == n * d * bits // 8
    # single-bit probes of the two index formulas (tests/golden/pack_format.txt)
    for line in open(os.path.join(GOLDEN, "pack_format.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        side, b, t, c, j, unit, bit = line.split()
        if int(b) != bits:
            continue
        one = np.zeros((n, d), np.uint8)
        one[int(t), int(c)] = 1 << int(j)
        if side == "K":
            w = oracle.pack_k(one, bits).reshape(-1)
            assert np.flatnonzero(w).tolist() == [int(unit)] and w[int(unit)] == 1 << int(bit)
        else:
            w = oracle.pack_v(one, bits)
            assert w.dtype == np.uint32 and np.flatnonzero(w).tolist() == [int(unit)] and w[int(unit)] == 1 << int(bit)


def test_eq1_worked_examples(oracle):
    # tests/golden/eq1_cases.txt: Eq. 1 evaluated by hand on exactly representable values
    for line in open(os.path.join(GOLDEN, "eq1_cases.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        bits, vals, s_want, z_want, codes_want = [f.strip() for f in line.split("|")]
        vals = [float(v) for v in vals.split()]
        G = 32
        x = np.zeros((1, 2 * G, 128), np.float16)      # second group of the stream stays zero
        x[0, :len(vals), 0] = vals
        x[0, len(vals):G, 0] = vals[0]
        res = oracle.quantize_streams(x.view(np.uint16), np.zeros(1, np.int32), np.zeros((1, 1, 128), np.uint16),
                                      0, int(bits), G, 0, want_codes=True)
        assert float(res["scale"][0, 0, 0:1].view(np.float16)[0]) == float(s_want)
        assert float(res["zero"][0, 0, 0:1].view(np.float16)[0]) == float(z_want)
        assert res["codes"][0, :len(vals), 0].tolist() == [int(c) for c in codes_want.split()]


# ---------------------------------------------------------------- cache bookkeeping + layout

def _cfg(oracle, **kw):
    base = dict(n_seq=2, n_kv_heads=2, n_q_heads=4, head_dim=128, n_patterns=8, seqs_per_set=0, bits=2,
                group=32, recent=16, flush=64, t_capacity=512, metric=0)
    base.update(kw)
    return oracle.Config(**base)


def test_append_bookkeeping(oracle):
    cfg = _cfg(oracle)
    spec = synth.KVSpec(1, 2, 2, 4, 400, 128, 8)
    K, V = synth.make_kv(15, spec)
    pk, pv = K[0, :, :8].copy().view(np.uint16), V[0, :, :8].copy().view(np.uint16)
    a = oracle.Cache(cfg)
    b = oracle.Cache(cfg)
    a.append(K.view(np.uint16), V.view(np.uint16), pk, pv)          # one call
    pos = 0
    for n in (1, 7, 64, 100, 3, 225):                                # same tokens in pieces
        b.append(K[:, :, pos:pos + n].view(np.uint16), V[:, :, pos:pos + n].view(np.uint16), pk, pv)
        pos += n
        assert b.t_quant + b.t_tail == pos
        assert b.t_tail < cfg.recent + cfg.flush
        if b.t_quant:
            assert b.t_tail >= cfg.recent
    assert pos == 400 and a.t_quant == b.t_quant == 384 and a.t_tail == b.t_tail == 16
    for name in ("k_codes", "k_scale", "k_zero", "k_idx", "v_codes", "v_scale", "v_zero", "v_idx"):
        assert np.array_equal(getattr(a, name), getattr(b, name)), name
    assert np.array_equal(a.tail("k"), b.tail("k")) and np.array_equal(a.tail("k"), K.reshape(4, 400, 128)[:, 384:].view(np.uint16))
    # nothing is flushed while the window is short
    c = oracle.Cache(cfg)
    c.append(K[:, :, :79].view(np.uint16), V[:, :, :79].view(np.uint16), pk, pv)
    assert c.t_quant == 0 and c.t_tail == 79


def test_layout_bits_per_element_and_pattern_ratio(oracle):
    # byte accounting of the cache arrays; App. H: pattern table / fp16 KV = P / (B*S) = 0.39 % at P=32, S=8192, B=1
    cfg = _cfg(oracle, n_seq=1, n_kv_heads=1, n_q_heads=1, group=64, recent=0, flush=64, t_capacity=8192, n_patterns=32)
    c = oracle.Cache(cfg)
    packed_bytes = sum(getattr(c, n).nbytes for n in ("k_codes", "k_scale", "k_zero", "k_idx", "v_codes", "v_scale", "v_zero", "v_idx"))
    bits_per_elem = packed_bytes * 8 / (2 * 8192 * 128)
    assert abs(bits_per_elem - (2 + 32 / 64 + 8 / 128)) < 1e-12          # 2.5625 bits
    pattern_bytes = 2 * 32 * 128 * 2
    kv_fp16_bytes = 2 * 8192 * 128 * 2
    assert abs(pattern_bytes / kv_fp16_bytes - 32 / 8192) < 1e-15 and round(100 * pattern_bytes / kv_fp16_bytes, 2) == 0.39


# ---------------------------------------------------------------- attention

def _small_cache(oracle, seed=16, **kw):
    cfg = _cfg(oracle, **kw)
    spec = synth.KVSpec(1, cfg.n_seq, cfg.n_kv_heads, cfg.n_q_heads, 150, 128, 8)
    K, V = synth.make_kv(seed, spec)
    M_k, _, _, _ = oracle.mine(K[0].view(np.uint16), cfg.n_patterns, 3)
    M_v, _, _, _ = oracle.mine(V[0].view(np.uint16), cfg.n_patterns, 3)
    c = oracle.Cache(cfg)
    c.append(K.view(np.uint16), V.view(np.uint16), M_k, M_v)
    q = synth.make_queries(seed, cfg.n_seq, cfg.n_q_heads, 128)
    return cfg, c, K, V, M_k, M_v, q


def test_attention_matches_torch_sdpa(oracle):
    import torch
    cfg, c, K, V, M_k, M_v, q = _small_cache(oracle)
    assert c.t_quant == 128 and c.t_tail == 22
    out, lse = oracle.decode_attention(c, q.view(np.uint16), M_k, M_v, 128 ** -0.5)
    Kh, Vh = c.materialize(M_k, M_v)
    Kh = torch.from_numpy(Kh).reshape(2, 2, 150, 128).repeat_interleave(2, dim=1).double()
    Vh = torch.from_numpy(Vh).reshape(2, 2, 150, 128).repeat_interleave(2, dim=1).double()
    Q = torch.from_numpy(q.astype(np.float64)).reshape(2, 4, 1, 128)
    ref = torch.nn.functional.scaled_dot_product_attention(Q, Kh, Vh, scale=128 ** -0.5)
    assert np.allclose(out, ref.reshape(2, 4, 128).numpy(), rtol=1e-5, atol=1e-6)
    ref_lse = torch.logsumexp((Q @ Kh.transpose(-1, -2)) * 128 ** -0.5, dim=-1).reshape(2, 4).numpy()
    assert np.allclose(lse, ref_lse, rtol=1e-6)
    # the reconstruction is close to the source: attention over it is close to fp16 attention
    Kf = torch.from_numpy(K.astype(np.float64)).repeat_interleave(2, dim=1)
    Vf = torch.from_numpy(V.astype(np.float64)).repeat_interleave(2, dim=1)
    full = torch.nn.functional.scaled_dot_product_attention(Q, Kf, Vf, scale=128 ** -0.5).reshape(2, 4, 128).numpy()
    assert np.linalg.norm(out - full) / np.linalg.norm(full) < 0.35


def test_v_parameter_layout(oracle):
    # V (s, z) are stored in slices of 16 tokens: parameter of token t, channel group j at ((t/16)*groups + j)*16 + t%16
    rng = np.random.default_rng(21)
    x = f16(rng.standard_normal((1, 64, 128)) * (1 + np.arange(64))[None, :, None])   # scale grows with the token index
    res = oracle.quantize_streams(x.view(np.uint16), np.zeros(1, np.int32), np.zeros((1, 1, 128), np.uint16), 0, 2, 32, 1)
    flat = res["scale"][0].reshape(-1).view(np.float16).astype(np.float32)
    r = x[0].astype(np.float32).reshape(64, 4, 32)
    want = (r.max(2) - r.min(2)) / 3
    for t in (0, 5, 16, 37, 63):
        for j in range(4):
            got = flat[((t // 16) * 4 + j) * 16 + t % 16]
            assert abs(got - want[t, j]) <= 2e-3 * want[t, j]


def test_attention_factorised_form_equals_plain(oracle):
    """The algebra the GPU kernels rely on: scores = q.M[idx] + sum_c (q_c s_c) code_c + q.z, and
    output = W.M_V + sum_t p_t (s code + z) with W[p] = sum of p_t over tokens assigned to p."""
    cfg, c, K, V, M_k, M_v, q = _small_cache(oracle, seed=17, recent=0, flush=64)
    assert c.t_tail == 22 and c.t_quant == 128
    out, _ = oracle.decode_attention(c, q.view(np.uint16), M_k, M_v, 128 ** -0.5)
    d, G, tq = 128, cfg.group, c.t_quant
    set_of = cfg.set_of()
    for seq in range(cfg.n_seq):
        for h in range(cfg.n_q_heads):
            s = seq * cfg.n_kv_heads + h // 2
            qd = q[seq, h].astype(np.float64)
            ck = oracle.unpack_k(c.k_codes[s, :tq], tq, d, 2).astype(np.float64)
            cv = oracle.unpack_v(c.v_codes[s, :tq * 8], tq, d, 2).astype(np.float64)
            ks = np.repeat(c.k_scale[s, :tq // G].view(np.float16).astype(np.float64), G, axis=0)
            kz = np.repeat(c.k_zero[s, :tq // G].view(np.float16).astype(np.float64), G, axis=0)
            vs = np.repeat(oracle.v_params_by_token(c.v_scale[s, :tq // 16]).view(np.float16).astype(np.float64), G, axis=1)
            vz = np.repeat(oracle.v_params_by_token(c.v_zero[s, :tq // 16]).view(np.float16).astype(np.float64), G, axis=1)
            Mk = M_k[set_of[s]].view(np.float16).astype(np.float64)
            Mv = M_v[set_of[s]].view(np.float16).astype(np.float64)
            QM = Mk @ qd
            sc_packed = QM[c.k_idx[s, :tq]] + ((qd[None] * ks) * ck).sum(1) + (kz @ qd)
            sc_tail = c.tail("k")[s].view(np.float16).astype(np.float64) @ qd
            sc = np.concatenate([sc_packed, sc_tail]) * 128 ** -0.5
            p = np.exp(sc - sc.max()); p /= p.sum()
            W = np.bincount(c.v_idx[s, :tq], weights=p[:tq], minlength=cfg.n_patterns)
            o = W @ Mv + (p[:tq, None] * (vs * cv + vz)).sum(0) + p[tq:] @ c.tail("v")[s].view(np.float16).astype(np.float64)
            assert np.allclose(o, out[seq, h], rtol=2e-5, atol=2e-6)


def test_attention_special_cases(oracle):
    cfg, c, K, V, M_k, M_v, q = _small_cache(oracle, seed=18)
    # zero query: all scores equal, output is the mean of V^
    q0 = np.zeros_like(q)
    out, lse = oracle.decode_attention(c, q0.view(np.uint16), M_k, M_v, 128 ** -0.5)
    _, Vh = c.materialize(M_k, M_v)
    Vh = Vh.reshape(2, 2, 150, 128)
    assert np.allclose(out[:, ::2], Vh.astype(np.float64).mean(2), rtol=1e-6, atol=1e-6)
    assert np.allclose(lse, np.log(150.0))
    # nothing quantized yet: plain attention over the fp16 window
    cfg2 = _cfg(oracle, recent=128, flush=64)
    c2 = oracle.Cache(cfg2)
    c2.append(K[:, :, :100].view(np.uint16), V[:, :, :100].view(np.uint16), M_k, M_v)
    assert c2.t_quant == 0
    out2, _ = oracle.decode_attention(c2, q.view(np.uint16), M_k, M_v, 128 ** -0.5)
    Kd, Vd, Qd = K[:, :, :100].astype(np.float64), V[:, :, :100].astype(np.float64), q.astype(np.float64)
    for seq in range(2):
        for h in range(4):
            sc = Kd[seq, h // 2] @ Qd[seq, h] * 128 ** -0.5
            p = np.exp(sc - sc.max()); p /= p.sum()
            assert np.allclose(out2[seq, h], p @ Vd[seq, h // 2], rtol=1e-6, atol=1e-7)


def test_attention_shared_prefix_equals_concatenation(oracle):
    """A shared prompt cache in front of each sequence's own cache is the same as one cache holding
    both, when both are quantized against the same patterns."""
    cfg_own = _cfg(oracle, recent=0, flush=64, n_seq=2)
    cfg_pre = _cfg(oracle, recent=0, flush=64, n_seq=1)
    spec = synth.KVSpec(1, 2, 2, 4, 160, 128, 8)
    K, V = synth.make_kv(19, spec)
    Kp, Vp = K[:1, :, :64], V[:1, :, :64]                   # prompt of sequence 0 is the shared prefix
    M_k, _, _, _ = oracle.mine(K[0].view(np.uint16), 8, 2)
    M_v, _, _, _ = oracle.mine(V[0].view(np.uint16), 8, 2)
    pre = oracle.Cache(cfg_pre); pre.append(Kp.view(np.uint16), Vp.view(np.uint16), M_k, M_v)
    own = oracle.Cache(cfg_own); own.append(K[:, :, 64:].view(np.uint16), V[:, :, 64:].view(np.uint16), M_k, M_v)
    q = synth.make_queries(19, 2, 4, 128)
    out, _ = oracle.decode_attention(own, q.view(np.uint16), M_k, M_v, 128 ** -0.5, prefix=pre,
                                     prefix_patterns_k=M_k, prefix_patterns_v=M_v)
    K2 = K.copy(); V2 = V.copy(); K2[1, :, :64] = Kp[0]; V2[1, :, :64] = Vp[0]
    both = oracle.Cache(cfg_own); both.append(K2.view(np.uint16), V2.view(np.uint16), M_k, M_v)
    ref, _ = oracle.decode_attention(both, q.view(np.uint16), M_k, M_v, 128 ** -0.5)
    assert np.allclose(out, ref, rtol=1e-6, atol=1e-7)


def test_ragged_batch_is_attention_per_sequence(oracle):
    """A batch of sequences filled to different lengths: equal lengths give the uniform batch's result, and a
    sequence's rows are the plain softmax attention over exactly its own vectors (tail-only sequences, so the
    reference needs no quantizer), whatever the other sequences hold."""
    spec = synth.KVSpec(1, 3, 2, 4, 200, 128, 8)
    K, V = synth.make_kv(23, spec)
    M_k, _, _, _ = oracle.mine(K[0].view(np.uint16), 8, 2)
    M_v, _, _, _ = oracle.mine(V[0].view(np.uint16), 8, 2)
    q = synth.make_queries(23, 3, 4, 128)
    one = _cfg(oracle, recent=32, flush=64, n_seq=1)
    # equal lengths == the uniform batch
    uni = oracle.Cache(_cfg(oracle, recent=32, flush=64, n_seq=3))
    uni.append(K.view(np.uint16), V.view(np.uint16), M_k, M_v)
    per = []
    for i in range(3):
        c = oracle.Cache(one); c.append(K[i:i + 1].view(np.uint16), V[i:i + 1].view(np.uint16), M_k, M_v); per.append(c)
    ref, ref_lse = oracle.decode_attention(uni, q.view(np.uint16), M_k, M_v, 128 ** -0.5)
    out, lse = oracle.decode_attention_ragged(per, q.view(np.uint16), M_k, M_v, 128 ** -0.5)
    assert np.array_equal(out, ref) and np.array_equal(lse, ref_lse)
    # different lengths, short enough to stay in the fp16 tail: plain attention over each sequence's own vectors
    lens = [0, 17, 90]
    per = []
    for i, n in enumerate(lens):
        c = oracle.Cache(_cfg(oracle, recent=128, flush=64, n_seq=1))
        if n:
            c.append(K[i:i + 1, :, :n].view(np.uint16), V[i:i + 1, :, :n].view(np.uint16), M_k, M_v)
        assert c.t_quant == 0 and c.t_tail == n
        per.append(c)
    out, lse = oracle.decode_attention_ragged(per, q.view(np.uint16), M_k, M_v, 128 ** -0.5)
    assert np.all(out[0] == 0) and np.all(np.isneginf(lse[0]))
    Qd = q.astype(np.float64)
    for i, n in enumerate(lens):
        for h in range(4):
            if n == 0:
                continue
            sc = K[i, h // 2, :n].astype(np.float64) @ Qd[i, h] * 128 ** -0.5
            p = np.exp(sc - sc.max()); p /= p.sum()
            assert np.allclose(out[i, h], p @ V[i, h // 2, :n].astype(np.float64), rtol=1e-6, atol=1e-7)
            assert abs(lse[i, h] - (sc.max() + np.log(np.exp(sc - sc.max()).sum()))) < 1e-5


@pytest.mark.parametrize("n_seq,hkv,k,expected", [
    # streams in order (sequence-major, then KV head) -> the pattern table each one must use, written out by hand
    (3, 2, 0, [0, 1, 0, 1, 0, 1]),                               # one table per KV head, shared by all sequences
    (3, 2, 1, [0, 1, 2, 3, 4, 5]),                               # one table per (sequence, head)
    (6, 2, 3, [0, 1, 0, 1, 0, 1, 2, 3, 2, 3, 2, 3]),             # 2 layers x batch 3: one table per (layer, head)
    (7, 1, 3, [0, 0, 0, 1, 1, 1, 2]),                            # a last, partly filled set
])
def test_stream_to_pattern_set_mapping(oracle, n_seq, hkv, k, expected):
    """Which table a stream is quantized against (seqs_per_set).  Made visible through the stored zero points:
    all vectors are zero, table s holds the single pattern (s+1, s+1, ...), so every residual is -(s+1), the group's
    minimum - and with it the stored K zero point and V zero point - names the table that was used."""
    d, G = 128, 64
    cfg = oracle.Config(n_seq=n_seq, n_kv_heads=hkv, n_q_heads=hkv, head_dim=d, n_patterns=1, seqs_per_set=k, bits=2,
                        group=G, recent=0, flush=64, t_capacity=64, metric=0)
    n_sets = len(set(expected))
    assert cfg.n_sets == n_sets
    tables = np.empty((n_sets, 1, d), np.float16)
    for s in range(n_sets):
        tables[s] = s + 1
    zeros = np.zeros((n_seq, hkv, 64, d), np.uint16)
    c = oracle.Cache(cfg)
    c.append(zeros, zeros, tables.view(np.uint16), tables.view(np.uint16))
    zk = c.k_zero[:, 0, :].view(np.float16).astype(np.float64)              # [streams, d]
    zv = c.v_zero[:, 0].view(np.float16).astype(np.float64)                 # [streams, groups, 16 tokens]
    for n, s in enumerate(expected):
        assert np.all(zk[n] == -(s + 1)) and np.all(zv[n] == -(s + 1)), (n, s)
    # and the reconstruction with the same tables gives the zero vectors back
    kh, vh = c.dequantize(tables.view(np.uint16), tables.view(np.uint16))
    assert not kh.any() and not vh.any()


# ---------------------------------------------------------------- head dimensions 96 and 256

@pytest.mark.parametrize("d,G", [(96, 32), (96, 128), (256, 64), (256, 128)])
@pytest.mark.parametrize("bits", [2, 4])
def test_other_head_dimensions_quantizer_and_format(oracle, d, G, bits):
    """The oracle at the other head sizes of Sec. 3.3: with a zero pattern both quantizers are the textbook asymmetric
    quantizer (numpy, written separately) over K's token groups and V's channel groups of min(G, d); the packed
    words follow the stated index formulas (hand-worked probes in tests/golden/pack_format_other_d.txt) and
    round-trip."""
    rng = np.random.default_rng(40 + d + G + bits)
    n = 256
    x = f16(rng.standard_normal((1, n, d)) * np.exp(rng.standard_normal((1, 1, d))))
    M = np.zeros((1, 1, d), np.uint16)
    set_of = np.zeros(1, np.int32)
    rk = oracle.quantize_streams(x.view(np.uint16), set_of, M, 0, bits, G, 0, want_codes=True)
    rv = oracle.quantize_streams(x.view(np.uint16), set_of, M, 0, bits, G, 1, want_codes=True)
    r = x[0].astype(np.float32)
    qk, sk, zk = _numpy_asym_quant(r.reshape(n // G, G, d), bits, axis=1)
    assert np.array_equal(rk["codes"][0], qk.reshape(n, d))
    assert np.array_equal(rk["scale"][0], sk.reshape(n // G, d).view(np.uint16))
    assert np.array_equal(rk["zero"][0], zk.reshape(n // G, d).view(np.uint16))
    Gc = min(G, d)
    qv, sv, zv = _numpy_asym_quant(r.reshape(n, d // Gc, Gc), bits, axis=2)
    assert np.array_equal(rv["codes"][0], qv.reshape(n, d))
    assert np.array_equal(oracle.v_params_by_token(rv["scale"][0]), sv.reshape(n, d // Gc).view(np.uint16))
    assert np.array_equal(oracle.v_params_by_token(rv["zero"][0]), zv.reshape(n, d // Gc).view(np.uint16))
    # format
    codes = rk["codes"][0][:48]
    wk, wv = oracle.pack_k(codes, bits), oracle.pack_v(codes, bits)
    assert wk.nbytes == wv.nbytes == 48 * d * bits // 8
    assert np.array_equal(oracle.unpack_k(wk, 48, d, bits), codes) and np.array_equal(oracle.unpack_v(wv, 48, d, bits), codes)
    probed = 0
    for line in open(os.path.join(GOLDEN, "pack_format_other_d.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        side, b, dd, t, c, j, unit, bit = line.split()
        if int(b) != bits or int(dd) != d:
            continue
        one = np.zeros((48, d), np.uint8)
        one[int(t), int(c)] = 1 << int(j)
        w = (oracle.pack_k(one, bits) if side == "K" else oracle.pack_v(one, bits)).reshape(-1)
        assert w.dtype == np.uint32 and np.flatnonzero(w).tolist() == [int(unit)] and w[int(unit)] == 1 << int(bit)
        probed += 1
    assert probed == 2


@pytest.mark.parametrize("d,G", [(96, 32), (256, 128)])
def test_other_head_dimensions_attention_matches_torch_sdpa(oracle, d, G):
    """Decode over a cache with a packed part, a tail and a shared prefix at head dimensions 96 and 256 equals
    torch's scaled_dot_product_attention over the reconstructed keys and values."""
    import torch
    cfg = _cfg(oracle, head_dim=d, group=G, flush=128, recent=16, t_capacity=512)
    spec = synth.KVSpec(1, cfg.n_seq, cfg.n_kv_heads, cfg.n_q_heads, 300, d, 8)
    K, V = synth.make_kv(41, spec)
    M_k, _, _, _ = oracle.mine(K[0].view(np.uint16), cfg.n_patterns, 2)
    M_v, _, _, _ = oracle.mine(V[0].view(np.uint16), cfg.n_patterns, 2)
    c = oracle.Cache(cfg)
    c.append(K.view(np.uint16), V.view(np.uint16), M_k, M_v)
    assert c.t_quant == 256 and c.t_tail == 44
    q = synth.make_queries(41, cfg.n_seq, cfg.n_q_heads, d)
    out, lse = oracle.decode_attention(c, q.view(np.uint16), M_k, M_v, d ** -0.5)
    Kh, Vh = c.materialize(M_k, M_v)
    Kh = torch.from_numpy(Kh).reshape(2, 2, 300, d).repeat_interleave(2, dim=1).double()
    Vh = torch.from_numpy(Vh).reshape(2, 2, 300, d).repeat_interleave(2, dim=1).double()
    Q = torch.from_numpy(q.astype(np.float64)).reshape(2, 4, 1, d)
    ref = torch.nn.functional.scaled_dot_product_attention(Q, Kh, Vh, scale=d ** -0.5)
    assert np.allclose(out, ref.reshape(2, 4, d).numpy(), rtol=1e-5, atol=1e-6)
    ref_lse = torch.logsumexp((Q @ Kh.transpose(-1, -2)) * d ** -0.5, dim=-1).reshape(2, 4).numpy()
    assert np.allclose(lse, ref_lse, rtol=1e-6)
    # the reconstruction stays close to the source
    Kf = torch.from_numpy(K.astype(np.float64)).repeat_interleave(2, dim=1)
    Vf = torch.from_numpy(V.astype(np.float64)).repeat_interleave(2, dim=1)
    full = torch.nn.functional.scaled_dot_product_attention(Q, Kf, Vf, scale=d ** -0.5).reshape(2, 4, d).numpy()
    assert np.linalg.norm(out - full) / np.linalg.norm(full) < 0.35
