"""Pins for the oracle's general operands (per-group zero points), the Eq. 4 clip and the
two-phase grid search of Section 3.3 (no GPU).  None of them goes through the oracle's own
formulas: constructed inputs that must be recovered exactly, brute force over every
(S2, ZP, u), hand-worked values and offsets, special cases that reduce to already pinned
routines, and an independent slow search on tiny inputs."""
import json
import os

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


# ---------------------------------------------------------------- Eq. 2 with a zero point
def test_expand_zp_hand_values():
    # S2 * (u - ZP), worked by hand: 9*(3-11) = -72, 127*(1-0) = 127, 15*(15-8) = 105, 1*(0-15) = -15
    u4 = np.array([[3, 1, 15, 0]], np.uint8).repeat(4, axis=0)
    s2 = np.array([[9, 127, 15, 1]], np.uint8)
    zp = np.array([[11, 0, 8, 15]], np.uint8)
    ws8, bad = oracle.expand_zp(u4, s2, zp, 4)
    assert bad == 0 and (ws8 == np.array([-72, 127, 105, -15], np.int8)).all()


def test_expand_zp_counts_and_saturates_overflow():
    u4 = np.array([[15, 0]], np.uint8).repeat(2, axis=0)
    ws8, bad = oracle.expand_zp(u4, np.array([[20, 20]], np.uint8), np.array([[0, 15]], np.uint8), 2)
    assert bad == 4 and (ws8[:, 0] == 127).all() and (ws8[:, 1] == -128).all()     # 300 and -300


def test_expand_zp_with_zero_point_8_is_the_signed_nibble_form():
    rng = np.random.default_rng(1)
    w4 = rng.integers(-8, 8, (256, 48), dtype=np.int8)
    s2 = rng.integers(1, 16, (4, 48), dtype=np.uint8)
    ref, _ = oracle.expand(w4, s2, 64)                               # pinned in test_oracle_pins.py
    got, bad = oracle.expand_zp((w4 + 8).astype(np.uint8), s2, np.full_like(s2, 8), 64)
    assert bad == 0 and np.array_equal(ref, got)


def test_expand_zp_shift_identity():
    # moving the zero point by d moves every expanded weight of the group by -S2*d
    rng = np.random.default_rng(2)
    u4 = rng.integers(0, 16, (128, 16), dtype=np.uint8)
    s2 = rng.integers(1, 5, (2, 16), dtype=np.uint8)
    a, _ = oracle.expand_zp(u4, s2, np.full_like(s2, 3), 64)
    b, _ = oracle.expand_zp(u4, s2, np.full_like(s2, 9), 64)
    assert np.array_equal(a.astype(int) - b.astype(int), 6 * np.repeat(s2.astype(int), 64, axis=0))


# ---------------------------------------------------------------- Eq. 4
def test_clip_interval_brute_force():
    """u is inside the interval exactly when S2*(u-ZP) fits [-127, 127] (and u is a nibble)."""
    for s2 in range(1, 128):
        for zp in range(16):
            lo, hi = oracle.clip_interval(s2, zp)
            ok = [u for u in range(16) if abs(s2 * (u - zp)) <= 127]
            assert ok == list(range(lo, hi + 1)), (s2, zp)
            assert lo <= zp <= hi                                    # zero is always representable


# ---------------------------------------------------------------- format
def test_pack_zp_offsets_match_hand_computed_golden():
    cases = json.load(open(os.path.join(HERE, "golden", "layout_offsets_zp.json")))["cases"]
    for c in cases:
        K, N, g = c["K"], c["N"], c["group"]
        u4 = np.zeros((K, N), np.uint8)
        s2 = np.ones((K // g, N), np.uint8)
        zp = np.zeros((K // g, N), np.uint8)
        s2[c["gi"], c["n"]], zp[c["gi"], c["n"]] = 77, 13
        u4[c["gi"] * g:(c["gi"] + 1) * g, c["n"]] = 13              # zero weights: 77*(13-13) = 0
        _, sc, bad = oracle.pack_zp(u4, s2, zp, g)
        assert bad == 0
        assert sc[c["s2_offset"]] == 77 and sc[c["s2_offset"] + 1] == 13, c
        assert (sc == 77).sum() == 1 and (sc == 13).sum() == 1


def test_pack_zp_nibbles_equal_the_signed_format_and_round_trip():
    rng = np.random.default_rng(3)
    K, N, g = 384, 48, 128
    w4 = rng.integers(-8, 8, (K, N), dtype=np.int8)
    s2 = rng.integers(1, 16, (K // g, N), dtype=np.uint8)
    q1, _, _ = oracle.pack(w4, s2, g)                                # pinned against golden offsets
    q2, sc, bad = oracle.pack_zp((w4 + 8).astype(np.uint8), s2, np.full_like(s2, 8), g)
    assert bad == 0 and np.array_equal(q1, q2)
    zp = rng.integers(6, 10, (K // g, N), dtype=np.uint8)
    u4 = rng.integers(0, 16, (K, N), dtype=np.uint8)
    q, sc, bad = oracle.pack_zp(u4, np.minimum(s2, 12), zp, g)       # 12*9 = 108 fits
    assert bad == 0
    ru, rs, rz = oracle.unpack_zp(q, sc, K, N, g)
    assert np.array_equal(ru, u4) and np.array_equal(rs, np.minimum(s2, 12)) and np.array_equal(rz, zp)
    assert sc.size == (N // 16) * 2 * 64                             # ng = 3 padded to 4 entries
    pad = sc.reshape(N // 16, 2, 16, 2, 2)[:, 1, :, 1, :]            # entry gi = 3 does not exist
    assert (pad == 0).all()


def test_pack_zp_counts_rule_breakers():
    K, N, g = 128, 16, 64
    u4 = np.zeros((K, N), np.uint8)
    s2 = np.ones((2, N), np.uint8)
    zp = np.zeros((2, N), np.uint8)
    s2[0, 0] = 0            # scale below 1
    s2[1, 1] = 128          # scale above 127
    zp[0, 2] = 16           # zero point above 15
    u4[5, 3] = 16           # not a nibble
    s2[1, 4], u4[70, 4] = 20, 7      # 140 > 127
    q, sc, bad = oracle.pack_zp(u4, s2, zp, g)
    assert bad == 5
    ru, rs, rz = oracle.unpack_zp(q, sc, K, N, g)
    assert rs[0, 0] == 1 and rs[1, 1] == 1 and rz[0, 2] == 0 and ru[5, 3] == 0 and ru[70, 4] == 0


# ---------------------------------------------------------------- grid search
def _constructed(seed, K=256, N=8, g=64):
    """Weights that are exactly s1*S2*(u-ZP) with every group using nibbles 0 and 15, S2*max|u-ZP| <= 127
    and the largest S2 of each column equal to 15: both phases must find alpha = 1 with zero error."""
    rng = np.random.default_rng(seed)
    ng = K // g
    s1 = (2.0 ** rng.integers(-12, -6, N)).astype(np.float32)
    s2 = rng.integers(8, 16, (ng, N)).astype(np.uint8)
    s2[rng.integers(0, ng, N), np.arange(N)] = 15
    room = 127 // s2.astype(int)                                     # largest |u - ZP| allowed
    zlo, zhi = 15 - room, room                                       # 15-ZP <= room and ZP <= room
    assert (zlo <= zhi).all()
    zp = (zlo + (rng.random((ng, N)) * (zhi - zlo + 1)).astype(int)).astype(np.uint8)
    u4 = rng.integers(0, 16, (K, N)).astype(np.uint8)
    for j in range(ng):
        for n in range(N):
            rows = rng.choice(g, 2, replace=False) + j * g
            u4[rows[0], n], u4[rows[1], n] = 0, 15
    W = (u4.astype(np.float32) - np.repeat(zp, g, axis=0).astype(np.float32)) * \
        (np.repeat(s2, g, axis=0).astype(np.float32) * s1[None, :])
    return W, u4, zp, s2, s1


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_grid_search_recovers_exactly_representable_weights(seed):
    W, u4, zp, s2, s1 = _constructed(seed)
    for g in (64,):
        gu, gz, gs2, gs1 = oracle.quantize_weights_grid(W, g, n_alpha=11, step=0.05)
        assert np.array_equal(gz, zp) and np.array_equal(gs2, s2) and np.array_equal(gs1, s1)
        assert np.array_equal(gu, u4)


def _slow_search(W, g, alphas):
    """Independent, slow restatement of Section 3.3 on one column (float32 numpy scalars)."""
    f = np.float32
    K = W.shape[0]
    ng = K // g
    Sp, Z = [], []
    for j in range(ng):
        w = W[j * g:(j + 1) * g]
        lo, hi = min(f(0), w.min()), max(f(0), w.max())
        cand = []
        for a in alphas:
            s = f(f(a * f(hi - lo)) / f(15))
            z = f(np.clip(np.rint(f(-(f(a * lo))) / s), 0, 15))
            u = np.clip(np.rint(w / s) + z, 0, 15).astype(f)
            d = (w - (u - z) * s).astype(f)
            e = f(0)
            for v in d:
                e = f(e + f(v * v))
            cand.append((e, s, int(z)))
        e, s, z = min(cand, key=lambda t: t[0])                       # min() keeps the first of equals
        Sp.append(s), Z.append(z)
    smax = max(Sp)
    best = None
    for a in alphas:
        c1 = f(f(a * smax) / f(15))
        e = f(0)
        U, S2 = [], []
        for j in range(ng):
            q2 = int(np.clip(np.rint(f(Sp[j] / c1)), 1, 127))
            S = f(c1 * f(q2))
            r = 127 // q2
            lo4, hi4 = max(0, Z[j] - r), min(15, Z[j] + r)
            w = W[j * g:(j + 1) * g]
            u = np.clip(np.rint(w / S) + f(Z[j]), lo4, hi4).astype(f)
            for v in (w - (u - f(Z[j])) * S).astype(f):
                e = f(e + f(v * v))
            U.append(u.astype(np.uint8)), S2.append(q2)
        if best is None or e < best[0]:
            best = (e, c1, S2, np.concatenate(U))
    return best[3], np.array(Z, np.uint8), np.array(best[2], np.uint8), best[1]


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_grid_search_equals_an_independent_slow_search_on_tiny_inputs(seed):
    rng = np.random.default_rng(100 + seed)
    K, N, g = 32, 3, 8
    W = rng.normal(0, 0.02, (K, N)).astype(np.float16).astype(np.float32)
    W[rng.integers(0, K, 2), rng.integers(0, N, 2)] *= 6             # outliers make clipping pay
    alphas = [np.float32(1.0) - np.float32(i) * np.float32(0.05) for i in range(9)]
    u4, zp, s2, s1 = oracle.quantize_weights_grid(W, g, n_alpha=9, step=0.05)
    for n in range(N):
        su, sz, ss2, ss1 = _slow_search(W[:, n].copy(), g, alphas)
        assert np.array_equal(zp[:, n], sz) and np.array_equal(s2[:, n], ss2) and s1[n] == ss1
        assert np.array_equal(u4[:, n], su)


def test_grid_search_invariants_and_error_bounds():
    rng = np.random.default_rng(5)
    K, N, g = 512, 64, 128
    W = rng.normal(0, 0.02, (K, N)).astype(np.float16).astype(np.float32)
    W[:, 7] = 0                                                      # an all-zero column
    W[128:256, 9] = 0                                                # an all-zero group
    W[:, 11] = np.abs(W[:, 11])                                      # one-sided groups: ZP = 0
    u4, zp, s2, s1 = oracle.quantize_weights_grid(W, g)
    assert u4.max() <= 15 and zp.max() <= 15 and s2.min() >= 1 and s2.max() <= 127
    ws8, bad = oracle.expand_zp(u4, s2, zp, g)
    assert bad == 0 and np.abs(ws8.astype(int)).max() <= 127         # Eq. 4 did its job
    assert s1[7] == 1 and (u4[:, 7] == 0).all() and (zp[:, 7] == 0).all()
    assert (ws8[128:256, 9] == 0).all() and (zp[:, 11] == 0).all()
    deq = ws8.astype(np.float64) * s1[None, :]
    S = np.repeat(s2, g, axis=0) * s1[None, :].astype(np.float64)
    inner = (u4 > 0) & (u4 < 15)                                     # not at the end of the nibble range
    lo_hi = np.array([[oracle.clip_interval(int(a), int(b)) for a, b in zip(r1, r2)] for r1, r2 in zip(s2, zp)])
    lo = np.repeat(lo_hi[:, :, 0], g, axis=0)
    hi = np.repeat(lo_hi[:, :, 1], g, axis=0)
    inner &= (u4 > lo) & (u4 < hi)
    assert (np.abs(W - deq)[inner] <= 0.5 * S[inner] * (1 + 1e-5)).all()   # round to nearest: half a step


def test_grid_search_beats_direct_rounding_on_gaussian_weights():
    """Direction of Table 1: direct rounding into (s1, S2) loses accuracy, the search recovers it."""
    rng = np.random.default_rng(6)
    K, N, g = 1024, 96, 128
    W = rng.normal(0, 0.02, (K, N)).astype(np.float16).astype(np.float32)

    def mse(ws8, s1):
        return float(((W - ws8.astype(np.float32) * s1[None, :]) ** 2).mean())
    u4, zp, s2, s1 = oracle.quantize_weights_grid(W, g)
    e_grid = mse(oracle.expand_zp(u4, s2, zp, g)[0], s1)
    u1, z1, s21, s11 = oracle.quantize_weights_grid(W, g, n_alpha=1)
    e_minmax = mse(oracle.expand_zp(u1, s21, z1, g)[0], s11)
    w4, r2, r1 = oracle.quantize_weights_rtn(W, g)
    e_rtn = mse(oracle.expand(w4, r2, g)[0], r1)
    assert e_grid < e_minmax and e_grid < e_rtn


# ---------------------------------------------------------------- Eq. 6 smoothing
def test_smooth_scales_hand_example():
    # 400 channels, pct 0.5 % -> r = 2: the threshold is the second largest channel maximum.
    # Channel maxima: 40 at j=7, 10 at j=3, 4 at j=11, 2 elsewhere -> t = 10, k = 4 at j=7, 1 everywhere else
    X = np.full((3, 400), 2.0, np.float32)
    X[1, 7], X[2, 3], X[0, 11] = -40.0, 10.0, 4.0
    k = oracle.smooth_scales(X, 0.005)
    assert k[7] == 4.0 and (np.delete(k, 7) == 1.0).all()


def test_smooth_scales_properties_and_product_is_preserved():
    rng = np.random.default_rng(12)
    M, K, N = 64, 4096, 32
    X = rng.normal(0, 1, (M, K)).astype(np.float32)
    hot = rng.choice(K, 41, replace=False)
    X[:, hot] *= 20                                                   # 1 % outlier channels
    k = oracle.smooth_scales(X, 0.005)
    r = int(np.ceil(0.005 * K))
    z = np.abs(X).max(axis=0)
    assert (k >= 1).all() and (k > 1).sum() == r - 1                  # strictly above the r-th largest
    assert set(np.nonzero(k > 1)[0]) <= set(hot)
    assert np.isclose((z / k).max(), np.sort(z)[-r])                  # outliers are clipped to the threshold
    W = rng.normal(0, 0.02, (K, N)).astype(np.float32)
    lhs = (X.astype(np.float64) / k) @ (W.astype(np.float64) * k[:, None])
    assert np.allclose(lhs, X.astype(np.float64) @ W.astype(np.float64), rtol=1e-12, atol=1e-12)
    Wo, Xo = oracle.smooth_apply(W, X, k)
    assert np.array_equal(Wo, (W * k[:, None]).astype(np.float16)) and np.array_equal(Xo[:, k == 1], X[:, k == 1].astype(np.float16))


def test_smooth_apply_hand_values():
    """Section 3.4: the scale leaves the activations (X / k) and enters the weights (k * W).  Hand values with a
    channel whose scale is above 1, so that a swapped direction, a transposed index or a missing rounding shows:
    channel 1 has k = 4: X 6 -> 1.5, W 0.25 -> 1.0; channel 2 has k = 3: X 1 -> 1/3 (rounded once to fp16)."""
    k = np.array([1.0, 4.0, 3.0], np.float32)
    X = np.array([[2.0, 6.0, 1.0], [-8.0, -0.5, 9.0]], np.float32)
    W = np.array([[5.0, -7.0], [0.25, 0.5], [-1.0, 0.125]], np.float32)
    Wo, Xo = oracle.smooth_apply(W, X, k)
    assert Wo.dtype == np.float16 and Xo.dtype == np.float16
    assert Xo.tolist() == [[2.0, 1.5, float(np.float16(1.0 / 3.0))], [-8.0, -0.125, 3.0]]
    assert Wo.tolist() == [[5.0, -7.0], [1.0, 2.0], [-3.0, 0.375]]
    # the product of Eq. 2's operands is what the transfer preserves (here exactly: all factors are small integers
    # over powers of two except the thirds, which are left out)
    assert np.array_equal(Xo[:, :2].astype(np.float64) @ Wo[:2].astype(np.float64), X[:, :2].astype(np.float64) @ W[:2].astype(np.float64))


def test_smooth_scales_without_activations_is_the_identity():
    assert (oracle.smooth_scales(np.zeros((2, 256), np.float32)) == 1).all()


# ---------------------------------------------------------------- Eq. 3 with calibration activations
def test_activation_weighted_search_with_identity_activations_is_the_weight_only_search():
    """X = X^ = I makes ||X W - X^ Q(W)||^2 the weight-only objective term by term (the other products are
    exact zeros), so the result must equal the already pinned weight-only search bit for bit."""
    rng = np.random.default_rng(31)
    K, N, g = 64, 24, 16
    W = rng.normal(0, 0.02, (K, N)).astype(np.float32)
    W[:, 3] = 0
    W[16:32, 5] = 0
    I = np.eye(K, dtype=np.float32)
    a = oracle.quantize_weights_grid_act(W, I, g, n_alpha=21, step=0.025, Xh=I)
    b = oracle.quantize_weights_grid(W, g, n_alpha=21, step=0.025)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_activation_weighted_search_hand_worked_flip():
    """One group of two weights (1.0, 0.1), alpha in {1, 0.5}, one calibration token that only excites channel 1.
    Weight-only: alpha = 1 keeps 1.0 exact (s = 1/15, u = (15, 2), error 0.0011 on the small weight) and wins.
    With the activations only the small weight counts: alpha = 0.5 gives s = 1/30, u = (15, 3): 3/30 = 0.1 exactly,
    error 0, and wins phase 1 (S' = 1/30).  Phase 2 at alpha = 1: s1 = S'/15 = 1/450, S2 = 15, the Eq. 4 clip of
    S2 = 15, ZP = 0 is [0, 8], so u = (8, 3), error 0 again."""
    W = np.array([[1.0], [0.1]], np.float32)
    X = np.array([[0.0, 1.0]], np.float32)
    u4, zp, s2, s1 = oracle.quantize_weights_grid_act(W, X, 2, n_alpha=2, step=0.5, Xh=X)
    assert u4[:, 0].tolist() == [8, 3] and zp[0, 0] == 0 and s2[0, 0] == 15
    assert abs(s1[0] * 450 - 1) < 1e-6
    wu, wz, ws2, ws1 = oracle.quantize_weights_grid(W, 2, n_alpha=2, step=0.5)
    assert abs(ws1[0] * 225 - 1) < 1e-6 and wu[:, 0].tolist() == [8, 2]     # the weight-only search keeps alpha = 1


def test_activation_weighted_search_recovers_representable_weights_and_lowers_the_output_error():
    rng = np.random.default_rng(32)
    # weights that are exactly s1 * S2 * (u - ZP) (the construction of the weight-only pin): with X^ = X the
    # error zero is reachable at alpha = 1 in both phases and nothing else can beat it, whatever X is
    W, u4, zp, s2, s1 = _constructed(5)
    K, N = W.shape
    g, M = 64, 40
    X = rng.normal(0, 1, (M, K)).astype(np.float32)
    X[:, rng.choice(K, 4, replace=False)] *= 20
    gu, gz, gs2, gs1 = oracle.quantize_weights_grid_act(W, X, g, n_alpha=11, step=0.05, Xh=X)
    assert np.array_equal(gz, zp) and np.array_equal(gs2, s2) and np.array_equal(gs1, s1) and np.array_equal(gu, u4)
    # on Gaussian weights the activation-weighted search gives a smaller output error than the weight-only one
    Xh = oracle.dequant_act(X)
    Wg = rng.normal(0, 0.02, (K, N)).astype(np.float32)
    ref = X.astype(np.float64) @ Wg.astype(np.float64)

    def out_err(res):
        a4, az, a2, a1 = res
        d = a1[None, :].astype(np.float64) * np.repeat(a2, g, 0) * (a4.astype(np.float64) - np.repeat(az, g, 0))
        return np.linalg.norm(Xh.astype(np.float64) @ d - ref)
    assert out_err(oracle.quantize_weights_grid_act(Wg, X, g)) < out_err(oracle.quantize_weights_grid(Wg, g))
