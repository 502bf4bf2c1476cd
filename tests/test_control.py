"""Control-plane formulas (predictor Eq. 1-3, prewarming scores, placement Alg. 1):
pins for the plain-Python oracle, then the library against it.  Host arithmetic
in double precision only; no GPU involved.

Tolerances: the predictor is at most D + N*(D+1) <= 87 additions and one
division on values of magnitude |L|; the library sums left to right, the oracle
with correctly rounded sums, so they differ by at most ~100 ulp of max|L|:
1e-12 * max|L| is used.  Scores are one exp, one division and two products in the
same order on both sides (same libm): compared to 4 ulp.  Placement decisions are
integers decided in double precision on both sides: compared exactly."""
import math

import numpy as np
import pytest

import paper_2512_09472_amd as wk
from oracle import control as oc


# ------------------------------------------------------------ oracle pins
def test_predictor_closed_forms():
    D, N, W = 7, 10, 24
    const = [[5.0] * W for _ in range(9)]
    assert oc.predict(const, 8, 13, D, N) == 5.0
    pattern = [[100 + 10 * math.sin(j) for j in range(W)] for _ in range(9)]
    for i in (0, 1, 5, 23):
        assert oc.predict(pattern, 8, i, D, N) == pytest.approx(pattern[0][i], abs=1e-12)
    # today runs e above the pattern in every window: the normalised weights give Delta = e
    e = 3.25
    shifted = [row[:] for row in pattern]
    shifted[8] = [v + e for v in pattern[8]]
    for i in (1, 4, 10, 17):
        assert oc.predict(shifted, 8, i, D, N) == pytest.approx(pattern[0][i] + e, abs=1e-11)
    assert oc.predict(shifted, 8, 0, D, N) == pytest.approx(pattern[0][0], abs=1e-12)   # no window before the first


def test_predictor_hand_case_and_lookback():
    # D = 2, seasonal terms 10 everywhere; today's errors e1 (window i-1) and e2 (window i-2):
    # Delta = (e1 * 1 + e2 * 2) / 3, as printed in Eq. 2
    hist = [[10.0] * 6, [10.0] * 6, [10.0, 16.0, 13.0, 0, 0, 0]]
    assert oc.predict(hist, 2, 3, D=2, N=2) == pytest.approx(10 + (3.0 * 1 + 6.0 * 2) / 3)
    assert oc.predict(hist, 2, 3, D=2, N=10) == pytest.approx(10 + (3.0 * 1 + 6.0 * 2 + 0.0 * 4) / 7)   # m = min(3, 10)
    assert oc.predict(hist, 2, 3, D=2, N=1) == pytest.approx(10 + 3.0)          # only the last window
    far = [row[:] for row in hist]
    far[2][0] = 1000.0                                                           # window i-3
    assert oc.predict(far, 2, 3, D=2, N=2) == oc.predict(hist, 2, 3, D=2, N=2)  # outside the lookback
    assert oc.predict(far, 2, 3, D=2, N=3) != oc.predict(hist, 2, 3, D=2, N=3)
    # seasonal term is the mean over exactly D days
    hist2 = [[99.0] * 3, [4.0] * 3, [8.0] * 3, [0.0] * 3]
    assert oc.predict(hist2, 3, 0, D=2, N=10) == 6.0
    assert oc.predict(hist2, 3, 0, D=3, N=10) == pytest.approx(37.0)


def test_scores_hand_case():
    # K = 1, B = 32, L_A = 70 -> ceil = 3 -> 2 basic; L_P = 150 -> ceil = 5 -> 5 - 2 - 1 = 2 burst
    nb, nu, s = oc.replica_scores(70.0, 150.0, 32, 1, 20.0)
    assert (nb, nu) == (2, 2)
    want = [20.0, math.exp(-0.25) * 20.0, math.exp(-0.5) * 20.0 * 80 / 70, math.exp(-0.75) * 20.0 * 80 / 70]
    assert s == pytest.approx(want, rel=1e-15)
    assert oc.replica_scores(70.0, 150.0, 32, 5, 20.0)[:2] == (0, 0)             # enough instances already
    assert oc.replica_scores(0.0, 40.0, 32, 0, 2.0) == (0, 2, [math.inf, math.inf])
    for L_A, L_P, B, K in ((10, 10, 4, 0), (33, 64, 32, 1), (1, 1000, 7, 3)):
        nb, nu, s = oc.replica_scores(L_A, L_P, B, K, 1.0)
        assert nb + nu == max(math.ceil(L_P / B) - K, 0)                          # Alg. 1's replica count
        assert all(a >= b for a, b in zip(s[:nb], s[1:nb])) and all(a >= b for a, b in zip(s[nb:], s[nb + 1:]))


def _model(S, D, B, K, L_A, L_P, T_c):
    return dict(S=S, D=D, B=B, K=K, L_A=L_A, L_P=L_P, T_c=T_c)


def test_placement_hand_case():
    # one server of 4 GPUs.  A: degree 2, one basic replica, score 10.  B: degree 1, two basic
    # replicas, scores 5 and 5*exp(-1/2).  C: degree 1, one basic replica, score 1.
    A = _model(40, 2, 10, 0, 10, 10, 10.0)
    B = _model(10, 1, 10, 0, 20, 20, 5.0)
    C = _model(10, 1, 10, 0, 10, 10, 1.0)
    free = [100.0] * 4
    got = oc.place([A, B, C], free, 4)
    assert [(m, r, g) for m, r, g, _, _ in got] == [(0, 0, 0),   # A: all groups untouched, lowest index
                                                    (1, 0, 2),   # B#0: GPUs 0,1 hold a higher score; 2 and 3 are untouched
                                                    (1, 1, 3),   # B#1: only GPU 3 holds nothing higher
                                                    (2, 0, 3)]   # C: nothing to isolate from; least sum is GPU 3 (3.03)
    assert free == [80.0, 80.0, 90.0, 80.0]
    # no room: the replica is skipped, later ones still placed
    free = [100.0, 100.0, 5.0, 5.0]
    got = oc.place([_model(300, 2, 10, 0, 10, 10, 9.0), C], free, 4)
    assert [(m, r, g) for m, r, g, _, _ in got] == [(1, 0, 0)]
    # basic replicas outrank burst replicas whatever their scores
    X = _model(10, 1, 10, 0, 10, 10, 1.0)          # one basic, score 1
    Y = _model(10, 1, 10, 1, 10, 100, 50.0)        # nine burst, large scores
    got = oc.place([Y, X], [100.0] * 4, 4)
    assert got[0][0] == 1 and got[0][3] == 0 and all(b == 1 for _, _, _, b, _ in got[1:])


def _check_placement_invariants(models, free0, free1, gps, placed):
    for a in range(len(placed)):
        ma, _, ga, _, _ = placed[a]
        Da = models[ma]["D"]
        assert ga % Da == 0 and ga // gps == (ga + Da - 1) // gps, "aligned, one server"
        for b in range(a):
            mb, _, gb, _, _ = placed[b]
            Db = models[mb]["D"]
            sa, sb = set(range(ga, ga + Da)), set(range(gb, gb + Db))
            assert not (sa & sb) or sa <= sb or sb <= sa, "no partial overlap"
    used = [0.0] * len(free0)
    for m, _, g, _, _ in placed:
        for j in range(g, g + models[m]["D"]):
            used[j] += math.ceil(models[m]["S"] / models[m]["D"])
    assert all(abs(f0 - u - f1) < 1e-6 and f1 >= 0 for f0, u, f1 in zip(free0, used, free1))
    order = [(b, -s) for _, _, _, b, s in placed]
    assert order == sorted(order), "basic first, then by score"


def _random_models(rs, n):
    out = []
    for _ in range(n):
        L_A = float(rs.integers(0, 200))
        out.append(_model(float(rs.integers(1, 60)) * 1e9, int(rs.choice([1, 2, 4])), int(rs.choice([8, 16, 32])),
                          int(rs.integers(0, 3)), L_A, L_A + float(rs.integers(0, 150)), float(rs.integers(1, 40))))
    return out


def test_placement_invariants_on_random_clusters():
    rs = np.random.default_rng(0)
    for _ in range(60):
        models = _random_models(rs, int(rs.integers(1, 6)))
        gps = 8
        free0 = [float(rs.integers(0, 80)) * 1e9 for _ in range(16)]
        free1 = free0[:]
        placed = oc.place(models, free1, gps)
        _check_placement_invariants(models, free0, free1, gps, placed)


# ------------------------------------------------- library against the oracle
def test_library_predictor_matches_oracle():
    rs = np.random.default_rng(1)
    for _ in range(200):
        D, N = int(rs.integers(1, 9)), int(rs.integers(0, 14))
        days, W = D + int(rs.integers(1, 4)), int(rs.integers(1, 40))
        hist = rs.random((days, W)) * float(rs.choice([1.0, 1e3, 1e6]))
        k, i = int(rs.integers(D, days)), int(rs.integers(0, W))
        want = oc.predict(hist.tolist(), k, i, D, N)
        assert wk.ws_predict_load(hist, k, i, D, N) == pytest.approx(want, abs=1e-12 * hist.max(), rel=0)
    h = np.ones((8, 4))
    for args in ((7, 4), (8, 0), (6, 0)):                       # window / day out of range, too few days
        with pytest.raises(wk.WarmKVError):
            wk.ws_predict_load(h, *args, 7, 10)
    assert wk.ws_predict_load(h, 7, 3, 7, 10) == 1.0


def test_library_scores_match_oracle():
    rs = np.random.default_rng(2)
    for _ in range(300):
        L_A = float(rs.integers(0, 500)) / 2
        L_P = L_A + float(rs.integers(0, 900)) / 2
        B, K, T_c = int(rs.choice([1, 8, 32])), int(rs.integers(0, 5)), float(rs.random() * 40)
        nb, nu, s = wk.ws_replica_scores(wk.make_model(1e9, L_A, L_P, T_c, 1, B, K))
        onb, onu, os_ = oc.replica_scores(L_A, L_P, B, K, T_c)
        assert (nb, nu) == (onb, onu)
        for a, b in zip(s, os_):
            assert a == b or abs(a - b) <= 4 * math.ulp(b)
    with pytest.raises(wk.WarmKVError):
        wk.ws_replica_scores(wk.make_model(1e9, 1.0, 2.0, 1.0, 1, 0, 0))


def test_library_placement_matches_oracle():
    rs = np.random.default_rng(3)
    for _ in range(150):
        models = _random_models(rs, int(rs.integers(1, 7)))
        gps = int(rs.choice([4, 8]))
        free0 = [float(rs.integers(0, 80)) * 1e9 for _ in range(gps * int(rs.integers(1, 4)))]
        ofree = free0[:]
        want = oc.place(models, ofree, gps)
        lfree = np.array(free0)
        got = wk.ws_place_replicas([wk.make_model(m["S"], m["L_A"], m["L_P"], m["T_c"], m["D"], m["B"], m["K"])
                                    for m in models], lfree, gps)
        assert [(a, b, c, d) for a, b, c, d, _ in got] == [(a, b, c, d) for a, b, c, d, _ in want]
        assert np.array_equal(lfree, np.array(ofree))
        _check_placement_invariants(models, free0, lfree.tolist(), gps, got)
    with pytest.raises(wk.WarmKVError):                          # degree must divide the server size
        wk.ws_place_replicas([wk.make_model(1e9, 10, 10, 1, 3, 8, 0)], np.array([1e10] * 8), 8)
