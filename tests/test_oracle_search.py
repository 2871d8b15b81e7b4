"""Pins of the search oracle (Sec. III-C, Eq. 3, Eq. 4, Alg. 1) and of the tensor error metric
(Eq. 2) it is driven by: hand-traced runs, the reduction to a plain greedy descent, constraint
checks on random tables, and closed forms of the quantization error."""
import numpy as np
import pytest

from oracle import dybit_ref as R
from oracle import search_ref as S


# ---- hand-traced example -----------------------------------------------------------------------
# Three layers whose latency follows the paper's (8/P1)(8/P2) scaling (Sec. III-B) from 8, 4 and 2
# time units at (8, 8); per-tensor errors below, the same table for weights and activations.
BASE = (8.0, 4.0, 2.0)
ERR = ((0.01, 0.1, 0.5), (0.005, 0.05, 0.3), (0.02, 0.2, 0.6))
LAT = [[[b * (pw / 8) * (pa / 8) for pa in S.LEVELS] for pw in S.LEVELS] for b in BASE]


def test_speedup_strategy_hand_trace_alpha_2():
    """Total 14.  Round 1: the two slowest are layers 0 and 1; least error first: 1 (0.01) then 0 (0.02).
    W pass: L1 8->4 (total 12, 1.17x), L0 8->4 (total 8, 1.75x).  A pass: L1 8->4 (total 7, 2.0x): met."""
    w, a, ratio, met = S.search(LAT, ERR, ERR, "speedup", 2.0, 2)
    assert (w, a) == ([4, 4, 8], [8, 4, 8])
    assert ratio == pytest.approx(2.0) and met


def test_speedup_strategy_hand_trace_alpha_3():
    """Continues the trace above: L0 A 8->4 (total 5, 2.8x).  Round 2: latencies (2, 1, 2), the two
    slowest are 0 and 2 (tie with layer 0 listed first); errors 0.2 and 0.04, so 2 goes first:
    L2 W 8->4 (total 4, 3.5x): met."""
    w, a, ratio, met = S.search(LAT, ERR, ERR, "speedup", 3.0, 2)
    assert (w, a) == ([4, 4, 4], [4, 4, 8])
    assert ratio == pytest.approx(3.5) and met


def test_rmse_strategy_hand_trace_beta_5():
    """Base error 0.02 + 0.01 + 0.04 = 0.07, budget 0.35.  Round 1: least error: layers 1 and 0, slowest
    first: 0 then 1.  W pass: L0 (total 0.16), L1 (0.205).  A pass: L0 (0.295), L1 (0.34 = 4.86x).
    Round 2: errors (0.2, 0.1, 0.04): layers 2 and 1; latencies (2, 1, 2): 2 first; L2 W 8->4 would give
    0.52 = 7.4x: taken back, search ends."""
    w, a, ratio, met = S.search(LAT, ERR, ERR, "rmse", 5.0, 2)
    assert (w, a) == ([4, 4, 8], [4, 4, 8])
    assert ratio == pytest.approx(0.34 / 0.07) and met
    assert S.total_latency(LAT, [1, 1, 0], [1, 1, 0]) == pytest.approx(5.0)


def test_rmse_strategy_hand_trace_k1():
    """k = 1, beta = 2.5 (budget 0.175).  Round 1: least error is layer 1: W 8->4 (0.115), A 8->4 (0.16).
    Round 2: errors (0.02, 0.1, 0.04): layer 0: W 8->4 gives 0.25 > 0.175: taken back, end."""
    w, a, ratio, met = S.search(LAT, ERR, ERR, "rmse", 2.5, 1)
    assert (w, a) == ([8, 4, 8], [8, 4, 8])
    assert ratio == pytest.approx(0.16 / 0.07) and met


# ---- reductions and invariants --------------------------------------------------------------------
def random_tables(rng, n):
    """Latencies that fall and errors that grow as the widths shrink, with noise."""
    lat = [[[float(b * (0.3 + pw / 8) * (0.3 + pa / 8) * rng.uniform(0.8, 1.2)) for pa in S.LEVELS] for pw in S.LEVELS]
           for b in rng.uniform(1, 20, n)]
    def err():
        return [sorted(float(v) for v in rng.uniform(0.001, 1.0, 3) * (0.01, 0.1, 1.0)) for _ in range(n)]
    return lat, err(), err()


def greedy_slowest_first(lat, alpha):
    """What Alg. 1 comes to for k = 1 in the speedup strategy: lower W, then A, of the slowest layer
    that can still be lowered, until the speedup is reached."""
    n = len(lat)
    wi, ai = [0] * n, [0] * n
    total = lambda: sum(lat[l][wi[l]][ai[l]] for l in range(n))
    base = total()
    while base / total() < alpha:
        open_ = [l for l in range(n) if wi[l] < 2 or ai[l] < 2]
        if not open_:
            break
        l = max(open_, key=lambda j: (lat[j][wi[j]][ai[j]], -j))
        if wi[l] < 2:
            wi[l] += 1
            if base / total() >= alpha:
                break
        if ai[l] < 2:
            ai[l] += 1
    return [S.LEVELS[i] for i in wi], [S.LEVELS[i] for i in ai]


@pytest.mark.parametrize("seed", range(8))
def test_k1_speedup_is_greedy_descent(seed):
    rng = np.random.default_rng(seed)
    lat, ew, ea = random_tables(rng, 7)
    for alpha in (1.3, 2.0, 4.0, 100.0):
        w, a, _, _ = S.search(lat, ew, ea, "speedup", alpha, 1)
        assert (w, a) == greedy_slowest_first(lat, alpha)


@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("k", [1, 3, 9])
def test_constraints_hold(seed, k):
    rng = np.random.default_rng(100 + seed)
    n = 6
    lat, ew, ea = random_tables(rng, n)
    idx = {8: 0, 4: 1, 2: 2}
    best_speedup = S.total_latency(lat, [0] * n, [0] * n) / S.total_latency(lat, [2] * n, [2] * n)
    for alpha in (0.5, 1.0, 1.5, 3.0, 1000.0):
        w, a, ratio, met = S.search(lat, ew, ea, "speedup", alpha, k)
        wi, ai = [idx[b] for b in w], [idx[b] for b in a]
        assert ratio == pytest.approx(S.total_latency(lat, [0] * n, [0] * n) / S.total_latency(lat, wi, ai))
        assert met == (ratio >= alpha)
        if alpha <= 1.0:
            assert w == [8] * n and a == [8] * n                   # nothing to do
        if not met:
            assert w == [2] * n and a == [2] * n                   # gave up only when nothing was left
            assert alpha > best_speedup
    base = S.total_rmse(ew, ea, [0] * n, [0] * n)
    for beta in (0.5, 1.0, 2.0, 10.0, 1e9):
        w, a, ratio, met = S.search(lat, ew, ea, "rmse", beta, k)
        wi, ai = [idx[b] for b in w], [idx[b] for b in a]
        assert ratio == pytest.approx(S.total_rmse(ew, ea, wi, ai) / base)
        if beta >= 1.0:
            assert met and ratio <= beta                           # Eq. 4 holds
        else:
            assert not met and w == [8] * n and a == [8] * n
        if beta == 1e9:
            assert w == [2] * n and a == [2] * n


def test_search_rejects_bad_arguments():
    with pytest.raises(ValueError):
        S.search(LAT, ERR, ERR, "latency", 2.0, 2)
    with pytest.raises(ValueError):
        S.search(LAT, ERR, ERR, "speedup", 2.0, 0)
    with pytest.raises(ValueError):
        S.search(LAT, [(0.0, 0.0, 0.0)] * 3, [(0.0, 0.0, 0.0)] * 3, "rmse", 2.0, 1)


# ---- Eq. 2 on a quantized tensor ----------------------------------------------------------------
@pytest.mark.parametrize("bits,signed", [(8, False), (6, False), (4, False), (8, True), (4, True)])
def test_rmse_of_a_uniform_tensor_below_one(bits, signed):
    """x on a fine regular grid over [0, s): only the fraction codes c / 2^(m-1) are used, the error is
    uniform over one step, so its root mean square is step / sqrt(12); sigma of the grid is
    s / sqrt(12) (both up to the grid's own spacing), hence RMSE -> 2^-(m-1)."""
    m = R.magnitude_bits(bits, signed)
    s = np.float32(0.75)
    n = 1 << 16
    x = ((np.arange(n) + 0.5) / n * s).astype(np.float32)
    assert R.quantization_rmse(x, s, bits, signed) == pytest.approx(2.0 ** -(m - 1), rel=2e-3)


def test_rmse_hand_values():
    """4-bit unsigned, s = 1 (Table I: 0, 1/8, ..., 7/8, 1, 1.25, 1.5, 1.75, 2, 3, 4, 8).
    x = (0.3, 1.3, 5, -2, 2.5): nearest values 0.25, 1.25, 4, 0 (negative in an unsigned format) and 2
    (tie between 1100 = 2 and 1101 = 3 goes to the even code); errors 0.05, 0.05, 1, -2, 0.5."""
    x = np.array([0.3, 1.3, 5.0, -2.0, 2.5], dtype=np.float32)
    want = np.sqrt((0.05 ** 2 + 0.05 ** 2 + 1.0 + 4.0 + 0.25) / 5) / np.std(x.astype(np.float64))
    assert R.quantization_rmse(x, 1.0, 4, False) == pytest.approx(want, rel=1e-6)


def test_rmse_is_zero_on_representable_values_and_scales_out():
    for bits, signed in [(2, True), (4, True), (6, False), (8, True)]:
        cb = R.codebook(bits, signed)
        x = (np.float32(0.5) * cb.astype(np.float32))
        assert R.quantization_rmse(x, 0.5, bits, signed) == 0.0
    rng = np.random.default_rng(5)
    x = rng.normal(0, 1, 5000).astype(np.float32)
    s = R.absmax_scale(x, 4, True)
    # a power-of-two factor on tensor and scale changes neither the codes nor the ratio to sigma
    assert R.quantization_rmse(x * np.float32(8), s * np.float32(8), 4, True) == pytest.approx(
        R.quantization_rmse(x, s, 4, True), rel=1e-12)


def test_rmse_grows_as_bits_shrink():
    rng = np.random.default_rng(6)
    x = rng.laplace(0, 0.02, 20000).astype(np.float32)
    e = [R.quantization_rmse(x, R.absmax_scale(x, b, True), b, True) for b in (8, 6, 4, 2)]
    assert e[0] < e[1] < e[2] < e[3]
