"""Pins of the oracle's max pooling on codes (Sec. III-B: activations are stored as DyBit codes).

What fixes it independently of its own code: (1) the encoder is monotone, so pooling the codes of a tensor
must equal encoding the pooled tensor -- the right-hand side uses only numpy's maximum over explicitly
gathered windows and the oracle's (separately pinned) quantize; (2) a hand-worked 4 x 4 example;
(3) k = stride = 1 is the identity up to the canonical zero; (4) brute force over scalar loops."""
import numpy as np
import pytest

from oracle import dybit_ref as R

FMTS = [(2, False), (2, True), (4, False), (4, True), (8, False), (8, True)]


def pool_values(x, k, stride, pad):
    Bn, H, W, C = x.shape
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    xp = np.full((Bn, H + 2 * pad, W + 2 * pad, C), -np.inf)
    xp[:, pad:pad + H, pad:pad + W, :] = x
    out = np.empty((Bn, Ho, Wo, C))
    for i in range(Ho):
        for j in range(Wo):
            out[:, i, j, :] = xp[:, i * stride:i * stride + k, j * stride:j * stride + k, :].max(axis=(1, 2))
    return out


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("geom", [(3, 2, 1), (2, 2, 0), (3, 1, 1), (5, 3, 2)])
def test_pooling_commutes_with_the_encoder(fmt, geom):
    k, stride, pad = geom
    rng = np.random.default_rng(5 + fmt[0])
    x = rng.normal(0, 1, (2, 9, 11, 8)).astype(np.float32)
    if not fmt[1]:
        x = np.abs(x)
    s = R.absmax_scale(x, *fmt)
    q = R.quantize(x, s, *fmt).reshape(x.shape)
    got = R.maxpool2d_codes(q, *fmt, k, stride, pad)
    want = R.quantize(pool_values(x.astype(np.float64), k, stride, pad).astype(np.float32), s, *fmt).reshape(got.shape)
    assert np.array_equal(got, want)


def test_hand_worked_example():
    # 4-bit signed codes (3 magnitude bits, sign in bit 3): values 0 .25 .5 .75 1 1.5 2 4 and their negatives
    q = np.array([[1, 9, 2, 10],
                  [12, 8, 11, 15],
                  [0, 3, 5, 13],
                  [14, 6, 7, 4]], dtype=np.uint8).reshape(1, 4, 4, 1)
    # 2 x 2 windows, stride 2: {.25, -.25, -1, -0} -> .25 (code 1); {.5, -.5, -.75, -4} -> .5 (code 2);
    # {0, .75, -2, 2} -> 2 (code 6); {1.5, -1.5, 4, 1} -> 4 (code 7)
    assert R.maxpool2d_codes(q, 4, True, 2, 2, 0).reshape(2, 2).tolist() == [[1, 2], [6, 7]]
    # a window of negative values only, and one whose maximum is the negative zero: canonical code 0
    q2 = np.array([[9, 12], [15, 10]], dtype=np.uint8).reshape(1, 2, 2, 1)
    assert R.maxpool2d_codes(q2, 4, True, 2, 2, 0).reshape(-1).tolist() == [9]
    q3 = np.array([[8, 12], [15, 10]], dtype=np.uint8).reshape(1, 2, 2, 1)
    assert R.maxpool2d_codes(q3, 4, True, 2, 2, 0).reshape(-1).tolist() == [0]


@pytest.mark.parametrize("fmt", FMTS)
def test_unit_window_is_the_identity_up_to_the_canonical_zero(fmt):
    rng = np.random.default_rng(9)
    q = rng.integers(0, 1 << fmt[0], (1, 5, 6, 4)).astype(np.uint8)
    got = R.maxpool2d_codes(q, *fmt, 1, 1, 0)
    want = q.copy()
    if fmt[1]:
        want[q == (1 << (fmt[0] - 1))] = 0
    assert np.array_equal(got, want)


@pytest.mark.parametrize("fmt", [(4, True), (8, False)])
def test_against_scalar_loops(fmt):
    rng = np.random.default_rng(11)
    q = rng.integers(0, 1 << fmt[0], (2, 6, 5, 3)).astype(np.uint8)
    k, stride, pad = 3, 2, 1
    cb = [float(v) for v in R.codebook(*fmt)]
    got = R.maxpool2d_codes(q, *fmt, k, stride, pad)
    for b in range(2):
        for ho in range(got.shape[1]):
            for wo in range(got.shape[2]):
                for c in range(3):
                    taps = [int(q[b, r, s, c]) for r in range(ho * stride - pad, ho * stride - pad + k)
                            for s in range(wo * stride - pad, wo * stride - pad + k) if 0 <= r < 6 and 0 <= s < 5]
                    best = max(cb[t] for t in taps)
                    assert cb[int(got[b, ho, wo, c])] == best
                    assert int(got[b, ho, wo, c]) == min(t for t in range(1 << fmt[0]) if cb[t] == best)
