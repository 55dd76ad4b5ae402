"""Independent pins of the oracle's two FP8 attention emulations (diagnostics of the FP8
attention variant; the binding bar of that variant is exact attention at 6e-2).

Each emulation is restated here one value at a time, in scalar Python, with a rounding routine of
its own (nearest value in the table of all E4M3 codes, ties to the even code), and checked (a) on
a case small enough to work out by hand, whose expected weights are written below with their
derivation, and (b) against the vectorised oracle on a small random case.  A wrong score bound,
a wrong weight top or a wrong normaliser each changes a hand-derived number (see the asserts).
"""
import math

import numpy as np

from oracle import litevggt_oracle as O


# ------------------------------------------------------------------ scalar E4M3, by table
def _e4m3_table():
    """Every finite E4M3 ("fn": bias 7, no infinities, 0x7f is NaN) value with its code."""
    vals = []
    for code in range(0x7f):                       # positive codes below NaN
        e, m = code >> 3, code & 7
        vals.append((m / 8.0) * 2.0 ** -6 if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7))
    return vals


_TABLE = _e4m3_table()
assert _TABLE[-1] == 448.0 and _TABLE[1] == 2.0 ** -9 and len(_TABLE) == 127


def e4m3(x: float) -> float:
    """Nearest E4M3 value, ties to the even code, saturating at +-448."""
    a = min(abs(x), 448.0)
    best = min(range(len(_TABLE)), key=lambda c: (abs(_TABLE[c] - a), c & 1))
    return math.copysign(_TABLE[best], x) if _TABLE[best] != 0.0 else 0.0


def test_scalar_e4m3_against_the_oracle_rounder():
    rng = np.random.default_rng(3)
    xs = np.concatenate([rng.standard_normal(400) * 10 ** rng.uniform(-4, 3, 400),
                         [17.0, 18.0, 19.0, 2.0 ** -10, 1.5 * 2.0 ** -9, 464.0, 1e9, 0.0]])
    assert [e4m3(float(x)) for x in xs] == list(O.round_e4m3(xs))


# ------------------------------------------------------------------ scalar restatements
def scalar_fp8_bounded(q, k, v, scale=None):
    """The fixed-reference scheme for unit-RMS q, k, one value at a time.  Returns (out, weights,
    totals): weights[i][j] is the E4M3 weight of key j for query i (one head)."""
    n, d = len(k), len(k[0])
    f32 = np.float32
    c = f32((1.0 / math.sqrt(d) if scale is None else scale) * math.log2(math.e))
    amax = lambda rows: max(abs(x) for r in rows for x in r)
    inv_k = f32(448.0) / f32(amax(k))
    inv_q0 = f32(448.0) / f32(amax(q))
    e = math.ceil(math.log2(float(c) / (float(inv_q0) * float(inv_k))))     # power-of-two block scale
    inv_q = f32(float(c) / (float(inv_k) * 2.0 ** e))
    q8 = [[e4m3(float(f32(x) * inv_q)) for x in r] for r in q]
    k8 = [[e4m3(float(f32(x) * inv_k)) for x in r] for r in k]
    sv = amax(v) / 448.0
    v8 = [[e4m3(x / sv) for x in r] for r in v]
    ref = 73.0 * float(c) - 8.75            # largest reachable score, stored as 2^8.75
    out, weights, totals = [], [], []
    for qi in q8:
        w = [e4m3(2.0 ** (sum(a * b for a, b in zip(qi, kj)) * 2.0 ** e - ref)) for kj in k8]
        tot = sum(w)                        # the normaliser is the sum of the E4M3 weights
        weights.append(w)
        totals.append(tot)
        out.append([sum(w[j] * v8[j][t] for j in range(n)) * sv / tot if tot > 0 else 0.0
                    for t in range(len(v[0]))])
    return out, weights, totals


def scalar_fp8_running(q, k, v, scale=None, p_scale=256.0):
    """The running-maximum scheme: per-tensor scales amax / 448, weights relative to the row
    maximum stored as E4M3(p_scale * w), normaliser from the unrounded weights."""
    n, d = len(k), len(k[0])
    amax = lambda rows: max(abs(x) for r in rows for x in r)
    sq, sk, sv = amax(q) / 448.0, amax(k) / 448.0, amax(v) / 448.0
    q8 = [[e4m3(x / sq) for x in r] for r in q]
    k8 = [[e4m3(x / sk) for x in r] for r in k]
    v8 = [[e4m3(x / sv) for x in r] for r in v]
    sc = (1.0 / math.sqrt(d) if scale is None else scale) * sq * sk
    out, weights = [], []
    for qi in q8:
        s = [sum(a * b for a, b in zip(qi, kj)) * sc for kj in k8]
        m = max(s)
        w = [math.exp(x - m) for x in s]
        w8 = [e4m3(x * p_scale) / p_scale for x in w]
        weights.append(w8)
        out.append([sum(w8[j] * v8[j][t] for j in range(n)) * sv / sum(w) for t in range(len(v[0]))])
    return out, weights


# ------------------------------------------------------------------ the hand-worked case
def _hadamard_case():
    """Four keys of +-1 entries (unit RMS, amax 1): all ones, two Walsh rows orthogonal to it, and
    minus all ones; the query is the all-ones row.  Values: constant rows 1, -1, 0.25, 0.5."""
    d = 64
    h0 = [1.0] * d
    h1 = [1.0 if (t >> 0) & 1 == 0 else -1.0 for t in range(d)]
    h2 = [1.0 if (t >> 1) & 1 == 0 else -1.0 for t in range(d)]
    k = [h0, h1, h2, [-1.0] * d]
    v = [[1.0] * d, [-1.0] * d, [0.25] * d, [0.5] * d]
    return [h0], k, v


def test_fp8_bounded_weights_worked_out_by_hand():
    q, k, v = _hadamard_case()
    out, w, tot = scalar_fp8_bounded(q, k, v)
    # c = fp32(0.125 log2 e) = 0.18033688.  amax(q) = amax(k) = 1: inv_k = 448, and the block scale
    # is 2^e with e = ceil(log2(c / 448^2)) = ceil(-20.086) = -20, so inv_q = c 2^20 / 448 = 422.09
    # and q's codes are E4M3(+-422.09) = +-416 (step 32 between 256 and 512); k's codes are +-448.
    # Scores in log2 units: parallel 64 * 416 * 448 * 2^-20 = 11.375, orthogonal 0, opposite -11.375.
    # Reference: 73 c - 8.75 = 4.414592.
    #   parallel:   2^(11.375 - 4.414592) = 2^6.960408 = 124.53  -> E4M3 128 (step 8 above 64)
    #   orthogonal: 2^-4.414592 = 0.046890                     -> E4M3 0.046875 (= 12 * 2^-8)
    #   opposite:   2^-15.79 = 1.8e-5, below half the smallest subnormal 2^-10 -> 0
    assert w[0] == [128.0, 0.046875, 0.046875, 0.0]
    # a bound of 64 instead of 73 would give 2^8.583 = 383.6 -> 384; a weight top of 8 instead of
    # 8.75 would give 2^6.2104 = 74.05 -> 72: both change the first weight
    assert e4m3(2.0 ** (11.375 - (64.0 * 0.18033688 - 8.75))) == 384.0
    assert e4m3(2.0 ** (11.375 - (73.0 * 0.18033688 - 8.0))) == 72.0
    # normaliser: the sum of the E4M3 weights, 128.09375 (the unrounded weights sum to 124.62, which
    # would give 1.027 instead of 0.99899)
    assert tot[0] == 128.09375
    want = (128.0 * 1.0 + 0.046875 * -1.0 + 0.046875 * 0.25) / 128.09375       # v's codes are exact
    assert abs(out[0][0] - want) < 1e-15 and abs(want - 0.99899) < 1e-5
    got = O.attention_fp8_bounded(np.array(q)[:, None, :], np.array(k)[:, None, :], np.array(v)[:, None, :])
    assert np.allclose(got[0, 0], want, rtol=0, atol=1e-13)
    assert abs(128.0 / (124.53 + 2 * 0.04689) - 1.027) < 1e-3


def test_fp8_running_weights_worked_out_by_hand():
    q, k, v = _hadamard_case()
    out, w = scalar_fp8_running(q, k, v)
    # q and k quantise exactly (codes +-448, scales 1/448): scores 64/8 = 8, 0, 0, -8; row maximum 8.
    #   parallel:   exp(0) = 1          -> 256 -> E4M3 256            -> 1
    #   orthogonal: exp(-8) = 3.3546e-4 -> 0.085878 -> E4M3 0.0859375 (= 11 * 2^-7) -> 3.35693e-4
    #   opposite:   exp(-16) * 256 = 2.9e-5, below 2^-10 -> 0
    assert w[0] == [1.0, 0.0859375 / 256, 0.0859375 / 256, 0.0]
    norm = 1.0 + 2.0 * math.exp(-8.0) + math.exp(-16.0)          # the unrounded weights
    want = (1.0 - 0.0859375 / 256 + 0.25 * 0.0859375 / 256) / norm
    assert abs(out[0][0] - want) < 1e-15 and abs(want - 0.999078) < 1e-6
    # the E4M3 weights as normaliser would differ in the seventh digit
    assert abs(want - (1.0 - 0.75 * 0.0859375 / 256) / (1.0 + 2 * 0.0859375 / 256)) > 3e-7
    got = O.attention_fp8(np.array(q)[:, None, :], np.array(k)[:, None, :], np.array(v)[:, None, :])
    assert np.allclose(got[0, 0], want, rtol=0, atol=1e-13)


# ------------------------------------------------------------------ small random cases
def _unit_rms_bf16(rng, n, d):
    return O.round_bf16(O.qk_normalize(rng.standard_normal((n, 1, d))))[:, 0, :]


def test_fp8_bounded_scalar_restatement_matches_the_oracle():
    rng = np.random.default_rng(71)
    n, d = 7, 64
    q = _unit_rms_bf16(rng, n, d)
    k = O.round_bf16(O.qk_normalize((q + 0.4 * rng.standard_normal((n, d)))[:, None, :]))[:, 0, :]
    v = rng.standard_normal((n, d))
    out, w, tot = scalar_fp8_bounded(q.tolist(), k.tolist(), v.tolist())
    assert min(tot) >= 1.0                                   # no row leaves the scheme
    got = O.attention_fp8_bounded(q[:, None, :], k[:, None, :], v[:, None, :])[:, 0, :]
    assert np.allclose(got, np.array(out), rtol=1e-12, atol=1e-12)
    assert max(abs(sum(r) / t - 1.0) for r, t in zip(w, tot)) < 1e-15


def test_fp8_bounded_rows_below_the_range_follow_the_running_scheme():
    rng = np.random.default_rng(72)
    n, d = 6, 64
    u = rng.standard_normal(d)
    k = O.round_bf16(O.qk_normalize((u + 0.05 * rng.standard_normal((n, d)))[:, None, :]))[:, 0, :]
    q = O.round_bf16(O.qk_normalize((-u + 0.05 * rng.standard_normal((n, d)))[:, None, :]))[:, 0, :]
    v = rng.standard_normal((n, d))
    _, _, tot = scalar_fp8_bounded(q.tolist(), k.tolist(), v.tolist())
    assert max(tot) < 1.0                                    # every row is out of range
    want, _ = scalar_fp8_running(q.tolist(), k.tolist(), v.tolist())
    got = O.attention_fp8_bounded(q[:, None, :], k[:, None, :], v[:, None, :])[:, 0, :]
    assert np.allclose(got, np.array(want), rtol=1e-12, atol=1e-12)


def test_fp8_running_scalar_restatement_matches_the_oracle():
    rng = np.random.default_rng(73)
    n, d = 8, 16
    q, k, v = (rng.standard_normal((n, d)) for _ in range(3))
    want, _ = scalar_fp8_running(q.tolist(), k.tolist(), v.tolist(), scale=0.3)
    got = O.attention_fp8(q[:, None, :], k[:, None, :], v[:, None, :], scale=0.3)[:, 0, :]
    assert np.allclose(got, np.array(want), rtol=1e-12, atol=1e-12)
