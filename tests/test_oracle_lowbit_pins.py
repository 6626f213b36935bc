"""Hand-worked pins for the low-bit sparse branch of the oracle (Sec. 5; Alg. 2, the block loop with
quant / dequant) and for the float32 smoothing that precedes the quantiser.

The paper leaves the quantisation scheme open; the definition taken is in the docstring of
oracle.sparse_branch_lowbit.  These cases fix that definition from the outside: every expected value
below is worked out on paper from the definition (e4m3 grid, scale 2^8 on P, the denominator from the
un-rounded P, float32 smoothing) and written as literal numbers, so a slip in the oracle - another
scale, a flushed subnormal, the denominator taken from the rounded P, a smoothing done in another
precision - fails here.  The last test plants exactly those slips into a copy of the oracle and
checks that the cases notice.

Construction shared by cases (a) and (b).  d = 2, b_q = b_k = 2, N = 6 (three key blocks); query
block 0 keeps key blocks 0 and 2.  Q rows are sqrt(2) (1, 1) and sqrt(2) (0, 1): the block's
largest magnitude is sqrt 2, so the e4m3 codes are 448 and 0, exact.  Smoothed keys are
beta (n, m) with small integers; a key block whose largest |integer| is 7 or 14 has codes
448 n / 7 = 64 n or 448 n / 14 = 32 n, all on the e4m3 grid (four significant bits), so the
dequantised products are exact up to float32 rounding of the two scales (relative 1e-7):
row 0 scores beta (n + m), row 1 scores beta m.  Key block 1 is not selected; its keys only make
the columns of the smoothed K sum to zero.  The keys handed in carry an offset that the smoothing
step must remove.
"""
import importlib.util
import math
import os

import numpy as np
import pytest

import sla2_oracle as O

S2 = math.sqrt(2.0)
SEL = np.array([[0, 2], [0, 2], [0, 2]], dtype=np.int32)      # only query block 0 is evaluated


def _inputs(beta, ints, V):
    Kp = beta * np.array(ints, dtype=np.float64)
    assert np.allclose(Kp.sum(axis=0), 0.0)
    K = Kp + np.array([0.75, -1.25])                           # offset, removed by the smoothing step
    Q = np.zeros((6, 2))
    Q[0], Q[1] = (S2, S2), (0.0, S2)
    Q[2:] = [[0.5, -0.5], [0.25, 1.0], [-1.0, 0.5], [0.5, 0.5]]   # other query blocks: not evaluated
    return Q, K, np.array(V, dtype=np.float64)


# smoothed keys of case (a), in units of ln 2:  (n, m)
INTS_A = [(7, -7), (4, -6),          # block 0 (largest 7):  row 0 scores 0, -2;    row 1 scores -7, -6
          (5, 1), (0, 14),           # block 1: filler, columns then sum to zero
          (-14, -3), (-2, 1)]        # block 2 (largest 14): row 0 scores -17, -1;  row 1 scores -3, 1
V_A = [(1, 0), (0, 4), (9, 9), (-9, 9), (2.0 ** 17, -2.0 ** 17), (2, 2)]


def case_a(mod):
    """Every probability is a power of two that the 2^8-scaled e4m3 grid holds exactly (the smallest,
    2^-17, lands on the smallest subnormal 2^-9), so the low-bit loop must return the exact softmax:

      row 0: block 0  P = (1, 1/4),     l = 5/4
             block 2  P = (2^-17, 1/2), max unchanged, l = 7/4 + 2^-17
             O = (v0 + v1/4 + 2^-17 v4 + v5/2) / l = (3, 1) / (7/4 + 2^-17),   L = ln l
      row 1: block 0  scores (-7, -6) ln 2: m = -6 ln 2, P = (1/2, 1), l = 3/2
             block 2  scores (-3, 1) ln 2: m = ln 2, rescale 2^-7, P = (1/16, 1), l = 3/256 + 17/16 = 275/256
             O = (2^-7 (v0/2 + v1) + v4/16 + v5) / l,                          L = ln 2 + ln(275/256)
    """
    Q, K, V = _inputs(math.log(2.0), INTS_A, V_A)
    got, L = mod.sparse_branch_lowbit(Q, K, V, SEL, 2, 2, q_blocks=[0])
    l0 = 7 / 4 + 2.0 ** -17
    np.testing.assert_allclose(got[0], np.array([3.0, 1.0]) / l0, rtol=3e-6)
    l1 = 275 / 256
    v = V
    np.testing.assert_allclose(got[1], (2.0 ** -7 * (v[0] / 2 + v[1]) + v[4] / 16 + v[5]) / l1, rtol=3e-6)
    np.testing.assert_allclose(L[:2], [math.log(l0), math.log(2.0) + math.log(l1)], rtol=0, atol=3e-6)
    assert not got[2:].any() and np.all(np.isneginf(L[2:]))     # blocks that were not asked for
    # and, all weights being exact, the un-quantised branch gives the same
    ex, Lex = mod.sparse_branch(Q, mod.smooth_k(K), V, SEL, 2, 2, q_blocks=[0])
    np.testing.assert_allclose(got[:2], ex[:2], rtol=3e-6)
    np.testing.assert_allclose(L[:2], Lex[:2], rtol=0, atol=3e-6)


# smoothed keys of case (b), in natural units (beta = 1)
INTS_B = [(7, -7), (1, -2),          # block 0 (largest 7):  row 0 scores 0, -1;     row 1 scores -7, -2
          (10, 2), (10, 3),          # block 1: filler
          (-14, 1), (-14, 3)]        # block 2 (largest 14): row 0 scores -13, -11;  row 1 scores 1, 3
V_B = [(1, 2), (3, -1), (9, 9), (-9, 9), (2.0 ** 10, 5), (2.0 ** 16, -2.0 ** 16)]


def case_b(mod):
    """Probabilities that are not on the grid.  Rounding of 256 P to e4m3 (grid spacing 8 in [64, 128),
    4 in [32, 64), 1 in [8, 16), 1/8 in [1, 2), 2^-9 below 2^-6):

      256 e^-1  = 94.18   -> 96          256 e^-2  = 34.65   -> 36        256 e^-3 = 12.745 -> 13
      256 e^-5  = 1.7249  -> 1.75        256 e^-11 = 2.19 2^-9 -> 2 2^-9  256 e^-13 = 0.30 2^-9 -> 0

      row 0: block 0  P = (1, e^-1) -> (1, 96/256);  block 2  P = (e^-13, e^-11) -> (0, 2^-16); max stays 0
             l = 1 + e^-1 + e^-13 + e^-11   (the un-rounded P)
             O = (v0 + 96/256 v1 + 2^-16 v5) / l
      row 1: block 0  scores (-7, -2): m = -2, P = (e^-5, 1) -> (1.75/256, 1), l = 1 + e^-5
             block 2  scores (1, 3):  m = 3, rescale e^-5, P = (e^-2, 1) -> (36/256, 1)
             l = e^-5 (1 + e^-5) + e^-2 + 1
             O = (e^-5 (1.75/256 v0 + v1) + 36/256 v4 + v5) / l,   L = 3 + ln l
    Row 1 rounds its first block against the maximum it had then (-2), not the final one.
    """
    Q, K, V = _inputs(1.0, INTS_B, V_B)
    got, L = mod.sparse_branch_lowbit(Q, K, V, SEL, 2, 2, q_blocks=[0])
    e = math.exp
    v = V
    l0 = 1 + e(-1) + e(-13) + e(-11)
    np.testing.assert_allclose(got[0], (v[0] + 96 / 256 * v[1] + 2.0 ** -16 * v[5]) / l0, rtol=3e-6)
    l1 = e(-5) * (1 + e(-5)) + e(-2) + 1
    np.testing.assert_allclose(got[1], (e(-5) * (1.75 / 256 * v[0] + v[1]) + 36 / 256 * v[4] + v[5]) / l1, rtol=3e-6)
    np.testing.assert_allclose(L[:2], [math.log(l0), 3 + math.log(l1)], rtol=0, atol=3e-6)
    # the same case with moderate values everywhere, so that the large entries above hide nothing
    V2 = np.array([(1, 2), (3, -1), (9, 9), (-9, 9), (-2, 5), (4, 1)], dtype=np.float64)
    got2, _ = mod.sparse_branch_lowbit(Q, K, V2, SEL, 2, 2, q_blocks=[0])
    np.testing.assert_allclose(got2[0], (V2[0] + 96 / 256 * V2[1] + 2.0 ** -16 * V2[5]) / l0, rtol=3e-6)
    np.testing.assert_allclose(got2[1], (e(-5) * (1.75 / 256 * V2[0] + V2[1]) + 36 / 256 * V2[4] + V2[5]) / l1,
                               rtol=3e-6)


def case_b_quantised_v(mod):
    """The same weights with V quantised as well (the second product as Alg. 2 prints it).  Block 0 of V
    is ((7, 14), (3.5, -1)): largest 14, codes 448 x / 14 = 32 x on the grid for 7, 14, 3.5 and 1, so it
    is reproduced exactly.  Block 2 is ((-2, 5), (4, 1)): largest 5, codes of 448 x / 5 = -179.2, 448,
    358.4, 89.6 -> -176, 448, 352, 88 (grid spacing 16 in [128, 256), 32 in [256, 448], 8 in [64, 128)),
    i.e. V is read as (-176, 448) 5/448 = (-55/28, 5) and (352, 88) 5/448 = (55/14, 55/56)."""
    Q, K, _ = _inputs(1.0, INTS_B, V_B)
    V = np.array([(7, 14), (3.5, -1), (9, 9), (-9, 9), (-2, 5), (4, 1)], dtype=np.float64)
    got, _ = mod.sparse_branch_lowbit(Q, K, V, SEL, 2, 2, q_blocks=[0], quant_v=True)
    e = math.exp
    v4, v5 = np.array([-55 / 28, 5.0]), np.array([55 / 14, 55 / 56])
    l0 = 1 + e(-1) + e(-13) + e(-11)
    np.testing.assert_allclose(got[0], (V[0] + 96 / 256 * V[1] + 2.0 ** -16 * v5) / l0, rtol=3e-6)
    l1 = e(-5) * (1 + e(-5)) + e(-2) + 1
    np.testing.assert_allclose(got[1], (e(-5) * (1.75 / 256 * V[0] + V[1]) + 36 / 256 * v4 + v5) / l1, rtol=3e-6)


def case_int8(mod):
    """The INT8 quantiser in the same loop.  Q codes 127 and 0.  Key block 0 (largest 7): codes of
    127 n / 7 = 18.14 n, i.e. (7, -7) -> (127, -127), (1, -2) -> (18, -36); the block is read as
    (7, -7) and (18, -36) 7/127.  Key block 2 (largest 14): (-14, 1) -> (-127, 9), (-14, 3) -> (-127, 27),
    read as (-14, 9 x 14/127) and (-14, 27 x 14/127).  Scores, row 0 = n + m of the values as read,
    row 1 = m; P is rounded as in FP8 mode."""
    Q, K, V = _inputs(1.0, INTS_B, [(1, 2), (3, -1), (9, 9), (-9, 9), (-2, 5), (4, 1)])
    got, L = mod.sparse_branch_lowbit(Q, K, V, SEL, 2, 2, q_blocks=[0], quant_block=mod.quant_block_int8)
    k = np.array([(7.0, -7.0), (18 * 7 / 127, -36 * 7 / 127), (0, 0), (0, 0),
                  (-14.0, 9 * 14 / 127), (-14.0, 27 * 14 / 127)])
    e4 = lambda p: float(O_e4m3_reference(p * 256.0)) / 256.0   # noqa: E731
    for r, s in enumerate((k[:, 0] + k[:, 1], k[:, 1])):
        m = max(s[0], s[1])
        p0 = [math.exp(s[0] - m), math.exp(s[1] - m)]
        l = sum(p0)
        acc = e4(p0[0]) * V[0] + e4(p0[1]) * V[1]
        m2 = max(m, s[4], s[5])
        c = math.exp(m - m2)
        p2 = [math.exp(s[4] - m2), math.exp(s[5] - m2)]
        l = c * l + sum(p2)
        acc = c * acc + e4(p2[0]) * V[4] + e4(p2[1]) * V[5]
        np.testing.assert_allclose(got[r], acc / l, rtol=3e-6)
        np.testing.assert_allclose(L[r], m2 + math.log(l), rtol=0, atol=3e-6)


def O_e4m3_reference(x):
    """Nearest e4m3 value by search over the table of all codes (format definition: 4 exponent bits,
    bias 7, 3 mantissa bits, subnormals, largest 448), ties to the even mantissa."""
    best, best_d, best_even = 0.0, abs(x), True
    for code in range(127):                                   # positive finite codes (0x7F is NaN)
        ex, man = code >> 3, code & 7
        val = (man / 8.0) * 2.0 ** -6 if ex == 0 else (1 + man / 8.0) * 2.0 ** (ex - 7)
        dist = abs(abs(x) - val)
        if dist < best_d or (dist == best_d and man % 2 == 0 and not best_even):
            best, best_d, best_even = val, dist, man % 2 == 0
    return math.copysign(min(best, 448.0), x)


def case_c(mod):
    """Smoothing as it enters the quantiser: float32(K) - float32(mean), the mean taken in float64 and
    rounded once.  One channel, K = (1, 2^-24): the mean 1/2 + 2^-25 needs 25 bits and rounds (tie to
    even) to 1/2, so the smoothed column is (1/2, 2^-24 - 1/2), both exact in float32.  Subtracting in
    float64 and rounding afterwards would give (1/2 - 2^-25, 2^-25 - 1/2) instead."""
    K = np.array([[1.0], [2.0 ** -24]])
    got = mod.smooth_k_f32(K)
    assert got.dtype == np.float32
    assert got[0, 0] == np.float32(0.5) and got[1, 0] == np.float32(2.0 ** -24 - 0.5)
    # a key that float32 cannot hold is rounded before the subtraction: 1 + 3 2^-25 -> 1 + 2^-23
    K = np.array([[1.0 + 3 * 2.0 ** -25], [-1.0]])
    got = mod.smooth_k_f32(K)
    assert got[0, 0] == np.float32(1.0 + 2.0 ** -23) and got[1, 0] == np.float32(-1.0)


CASES = [case_a, case_b, case_b_quantised_v, case_int8, case_c]


@pytest.mark.parametrize("case", CASES, ids=lambda c: c.__name__)
def test_lowbit_hand_worked(case):
    case(O)


# ---- the same cases must notice a slip planted into the oracle ---------------------------------- #
SLIPS = {
    "P scaled by 2^7": ("P_SCALE_LOG2 = 8", "P_SCALE_LOG2 = 7"),
    "P scaled by 2^9 (saturates P = 1)": ("P_SCALE_LOG2 = 8", "P_SCALE_LOG2 = 9"),
    "denominator from the rounded P": ("l_new = keep * l + w.sum(axis=1, keepdims=True)",
                                       "l_new = keep * l + (e4m3_round((w * 256.0).astype(np.float32)).astype(np.float64) / 256.0).sum(axis=1, keepdims=True)"),
    "subnormals flushed to zero": ("e = np.maximum(e - 1, -6)", "e = e - 1; a = np.where(a < 2.0 ** -6, 0.0, a)"),
    "no subnormals (normal spacing all the way down)": ("e = np.maximum(e - 1, -6)", "e = e - 1"),
    "P truncated instead of rounded": ("r = np.rint(a / quantum) * quantum", "r = np.floor(a / quantum) * quantum"),
    "smoothing in float64, rounded afterwards": ("return K.astype(np.float32) - mu32[None, :]",
                                                 "return (K - K.mean(axis=0)[None, :]).astype(np.float32)"),
    "block scale applied once": ("* (float(sQ) * float(sK[j])) / math.sqrt(d)", "* float(sK[j]) / math.sqrt(d)"),
    "P rounded against the final maximum": ("w_rounded = e4m3_round((w * 2.0 ** P_SCALE_LOG2)",
                                            "w_rounded = e4m3_round((np.exp(S - _FINAL_M) * 2.0 ** P_SCALE_LOG2)"),
    "V scale dropped": ("A_new = keep * A + (w_rounded @ Vj) * v_scale", "A_new = keep * A + (w_rounded @ Vj)"),
    "old sum not carried to the new maximum": ("l_new = keep * l + w.sum(axis=1, keepdims=True)",
                                               "l_new = l + w.sum(axis=1, keepdims=True)"),
    "blocks absorbed in descending order": ("for j in sel[i]:", "for j in sel[i][::-1]:"),
}


def _oracle_with(old, new):
    path = os.path.abspath(O.__file__)
    src = open(path).read()
    assert src.count(old) >= 1, "the oracle no longer contains: " + old
    src = src.replace(old, new)
    spec = importlib.util.spec_from_loader("sla2_oracle_slip", loader=None)
    mod = importlib.util.module_from_spec(spec)
    exec(compile(src, path + " (with a planted slip)", "exec"), mod.__dict__)
    return mod


@pytest.mark.parametrize("name", sorted(SLIPS))
def test_planted_slip_is_noticed(name):
    old, new = SLIPS[name]
    mod = _oracle_with(old, new)
    if "_FINAL_M" in new:
        # the row maxima over all selected blocks of case (b): row 0 -> 0, row 1 -> 3
        mod._FINAL_M = np.array([[0.0], [3.0]])
    failed = []
    for case in ([case_b] if "_FINAL_M" in new else CASES):
        try:
            case(mod)
        except AssertionError:
            failed.append(case.__name__)
    assert failed, "no hand-worked case notices: " + name
