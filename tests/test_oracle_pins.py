"""Pins for oracle/sla2_oracle.py: every check compares the oracle with
something that is not the oracle - a closed form, a textbook routine, a library
routine, brute force over the expanded N x N mask, an invariance the paper's
text implies, or a case worked by hand below."""
import math
from fractions import Fraction as F

import numpy as np
import pytest

import sla2_oracle as O

RTOL = 1e-10


def rand_head(seed, N, d, scale=1.0):
    rng = np.random.default_rng(seed)
    Q, K, V = rng.normal(size=(3, N, d)) * scale
    Wq, Wk = rng.normal(size=(2, d, d)) / math.sqrt(d)
    return Q, K, V, Wq, Wk


def dense_attention(Q, K, V):
    """Textbook softmax(QK^T/sqrt(d))V, written with explicit row loops."""
    N, d = Q.shape
    out = np.zeros_like(V)
    for r in range(N):
        s = np.array([Q[r] @ K[c] for c in range(K.shape[0])]) / math.sqrt(d)
        p = np.exp(s - s.max())
        out[r] = (p / p.sum()) @ V
    return out


def expanded_mask(sel, N, b_q, b_k):
    """M in {0,1}^{N x N} obtained by expanding M_c (Sec. 2.1)."""
    M = np.zeros((N, N), dtype=bool)
    for i in range(sel.shape[0]):
        for j in sel[i]:
            M[i * b_q:(i + 1) * b_q, j * b_k:(j + 1) * b_k] = True
    return M


def brute_force(Q, K, V, sel, alpha_rows, b_q, b_k):
    """Eq. 13-14 with dense N x N matrices and the expanded mask.  Masked-out
    score entries are excluded from the softmax; norm() divides each row by its
    sum."""
    N, d = Q.shape
    M = expanded_mask(sel, N, b_q, b_k)
    Ks = K - K.mean(axis=0)
    S = Q @ Ks.T / math.sqrt(d)
    E = np.where(M, np.exp(S - S.max(axis=1, keepdims=True)), 0.0)
    rs = E.sum(axis=1, keepdims=True)
    Ps = np.divide(E, rs, out=np.zeros_like(E), where=rs > 0)
    Os = Ps @ V

    def softmax_d(X):
        e = np.exp(X - X.max(axis=1, keepdims=True))
        return e / e.sum(axis=1, keepdims=True)
    A = (softmax_d(Q) @ softmax_d(Ks).T) * (~M)
    ra = A.sum(axis=1, keepdims=True)
    Pl = np.divide(A, ra, out=np.zeros_like(A), where=ra > 0)
    Ol = Pl @ V
    a = alpha_rows[:, None]
    return a * Os + (1 - a) * Ol, Os, Ol


# ---- (i) every block kept, alpha = 1: dense softmax attention ------------- #
@pytest.mark.parametrize("N,d,bq,bk", [(64, 8, 16, 8), (70, 8, 16, 8), (33, 4, 32, 16)])
def test_all_blocks_alpha1_is_dense_attention(N, d, bq, bk):
    Q, K, V, Wq, Wk = rand_head(1, N, d)
    r = O.forward_head(Q, K, V, Wq, Wk, 1.0, 1.0, bq, bk)
    assert r["sel"].shape[1] == O.num_blocks(N, bk)
    ref = dense_attention(Q, K, V)
    np.testing.assert_allclose(r["O"], ref, rtol=RTOL, atol=1e-12)


def test_dense_case_against_library_sdpa():
    torch = pytest.importorskip("torch")
    Q, K, V, Wq, Wk = rand_head(2, 96, 16)
    r = O.forward_head(Q, K, V, Wq, Wk, 1.0, 1.0, 32, 16)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q)[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None])[0].numpy()
    np.testing.assert_allclose(r["O"], ref, rtol=1e-9, atol=1e-12)


def test_lse_output_matches_logsumexp():
    Q, K, V, Wq, Wk = rand_head(3, 48, 8)
    r = O.forward_head(Q, K, V, Wq, Wk, 1.0, 1.0, 16, 8)
    S = Q @ K.T / math.sqrt(8)
    # smoothing K shifts every score of a row by q . mu
    mu = K.mean(axis=0)
    ref = np.log(np.exp(S).sum(axis=1)) - (Q @ mu) / math.sqrt(8)
    np.testing.assert_allclose(r["L"], ref, rtol=1e-10)


# ---- (ii) no block kept, alpha = 0: linear attention closed form ---------- #
@pytest.mark.parametrize("N,d,bq,bk", [(64, 8, 16, 8), (75, 8, 16, 8)])
def test_no_blocks_alpha0_is_linear_attention(N, d, bq, bk):
    Q, K, V, Wq, Wk = rand_head(4, N, d)
    r = O.forward_head(Q, K, V, Wq, Wk, 0.0, 0.0, bq, bk)
    assert r["sel"].shape[1] == 0

    def sm(X):
        e = np.exp(X)
        return e / e.sum(axis=1, keepdims=True)
    qf, kf = sm(Q), sm(K - K.mean(axis=0))
    ref = (qf @ (kf.T @ V)) / (qf @ (kf.T @ np.ones((N, 1))))      # Eq. 3 with M = 0
    np.testing.assert_allclose(r["O"], ref, rtol=RTOL)


# ---- (iii) complement identity ------------------------------------------- #
def test_complement_identity():
    N, d, bq, bk = 160, 8, 32, 16
    Q, K, V, Wq, Wk = rand_head(5, N, d)
    r = O.forward_head(Q, K, V, Wq, Wk, 0.4, 0.3, bq, bk)
    Ks = K - K.mean(axis=0)
    h, z = O.kv_state(O.phi(Ks), V, bk)
    for i in range(r["sel"].shape[0]):
        Hsub = h.sum(axis=0) - h[r["sel"][i]].sum(axis=0)
        Zsub = z.sum(axis=0) - z[r["sel"][i]].sum(axis=0)
        np.testing.assert_allclose(r["H"][i], Hsub, rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(r["Z"][i], Zsub, rtol=1e-9, atol=1e-12)


def test_kv_state_is_sum_of_outer_products():
    rng = np.random.default_rng(6)
    Kphi, V = rng.uniform(size=(20, 4)), rng.normal(size=(20, 4))
    h, z = O.kv_state(Kphi, V, 8)
    assert h.shape == (3, 4, 4)
    ref = sum(np.outer(Kphi[t], V[t]) for t in range(16, 20))
    np.testing.assert_allclose(h[2], ref, rtol=1e-12)
    np.testing.assert_allclose(z[2], Kphi[16:].sum(axis=0), rtol=1e-12)
    # orientation: h[c, e] pairs key channel c with value channel e
    assert not np.allclose(h[2], ref.T)


# ---- (iv) brute force with the expanded mask ------------------------------ #
@pytest.mark.parametrize("N,d,bq,bk,frac", [(128, 8, 32, 16, 0.25), (128, 8, 16, 16, 0.125),
                                            (150, 8, 32, 16, 0.3), (97, 4, 32, 8, 0.5)])
def test_brute_force_expanded_mask(N, d, bq, bk, frac):
    Q, K, V, Wq, Wk = rand_head(7, N, d, scale=1.5)
    T_m = O.num_blocks(N, bq)
    alpha = np.random.default_rng(8).uniform(size=T_m)
    r = O.forward_head(Q, K, V, Wq, Wk, alpha, frac, bq, bk)
    a_rows = np.repeat(alpha, bq)[:N]
    ref, ref_s, ref_l = brute_force(Q, K, V, r["sel"], a_rows, bq, bk)
    np.testing.assert_allclose(r["O_s"], ref_s, rtol=RTOL, atol=1e-13)
    np.testing.assert_allclose(r["O_l"], ref_l, rtol=RTOL, atol=1e-13)
    np.testing.assert_allclose(r["O"], ref, rtol=RTOL, atol=1e-13)


def test_q_blocks_subset_matches_full():
    Q, K, V, Wq, Wk = rand_head(9, 150, 8)
    full = O.forward_head(Q, K, V, Wq, Wk, 0.3, 0.3, 32, 16)
    for quant in (O.QUANT_NONE, O.QUANT_FP8):
        full = O.forward_head(Q, K, V, Wq, Wk, 0.3, 0.3, 32, 16, quant=quant)
        part = O.forward_head(Q, K, V, Wq, Wk, 0.3, 0.3, 32, 16, quant=quant, q_blocks=[4, 1])
        np.testing.assert_array_equal(part["O"][32:64], full["O"][32:64])
        np.testing.assert_array_equal(part["O"][128:], full["O"][128:])
        assert not part["O"][:32].any()


# ---- (v) alpha identity of Sec. 2.2 --------------------------------------- #
def test_alpha_identity():
    N, d, bq, bk = 96, 8, 32, 16
    Q, K, V, Wq, Wk = rand_head(10, N, d)
    r = O.forward_head(Q, K, V, Wq, Wk, 0.5, 0.34, bq, bk, smooth=False)
    S = Q @ K.T / math.sqrt(d)
    P = np.exp(S - S.max(axis=1, keepdims=True))
    P /= P.sum(axis=1, keepdims=True)                    # full attention
    M = expanded_mask(r["sel"], N, bq, bk)
    P1 = P * M
    a = P1.sum(axis=1, keepdims=True)                    # Eq. 7
    np.testing.assert_allclose(a * r["O_s"], P1 @ V, rtol=1e-9, atol=1e-13)   # Eq. 9


# ---- (vi) row normalisation: constant V rows ------------------------------ #
@pytest.mark.parametrize("quant", [O.QUANT_NONE])
def test_constant_value_rows(quant):
    N, d, bq, bk = 128, 8, 32, 16
    Q, K, V, Wq, Wk = rand_head(11, N, d)
    c = np.arange(1.0, d + 1.0)
    V = np.tile(c, (N, 1))
    alpha = np.random.default_rng(12).uniform(size=O.num_blocks(N, bq))
    r = O.forward_head(Q, K, V, Wq, Wk, alpha, 0.25, bq, bk, quant=quant)
    np.testing.assert_allclose(r["O"], V, rtol=1e-10)


# ---- (vii) router: orientation, brute-force ranking, invariances ---------- #
def test_router_projection_orientation():
    N, d, bq, bk = 64, 8, 16, 8
    Q, K, V, _, _ = rand_head(13, N, d)
    a, b, c = 2, 5, 6
    Wq = np.zeros((d, d)); Wq[a, b] = 1.0      # (x Wq)[b] = x[a]
    Wk = np.zeros((d, d)); Wk[c, b] = 1.0      # (x Wk)[b] = x[c]
    R = O.router_scores(Q, K, Wq, Wk, bq, bk)
    Qbar = Q.reshape(N // bq, bq, d).mean(axis=1)
    Kbar = K.reshape(N // bk, bk, d).mean(axis=1)
    ref = np.outer(Qbar[:, a], Kbar[:, c]) / math.sqrt(d)
    np.testing.assert_allclose(R, ref, rtol=1e-12, atol=1e-15)


def test_pool_ragged_tail():
    X = np.arange(22.0).reshape(11, 2)
    P = O.pool(X, 4)
    assert P.shape == (3, 2)
    np.testing.assert_allclose(P[0], [3.0, 4.0])
    np.testing.assert_allclose(P[2], [18.0, 19.0])     # mean of rows 8, 9, 10


def test_topk_is_brute_force_rank_with_low_index_ties():
    rng = np.random.default_rng(14)
    R = rng.integers(0, 6, size=(9, 20)).astype(float)     # many ties
    k = 7
    sel = O.topk_rows(R, k)
    for i in range(R.shape[0]):
        # entry j is kept iff fewer than k entries beat it, where "beats" is
        # strictly larger, or equal with a lower index
        kept = [j for j in range(R.shape[1])
                if sum(1 for t in range(R.shape[1])
                       if R[i, t] > R[i, j] or (R[i, t] == R[i, j] and t < j)) < k]
        assert list(sel[i]) == kept
    assert O.topk_rows(R, 0).shape == (9, 0)
    assert np.array_equal(O.topk_rows(R, 20), np.tile(np.arange(20), (9, 1)))


def test_num_selected_matches_stated_workloads():
    # "top 2 of 16"; 5 % of 512 -> 26; 3 % of 512 -> 15; 3 % of 1182 -> 35
    assert O.num_selected(0.125, 16) == 2
    assert O.num_selected(0.05, 512) == 26
    assert O.num_selected(0.03, 512) == 15
    assert O.num_selected(0.03, 1182) == 35
    assert O.num_selected(0.0, 10) == 0 and O.num_selected(1.0, 10) == 10


def test_mask_invariances():
    N, d, bq, bk = 256, 8, 32, 16
    Q, K, V, Wq, Wk = rand_head(15, N, d)
    base = O.forward_head(Q, K, V, Wq, Wk, 0.5, 0.25, bq, bk)
    # adding one vector to every key changes nothing downstream (K is smoothed)
    shift = O.forward_head(Q, K + np.linspace(-3, 3, d), V, Wq, Wk, 0.5, 0.25, bq, bk)
    assert np.array_equal(base["sel"], shift["sel"])
    np.testing.assert_allclose(shift["O"], base["O"], rtol=1e-9, atol=1e-12)
    # without smoothing the mask and the sparse branch still do not move
    raw = O.forward_head(Q, K, V, Wq, Wk, 0.5, 0.25, bq, bk, smooth=False)
    assert np.array_equal(base["sel"], raw["sel"])
    np.testing.assert_allclose(raw["O_s"], base["O_s"], rtol=1e-9, atol=1e-12)
    # the row softmax and the 1/sqrt(d) of Alg. 2's router step keep the top-k
    R = base["R"]
    Pc = np.exp(R - R.max(axis=1, keepdims=True))
    Pc /= Pc.sum(axis=1, keepdims=True)
    k = base["sel"].shape[1]
    assert np.array_equal(O.topk_rows(Pc, k), base["sel"])
    assert np.array_equal(O.topk_rows(R * math.sqrt(d), k), base["sel"])
    # proj = I recovers the pooled-QK router of SLA (Sec. 8, insight 1.c)
    eye = O.forward_head(Q, K, V, np.eye(d), np.eye(d), 0.5, 0.25, bq, bk, smooth=False)
    Qbar = Q.reshape(-1, bq, d).mean(axis=1)
    Kbar = K.reshape(-1, bk, d).mean(axis=1)
    assert np.array_equal(eye["sel"], O.topk_rows(Qbar @ Kbar.T, k))


# ---- (viii) permuting whole key/value blocks ------------------------------ #
def test_kv_block_permutation():
    N, d, bq, bk = 128, 8, 32, 16
    Q, K, V, Wq, Wk = rand_head(16, N, d)
    T_n = N // bk
    perm = np.random.default_rng(17).permutation(T_n)
    rows = np.concatenate([np.arange(p * bk, (p + 1) * bk) for p in perm])
    a = O.forward_head(Q, K, V, Wq, Wk, 0.6, 0.25, bq, bk)
    b = O.forward_head(Q, K[rows], V[rows], Wq, Wk, 0.6, 0.25, bq, bk)
    np.testing.assert_allclose(b["O"], a["O"], rtol=1e-9, atol=1e-12)
    inv = np.argsort(perm)                 # old block p sits at new position inv[p]
    for i in range(a["sel"].shape[0]):
        assert sorted(inv[a["sel"][i]]) == list(b["sel"][i])


# ---- (ix) a case worked by hand ------------------------------------------- #
def test_hand_worked_micro_case():
    """N = 4, d = 2, b_q = b_k = 2, k = 1, Wq = Wk = I.

    Smoothed keys K' = ln2 * [[1,0],[0,2],[-1,-1],[0,-1]] (columns sum to 0);
    the keys handed in are K' + ln2 * (3,-1), so the smoothing step must undo
    the offset.  Q = sqrt2 * [[1,0],[1,2],[-1,0],[0,-2]], so that every score
    q.k'/sqrt2 is an integer multiple of ln2 and every softmax weight is a ratio
    of powers of two.  V = [[1,0],[0,1],[2,2],[-1,1]].

    Router: Qbar = sqrt2*[(1,1),(-1/2,-1)], Kbar = ln2*[(1/2,1),(-1/2,-1)];
    R = ln2*[[3/2,-3/2],[-5/4,5/4]] / ... > block 0 keeps kv block 0, block 1
    keeps kv block 1.

    Sparse branch (weights 2^(q.k'/ (sqrt2 ln2))):
      row0: (2,1)/3  -> (2/3,1/3)         L = ln 3
      row1: (2,16)/18-> (1/9,8/9)         L = ln 18
      row2: (2,1)/3  -> (2*2-1, 2*2+1)/3 = (1,5/3)   L = ln 3
      row3: (4,4)/8  -> (1/2,3/2)         L = ln 8
    phi(K') rows: (2,1)/3, (1,4)/5, (1,1)/2, (2,1)/3.
      h_0 = [[2/3,1/5],[1/3,4/5]]  z_0 = (13/15,17/15)
      h_1 = [[1/3,5/3],[2/3,4/3]]  z_1 = (7/6,5/6)
    Linear branch, phi(q) = (p, 1-p), p = sigmoid(q_0 - q_1):
      block 0 uses (h_1, z_1): O_l = (2(2-p), 2(4+p)) / (5+2p)
      block 1 uses (h_0, z_0): O_l = (5(1+p), 3(4-3p)) / (17-4p)
    alpha = (1/4, 3/4) per query block.
    """
    ln2, s2 = math.log(2.0), math.sqrt(2.0)
    Kp = ln2 * np.array([[1, 0], [0, 2], [-1, -1], [0, -1]], dtype=float)
    K = Kp + ln2 * np.array([3.0, -1.0])
    Q = s2 * np.array([[1, 0], [1, 2], [-1, 0], [0, -2]], dtype=float)
    V = np.array([[1, 0], [0, 1], [2, 2], [-1, 1]], dtype=float)
    alpha = np.array([0.25, 0.75])
    r = O.forward_head(Q, K, V, np.eye(2), np.eye(2), alpha, 0.5, 2, 2)

    np.testing.assert_allclose(r["R"], ln2 * np.array([[1.5, -1.5], [-1.25, 1.25]]), rtol=1e-12)
    assert r["sel"].tolist() == [[0], [1]]
    Os = np.array([[F(2, 3), F(1, 3)], [F(1, 9), F(8, 9)], [F(1), F(5, 3)], [F(1, 2), F(3, 2)]], dtype=float)
    np.testing.assert_allclose(r["O_s"], Os, rtol=1e-12)
    np.testing.assert_allclose(r["L"], np.log([3.0, 18.0, 3.0, 8.0]), rtol=1e-12)
    np.testing.assert_allclose(r["H"][0], np.array([[F(1, 3), F(5, 3)], [F(2, 3), F(4, 3)]], dtype=float), rtol=1e-12)
    np.testing.assert_allclose(r["H"][1], np.array([[F(2, 3), F(1, 5)], [F(1, 3), F(4, 5)]], dtype=float), rtol=1e-12)
    np.testing.assert_allclose(r["Z"][0], [7 / 6, 5 / 6], rtol=1e-12)
    np.testing.assert_allclose(r["Z"][1], [13 / 15, 17 / 15], rtol=1e-12)

    def sig(x):
        return 1.0 / (1.0 + math.exp(-x))
    p = [sig(s2 * 1), sig(s2 * -1), sig(s2 * -1), sig(s2 * 2)]
    Ol = np.array([
        [2 * (2 - p[0]) / (5 + 2 * p[0]), 2 * (4 + p[0]) / (5 + 2 * p[0])],
        [2 * (2 - p[1]) / (5 + 2 * p[1]), 2 * (4 + p[1]) / (5 + 2 * p[1])],
        [5 * (1 + p[2]) / (17 - 4 * p[2]), 3 * (4 - 3 * p[2]) / (17 - 4 * p[2])],
        [5 * (1 + p[3]) / (17 - 4 * p[3]), 3 * (4 - 3 * p[3]) / (17 - 4 * p[3])]])
    np.testing.assert_allclose(r["O_l"], Ol, rtol=1e-12)
    a = np.array([0.25, 0.25, 0.75, 0.75])[:, None]
    np.testing.assert_allclose(r["O"], a * Os + (1 - a) * Ol, rtol=1e-12)


# ---- (x) low-bit branch ---------------------------------------------------- #
def e4m3_table():
    """All finite e4m3 values from the format's definition: sign, 4 exponent
    bits (bias 7), 3 mantissa bits; exponent 0 is subnormal; code S.1111.111 is
    NaN, every other code is finite (no infinities)."""
    vals = []
    for code in range(256):
        s, e, m = code >> 7, (code >> 3) & 15, code & 7
        if e == 15 and m == 7:
            continue
        mag = (m / 8.0) * 2.0 ** -6 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7)
        vals.append(-mag if s else mag)
    return np.array(sorted(set(vals)))


def test_e4m3_round_is_nearest_even_saturating():
    tab = e4m3_table()
    assert tab.max() == 448.0 and np.min(tab[tab > 0]) == 2.0 ** -9 and len(tab) == 253
    # every representable value is a fixed point
    np.testing.assert_array_equal(O.e4m3_round(tab.astype(np.float32)), tab.astype(np.float32))
    rng = np.random.default_rng(18)
    x = np.concatenate([rng.normal(size=4000) * 3, rng.normal(size=4000) * 200,
                        rng.normal(size=2000) * 0.01, rng.uniform(-470, 470, size=2000),
                        (tab[:-1] + tab[1:]) / 2,                 # exact midpoints
                        [0.0, 448.0, 449.0, 463.9, 464.0, 480.0, 1e6, -1e6, 2.0 ** -10, 2.0 ** -10 * 1.01]]
                       ).astype(np.float32)
    got = O.e4m3_round(x)
    pos = tab[tab >= 0]
    mant_even = {v: (int(round(v / 2.0 ** -9)) if v < 2.0 ** -6 else
                     int(round(v / 2.0 ** (math.floor(math.log2(v)) - 3)))) % 2 == 0 for v in pos if v > 0}
    mant_even[0.0] = True
    for xi, gi in zip(x.astype(np.float64), got.astype(np.float64)):
        a = abs(xi)
        if a >= 448.0:
            want = 448.0
        else:
            dist = np.abs(pos - a)
            best = np.nonzero(dist == dist.min())[0]
            want = pos[best[0]] if len(best) == 1 else next(pos[b] for b in best if mant_even[pos[b]])
        assert gi == math.copysign(want, xi), (xi, gi, want)


def test_quant_block_scale_and_grid():
    rng = np.random.default_rng(19)
    X = (rng.normal(size=(16, 8)) * 2.5).astype(np.float32)
    v, s = O.quant_block_e4m3(X)
    tab = set(e4m3_table().tolist())
    assert all(float(t) in tab for t in v.ravel())
    assert np.abs(v).max() == 448.0                      # the block's largest entry maps to the top code
    assert s == np.float32(np.abs(X).max()) / np.float32(448)
    # dequantised values stay within half a grid step (relative 2^-4) of x
    assert np.all(np.abs(v * s - X) <= np.abs(X) * 2.0 ** -4 + s * 2.0 ** -10)
    v0, s0 = O.quant_block_e4m3(np.zeros((4, 4), np.float32))
    assert not v0.any() and s0 == 1.0


def test_lowbit_branch_reduces_to_exact_when_quantisers_are_exact(monkeypatch):
    """With rounding switched off the step-by-step online softmax of Alg. 2 must
    reproduce the plain definition - this pins the loop (running max, rescale,
    running sum, final division) independently of the number format."""
    N, d, bq, bk = 150, 8, 32, 16
    Q, K, V, Wq, Wk = rand_head(20, N, d)
    Q, K, V = (a.astype(np.float32).astype(np.float64) for a in (Q, K, V))
    sel = O.forward_head(Q, K, V, Wq, Wk, 1.0, 0.3, bq, bk)["sel"]
    monkeypatch.setattr(O, "e4m3_round", lambda x: np.asarray(x, dtype=np.float32))
    monkeypatch.setattr(O, "quant_block_e4m3", lambda X: (np.asarray(X, np.float32), np.float32(1.0)))
    lo, Llo = O.sparse_branch_lowbit(Q, K, V, sel, bq, bk)
    ex, Lex = O.sparse_branch(Q, O.smooth_k(K), V, sel, bq, bk)
    # float32 P and float32 smoothed K are the only roundings left
    np.testing.assert_allclose(lo, ex, rtol=0, atol=5e-6)
    np.testing.assert_allclose(Llo, Lex, rtol=0, atol=5e-6)


def test_lowbit_branch_close_to_exact_and_order_sensitive():
    N, d, bq, bk = 512, 64, 64, 64
    Q, K, V, Wq, Wk = rand_head(21, N, d)
    ex = O.forward_head(Q, K, V, Wq, Wk, 1.0, 0.25, bq, bk)
    lo = O.forward_head(Q, K, V, Wq, Wk, 1.0, 0.25, bq, bk, quant=O.QUANT_FP8)
    rel = np.linalg.norm(lo["O"] - ex["O"]) / np.linalg.norm(ex["O"])
    assert 1e-4 < rel < 5e-2, rel
    np.testing.assert_allclose(lo["L"], ex["L"], atol=0.1)


def test_lowbit_products_are_exact_in_float64():
    """Products of two e4m3 values have at most 8 significant bits, sums of 128
    of them (|.| <= 448^2) fit float64 exactly: the oracle's Qhat Khat^T is the
    exact integer-grid result."""
    rng = np.random.default_rng(22)
    a = O.e4m3_round((rng.normal(size=(8, 128)) * 100).astype(np.float32)).astype(np.float64)
    b = O.e4m3_round((rng.normal(size=(8, 128)) * 100).astype(np.float32)).astype(np.float64)
    S = a @ b.T
    exact = np.array([[sum(F(x) * F(y) for x, y in zip(ra, rb)) for rb in b] for ra in a], dtype=object)
    assert all(F(S[i, j]) == exact[i, j] for i in range(8) for j in range(8))


# ---- backward pass (Alg. 3) ------------------------------------------------- #
def _expanded_forward_torch(Q, K, V, M, a_rows, smooth):
    """Eq. 13-14 with the N x N mask, in library tensor ops (no blocks, no online softmax)."""
    import torch
    d = Q.shape[1]
    Ks = K - K.mean(dim=0, keepdim=True) if smooth else K
    S = (Q @ Ks.T) / math.sqrt(d)
    S = S.masked_fill(~M, float("-inf"))
    Ps = torch.softmax(S, dim=1)
    Ps = torch.nan_to_num(Ps, nan=0.0)                 # rows with no selected key
    Os = Ps @ V
    A = (torch.softmax(Q, dim=1) @ torch.softmax(Ks, dim=1).T) * (~M)
    den = A.sum(dim=1, keepdim=True)
    Ol = torch.where(den > 0, (A @ V) / torch.where(den > 0, den, torch.ones_like(den)), torch.zeros_like(A @ V))
    return a_rows * Os + (1 - a_rows) * Ol


@pytest.mark.parametrize("N,d,bq,bk,frac,smooth,per_block", [
    (150, 8, 32, 16, 0.3, True, False), (96, 16, 32, 16, 0.34, False, True), (70, 8, 32, 16, 0.0, True, True),
    (64, 8, 32, 16, 1.0, True, False), (130, 4, 64, 64, 0.5, True, True),
])
def test_backward_matches_autograd_of_the_expanded_mask_definition(N, d, bq, bk, frac, smooth, per_block):
    import torch
    Q, K, V, Wq, Wk = rand_head(40 + N, N, d)
    rng = np.random.default_rng(41)
    T_m, T_n = O.num_blocks(N, bq), O.num_blocks(N, bk)
    alpha = rng.uniform(0.1, 0.9, size=T_m) if per_block else 0.37
    sel = O.topk_rows(O.router_scores(Q, O.smooth_k(K) if smooth else K, Wq, Wk, bq, bk), O.num_selected(frac, T_n))
    dO = rng.normal(size=(N, d))
    got = O.backward_head(Q, K, V, sel, alpha, dO, bq, bk, smooth=smooth)

    M = np.kron(O.mask_from_sel(sel, T_n), np.ones((bq, bk), dtype=bool))[:N, :N]
    a_blk = np.broadcast_to(np.asarray(alpha, dtype=np.float64).reshape(-1), (T_m,))
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (Q, K, V))
    ta = torch.tensor(a_blk.copy(), dtype=torch.float64, requires_grad=True)
    a_rows = ta.repeat_interleave(bq)[:N, None]
    out = _expanded_forward_torch(tq, tk, tv, torch.tensor(M), a_rows, smooth)
    # the oracle's forward and the expanded form agree, so the same dO is the same cotangent
    fwd = O.forward_head(Q, K, V, Wq, Wk, alpha, frac, bq, bk, smooth=smooth, sel=sel)["O"]
    np.testing.assert_allclose(out.detach().numpy(), fwd, rtol=0, atol=1e-12)
    out.backward(torch.tensor(dO))
    np.testing.assert_allclose(got["dQ"], tq.grad.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(got["dK"], tk.grad.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(got["dV"], tv.grad.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(got["dalpha"], ta.grad.numpy(), rtol=0, atol=1e-11)


def test_backward_central_differences():
    N, d, bq, bk = 48, 4, 16, 16
    Q, K, V, Wq, Wk = rand_head(45, N, d)
    rng = np.random.default_rng(46)
    sel = O.topk_rows(O.router_scores(Q, O.smooth_k(K), Wq, Wk, bq, bk), 1)
    dO = rng.normal(size=(N, d))
    g = O.backward_head(Q, K, V, sel, 0.6, dO, bq, bk)
    f = lambda q, k, v: (O.forward_head(q, k, v, Wq, Wk, 0.6, 0.3, bq, bk, sel=sel)["O"] * dO).sum()
    eps = 1e-6
    for name, X, idx in (("dQ", Q, (5, 2)), ("dK", K, (17, 1)), ("dV", V, (40, 3)), ("dK", K, (47, 0))):
        Xp, Xm = X.copy(), X.copy()
        Xp[idx] += eps; Xm[idx] -= eps
        args_p = [Xp if A is X else A for A in (Q, K, V)]
        args_m = [Xm if A is X else A for A in (Q, K, V)]
        fd = (f(*args_p) - f(*args_m)) / (2 * eps)
        assert abs(fd - g[name][idx]) < 1e-7 * max(1.0, abs(fd)), (name, idx, fd, g[name][idx])


@pytest.mark.parametrize("quant", [O.QUANT_FP8, O.QUANT_INT8, O.QUANT_FP8_V])
def test_backward_after_a_low_bit_forward(quant):
    """Sec. 5: the backward pass runs in high precision on the original Q, K, V and takes from a low-bit
    forward only that forward's outputs.  Against the backward of the exact forward: nothing of the
    linear branch moves; the sparse branch moves exactly as the N x N expanded form says when its L and
    O^s are replaced by the low-bit forward's (P = exp(S - L), D^s = rowsum(dO^s (.) O^s))."""
    N, d, bq, bk = 96, 16, 32, 16
    Q, K, V, Wq, Wk = rand_head(50, N, d)
    rng = np.random.default_rng(51)
    alpha = 0.4
    T_n = O.num_blocks(N, bk)
    Ks = O.smooth_k(K)
    sel = O.topk_rows(O.router_scores(Q, Ks, Wq, Wk, bq, bk), O.num_selected(0.34, T_n))
    dO = rng.normal(size=(N, d))
    g0 = O.backward_head(Q, K, V, sel, alpha, dO, bq, bk)
    g8 = O.backward_head(Q, K, V, sel, alpha, dO, bq, bk, quant=quant)
    assert np.array_equal(g0["Dl"], g8["Dl"]) and np.array_equal(g0["dQphi"], g8["dQphi"])
    assert np.array_equal(g0["dKphi"], g8["dKphi"])
    ex = O.forward_head(Q, K, V, Wq, Wk, alpha, 0.34, bq, bk, sel=sel)
    lo = O.forward_head(Q, K, V, Wq, Wk, alpha, 0.34, bq, bk, sel=sel, quant=quant)
    assert not np.array_equal(ex["O_s"], lo["O_s"])
    M = np.kron(O.mask_from_sel(sel, T_n), np.ones((bq, bk), dtype=bool))[:N, :N]
    S = Q @ Ks.T / math.sqrt(d)
    dOs = alpha * dO
    dP = dOs @ V.T

    def sparse_terms(L, Os):
        P = np.where(M, np.exp(S - L[:, None]), 0.0)
        dS = P * (dP - (dOs * Os).sum(axis=1)[:, None])
        return P.T @ dOs, dS @ Ks / math.sqrt(d), dS.T @ Q / math.sqrt(d)

    dv0, dq0, dk0 = sparse_terms(ex["L"], ex["O_s"])
    dv8, dq8, dk8 = sparse_terms(lo["L"], lo["O_s"])
    np.testing.assert_allclose(g8["dV"] - g0["dV"], dv8 - dv0, rtol=0, atol=1e-12)
    np.testing.assert_allclose(g8["dQ"] - g0["dQ"], dq8 - dq0, rtol=0, atol=1e-12)
    dk_shift = dk8 - dk0
    np.testing.assert_allclose(g8["dK"] - g0["dK"], dk_shift - dk_shift.mean(axis=0, keepdims=True), rtol=0, atol=1e-12)
    np.testing.assert_allclose(g8["dalpha"].sum() - g0["dalpha"].sum(), (dO * (lo["O_s"] - ex["O_s"])).sum(), rtol=0, atol=1e-12)
    # and the move is of the size of the forward's own quantisation error, not more
    fwd_err = np.linalg.norm(lo["O_s"] - ex["O_s"]) / np.linalg.norm(ex["O_s"])
    for name in ("dQ", "dK", "dV"):
        move = np.linalg.norm(g8[name] - g0[name]) / np.linalg.norm(g0[name])
        assert 0.0 < move <= 20.0 * fwd_err, (name, move, fwd_err)


# ---- SoftTop-k (Sec. 6) ---------------------------------------------------- #
def test_soft_topk_row_sums_range_and_order():
    rng = np.random.default_rng(30)
    R = rng.normal(size=(7, 40)) * 3.0
    for k in (1, 5, 39):
        M = O.soft_topk_rows(R, k, tau=0.1)
        np.testing.assert_allclose(M.sum(axis=1), k, rtol=0, atol=1e-9)
        assert np.all(M > 0) and np.all(M < 1)
        for i in range(R.shape[0]):                   # larger score, larger weight
            o = np.argsort(R[i])
            assert np.all(np.diff(M[i, o]) >= 0)
    assert not O.soft_topk_rows(R, 0).any()
    assert np.all(O.soft_topk_rows(R, 40) == 1.0)


def test_soft_topk_closed_forms():
    # equal scores: every entry k / T_n whatever tau
    M = O.soft_topk_rows(np.full((2, 10), 0.7), 3, tau=0.05)
    np.testing.assert_allclose(M, 0.3, rtol=0, atol=1e-12)
    # two columns, k = 1: sigmoid(a + l) + sigmoid(b + l) = 1  <=>  l = -(a + b) / 2
    R = np.array([[0.3, -1.1]])
    e = np.exp(R[0] - R[0].max()); p = e / e.sum()
    tau = 0.2
    lam = -(p[0] + p[1]) / (2 * tau)
    want = 1.0 / (1.0 + np.exp(-(p / tau + lam)))
    np.testing.assert_allclose(O.soft_topk_rows(R, 1, tau=tau)[0], want, rtol=0, atol=1e-12)
    # a per-row constant added to the scores changes nothing (softmax), a permutation permutes
    rng = np.random.default_rng(31)
    R = rng.normal(size=(3, 12))
    A = O.soft_topk_rows(R, 4)
    np.testing.assert_allclose(O.soft_topk_rows(R + np.array([[5.0], [-2.0], [0.5]]), 4), A, rtol=0, atol=1e-12)
    perm = rng.permutation(12)
    np.testing.assert_allclose(O.soft_topk_rows(R[:, perm], 4), A[:, perm], rtol=0, atol=1e-12)


def test_soft_topk_tends_to_the_hard_mask():
    rng = np.random.default_rng(32)
    R = rng.normal(size=(5, 16)) * 1.5               # softmax values spread over (0, 0.5)
    k = 3
    hard = O.mask_from_sel(O.topk_rows(R, k), 16).astype(np.float64)
    soft = O.soft_topk_rows(R, k, tau=1e-5)
    # entries of the softmax closer than a few tau to the k-th / (k+1)-th boundary stay soft
    e = np.exp(R - R.max(axis=1, keepdims=True)); P = e / e.sum(axis=1, keepdims=True)
    srt = np.sort(P, axis=1)[:, ::-1]
    clear = (np.abs(P - 0.5 * (srt[:, k - 1] + srt[:, k])[:, None]) > 30e-5)
    assert clear.mean() > 0.8
    np.testing.assert_allclose(soft[clear], hard[clear], rtol=0, atol=1e-6)
    # and the order of the soft weights is the order the hard mask cuts
    for i in range(5):
        assert set(np.argsort(-soft[i])[:k]) == set(np.nonzero(hard[i])[0])


# ---- INT8 form of the Q/K quantiser (Sec. 5) ------------------------------- #
def test_quant_block_int8_is_nearest_integer_symmetric():
    rng = np.random.default_rng(23)
    X = (rng.normal(size=(16, 8)) * 3.0).astype(np.float32)
    X[3, 2] = -np.abs(X).max() * np.float32(1.5)          # the extreme entry is negative: the range must be symmetric
    codes, s = O.quant_block_int8(X)
    amax = np.float32(np.abs(X).max())
    assert s == amax / np.float32(127)
    assert codes.min() == -127.0 and codes.max() <= 127.0   # -128 is never produced
    assert np.array_equal(codes, np.round(codes))
    # brute force: the nearest integer to the float32 product x * inv, ties to the even integer
    inv = np.float32(127) / amax
    grid = np.arange(-127, 128, dtype=np.float64)
    for x, c in zip(X.ravel(), codes.ravel()):
        y = float(np.float32(x) * inv)
        dist = np.abs(grid - y)
        best = grid[dist == dist.min()]
        want = best[0] if len(best) == 1 else next(b for b in best if int(b) % 2 == 0)
        assert c == want, (x, y, c, want)
    # dequantised values stay within half a step of x (plus the float32 rounding of the product)
    assert np.all(np.abs(codes * s - X) <= 0.5 * s * (1 + 1e-5))
    c0, s0 = O.quant_block_int8(np.zeros((4, 4), np.float32))
    assert not c0.any() and s0 == 1.0


def test_quant_block_int8_ties_go_to_even():
    # amax = 127 makes inv exactly 1: the codes are rint(x)
    X = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 63.5, 64.5]], dtype=np.float32)
    codes, s = O.quant_block_int8(X)
    assert s == 1.0
    np.testing.assert_array_equal(codes[0], [127, 0, 2, 2, -0.0, -2, -2, 64, 64])


def test_int8_branch_reduces_to_exact_when_quantiser_is_exact(monkeypatch):
    """The INT8 mode shares the block loop of the FP8 mode; only the quantiser of Q and K
    differs.  With both roundings switched off it must give the plain definition."""
    N, d, bq, bk = 150, 8, 32, 16
    Q, K, V, Wq, Wk = rand_head(24, N, d)
    Q, K, V = (a.astype(np.float32).astype(np.float64) for a in (Q, K, V))
    sel = O.forward_head(Q, K, V, Wq, Wk, 1.0, 0.3, bq, bk)["sel"]
    monkeypatch.setattr(O, "e4m3_round", lambda x: np.asarray(x, dtype=np.float32))
    monkeypatch.setattr(O, "quant_block_int8", lambda X: (np.asarray(X, np.float32), np.float32(1.0)))
    lo = O.forward_head(Q, K, V, Wq, Wk, 1.0, 0.3, bq, bk, quant=O.QUANT_INT8, sel=sel)
    ex = O.forward_head(Q, K, V, Wq, Wk, 1.0, 0.3, bq, bk, sel=sel)
    np.testing.assert_allclose(lo["O"], ex["O"], rtol=0, atol=5e-6)
    np.testing.assert_allclose(lo["L"], ex["L"], rtol=0, atol=5e-6)


def test_int8_branch_close_to_exact_and_tighter_than_fp8_scores():
    N, d, bq, bk = 512, 64, 64, 64
    Q, K, V, Wq, Wk = rand_head(21, N, d)
    ex = O.forward_head(Q, K, V, Wq, Wk, 1.0, 0.25, bq, bk)
    i8 = O.forward_head(Q, K, V, Wq, Wk, 1.0, 0.25, bq, bk, quant=O.QUANT_INT8)
    f8 = O.forward_head(Q, K, V, Wq, Wk, 1.0, 0.25, bq, bk, quant=O.QUANT_FP8)
    rel = np.linalg.norm(i8["O"] - ex["O"]) / np.linalg.norm(ex["O"])
    assert 1e-4 < rel < 5e-2, rel
    # the scores (seen through the log-sum-exp) carry 7 fraction bits of a block-wide scale in INT8
    # against 3 mantissa bits in e4m3: for Gaussian blocks the INT8 scores are the closer ones
    err_i8 = np.abs(i8["L"] - ex["L"]).mean()
    err_f8 = np.abs(f8["L"] - ex["L"]).mean()
    assert err_i8 < err_f8, (err_i8, err_f8)
    assert np.array_equal(i8["sel"], ex["sel"])                     # the router never sees the codes


# ---- FP8 V in the second product (Alg. 2 as printed) ------------------------ #
def test_fp8v_branch_reduces_to_exact_when_quantisers_are_exact(monkeypatch):
    N, d, bq, bk = 150, 8, 32, 16
    Q, K, V, Wq, Wk = rand_head(25, N, d)
    Q, K, V = (a.astype(np.float32).astype(np.float64) for a in (Q, K, V))
    sel = O.forward_head(Q, K, V, Wq, Wk, 1.0, 0.3, bq, bk)["sel"]
    monkeypatch.setattr(O, "e4m3_round", lambda x: np.asarray(x, dtype=np.float32))
    # an "exact quantiser" with a scale that is not 1: the scale must come back exactly once
    monkeypatch.setattr(O, "quant_block_e4m3", lambda X: (np.asarray(X, np.float32) * np.float32(4), np.float32(0.25)))
    lo = O.forward_head(Q, K, V, Wq, Wk, 1.0, 0.3, bq, bk, quant=O.QUANT_FP8_V, sel=sel)
    ex = O.forward_head(Q, K, V, Wq, Wk, 1.0, 0.3, bq, bk, sel=sel)
    np.testing.assert_allclose(lo["O"], ex["O"], rtol=0, atol=5e-6)
    np.testing.assert_allclose(lo["L"], ex["L"], rtol=0, atol=5e-6)


def test_fp8v_differs_from_fp8_only_through_v_and_leaves_the_linear_branch_alone():
    N, d, bq, bk = 512, 64, 64, 64
    Q, K, V, Wq, Wk = rand_head(21, N, d)
    f8 = O.forward_head(Q, K, V, Wq, Wk, 0.4, 0.25, bq, bk, quant=O.QUANT_FP8)
    f8v = O.forward_head(Q, K, V, Wq, Wk, 0.4, 0.25, bq, bk, quant=O.QUANT_FP8_V)
    ex = O.forward_head(Q, K, V, Wq, Wk, 0.4, 0.25, bq, bk)
    np.testing.assert_array_equal(f8v["O_l"], f8["O_l"])          # h_j is built from the input V
    np.testing.assert_array_equal(f8v["L"], f8["L"])              # the scores never see V
    rel = lambda a, b: np.linalg.norm(a - b) / np.linalg.norm(b)
    e8, e8v = rel(f8["O_s"], ex["O_s"]), rel(f8v["O_s"], ex["O_s"])
    assert e8 < e8v < 5e-2, (e8, e8v)                             # one more rounding, still small
    # a V that is exactly representable (all entries on the e4m3 grid after its block scale) changes nothing
    Vg = np.sign(V) * 2.0 ** np.round(np.log2(np.abs(V) + 1e-30))       # powers of two, spread < 2^15 per block
    Vg = np.clip(Vg, -2.0, 2.0)
    Vg[np.abs(Vg) < 2.0 ** -4] = 2.0 ** -4
    Vg[::bk] = 3.5                                                        # every block's amax, exactly on the grid: scale 2^-7
    a = O.forward_head(Q, K, Vg, Wq, Wk, 1.0, 0.25, bq, bk, quant=O.QUANT_FP8)
    b = O.forward_head(Q, K, Vg, Wq, Wk, 1.0, 0.25, bq, bk, quant=O.QUANT_FP8_V)
    np.testing.assert_allclose(b["O"], a["O"], rtol=1e-12, atol=1e-12)


# ---- Table 1: the shapes behind the dense-equivalent FLOP count ----------- #
def test_table1_flops_confirm_workload_shapes():
    import os
    rows = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "table1_flops.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                m, s, v = line.split()
                rows[(m, int(s))] = float(v)
    # C = 4 N^2 d per head (Sec. 9.1, "Metrics"); the table's full-attention rows
    # equal C*H times a constant (8 and 2.5: not explained in the paper)
    assert round(4 * 32760 ** 2 * 128 * 12 * 8 / 1e12, 2) == rows[("wan1.3b", 0)]
    assert round(4 * 75600 ** 2 * 128 * 40 * 2.5 / 1e12, 1) == rows[("wan14b", 0)]
    # "29x" of Sec. 9.2 is the ratio of the table's FLOPs at 97 %
    assert round(rows[("wan1.3b", 0)] / rows[("wan1.3b", 97)]) == 29
