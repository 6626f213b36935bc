"""fp64 CPU statement of the SLA2 attention forward pass.  TEST INFRASTRUCTURE ONLY.

This file is the yardstick the HIP kernels are measured against.  It is slow on
purpose: every function is the paper's definition (or, where the result depends
on the order of operations, the paper's algorithm step by step) written out
with numpy in float64, one (batch, head) at a time, with no blocking, fusion or
reordering beyond what the cited passage states.  It shares no code, table or
constant with the HIP path and is never imported by it; only tests, the smoke
check and the benchmark's CPU-baseline leg may call it.

Notation follows the paper: Q, K, V are N x d per head; b_q, b_k are the query
and key/value block sizes; T_m = ceil(N/b_q), T_n = ceil(N/b_k); M_c is the
T_m x T_n block mask, stored here as `sel`, an int array [T_m, k] holding for
each query block the ascending indices of its k selected key/value blocks.

Where the paper is silent or contradicts itself, the reading taken is stated in
the docstring of the function concerned.  Pins (what fixes each function
independently of itself) live in tests/test_oracle_pins.py:

  smooth_k, phi, pool        closed forms + brute force with the expanded mask
  router_scores, topk_rows   single-entry projections (orientation), brute-force
                             ranking, invariances the paper's text implies
  soft_topk_rows             row sums, the closed form for equal scores and for two
                             columns, order preservation, the hard mask as tau -> 0
  sparse_branch              dense softmax attention when every block is kept;
                             library SDPA; hand-worked micro case; alpha identity
  linear_branch              linear-attention closed form when no block is kept;
                             complement identity; hand-worked micro case
  forward_head               N x N expanded-mask evaluation of Eq. 13-14;
                             constant-V invariance; block permutation
  backward_head              automatic differentiation (library autograd, float64)
                             of the N x N expanded-mask evaluation of Eq. 13-14;
                             central differences
  e4m3_round                 nearest-with-ties-to-even search over the table of
                             all 256 codes built from the format's definition
  quant_block_int8           codes against a brute-force nearest-integer search;
                             range, symmetry, scale round trip
  sparse_branch_lowbit,      equal sparse_branch when the quantisers are made exact; cases worked by hand
  absorb_block, smooth_k_f32 (tests/test_oracle_lowbit_pins.py): weights that are powers of two and must
                             come out exact, weights that need a fourth mantissa bit, a subnormal
                             and a flushed weight, a maximum that moves between blocks, the
                             float32 smoothing on inputs where the order of rounding shows; each
                             of a dozen planted slips fails one of them.  The quantisation
                             scheme itself (granularity, scale of P) is NOT fixed by the paper:
                             what is pinned is the definition given in the docstrings.
"""
from __future__ import annotations

import math

import numpy as np

QUANT_NONE = 0
QUANT_FP8 = 1
QUANT_INT8 = 2
QUANT_FP8_V = 3           # FP8 mode with V quantised as well (Alg. 2 as printed: quant(P) quant(V_j))

E4M3_MAX = 448.0          # largest finite magnitude of the OCP e4m3 format
INT8_MAX = 127.0          # symmetric int8 range used for Q and K codes
P_SCALE_LOG2 = 8          # P is rounded on the e4m3 grid after scaling by 2**8


# --------------------------------------------------------------------------- #
# small definitions
# --------------------------------------------------------------------------- #
def num_blocks(N: int, b: int) -> int:
    """T = ceil(N / b).  Alg. 2 (forward pass) divides the sequence into N/b blocks and assumes b
    divides N; a ragged
    last block simply holds the remaining N - (T-1) b tokens."""
    return (N + b - 1) // b


def num_selected(topk_frac: float, T_n: int) -> int:
    """k = number of key/value blocks each query block keeps: "the top k%
    positions" of a row of P_c (Sec. 4, Eq. 16).  The paper does not say how
    k% * T_n is rounded; reading taken: round half up, clamp to [0, T_n]."""
    k = int(math.floor(float(topk_frac) * T_n + 0.5))
    return max(0, min(T_n, k))


def smooth_k(K: np.ndarray) -> np.ndarray:
    """K <- K - colmean(K)  (Alg. 2, the K-smoothing step).  The mean is over all N tokens of
    this head, one value per channel."""
    return K - K.mean(axis=0, keepdims=True)


def phi(X: np.ndarray) -> np.ndarray:
    """Activation of the linear branch: "we use the softmax function" (Sec. 3,
    below Eq. 14).  Reading taken: softmax over the d channels of each token,
    no temperature."""
    E = np.exp(X - X.max(axis=-1, keepdims=True))
    return E / E.sum(axis=-1, keepdims=True)


def pool(X: np.ndarray, b: int) -> np.ndarray:
    """Mean pooling over consecutive b tokens (Sec. 4, Eq. 15).  A ragged last
    block is averaged over the tokens it has."""
    N, d = X.shape
    T = num_blocks(N, b)
    out = np.empty((T, d), dtype=np.float64)
    for t in range(T):
        out[t] = X[t * b:min(N, (t + 1) * b)].mean(axis=0)
    return out


# --------------------------------------------------------------------------- #
# router (Sec. 4)
# --------------------------------------------------------------------------- #
def router_scores(Q, Ks, Wq, Wk, b_q: int, b_k: int) -> np.ndarray:
    """R = proj_q(pool(Q)) proj_k(pool(K))^T / sqrt(d)   (Eq. 16; Alg. 2, router step).

    `Ks` is the smoothed K (in Alg. 2 smoothing precedes pooling).  proj(x) = x W with
    W stored [d_in, d_out], no bias.  The router step of Alg. 2 also applies a row softmax
    and writes proj_k(K) for proj_k(pool K); Eq. 16 has neither the softmax nor
    the 1/sqrt(d).  A row-wise softmax and a positive factor do not change a
    row-wise top-k, so the scores returned here are the pre-softmax ones, with
    the 1/sqrt(d) of Alg. 2 kept; "router score" means this R everywhere."""
    d = Q.shape[1]
    Qbar = pool(Q, b_q)
    Kbar = pool(Ks, b_k)
    return (Qbar @ Wq) @ (Kbar @ Wk).T / math.sqrt(d)


def topk_rows(R: np.ndarray, k: int) -> np.ndarray:
    """M_c = Top-k(k%, P_c), row-wise (Eq. 16), as index lists: for each row the
    k largest entries, equal scores broken toward the lower column index, the
    kept indices returned in ascending order.  Shape [T_m, k], int32."""
    T_m, T_n = R.shape
    sel = np.empty((T_m, k), dtype=np.int32)
    for i in range(T_m):
        order = np.argsort(-R[i], kind="stable")      # descending, stable
        sel[i] = np.sort(order[:k])
    return sel


def _sigmoid(x: np.ndarray) -> np.ndarray:
    """1 / (1 + exp(-x)) without overflow for large |x|."""
    e = np.exp(-np.abs(x))
    return np.where(x >= 0, 1.0 / (1.0 + e), e / (1.0 + e))


def soft_topk_rows(R: np.ndarray, k: int, tau: float = 0.1) -> np.ndarray:
    """SoftTop-k(k%, P_c) of Sec. 6 (the differentiable stand-in for Top-k used in the
    first training stage), row-wise:

        P_c    = softmax over the row of R             (the router step of Alg. 2)
        M_ij   = sigmoid(P_c[i, j] / tau + lambda_i)
        lambda_i solved by bisection so that the row sums to k.

    The row sum is increasing in lambda_i, from 0 to T_n, so the root is unique
    for 0 < k < T_n.  Reading taken: k is the same integer as for the hard mask
    (num_selected), so that both masks keep the same mass per row; k = 0 gives
    the zero mask and k = T_n the all-ones mask (the limits lambda -> -inf, +inf).
    The bisection runs in float64 on a bracket that provably contains the root
    until the interval stops shrinking.  Returns [T_m, T_n] float64."""
    T_m, T_n = R.shape
    if k <= 0:
        return np.zeros((T_m, T_n))
    if k >= T_n:
        return np.ones((T_m, T_n))
    M = np.empty((T_m, T_n))
    for i in range(T_m):
        e = np.exp(R[i] - R[i].max())
        x = (e / e.sum()) / tau                       # P_c / tau, in [0, 1 / tau]
        # sigmoid(x + lam) <= sigmoid(x.max() + lam): sum < k once lam < logit(k / T_n) - x.max();
        # sigmoid(x + lam) >= sigmoid(x.min() + lam): sum > k once lam > logit(k / T_n) - x.min()
        logit = math.log(k / (T_n - k))
        lo, hi = logit - x.max() - 1e-9, logit - x.min() + 1e-9
        while True:
            mid = 0.5 * (lo + hi)
            if mid <= lo or mid >= hi:
                break
            if _sigmoid(x + mid).sum() < k:
                lo = mid
            else:
                hi = mid
        M[i] = _sigmoid(x + 0.5 * (lo + hi))
    return M


def mask_from_sel(sel: np.ndarray, T_n: int) -> np.ndarray:
    """M_c in {0,1}^{T_m x T_n} from the index lists."""
    T_m = sel.shape[0]
    M = np.zeros((T_m, T_n), dtype=bool)
    for i in range(T_m):
        M[i, sel[i]] = True
    return M


# --------------------------------------------------------------------------- #
# sparse branch (Eq. 14, O_s; Alg. 2, the M_c[i,j] = 1 arm of the block loop)
# --------------------------------------------------------------------------- #
def _block_cols(js, b_k: int, N: int) -> np.ndarray:
    if len(js) == 0:
        return np.zeros((0,), dtype=np.int64)
    return np.concatenate([np.arange(j * b_k, min(N, (j + 1) * b_k)) for j in js])


def sparse_branch(Q, Ks, V, sel, b_q: int, b_k: int, q_blocks=None):
    """O_s = softmax(Q K^T / sqrt(d) (.) M) V   (Eq. 14).

    Reading taken for "(.) M": positions with M = 0 are left out of the softmax
    (they get no weight), which is what Alg. 2 computes by skipping those blocks
    and what P_s = P_1 / alpha (Eq. 8) requires; a literal product would give
    them weight e^0.  Without quantisation the result does not depend on the
    order of the blocks, so it is evaluated here as the plain definition: a
    softmax over exactly the selected, existing key positions of each row.
    A query block with no selected block outputs 0 and L = -inf.  `q_blocks`
    restricts the evaluation to some query blocks (other rows stay 0 / -inf).

    Returns (O_s [N, d], L [N]) with L = log sum exp of the kept scores
    (the L_i of Alg. 2)."""
    N, d = Q.shape
    O = np.zeros((N, d), dtype=np.float64)
    L = np.full((N,), -np.inf, dtype=np.float64)
    for i in (range(sel.shape[0]) if q_blocks is None else q_blocks):
        r0, r1 = i * b_q, min(N, (i + 1) * b_q)
        cols = _block_cols(sel[i], b_k, N)
        if cols.size == 0:
            continue
        S = Q[r0:r1] @ Ks[cols].T / math.sqrt(d)
        m = S.max(axis=1, keepdims=True)
        E = np.exp(S - m)
        l = E.sum(axis=1, keepdims=True)
        O[r0:r1] = (E / l) @ V[cols]
        L[r0:r1] = (m + np.log(l))[:, 0]
    return O, L


# --------------------------------------------------------------------------- #
# low-bit sparse branch (Sec. 5; Alg. 2, the same arm with quant / dequant)
# --------------------------------------------------------------------------- #
def e4m3_round(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest value of the OCP FP8 e4m3 format
    (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; subnormals with
    quantum 2^-9; largest finite 448; no infinities), ties to even, magnitudes
    beyond the range saturating at 448.  Result returned as float32."""
    x = np.asarray(x, dtype=np.float32)
    a = np.abs(x).astype(np.float64)
    _, e = np.frexp(a)                       # a = f * 2^e, f in [0.5, 1)
    e = np.maximum(e - 1, -6)                # exponent of the leading bit, floored at the subnormal range
    quantum = np.ldexp(1.0, e - 3)           # spacing of representable values in that binade
    r = np.rint(a / quantum) * quantum       # rint = round half to even
    r = np.minimum(r, E4M3_MAX)
    return np.copysign(r, x).astype(np.float32)


def quant_block_e4m3(X32: np.ndarray):
    """quant(.) of Sec. 5 for one block of Q or of the smoothed K.

    The paper defers the scheme to another paper that is not available; the
    definition used (and shared, as a definition only, with the HIP path) is:
    one scale per block, amax = max |x| over the block's existing tokens;
    inv = 448 / amax and s = amax / 448, both float32 divisions; the stored
    value is e4m3_round(x * inv) with the product taken in float32.  An
    all-zero block uses inv = s = 1.  Returns (values on the e4m3 grid as
    float32, s as float32).  Every step that decides a code is in float32, the
    precision the kernels take that decision in."""
    X32 = np.asarray(X32, dtype=np.float32)
    amax = np.float32(np.max(np.abs(X32))) if X32.size else np.float32(0)
    if amax == 0:
        return np.zeros_like(X32), np.float32(1.0)
    inv = np.float32(E4M3_MAX) / amax
    s = amax / np.float32(E4M3_MAX)
    return e4m3_round(X32 * inv), np.float32(s)


def quant_block_int8(X32: np.ndarray):
    """The INT8 form of quant(.) for one block of Q or of the smoothed K
    (Sec. 5 names INT8 next to FP8 as the low-bit formats of Q K^T).

    Same granularity and the same float32 decisions as quant_block_e4m3: one
    scale per block, amax = max |x|; inv = 127 / amax and s = amax / 127, both
    float32 divisions; the code is the float32 product x * inv rounded to the
    nearest integer, ties to even, kept within [-127, 127] (the range is
    symmetric: -128 is never produced).  An all-zero block uses inv = s = 1.
    Returns (integer codes as float32, s as float32)."""
    X32 = np.asarray(X32, dtype=np.float32)
    amax = np.float32(np.max(np.abs(X32))) if X32.size else np.float32(0)
    if amax == 0:
        return np.zeros_like(X32), np.float32(1.0)
    inv = np.float32(INT8_MAX) / amax
    s = amax / np.float32(INT8_MAX)
    codes = np.clip(np.rint(X32 * inv), -INT8_MAX, INT8_MAX)     # rint = round half to even
    return codes.astype(np.float32), np.float32(s)


def smooth_k_f32(K: np.ndarray) -> np.ndarray:
    """The smoothed keys as they enter quantisation: float32(K) - float32(mu),
    mu = colmean(K) taken in float64 and rounded once to float32."""
    mu32 = K.mean(axis=0).astype(np.float32)
    return K.astype(np.float32) - mu32[None, :]


def absorb_block(state, S, Vj, v_scale=1.0):
    """One step of the running softmax of a block of query rows, with the weights rounded for the product.

    `state` = (m, l, A) summarises the key blocks absorbed so far, per query row:
        m   the largest score seen                                   [rows, 1]
        l   sum over the keys seen of exp(score - m)                 [rows, 1]
        A   sum over the keys seen of round(exp(score - m_then)) v, carried forward to the present m:
            every time m grows to m', what has been added so far is scaled by exp(m - m')   [rows, d]
    Absorbing a block with scores S [rows, keys] and values Vj [keys, d]:
        m'  = max(m, largest score of each row of S)
        w   = exp(S - m')                       the block's weights against the new maximum (<= 1)
        l'  = exp(m - m') l + rowsum(w)         the un-rounded weights: l is what an exact softmax would have
        A'  = exp(m - m') A + round(w) Vj v_scale
    where round(.) puts a weight on the e4m3 grid after scaling by 2^8: round(w) = e4m3_round(w 2^8) / 2^8
    (weights are at most 1 and 2^8 < 448, so nothing saturates; weights below 2^-18 round to zero).
    This is the M_c[i, j] = 1 arm of the block loop of Alg. 2 with quant(P); the order of the three updates
    - maximum, then the sum from the un-rounded weights, then the rounded product - is the algorithm's."""
    m, l, A = state
    m_new = np.maximum(m, S.max(axis=1, keepdims=True))
    w = np.exp(S - m_new)
    keep = np.exp(m - m_new)                                    # exp(-inf) = 0 for the first block
    l_new = keep * l + w.sum(axis=1, keepdims=True)
    w_rounded = e4m3_round((w * 2.0 ** P_SCALE_LOG2).astype(np.float32)).astype(np.float64) / 2.0 ** P_SCALE_LOG2
    A_new = keep * A + (w_rounded @ Vj) * v_scale
    return m_new, l_new, A_new


def sparse_branch_lowbit(Q, K, V, sel, b_q: int, b_k: int, *, smooth: bool = True,
                         q_blocks=None, quant_block=None, quant_v: bool = False):
    """Sparse branch with low-bit Q, K and P (Sec. 5; Alg. 2 with quant / dequant).  With a rounded P the
    result depends on the running maximum and therefore on the order of the blocks, so it is not a plain
    closed form: each query block starts from the empty state (m = -inf, l = 0, A = 0) and absorbs its
    selected key blocks in ascending order through absorb_block, with the scores of block j taken from
    the 8-bit codes,
        S = (Qhat_i Khat_j^T) s_Qi s_Kj / sqrt(d)      (exact products of codes, then the two scales),
    and O_s = A / l, L = m + log l at the end.

    Readings taken (the paper leaves all four open): FP8 e4m3 with one scale per b_q x d block of Q and per
    b_k x d block of the smoothed K (quant_block_e4m3); P is rounded with the fixed power-of-two scale 2^8;
    l is accumulated from the un-rounded P (Alg. 2 updates l before it quantises P); V stays at its input
    values although Alg. 2 also quantises V (the workload definition keeps V in bf16).
    K is the raw K: smoothing is done here in float32 (smooth_k_f32).
    `quant_block` is the quantiser of Q and K blocks: quant_block_e4m3 (the default) or quant_block_int8;
    everything after the codes is the same.  `quant_v` takes the second product the way Alg. 2 prints it,
    dequant(quant(P) quant(V_j)): V_j is quantised like a key block (e4m3, one scale per b_k x d block over
    its existing tokens) and its scale multiplies the block's product; the linear branch keeps the input V
    (Alg. 2 forms h_j from the unquantised V_j).  Returns (O_s, L) like sparse_branch."""
    if quant_block is None:
        quant_block = quant_block_e4m3
    N, d = Q.shape
    Kin = smooth_k_f32(K) if smooth else K.astype(np.float32)
    T_n = num_blocks(N, b_k)
    key_rows = [slice(j * b_k, min(N, (j + 1) * b_k)) for j in range(T_n)]
    Khat, sK = zip(*[quant_block(Kin[rows]) for rows in key_rows]) if T_n else ((), ())
    O = np.zeros((N, d), dtype=np.float64)
    L = np.full((N,), -np.inf, dtype=np.float64)
    for i in (range(sel.shape[0]) if q_blocks is None else q_blocks):
        rows = slice(i * b_q, min(N, (i + 1) * b_q))
        n_rows = rows.stop - rows.start
        Qhat, sQ = quant_block(Q[rows].astype(np.float32))
        state = (np.full((n_rows, 1), -np.inf), np.zeros((n_rows, 1)), np.zeros((n_rows, d)))
        for j in sel[i]:
            S = (Qhat.astype(np.float64) @ Khat[j].astype(np.float64).T) * (float(sQ) * float(sK[j])) / math.sqrt(d)
            if quant_v:
                Vhat, sV = quant_block_e4m3(V[key_rows[j]].astype(np.float32))
                state = absorb_block(state, S, Vhat.astype(np.float64), float(sV))
            else:
                state = absorb_block(state, S, V[key_rows[j]])
        if len(sel[i]):
            m, l, A = state
            O[rows] = A / l
            L[rows] = (m + np.log(l))[:, 0]
    return O, L


# --------------------------------------------------------------------------- #
# linear branch (Eq. 3; Eq. 14, O_l; Alg. 2: h, z, the M_c[i,j] = 0 arm, O^l_i)
# --------------------------------------------------------------------------- #
def kv_state(Kphi, V, b_k: int):
    """h_j = (K^phi_j)^T V_j  (d x d)  and  z_j = rowsum((K^phi_j)^T)  (d), per
    key/value block (Alg. 2, before the block loop).  Returns h [T_n, d, d], z [T_n, d]."""
    N, d = V.shape
    T_n = num_blocks(N, b_k)
    h = np.empty((T_n, d, d), dtype=np.float64)
    z = np.empty((T_n, d), dtype=np.float64)
    for j in range(T_n):
        c0, c1 = j * b_k, min(N, (j + 1) * b_k)
        h[j] = Kphi[c0:c1].T @ V[c0:c1]
        z[j] = Kphi[c0:c1].sum(axis=0)
    return h, z


def linear_branch(Q, Ks, V, sel, b_q: int, b_k: int, q_blocks=None):
    """O_l = norm(phi(Q) phi(K)^T (.) (1 - M)) V   (Eq. 14), computed the way
    Alg. 2 does: H_i = sum of h_j and Z_i = sum of z_j over the blocks with
    M_c[i, j] = 0, then O^l_i = Q^phi_i H_i / (Q^phi_i Z_i).
    The sums run directly over the unselected blocks (written as a product with
    the 0/1 matrix 1 - M_c).  phi is applied to the raw Q and to the smoothed
    K.  A query block whose every key/value block is selected has H = Z = 0 and
    outputs 0.  `q_blocks` restricts the evaluation to some query blocks (the
    other rows stay 0).  Returns (O_l [N, d], H [T_m, d, d], Z [T_m, d])."""
    N, d = Q.shape
    T_m, T_n = num_blocks(N, b_q), num_blocks(N, b_k)
    Qphi, Kphi = phi(Q), phi(Ks)
    h, z = kv_state(Kphi, V, b_k)
    rows = range(T_m) if q_blocks is None else list(q_blocks)
    notM = ~mask_from_sel(sel, T_n)
    H = np.zeros((T_m, d, d))
    Z = np.zeros((T_m, d))
    idx = np.asarray(list(rows), dtype=np.int64)
    W = notM[idx].astype(np.float64)
    H[idx] = (W @ h.reshape(T_n, d * d)).reshape(len(idx), d, d)
    Z[idx] = W @ z
    O = np.zeros((N, d), dtype=np.float64)
    for i in idx:
        r0, r1 = i * b_q, min(N, (i + 1) * b_q)
        den = Qphi[r0:r1] @ Z[i]
        if notM[i].any():
            O[r0:r1] = (Qphi[r0:r1] @ H[i]) / den[:, None]
    return O, H, Z


# --------------------------------------------------------------------------- #
# the operator  O = SLA2(Q, K, V, k%, R, alpha)   (Eq. 13; Alg. 2)
# --------------------------------------------------------------------------- #
def forward_head(Q, K, V, Wq, Wk, alpha, topk_frac: float, b_q: int, b_k: int,
                 quant: int = QUANT_NONE, smooth: bool = True, q_blocks=None,
                 sel=None):
    """One head of Alg. 2.  Q, K, V: [N, d] float64 holding the input values
    (already rounded to the storage type by the caller).  alpha: a scalar (one
    ratio for the head) or an array [T_m] (one per query block, as in the input
    line of Alg. 2; Sec. 3 gives alpha one entry per token instead - per block
    is the finer of the two forms the boundary accepts).  `sel` overrides the
    router (used by tests that fix the mask).  `q_blocks` limits the output to
    some query blocks; other rows are returned as 0.

    Returns a dict: O, O_s, O_l, L, sel, R, H, Z."""
    N, d = Q.shape
    T_m, T_n = num_blocks(N, b_q), num_blocks(N, b_k)
    Ks = smooth_k(K) if smooth else K                       # K smoothing
    R = router_scores(Q, Ks, Wq, Wk, b_q, b_k)              # pooled, projected scores
    if sel is None:
        sel = topk_rows(R, num_selected(topk_frac, T_n))    # hard top-k
    qb = None if q_blocks is None else sorted(int(i) for i in q_blocks)
    if quant == QUANT_NONE:
        O_s, L = sparse_branch(Q, Ks, V, sel, b_q, b_k, q_blocks=qb)
    elif quant == QUANT_FP8:
        O_s, L = sparse_branch_lowbit(Q, K, V, sel, b_q, b_k, smooth=smooth, q_blocks=qb)
    elif quant == QUANT_INT8:
        O_s, L = sparse_branch_lowbit(Q, K, V, sel, b_q, b_k, smooth=smooth, q_blocks=qb,
                                      quant_block=quant_block_int8)
    elif quant == QUANT_FP8_V:
        O_s, L = sparse_branch_lowbit(Q, K, V, sel, b_q, b_k, smooth=smooth, q_blocks=qb, quant_v=True)
    else:
        raise ValueError("unknown quant mode")
    O_l, H, Z = linear_branch(Q, Ks, V, sel, b_q, b_k, q_blocks=qb)
    a = np.broadcast_to(np.asarray(alpha, dtype=np.float64).reshape(-1), (T_m,)) \
        if np.ndim(alpha) else np.full((T_m,), float(alpha))
    a_rows = np.repeat(a, b_q)[:N, None]
    O = a_rows * O_s + (1.0 - a_rows) * O_l                 # Eq. 13
    return dict(O=O, O_s=O_s, O_l=O_l, L=L, sel=sel, R=R, H=H, Z=Z)


# --------------------------------------------------------------------------- #
# backward pass (Alg. 3 of the appendix, plus the steps it leaves to automatic
# differentiation: phi, the smoothing of K, the mix of Eq. 13)
# --------------------------------------------------------------------------- #
def backward_head(Q, K, V, sel, alpha, dO, b_q: int, b_k: int, smooth: bool = True, quant: int = QUANT_NONE):
    """Gradients of one head of the un-quantised operator with respect to Q, K,
    V and alpha, for a fixed block mask `sel` (hard Top-k passes no gradient to
    the router; Sec. 6).  dO: [N, d], the gradient of the output of Eq. 13.
    Sec. 5: the backward pass is always taken in high precision from the
    original Q, K, V, whatever precision the forward ran in; what it takes
    from a low-bit forward (`quant`) is that forward's O^s and L, as inputs.

    Steps, in the notation of Alg. 3 (P is the normalised softmax over the
    selected positions, P = exp(S - L)):

      mix         dO^s = a dO,  dO^l = (1 - a) dO,  d alpha_i = sum_rows dO . (O^s - O^l)
      D           D^s = rowsum(dO^s (.) O^s),  D^l = rowsum(dO^l (.) O^l)
      per i       dH_i = (Q^phi_i / (Q^phi_i Z_i))^T dO^l_i,   dZ_i = -(Q^phi_i / (Q^phi_i Z_i))^T D^l_i
                  dQ^phi_i = (dO^l_i H_i^T - D^l_i Z_i^T) / (Q^phi_i Z_i)
      per (i, j)  M_c = 1:  dV_j += P^T dO^s_i,  dP = dO^s_i V_j^T,  dS = P (.) (dP - D^s_i),
                            dQ_i += dS K_j / sqrt(d),  dK_j += dS^T Q_i / sqrt(d)
                  M_c = 0:  dH += dH_i,  dZ += dZ_i
      per j       dK^phi_j = V_j dH^T + 1 dZ^T,   dV_j += K^phi_j dH
      phi         y = softmax(x):  dx = y (.) (dy - rowsum(dy (.) y)), for Q^phi and K^phi
      smoothing   K' = K - colmean(K):  dK = dK' - colmean(dK')

    The 1/sqrt(d) of the score is written out (Alg. 3 leaves it inside S).  An
    empty branch contributes nothing.  Returns dict dQ, dK, dV [N, d], dalpha [T_m]
    (one entry per query block; a per-head alpha takes their sum) and the
    intermediates dQphi, dKphi, Ds, Dl."""
    N, d = Q.shape
    T_m, T_n = num_blocks(N, b_q), num_blocks(N, b_k)
    Ks = smooth_k(K) if smooth else K
    if quant == QUANT_NONE:
        O_s, L = sparse_branch(Q, Ks, V, sel, b_q, b_k)
    else:
        O_s, L = sparse_branch_lowbit(Q, K, V, sel, b_q, b_k, smooth=smooth,
                                      quant_block=quant_block_int8 if quant == QUANT_INT8 else None,
                                      quant_v=quant == QUANT_FP8_V)
    O_l, H, Z = linear_branch(Q, Ks, V, sel, b_q, b_k)
    a_blk = np.broadcast_to(np.asarray(alpha, dtype=np.float64).reshape(-1), (T_m,)) if np.ndim(alpha) \
        else np.full((T_m,), float(alpha))
    a_rows = np.repeat(a_blk, b_q)[:N, None]
    dOs, dOl = a_rows * dO, (1.0 - a_rows) * dO
    mix = (dO * (O_s - O_l)).sum(axis=1)
    dalpha = np.array([mix[i * b_q:min(N, (i + 1) * b_q)].sum() for i in range(T_m)])
    Ds, Dl = (dOs * O_s).sum(axis=1), (dOl * O_l).sum(axis=1)
    Qphi, Kphi = phi(Q), phi(Ks)
    notM = ~mask_from_sel(sel, T_n)
    rscale = 1.0 / math.sqrt(d)
    dQ, dKs, dV = np.zeros((N, d)), np.zeros((N, d)), np.zeros((N, d))
    dQphi, dKphi = np.zeros((N, d)), np.zeros((N, d))
    dH_i, dZ_i = np.zeros((T_m, d, d)), np.zeros((T_m, d))
    for i in range(T_m):
        r0, r1 = i * b_q, min(N, (i + 1) * b_q)
        if notM[i].any():                                   # linear branch of this query block exists
            w = Qphi[r0:r1] / (Qphi[r0:r1] @ Z[i])[:, None]
            dH_i[i] = w.T @ dOl[r0:r1]
            dZ_i[i] = -(w.T @ Dl[r0:r1])
            dQphi[r0:r1] = (dOl[r0:r1] @ H[i].T - np.outer(Dl[r0:r1], Z[i])) / (Qphi[r0:r1] @ Z[i])[:, None]
        for j in sel[i]:                                    # M_c[i, j] = 1
            c0, c1 = j * b_k, min(N, (j + 1) * b_k)
            S = Q[r0:r1] @ Ks[c0:c1].T * rscale
            P = np.exp(S - L[r0:r1, None])
            dV[c0:c1] += P.T @ dOs[r0:r1]
            dP = dOs[r0:r1] @ V[c0:c1].T
            dS = P * (dP - Ds[r0:r1, None])
            dQ[r0:r1] += dS @ Ks[c0:c1] * rscale
            dKs[c0:c1] += dS.T @ Q[r0:r1] * rscale
    for j in range(T_n):
        c0, c1 = j * b_k, min(N, (j + 1) * b_k)
        dH = dH_i[notM[:, j]].sum(axis=0)                   # M_c[i, j] = 0
        dZ = dZ_i[notM[:, j]].sum(axis=0)
        dKphi[c0:c1] = V[c0:c1] @ dH.T + dZ[None, :]
        dV[c0:c1] += Kphi[c0:c1] @ dH
    dQ += Qphi * (dQphi - (dQphi * Qphi).sum(axis=1, keepdims=True))
    dKs += Kphi * (dKphi - (dKphi * Kphi).sum(axis=1, keepdims=True))
    dK = dKs - dKs.mean(axis=0, keepdims=True) if smooth else dKs
    return dict(dQ=dQ, dK=dK, dV=dV, dalpha=dalpha, dQphi=dQphi, dKphi=dKphi, Ds=Ds, Dl=Dl)


def forward(q, k, v, router_w, alpha, topk_frac: float, b_q: int, b_k: int,
            quant: int = QUANT_NONE, smooth: bool = True):
    """All heads.  q, k, v: [B, H, N, d] arrays of input values; router_w:
    [2, d, d] (Wq, Wk shared by all heads) ; alpha: [H] or [H, T_m].  Batch
    items and heads are independent instances of the single-head operator.
    Returns (O [B, H, N, d] float64, sel [B, H, T_m, k] int32)."""
    B, H, N, d = q.shape
    Wq = np.asarray(router_w[0], dtype=np.float64)
    Wk = np.asarray(router_w[1], dtype=np.float64)
    O = np.empty((B, H, N, d), dtype=np.float64)
    sels = []
    for b in range(B):
        for h in range(H):
            r = forward_head(np.asarray(q[b, h], dtype=np.float64),
                             np.asarray(k[b, h], dtype=np.float64),
                             np.asarray(v[b, h], dtype=np.float64),
                             Wq, Wk, alpha[h], topk_frac, b_q, b_k, quant, smooth)
            O[b, h] = r["O"]
            sels.append(r["sel"])
    sel = np.stack(sels).reshape(B, H, *sels[0].shape)
    return O, sel
