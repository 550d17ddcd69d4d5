"""Float64 CPU oracle of the SliM-LLM per-layer quantisation pass.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the HIP
path is checked against.  It may be imported by `tests/`, by
`__graft_entry__.smoke()` and by the `cpu_baseline` leg of `bench.py`, and by
nothing else; it shares no code with the HIP path and imports nothing from it.

Every function follows the paper's steps in the paper's order and notation
(W in R^{n x m}, n output rows, m input channels; x in R^{t x m}; group size
beta along the input dimension; k = m / beta groups; target average width N):

  hessian_*           Eq. 3 and Alg. 1 line 1     H = (2/T) X X^T
  hessian_inverse     Def. 1, Alg. 1 line 2       U = upper Cholesky factor of (H + lambda I)^-1
  salience            Def. 1, Alg. 2 (SBA) line 6 delta_ij = w_ij^2 / [H^-1]_jj^2, group mean
  rtn_fakequant       Eq. 1 / Eq. 2               min-max round-to-nearest per (row, group)
  sba_allocate        Eq. 4, Alg. 2 (SBA), App. C/D  double-pointer search, KL of softmaxed outputs
  block_mask          Sec. 3.3.2, Alg. 1 line 8   3-sigma mask of the current block
  sqc_calibrate       Eq. 5, Alg. 2 (SQC)         tau grid search per (row, group)
  gptq_quantize       Alg. 1 lines 5-13           column-serial quantisation with compensation
  pack / unpack       App. B.2                    per-group bit-packing, group-bit array, offsets
  pack_zeros / unpack_zeros  App. B.2             zero points packed with one width along the channel direction
  sequential_layers   Sec. 3.4 (GPTQ backbone)    layers quantised one after another on their quantised predecessors' outputs
  lwc_*               Sec. 3.4, Sec. 4, App. B    SliM-LLM+: SBA widths + learnable weight clipping trained with AdamW
  dequant_matmul      App. B.2 (inference)        y = x dequant(W_int)^T straight from the packed tensors

Readings taken where the paper is silent or inconsistent are stated at the
function that needs them.  Pins (tests/test_oracle_*.py) tie each function to
closed forms, library routines, brute force or invariants; the points that no
pin can decide are marked "parity unpinned" here:

  parity unpinned: the choice of SQC loss weighting (MASK_MEAN / UNIFORM / ELEMENT),
  the 1-bit quantiser form (SIGN / AFFINE), the scope of the 3-sigma statistics
  (BLOCK / ROW), the salience denominator (diag of H^-1 vs diag of its Cholesky
  factor) and the token subset used by the SBA objective.  Each is a mode switch
  with the same default on both sides; the formula of each mode is pinned.
  Likewise the bit order inside the packed words and the meaning of the 2-bit group
  value (width minus bit_base, bit_base_for(N)): App. B.2 gives the structure only;
  the layout written here is pinned by hand-worked words and round trips.  The same holds
  for the packed zero points (what is stored: 2 z; the width; the direction): App. B.2
  says "uniform precision along the channel direction" and no more.
  parity unpinned: everything about SliM-LLM+ beyond "SBA widths, no SQC, the learnable weight
  clipping of OmniQuant, AdamW" (App. B, Sec. 4): the parametrisation of the clipping (sigmoid
  of a free parameter times the group's extreme value, start value 4), the straight-through
  derivative of the rounding, the loss (mean squared layer-output error over the calibration
  tokens, full batch), the optimiser's constants and the two-level affine form of 1-bit groups are
  taken from the published description of that method and are arguments where they are numbers;
  what is pinned is that the derivatives are those of the stated forward pass (autograd) and
  that full clipping strength reproduces Eq. 1.
"""
from __future__ import annotations

import numpy as np
import scipy.linalg

# --- mode switches (same numeric values as the C header, by interface contract) ---------
WEIGHT_MASK_MEAN, WEIGHT_UNIFORM, WEIGHT_ELEMENT = 0, 1, 2
Q1_SIGN, Q1_AFFINE = 0, 1
SCOPE_BLOCK, SCOPE_ROW = 0, 1
SAL_HINV_DIAG, SAL_CHOL_DIAG = 0, 1
OBJ_KL, OBJ_MSE = 0, 1


def tau_grid(lam: float = 0.1, n: int = 50) -> np.ndarray:
    """The 2n candidates of tau obtained by dividing [1-lam, 1+lam] linearly (Sec. 3.3.2,
    Alg. 2 SQC loop header): tau_c = (1 - lam) + c * (lam / n), c = 0 .. 2n-1.
    tau = 1 is candidate c = n."""
    c = np.arange(2 * n, dtype=np.float64)
    return (1.0 - lam) + c * (lam / n)


# ----------------------------------------------------------------------------------------
# Hessian (Eq. 3; Alg. 1 line 1)
# ----------------------------------------------------------------------------------------
def gram_accumulate(G: np.ndarray, X_chunk: np.ndarray) -> np.ndarray:
    """G += X_c X_c^T for one chunk of tokens; X_c is (m, t_c), any float dtype."""
    Xc = np.asarray(X_chunk, dtype=np.float64)
    G += Xc @ Xc.T
    return G


def hessian_from_gram(G: np.ndarray, n_tokens: int) -> np.ndarray:
    """H = (2 / T) * sum_tokens x x^T.  The constant factor is immaterial downstream
    because the damping is relative to mean(diag H); 2/T is the GPTQ convention."""
    return (2.0 / float(n_tokens)) * np.asarray(G, dtype=np.float64)


# ----------------------------------------------------------------------------------------
# Damped inverse and its Cholesky factor (Def. 1; Alg. 1 line 2; App. G.1)
# ----------------------------------------------------------------------------------------
def hessian_inverse(G: np.ndarray, n_tokens: int, percdamp: float = 0.01):
    """Returns (U, hinv_diag, lam).

    lam = percdamp * mean(diag H);  Hd = H + lam I;  Hinv = Hd^-1;
    U is the upper-triangular factor with Hinv = U^T U, so that row c of U to the
    right of the diagonal carries the compensation of Alg. 1 line 12;
    hinv_diag_j = [Hinv]_jj.  Raises numpy.linalg.LinAlgError if Hd is not
    positive definite."""
    H = hessian_from_gram(G, n_tokens)
    m = H.shape[0]
    lam = percdamp * float(np.mean(np.diag(H)))
    Hd = H + lam * np.eye(m)
    L = scipy.linalg.cholesky(Hd, lower=True)            # LAPACK potrf
    Hinv = scipy.linalg.cho_solve((L, True), np.eye(m))  # LAPACK potrs
    Hinv = 0.5 * (Hinv + Hinv.T)
    U = scipy.linalg.cholesky(Hinv, lower=False)         # Hinv = U^T U
    return U, np.diag(Hinv).copy(), lam


# ----------------------------------------------------------------------------------------
# Salience (Def. 1; Alg. 2 SBA line 6)
# ----------------------------------------------------------------------------------------
def salience(W: np.ndarray, hinv_diag: np.ndarray, beta: int, U: np.ndarray | None = None,
             sal_mode: int = SAL_HINV_DIAG):
    """Returns (col_sal[m], group_sal[k], elem_sal[n, m]).

    elem_sal_ij = w_ij^2 / d_j^2 with d_j = [H^-1]_jj (Def. 1), or d_j = U_jj in the
    mode that reads Alg. 2's [H^in]_diag literally.  col_sal_j = sum_i elem_sal_ij;
    group_sal_g = mean of elem_sal over all n rows and the beta columns of group g."""
    W = np.asarray(W, dtype=np.float64)
    n, m = W.shape
    d = np.asarray(hinv_diag, dtype=np.float64) if sal_mode == SAL_HINV_DIAG else np.diag(U).astype(np.float64)
    elem = (W * W) / (d * d)[None, :]
    col = elem.sum(axis=0)
    group = elem.reshape(n, m // beta, beta).mean(axis=(0, 2))
    return col, group, elem


# ----------------------------------------------------------------------------------------
# Quantiser primitives (Eq. 1, Eq. 2)
# ----------------------------------------------------------------------------------------
def minmax_params(w: np.ndarray, bits: int):
    """Eq. 1 parameters of one quantiser group (1-D array w), bits >= 2:
    delta0 = (w_max - w_min) / (2^bits - 1),  z = -round(w_min / delta0).

    Degenerate range (the paper is silent): if w_max == w_min the range is widened to
    include 0; if it is still empty (all zeros) delta0 = 1 and z = 0."""
    qmax = float(2 ** bits - 1)
    wmin = float(np.min(w))
    wmax = float(np.max(w))
    if wmax == wmin:
        wmin = min(wmin, 0.0)
        wmax = max(wmax, 0.0)
    if wmax == wmin:
        return 1.0, 0.0
    delta0 = (wmax - wmin) / qmax
    z = -np.rint(wmin / delta0)
    return delta0, float(z)


def quantize_affine(w, delta, z, bits: int):
    """Eq. 1: q = clamp(round(w / delta) + z, 0, 2^bits - 1); rounding is IEEE
    round-half-to-even."""
    qmax = float(2 ** bits - 1)
    return np.clip(np.rint(np.asarray(w, dtype=np.float64) / delta) + z, 0.0, qmax)


def dequantize(q, scale, zero):
    """w_hat = scale * (q - zero): one formula for every width.  For the sign quantiser
    of Eq. 2 the code is q = [w >= 0], scale = 2 alpha, zero = 1/2, so w_hat = +-alpha."""
    return scale * (np.asarray(q, dtype=np.float64) - zero)


def rtn_fakequant(W: np.ndarray, bits: np.ndarray, beta: int, q1_mode: int = Q1_SIGN) -> np.ndarray:
    """Round-to-nearest fake quantisation of W with the default parameters of Eq. 1
    (tau = 1) per (row, group); groups of width 1 use Eq. 2 (sign and mean absolute value
    of the (row, group) vector) unless q1_mode is AFFINE.  This is the fakequant of
    Alg. 2 (SBA) lines 8-10, applied to the original weights."""
    W = np.asarray(W, dtype=np.float64)
    n, m = W.shape
    out = np.empty_like(W)
    for g in range(m // beta):
        b = int(bits[g])
        for i in range(n):
            w = W[i, g * beta:(g + 1) * beta]
            if b == 1 and q1_mode == Q1_SIGN:
                alpha = np.mean(np.abs(w))
                out[i, g * beta:(g + 1) * beta] = np.where(w >= 0.0, alpha, -alpha)
            else:
                delta0, z = minmax_params(w, b)
                q = quantize_affine(w, delta0, z, b)
                out[i, g * beta:(g + 1) * beta] = dequantize(q, delta0, z)
    return out


# ----------------------------------------------------------------------------------------
# Salience-Determined Bit Allocation (Eq. 4; Alg. 2 SBA; App. C, App. D)
# ----------------------------------------------------------------------------------------
def softmax_kl(Y: np.ndarray, Yq: np.ndarray) -> float:
    """sum over tokens of KL(softmax(Y_t) || softmax(Yq_t)); rows are tokens and the
    softmax runs over the layer's n output features (App. D)."""
    def log_softmax(A):
        A = A - A.max(axis=1, keepdims=True)
        return A - np.log(np.exp(A).sum(axis=1, keepdims=True))
    lp = log_softmax(np.asarray(Y, dtype=np.float64))
    lq = log_softmax(np.asarray(Yq, dtype=np.float64))
    return float(np.sum(np.exp(lp) * (lp - lq)))


def bits_for_p(order: np.ndarray, k: int, N: int, p: int) -> np.ndarray:
    """Width N everywhere, N-1 for the p least salient groups, N+1 for the p most salient
    (the double pointer of App. C)."""
    bits = np.full(k, N, dtype=np.uint8)
    if p > 0:
        bits[order[:p]] = N - 1
        bits[order[k - p:]] = N + 1
    return bits


def sba_allocate(W: np.ndarray, group_sal: np.ndarray, beta: int, N: int, Xs: np.ndarray,
                 q1_mode: int = Q1_SIGN, objective: int = OBJ_KL):
    """Returns (bits[k] uint8, p_star, obj_curve[k//2 + 1], margin).

    Groups are ranked by salience (stable ascending sort: ties keep the lower group index
    first).  For p = 0 .. floor(k/2) -- p = 0 is uniform precision, the other extreme has
    no N-bit group left (App. C) -- the original W is fake-quantised with the bit vector
    of that p and the objective is KL(softmax(x W^T) || softmax(x W_p^T)) summed over the
    tokens of Xs (shape (m, t_s), channels x tokens).  The first p that attains the
    minimum wins (strict '<' in Alg. 2 line 12).  margin = relative gap between the best
    and the second-best objective.  objective = OBJ_MSE replaces the KL divergence by the
    squared error of the same layer outputs, || x W^T - x W_p^T ||_F^2 (the loss of Eq. 3; the
    variant the paper compares against in App. D)."""
    W = np.asarray(W, dtype=np.float64)
    n, m = W.shape
    k = m // beta
    Xs = np.asarray(Xs, dtype=np.float64)
    order = np.argsort(np.asarray(group_sal, dtype=np.float64), kind="stable")
    Y = Xs.T @ W.T
    pmax = k // 2
    obj = np.empty(pmax + 1, dtype=np.float64)
    for p in range(pmax + 1):
        Wp = rtn_fakequant_fast(W, bits_for_p(order, k, N, p), beta, q1_mode)
        Yp = Xs.T @ Wp.T
        obj[p] = softmax_kl(Y, Yp) if objective == OBJ_KL else float(np.sum((Y - Yp) ** 2))
    p_star = int(np.argmin(obj))            # numpy returns the first minimum
    rest = np.delete(obj, p_star)
    margin = float("inf") if rest.size == 0 else float((rest.min() - obj[p_star]) / max(abs(obj[p_star]), 1e-300))
    return bits_for_p(order, k, N, p_star), p_star, obj, margin


def rtn_fakequant_fast(W: np.ndarray, bits: np.ndarray, beta: int, q1_mode: int = Q1_SIGN) -> np.ndarray:
    """Same result as rtn_fakequant, evaluated a whole group at a time (all rows at once)
    so that the SBA search finishes in reasonable time; tested equal to the loop form."""
    W = np.asarray(W, dtype=np.float64)
    n, m = W.shape
    out = np.empty_like(W)
    for g in range(m // beta):
        b = int(bits[g])
        w = W[:, g * beta:(g + 1) * beta]
        if b == 1 and q1_mode == Q1_SIGN:
            alpha = np.mean(np.abs(w), axis=1, keepdims=True)
            out[:, g * beta:(g + 1) * beta] = np.where(w >= 0.0, alpha, -alpha)
            continue
        delta0, z = _minmax_params_rows(w, b)
        q = np.clip(np.rint(w / delta0[:, None]) + z[:, None], 0.0, float(2 ** b - 1))
        out[:, g * beta:(g + 1) * beta] = delta0[:, None] * (q - z[:, None])
    return out


def _minmax_params_rows(w: np.ndarray, bits: int):
    """minmax_params for every row of a (rows, beta) block at once."""
    qmax = float(2 ** bits - 1)
    wmin = w.min(axis=1)
    wmax = w.max(axis=1)
    deg = wmax == wmin
    wmin = np.where(deg, np.minimum(wmin, 0.0), wmin)
    wmax = np.where(deg, np.maximum(wmax, 0.0), wmax)
    empty = wmax == wmin
    delta0 = np.where(empty, 1.0, (wmax - wmin) / qmax)
    z = np.where(empty, 0.0, -np.rint(wmin / delta0))
    return delta0, z


# ----------------------------------------------------------------------------------------
# 3-sigma mask (Sec. 3.3.2; Alg. 1 line 8)
# ----------------------------------------------------------------------------------------
def block_mask(Wblk: np.ndarray, scope: int = SCOPE_BLOCK) -> np.ndarray:
    """Boolean mask of the locally salient elements: w < mu - 3 sigma or w > mu + 3 sigma,
    mu and sigma (population) taken over the whole current n x beta block (Alg. 1 applies
    sal_mask to w^b = w[:, b:b+beta]) or, in ROW scope, over each row's beta entries."""
    Wblk = np.asarray(Wblk, dtype=np.float64)
    if scope == SCOPE_BLOCK:
        mu = Wblk.mean()
        sigma = Wblk.std()
        return np.abs(Wblk - mu) > 3.0 * sigma
    mu = Wblk.mean(axis=1, keepdims=True)
    sigma = Wblk.std(axis=1, keepdims=True)
    return np.abs(Wblk - mu) > 3.0 * sigma


# ----------------------------------------------------------------------------------------
# Salience-Weighted Quantizer Calibration (Eq. 5; Alg. 2 SQC)
# ----------------------------------------------------------------------------------------
def sqc_weights(w: np.ndarray, mask: np.ndarray | None, weight_mode: int,
                d: np.ndarray | None = None) -> np.ndarray:
    """Per-element loss weights omega_j of one (row, group) vector w.

    MASK_MEAN : the salient and the non-salient part each contribute their mean squared
                error, omega_j = 1/|s| on the mask and 1/|us| off it (a part with no
                element contributes nothing) -- the reading under which the split of
                Eq. 5 / Alg. 2 lines 13-14 raises the sensitivity to salient elements;
    UNIFORM   : omega_j = 1, Eq. 5 exactly as printed;
    ELEMENT   : omega_j = w_j^2 / d_j^2, the element salience of Def. 1 (d = diag of H^-1
                for the group's columns)."""
    beta = w.shape[0]
    if weight_mode == WEIGHT_UNIFORM:
        return np.ones(beta)
    if weight_mode == WEIGHT_MASK_MEAN:
        ns = int(mask.sum())
        nus = beta - ns
        om = np.empty(beta)
        om[mask] = 1.0 / ns if ns else 0.0
        om[~mask] = 1.0 / nus if nus else 0.0
        return om
    if weight_mode == WEIGHT_ELEMENT:
        return (w * w) / (d * d)
    raise ValueError(weight_mode)


def sqc_search(w: np.ndarray, bits: int, tau: np.ndarray, omega: np.ndarray, q1_mode: int = Q1_SIGN):
    """Grid search of Alg. 2 (SQC) for one (row, group) vector w with loss weights omega.

    bits >= 2 (or AFFINE): delta0, z from Eq. 1 (z does not depend on tau: in Alg. 2 lines
    9-10 tau cancels); for each candidate delta = tau_c * delta0, the fake-quantised vector and
    L_c = sum_j omega_j (w_j - w_hat_j)^2; the first candidate attaining the minimum wins.
    bits == 1 with SIGN: alpha = mean |w| (Eq. 2), w_hat = tau_c * alpha * sign(w), reported
    as scale = 2 tau alpha, zero = 1/2.
    Returns (scale, zero, c_star, losses[ncand])."""
    w = np.asarray(w, dtype=np.float64)
    losses = np.empty(tau.shape[0], dtype=np.float64)
    if bits == 1 and q1_mode == Q1_SIGN:
        alpha = float(np.mean(np.abs(w)))
        sgn = np.where(w >= 0.0, 1.0, -1.0)
        for c, tc in enumerate(tau):
            err = w - (tc * alpha) * sgn
            losses[c] = np.sum(omega * err * err)
        c_star = int(np.argmin(losses))
        return 2.0 * tau[c_star] * alpha, 0.5, c_star, losses
    delta0, z = minmax_params(w, bits)
    for c, tc in enumerate(tau):
        delta = tc * delta0
        q = quantize_affine(w, delta, z, bits)
        err = w - dequantize(q, delta, z)
        losses[c] = np.sum(omega * err * err)
    c_star = int(np.argmin(losses))
    return tau[c_star] * delta0, z, c_star, losses


def sqc_calibrate(Wblk: np.ndarray, bits: int, tau: np.ndarray, weight_mode: int = WEIGHT_MASK_MEAN,
                  scope: int = SCOPE_BLOCK, q1_mode: int = Q1_SIGN, omega: np.ndarray | None = None,
                  d: np.ndarray | None = None):
    """SQC over every row of one n x beta block; each (row, group) minimises its own loss
    (Alg. 2 keeps a per-channel scale and zero, SQC lines 6-7).  `omega`, if given,
    replaces the weights derived from weight_mode.
    Returns (scale[n], zero[n], cand_idx[n], margin[n]); margin = relative gap between the
    best and the second-best *distinct candidate*'s loss."""
    Wblk = np.asarray(Wblk, dtype=np.float64)
    n, beta = Wblk.shape
    mask = block_mask(Wblk, scope) if (omega is None and weight_mode == WEIGHT_MASK_MEAN) else None
    scale = np.empty(n)
    zero = np.empty(n)
    idx = np.empty(n, dtype=np.int32)
    margin = np.empty(n)
    for i in range(n):
        om = omega[i] if omega is not None else sqc_weights(Wblk[i], None if mask is None else mask[i], weight_mode, d)
        scale[i], zero[i], idx[i], losses = sqc_search(Wblk[i], bits, tau, om, q1_mode)
        rest = np.delete(losses, idx[i])
        best = losses[idx[i]]
        margin[i] = float("inf") if rest.size == 0 else (rest.min() - best) / max(abs(best), 1e-300)
    return scale, zero, idx, margin


def _sqc_rows_fast(Wblk, bits, tau, omega, q1_mode):
    """sqc_search for all rows of a block at once (same arithmetic, vectorised over rows);
    tested equal to the per-row form.  omega is (n, beta)."""
    n, beta = Wblk.shape
    ncand = tau.shape[0]
    losses = np.empty((n, ncand))
    if bits == 1 and q1_mode == Q1_SIGN:
        alpha = np.mean(np.abs(Wblk), axis=1)
        sgn = np.where(Wblk >= 0.0, 1.0, -1.0)
        for c, tc in enumerate(tau):
            err = Wblk - (tc * alpha)[:, None] * sgn
            losses[:, c] = np.sum(omega * err * err, axis=1)
        idx = np.argmin(losses, axis=1)
        return 2.0 * tau[idx] * alpha, np.full(n, 0.5), idx, losses
    delta0, z = _minmax_params_rows(Wblk, bits)
    qmax = float(2 ** bits - 1)
    for c, tc in enumerate(tau):
        delta = (tc * delta0)[:, None]
        q = np.clip(np.rint(Wblk / delta) + z[:, None], 0.0, qmax)
        err = Wblk - delta * (q - z[:, None])
        losses[:, c] = np.sum(omega * err * err, axis=1)
    idx = np.argmin(losses, axis=1)
    return tau[idx] * delta0, z, idx, losses


def _omega_rows(Wblk, weight_mode, scope, d):
    n, beta = Wblk.shape
    if weight_mode == WEIGHT_UNIFORM:
        return np.ones((n, beta))
    if weight_mode == WEIGHT_ELEMENT:
        return (Wblk * Wblk) / (d * d)[None, :]
    mask = block_mask(Wblk, scope)
    ns = mask.sum(axis=1).astype(np.float64)
    nus = beta - ns
    ws = np.where(ns > 0, 1.0 / np.maximum(ns, 1.0), 0.0)
    wus = np.where(nus > 0, 1.0 / np.maximum(nus, 1.0), 0.0)
    return np.where(mask, ws[:, None], wus[:, None])


# ----------------------------------------------------------------------------------------
# Main loop (Alg. 1 lines 5-13) with GPTQ's column-serial compensation as the backbone
# ----------------------------------------------------------------------------------------
def gptq_quantize(W: np.ndarray, U: np.ndarray, bits: np.ndarray, beta: int, tau: np.ndarray,
                  weight_mode: int = WEIGHT_MASK_MEAN, scope: int = SCOPE_BLOCK, q1_mode: int = Q1_SIGN,
                  gptq_block: int | None = None, hinv_diag: np.ndarray | None = None):
    """Quantise W (n x m) group by group along the input dimension.

    For each block of `gptq_block` columns (default beta; a multiple of beta): at the first
    column of every group the quantiser parameters of that group are fixed by SQC on the
    *current* (already compensated) weights of the group; then column by column
    q = Q(w_c), w_hat = dequant(q), e = (w_c - w_hat) / U_cc, and the remaining columns of
    the block receive  w[:, j] -= e * U[c, j]  (GPTQ; Alg. 1 lines 10-12 are its block
    shorthand).  After the block, every later column receives
    W[:, later] -= E_block @ U[block, later]  (Alg. 1 line 12).

    Returns a dict: codes (n,m) uint8, scale (n,k), zero (n,k), What (n,m), E (n,m),
    sum_e2, cand_idx (n,k) int32, sqc_margin (n,k), round_margin (n,m): distance of
    w/delta from the nearest rounding tie (for the sign quantiser |w|/alpha), in code steps;
    np.inf where the clamp decides."""
    Wc = np.array(W, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    n, m = Wc.shape
    k = m // beta
    B = beta if gptq_block is None else gptq_block
    codes = np.zeros((n, m), dtype=np.uint8)
    scale = np.zeros((n, k))
    zero = np.zeros((n, k))
    cand = np.zeros((n, k), dtype=np.int32)
    sqc_margin = np.zeros((n, k))
    round_margin = np.full((n, m), np.inf)
    What = np.zeros((n, m))
    E = np.zeros((n, m))
    for b0 in range(0, m, B):
        b1 = min(m, b0 + B)
        for c in range(b0, b1):
            g = c // beta
            bt = int(bits[g])
            if c % beta == 0:
                blk = Wc[:, c:c + beta]
                d = None if hinv_diag is None else np.asarray(hinv_diag, dtype=np.float64)[c:c + beta]
                om = _omega_rows(blk, weight_mode, scope, d)
                s_, z_, idx_, losses = _sqc_rows_fast(blk, bt, tau, om, q1_mode)
                scale[:, g], zero[:, g], cand[:, g] = s_, z_, idx_
                best = losses[np.arange(n), idx_]
                tmp = losses.copy()
                tmp[np.arange(n), idx_] = np.inf
                sqc_margin[:, g] = (tmp.min(axis=1) - best) / np.maximum(np.abs(best), 1e-300)
            w = Wc[:, c]
            s_, z_ = scale[:, g], zero[:, g]
            if bt == 1 and q1_mode == Q1_SIGN:
                q = (w >= 0.0).astype(np.float64)
                with np.errstate(divide="ignore", invalid="ignore"):
                    round_margin[:, c] = np.where(s_ > 0, np.abs(w) / (0.5 * s_), np.inf)
            else:
                x = np.rint(w / s_)
                q = np.clip(x + z_, 0.0, float(2 ** bt - 1))
                free = (x + z_ >= 0.0) & (x + z_ <= float(2 ** bt - 1))
                round_margin[:, c] = np.where(free, 0.5 - np.abs(w / s_ - x), np.inf)
            what = s_ * (q - z_)
            codes[:, c] = q.astype(np.uint8)
            What[:, c] = what
            e = (w - what) / U[c, c]
            E[:, c] = e
            if c + 1 < b1:
                Wc[:, c + 1:b1] -= np.outer(e, U[c, c + 1:b1])
        if b1 < m:
            Wc[:, b1:] -= E[:, b0:b1] @ U[b0:b1, b1:]
    return dict(codes=codes, scale=scale, zero=zero, What=What, E=E, sum_e2=float(np.sum(E * E)),
                cand_idx=cand, sqc_margin=sqc_margin, round_margin=round_margin)


def reconstruction_error(W: np.ndarray, What: np.ndarray, G: np.ndarray) -> float:
    """|| (W - What) X ||_F^2 = tr(dW G dW^T) with G = X X^T (Eq. 3)."""
    dW = np.asarray(W, dtype=np.float64) - np.asarray(What, dtype=np.float64)
    return float(np.sum((dW @ np.asarray(G, dtype=np.float64)) * dW))


# ----------------------------------------------------------------------------------------
# Storage (App. B.2)
# ----------------------------------------------------------------------------------------
def bit_base_for(N: int) -> int:
    """The width that the 2-bit group value 0 stands for (App. B.2 gives the value 2 bits).  A layer of target
    width N holds the widths N - 1, N, N + 1 only (the constraint of Eq. 4), so three of the four values are
    ever used: value = width - 1 covers the targets 2 and 3 (widths 1..4); above them (the 4-bit setting of
    App. G) the values count from N - 2, which maps N - 1, N, N + 1 to 1, 2, 3 for every target."""
    return max(1, int(N) - 2)


def pack(codes: np.ndarray, bits: np.ndarray, beta: int, bit_base: int = 1):
    """Returns (packed uint32 (m_star, n), gbits uint32 (ceil(k/16),), row_off int32 (k+1,), m_star).

    W^T is split into groups along its rows; for each (group g, output row i) the beta codes,
    each bits[g] wide, form a little-endian bit stream (element r occupies bits
    [r*b, (r+1)*b)) cut into 32-bit words that are stacked along the row axis of packed,
    starting at row_off[g]; groups follow one another without padding and no word mixes two
    widths (beta * b is a multiple of 32).  row_off is the running sum of beta*b_g/32.
    gbits stores b_g - bit_base as a 2-bit value, 16 groups per word, least significant first."""
    codes = np.asarray(codes)
    assert all(0 <= int(b) - bit_base <= 3 for b in bits)
    n, m = codes.shape
    k = m // beta
    words = [(beta * int(b)) // 32 for b in bits]
    row_off = np.zeros(k + 1, dtype=np.int32)
    row_off[1:] = np.cumsum(words)
    m_star = int(row_off[-1])
    packed = np.zeros((m_star, n), dtype=np.uint32)
    for g in range(k):
        b = int(bits[g])
        assert (beta * b) % 32 == 0
        for i in range(n):
            stream = 0
            for r in range(beta):
                stream |= int(codes[i, g * beta + r]) << (r * b)
            for wi in range(words[g]):
                packed[row_off[g] + wi, i] = (stream >> (32 * wi)) & 0xFFFFFFFF
    gbits = np.zeros((k + 15) // 16, dtype=np.uint32)
    for g in range(k):
        gbits[g // 16] |= np.uint32((int(bits[g]) - bit_base) << (2 * (g % 16)))
    return packed, gbits, row_off, m_star


def pack_fast(codes: np.ndarray, bits: np.ndarray, beta: int, bit_base: int = 1):
    """Same result as pack, built from an explicit bit matrix instead of Python integers, for
    layers too large for the loop form; tested equal to it."""
    codes = np.asarray(codes, dtype=np.uint8)
    n, m = codes.shape
    k = m // beta
    words = [(beta * int(b)) // 32 for b in bits]
    row_off = np.zeros(k + 1, dtype=np.int32)
    row_off[1:] = np.cumsum(words)
    m_star = int(row_off[-1])
    packed = np.zeros((m_star, n), dtype=np.uint32)
    weights = (np.uint64(1) << np.arange(32, dtype=np.uint64))
    for g in range(k):
        b = int(bits[g])
        blk = codes[:, g * beta:(g + 1) * beta]                       # (n, beta)
        bitmat = (blk[:, :, None] >> np.arange(b, dtype=np.uint8)[None, None, :]) & 1   # (n, beta, b)
        stream = bitmat.reshape(n, beta * b).astype(np.uint64)      # element r at [r*b, (r+1)*b)
        w = (stream.reshape(n, words[g], 32) * weights[None, None, :]).sum(axis=2)
        packed[row_off[g]:row_off[g + 1], :] = w.T.astype(np.uint32)
    gbits = np.zeros((k + 15) // 16, dtype=np.uint32)
    for g in range(k):
        gbits[g // 16] |= np.uint32((int(bits[g]) - bit_base) << (2 * (g % 16)))
    return packed, gbits, row_off, m_star


def unpack(packed: np.ndarray, gbits: np.ndarray, beta: int, k: int, bit_base: int = 1) -> tuple:
    """Inverse of pack: returns (codes (n, m) uint8, bits (k,) uint8)."""
    n = packed.shape[1]
    bits = np.array([((int(gbits[g // 16]) >> (2 * (g % 16))) & 3) + bit_base for g in range(k)], dtype=np.uint8)
    codes = np.zeros((n, k * beta), dtype=np.uint8)
    off = 0
    for g in range(k):
        b = int(bits[g])
        nw = beta * b // 32
        for i in range(n):
            stream = 0
            for wi in range(nw):
                stream |= int(packed[off + wi, i]) << (32 * wi)
            for r in range(beta):
                codes[i, g * beta + r] = (stream >> (r * b)) & ((1 << b) - 1)
        off += nw
    return codes, bits


def dequant_matmul(packed: np.ndarray, gbits: np.ndarray, row_off: np.ndarray, scale: np.ndarray,
                   zero: np.ndarray, beta: int, X: np.ndarray, bit_base: int = 1) -> np.ndarray:
    """The linear layer on the stored form (App. B.2, inference): the weights are dequantised group by group from
    the packed integers, the group-width array and the start rows, W^_ij = scale[i, g] * (q_ij - zero[i, g]) with
    g = j // beta (Eq. 1), and multiplied with the activations: Y = X W^^T for X of shape (t, m).  Plain float64.

    Written against the stored tensors only: widths come from gbits, a group's words from row_off, the codes
    from the bit stream of every (group, output row) - nothing from the quantiser's own outputs."""
    n = packed.shape[1]
    k = len(row_off) - 1
    X = np.asarray(X, dtype=np.float64)
    Y = np.zeros((X.shape[0], n))
    for g in range(k):
        b = ((int(gbits[g // 16]) >> (2 * (g % 16))) & 3) + bit_base
        nw = int(row_off[g + 1]) - int(row_off[g])
        assert nw * 32 == beta * b
        words = packed[int(row_off[g]):int(row_off[g + 1]), :].astype(np.uint64)        # (nw, n)
        q = np.zeros((n, beta))
        for r in range(beta):
            lo = r * b                       # element r occupies bits [r b, (r + 1) b) of the group's stream
            w, sh = lo // 32, lo % 32
            v = words[w] >> np.uint64(sh)
            if sh + b > 32:
                v = v | (words[w + 1] << np.uint64(32 - sh))
            q[:, r] = (v & np.uint64((1 << b) - 1)).astype(np.float64)
        Wg = scale[:, g][:, None] * (q - zero[:, g][:, None])                            # (n, beta)
        Y += X[:, g * beta:(g + 1) * beta] @ Wg.T
    return Y


def zero_bits_for(N: int) -> int:
    """Width of a packed zero point for a layer of target width N: the stored value is 2 z (Eq. 1 gives integer
    zeros in 0 .. 2^b - 1 for a group that straddles zero, the sign form of width 1 has z = 1/2), and the widest
    group has N + 1 bits, so 2 z <= 2^(N+2) - 2 fits N + 2 bits."""
    return int(N) + 2


def pack_zeros(zero: np.ndarray, zbits: int):
    """Zero points as packed integers (App. B.2: packed with a uniform precision along the channel direction).

    zero is (n, k): output channels x groups.  For every group g the n values u_i = 2 z_ig (integers) form a
    little-endian bit stream along the output channels, element i at bits [i zbits, (i + 1) zbits), cut into
    32-bit words: zp[g, w].  Returns (zp uint32 (k, ceil(n zbits / 32)), n_bad): a value that is not a multiple of
    1/2 or does not fit zbits bits (Eq. 1 does not bound the zero of a group whose weights all have one sign) is
    counted in n_bad and stored as 0 or the largest value, whichever is nearer."""
    zero = np.asarray(zero, dtype=np.float64)
    n, k = zero.shape
    top = (1 << zbits) - 1
    nw = (n * zbits + 31) // 32
    zp = np.zeros((k, nw), dtype=np.uint32)
    n_bad = 0
    for g in range(k):
        stream = 0
        for i in range(n):
            u2 = 2.0 * zero[i, g]
            u = int(np.rint(u2))
            if u != u2 or u < 0 or u > top:
                n_bad += 1
                u = min(max(u, 0), top)
            stream |= u << (i * zbits)
        for w in range(nw):
            zp[g, w] = (stream >> (32 * w)) & 0xFFFFFFFF
    return zp, n_bad


def unpack_zeros(zp: np.ndarray, n: int, zbits: int) -> np.ndarray:
    """Inverse of pack_zeros: (n, k) float64 zero points z = u / 2."""
    k = zp.shape[0]
    zero = np.zeros((n, k))
    for g in range(k):
        stream = 0
        for w in range(zp.shape[1]):
            stream |= int(zp[g, w]) << (32 * w)
        for i in range(n):
            zero[i, g] = ((stream >> (i * zbits)) & ((1 << zbits) - 1)) / 2.0
    return zero


# ----------------------------------------------------------------------------------------
# Layers one after another (Sec. 3.4: SBA and SQC inside GPTQ, whose layers are calibrated on
# the outputs of their already quantised predecessors)
# ----------------------------------------------------------------------------------------
def next_layer_input(out: dict, beta: int, N: int, X: np.ndarray) -> np.ndarray:
    """Calibration activations of the next layer: the quantised layer applied to X (m x t, channels x tokens) FROM
    ITS STORED FORM (packed codes, group widths, start rows, scales, zeros), rounded to fp16 like every activation
    tensor of the path: returns (n x t) float16."""
    Y = dequant_matmul(out["packed"], out["gbits"], out["row_off"], out["scale"], out["zero"], beta,
                       np.asarray(X, dtype=np.float64).T, bit_base_for(N))
    return np.clip(Y, -65504.0, 65504.0).astype(np.float16).T.copy()


def sequential_layers(Ws, X0: np.ndarray, beta: int, N: int, percdamp: float = 0.01, t_sba: int = 2048, **kw):
    """A chain of linear layers y = W_l x, quantised in order.  Layer 0 is calibrated on X0 (m_0 x t); layer l + 1 on
    the outputs of the QUANTISED layer l for the same tokens (next_layer_input), so that each layer compensates for
    the error its predecessors have already made.  Returns the list of per-layer results of slim_layer, each with
    its calibration input under "X"."""
    X = np.asarray(X0)
    outs = []
    for W in Ws:
        out = slim_layer(W, [X], beta, N, percdamp, t_sba=t_sba, **kw)
        out["X"] = X
        outs.append(out)
        X = next_layer_input(out, beta, N, X)
    return outs


# ----------------------------------------------------------------------------------------
# SliM-LLM+ (Sec. 3.4; Sec. 4; App. B): SBA's widths, no SQC and no compensation, a quantiser with
# learnable weight clipping per (row, group) trained by AdamW on the layer-output error
# ----------------------------------------------------------------------------------------
def lwc_forward(W: np.ndarray, gamma: np.ndarray, beta_p: np.ndarray, bits: np.ndarray, beta: int):
    """Fake quantisation with learnable clipping.  For every (row i, group g), with M and m_ the largest and the
    smallest weight of the (row, group):  hi = sigmoid(gamma_ig) M,  lo = sigmoid(beta_ig) m_,
    delta = (hi - lo) / (2^b - 1),  z = -round(lo / delta),  q = clamp(round(w / delta) + z, 0, 2^b - 1),
    w_hat = delta (q - z)   (Eq. 1 on the clipped range; every width, 1 bit included, in this affine form).
    A (row, group) with hi <= lo (all weights zero) gets delta = 1, z = 0.
    Returns a dict: What (n, m), codes (n, m) uint8, scale, zero (n, k), and what the derivatives need."""
    W = np.asarray(W, dtype=np.float64)
    n, m = W.shape
    k = m // beta
    Wg = W.reshape(n, k, beta)
    Q = (2.0 ** np.asarray(bits, dtype=np.float64) - 1.0)[None, :]                 # (1, k)
    M, m_ = Wg.max(axis=2), Wg.min(axis=2)
    s_hi, s_lo = 1.0 / (1.0 + np.exp(-gamma)), 1.0 / (1.0 + np.exp(-beta_p))
    hi, lo = s_hi * M, s_lo * m_
    live = hi > lo
    delta = np.where(live, (hi - lo) / Q, 1.0)
    z = np.where(live, -np.rint(lo / delta), 0.0)
    u = np.rint(Wg / delta[:, :, None]) + z[:, :, None]
    q = np.clip(u, 0.0, Q[:, :, None])
    What = delta[:, :, None] * (q - z[:, :, None])
    inside = (u >= 0.0) & (u <= Q[:, :, None])
    return dict(What=What.reshape(n, m), codes=q.reshape(n, m).astype(np.uint8), scale=delta, zero=z, q=q, inside=inside,
                M=M, m_=m_, s_hi=s_hi, s_lo=s_lo, lo=lo, Q=Q, live=live, Wg=Wg,
                round_margin=np.where(inside, 0.5 - np.abs(Wg / delta[:, :, None] - np.rint(Wg / delta[:, :, None])),
                                      np.inf).reshape(n, m))


def lwc_loss_and_grads(W, G, n_tokens, gamma, beta_p, bits, beta):
    """Loss L = || (W - W_hat) X ||_F^2 / (n T) = tr(dW G dW^T) / (n T) (Eq. 3 with G = X X^T; the mean squared error
    of the layer's outputs) and its derivatives with respect to gamma and beta_p, the rounding taken as the identity
    in the backward pass (straight-through) and the clamp passing derivatives where it does not clip:
        g = dL/dW_hat = 2 (W_hat - W) G / (n T)
        dW_hat_j/d delta = (q_j - z) - w_j / delta   (not clipped),   (q_j - z) - lo / delta   (clipped)
        dW_hat_j/d lo at fixed delta = 0 (not clipped), 1 (clipped)            [through z = -round(lo / delta)]
        delta = (hi - lo) / Q,  hi = sigmoid(gamma) M,  lo = sigmoid(beta_p) m_."""
    f = lwc_forward(W, gamma, beta_p, bits, beta)
    W = np.asarray(W, dtype=np.float64)
    n, m = W.shape
    k = m // beta
    D = f["What"] - W
    DG = D @ np.asarray(G, dtype=np.float64)
    norm = float(n) * float(n_tokens)
    loss = float(np.sum(D * DG)) / norm
    g = (2.0 / norm) * DG.reshape(n, k, beta)
    delta, z, lo = f["scale"][:, :, None], f["zero"][:, :, None], f["lo"][:, :, None]
    dwd = np.where(f["inside"], (f["q"] - z) - f["Wg"] / delta, (f["q"] - z) - lo / delta)
    s1 = np.sum(g * dwd, axis=2)                          # dL/d delta
    s2 = np.sum(np.where(f["inside"], 0.0, g), axis=2)    # dL/d lo at fixed delta
    d_hi = np.where(f["live"], s1 / f["Q"], 0.0)
    d_lo = np.where(f["live"], -s1 / f["Q"] + s2, 0.0)
    g_gamma = d_hi * f["M"] * f["s_hi"] * (1.0 - f["s_hi"])
    g_beta = d_lo * f["m_"] * f["s_lo"] * (1.0 - f["s_lo"])
    return loss, g_gamma, g_beta, f


def adamw_step(p, grad, m1, v, step, lr, b1, b2, eps, weight_decay=0.0):
    """One AdamW update (decoupled weight decay) in place; step counts from 1."""
    p *= 1.0 - lr * weight_decay
    m1 *= b1
    m1 += (1.0 - b1) * grad
    v *= b2
    v += (1.0 - b2) * grad * grad
    mhat = m1 / (1.0 - b1 ** step)
    vhat = v / (1.0 - b2 ** step)
    p -= lr * mhat / (np.sqrt(vhat) + eps)


def lwc_quantize(W, G, n_tokens, bits, beta, steps=20, lr=1e-2, b1=0.9, b2=0.999, eps=1e-8, init=4.0):
    """SliM-LLM+ for one layer: the widths `bits` (from SBA) stay fixed; the clipping strengths gamma, beta_p of every
    (row, group) start at `init` and take `steps` full-batch AdamW steps on lwc_loss_and_grads; the layer is then
    quantised with the final strengths.  Returns the forward dict of the final strengths plus loss_curve
    (steps + 1 values: before every step and after the last), gamma, beta_p."""
    W = np.asarray(W, dtype=np.float64)
    n, m = W.shape
    k = m // beta
    gamma = np.full((n, k), float(init))
    beta_p = np.full((n, k), float(init))
    mg, vg, mb, vb = (np.zeros((n, k)) for _ in range(4))
    curve = np.empty(steps + 1)
    for it in range(1, steps + 1):
        curve[it - 1], gg, gb, _ = lwc_loss_and_grads(W, G, n_tokens, gamma, beta_p, bits, beta)
        adamw_step(gamma, gg, mg, vg, it, lr, b1, b2, eps)
        adamw_step(beta_p, gb, mb, vb, it, lr, b1, b2, eps)
    curve[steps], _, _, f = lwc_loss_and_grads(W, G, n_tokens, gamma, beta_p, bits, beta)
    f.update(loss_curve=curve, gamma=gamma, beta_p=beta_p)
    return f


# ----------------------------------------------------------------------------------------
# The whole pass (Alg. 1)
# ----------------------------------------------------------------------------------------
def slim_layer(W: np.ndarray, X_chunks, beta: int, N: int, percdamp: float = 0.01,
               tau: np.ndarray | None = None, t_sba: int = 2048, weight_mode: int = WEIGHT_MASK_MEAN,
               scope: int = SCOPE_BLOCK, q1_mode: int = Q1_SIGN, do_pack: bool = True):
    """Alg. 1 end to end.  X_chunks iterates over (m, t_c) chunks of calibration tokens; the
    SBA objective uses the first t_sba tokens."""
    W64 = np.asarray(W, dtype=np.float64)
    n, m = W64.shape
    tau = tau_grid() if tau is None else tau
    G = np.zeros((m, m))
    T = 0
    Xs_parts, have = [], 0
    for Xc in X_chunks:
        gram_accumulate(G, Xc)
        T += Xc.shape[1]
        if have < t_sba:
            take = min(t_sba - have, Xc.shape[1])
            Xs_parts.append(np.asarray(Xc[:, :take], dtype=np.float64))
            have += take
    Xs = np.concatenate(Xs_parts, axis=1)
    U, hinv_diag, lam = hessian_inverse(G, T, percdamp)
    col_sal, group_sal, _ = salience(W64, hinv_diag, beta)
    bits, p_star, obj, sba_margin = sba_allocate(W64, group_sal, beta, N, Xs, q1_mode)
    out = gptq_quantize(W64, U, bits, beta, tau, weight_mode, scope, q1_mode, hinv_diag=hinv_diag)
    out.update(G=G, n_tokens=T, U=U, hinv_diag=hinv_diag, lam=lam, col_sal=col_sal, group_sal=group_sal,
               bits=bits, p_star=p_star, obj_curve=obj, sba_margin=sba_margin,
               recon=reconstruction_error(W64, out["What"], G))
    if do_pack:
        out["packed"], out["gbits"], out["row_off"], out["m_star"] = pack(out["codes"], bits, beta, bit_base_for(N))
    return out
