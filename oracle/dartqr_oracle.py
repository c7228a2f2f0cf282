"""CPU oracle for the QR-Orth calibration step of DartQuant (arXiv 2511.04063).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain, fp64 statement of what
one QR-Orth step computes.  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import it.  It shares no code with the HIP
library (no kernels, headers, helpers or tables) and never imports the product
package; the product path never imports this module.

Everything runs in float64 with NumPy.  Matrix products use ``@`` (a library
primitive used as one step); everything else is written out.

What the paper fixes and what it leaves open
--------------------------------------------
* Alg. 1 (Sec. 4.3), loop body:  R <- qr(Z);  O <- X @ R;  L <- Whip(O);
  Z <- Z - eta * dL/dZ.
* Eq. 4 (Sec. 4.2):  Whip(x) = sum_i exp(-|x_i|) for ONE activation vector x.
* Sec. 4.3: QR of any Z gives an orthogonal R and an upper-triangular U, Z = R U.
  (The paper calls the orthogonal factor R and the triangular factor U.)
* Alg. 2 (App. B.1): Householder QR, v = x + sign(x_1) ||x|| e_1, v <- v/||v||,
  reflect the trailing block and accumulate the orthogonal factor.

Readings taken where the paper is silent (each is also listed in the design notes):
* sign convention of the QR: diag(U) >= 0 (sign(0) := +1), which makes R unique for
  nonsingular Z.  Loss and dZ do not depend on this choice.
* Whip over a block of T tokens: ``reduce="mean"`` -> (1/T) * sum over tokens of the
  per-token Whip (default);  ``reduce="sum"`` -> plain sum.  Parity unpinned by the
  paper (a pure scale, equivalent to rescaling eta).
* d|y|/dy at y = 0 is taken as 0.  Parity unpinned by the paper.
* dL/dZ is not written in the paper (it says only "dL/dZ" in the last step of Alg. 1).  It is
  derived here from Z = R U:  with B = R^T G, P = strict_lower(B - B^T),
  dZ = R P U^{-T}.  Pinned by finite differences of the whole map Z -> L, by the
  structural identities of the true gradient, and by a library autograd route
  (all in tests/).
* Alg. 2 as printed updates only a square sub-block of the orthogonal factor and
  stops at k = n-1; it is read as the textbook Householder QR (right-multiply ALL rows
  of the accumulated factor, columns k..n), and the last diagonal entry's sign is
  handled by the sign normalisation above.
* Sec. 4.3 and Table 4 say that Z may be driven by "SGD or Adam" and print neither rule
  nor hyper-parameters.  Adam is taken as the standard rule with bias correction and
  the usual defaults (beta1 0.9, beta2 0.999, eps 1e-8, step counter from 1); SGD with
  momentum as the heavy-ball form without dampening.  Both pinned against closed forms
  and a library optimiser (tests/).
* Alg. 1, token_sampling(X): the paper keeps a random 10 % of the tokens (App.,
  sample-size analysis) and does not say how they are drawn.  The draw is an INPUT here
  (a list of row numbers, repeats allowed); the step itself is the selection of those
  rows, in the given order.  Pinned by its invariants (tests/).
* App. (hyper-parameter settings): the latent starts from a randomised Hadamard matrix, construction not given.  Read
  as diag(s) H_n / sqrt(n) with Sylvester's H_n and random signs s supplied by the caller.  Pinned by orthogonality,
  the Kronecker form and the bit-count form of the entries (tests/).
* Sec. 4.1 and the ablation of Sec. 5 (comparison of four objectives) name variance, kurtosis and the quantisation loss
  as alternatives to Eq. 4 and print no formula for any of them.  PARITY UNPINNED BY THE PAPER; the readings taken, each
  per token row y of n channels and combined over the rows like Eq. 4 (sum, or mean over tokens):
    variance      m2 = (1/n) sum_i (y_i - mu)^2, mu the row mean;
    kurtosis      m4 / m2^2 with m_k = (1/n) sum_i (y_i - mu)^k (Pearson's, 3 for a Gaussian); 0 for a constant row;
    quantisation  (1/n) sum_i (y_i - yhat_i)^2 for the per-token asymmetric uniform quantiser the paper's experiments
                  use for activations (Sec. 5: per-token asymmetric, 4 bits): lo = min_i y_i, hi = max_i y_i,
                  delta = (hi - lo) / (2^bits - 1), code q_i = round((y_i - lo) / delta) (nearest level, ties to
                  even), yhat_i = lo + delta q_i; 0 for a constant row.  All of it in float64 on the given values.
                  Gradient: the codes are held fixed (the derivative that exists almost everywhere), lo and hi carry
                  gradient to the first position of the row minimum and maximum.  An entry whose grid position
                  (y_i - lo) / delta lies within rounding distance of a half-integer may legitimately take either
                  neighbouring code in a lower-precision implementation; ``quant_positions`` returns those positions
                  and ``quant_objective(codes=...)`` evaluates loss and gradient for a given set of codes, so that a
                  test can separate "a valid other code" from "a wrong result".
  Pinned by library routines (numpy.var, scipy.stats.kurtosis), closed forms, a brute-force nearest-level search,
  invariances and central finite differences (tests/).
* Alg. 3 (App. B.2), Cayley SGD with momentum, the optimiser QR-Orth is compared with (Sec. 5, optimiser comparison):
  it acts on the rotation itself (the algorithm's X is this module's R), with the Euclidean gradient dL/dR.  As
  printed, the skew-symmetrisation step reads "W_k <- W^_k - W_k^T"; it is read as W_k = W^_k - W^_k^T (the only
  reading that makes W_k skew-symmetric, which the Cayley transform needs).  The norm in the step-size rule
  alpha = min(l, 2q / (||W_k|| + eps)) is not named; the Frobenius norm is taken (it bounds the spectral norm, so
  the fixed-point iteration of the transform contracts at rate alpha ||W_k||_2 / 2 <= q either way).  The loop
  "for k = 0 to T" is run for the number of steps asked for.  Pinned by the exact Cayley transform (a linear solve),
  the contraction bound of the iteration, a 2 x 2 closed form, descent identities and orthogonality (tests/).
"""

from __future__ import annotations

import numpy as np

__all__ = [
    "householder_qr",
    "qr_orth",
    "rotate",
    "whip_loss",
    "whip_grad",
    "grad_wrt_rotation",
    "qr_backward",
    "sgd_update",
    "sgd_momentum_update",
    "adam_update",
    "calib_step",
    "calib_step_adam",
    "calibrate",
    "rotate_loss_grad",
    "token_sampling",
    "outlier_count",
    "hadamard_latent",
    "variance_objective",
    "kurtosis_objective",
    "quant_positions",
    "quant_objective",
    "objective_loss_grad",
    "calibrate_batches",
    "cayley_sgd_update",
    "cayley_step",
]


def _f64(a) -> np.ndarray:
    return np.array(a, dtype=np.float64, copy=True)


def _reduce_scale(reduce: str, n_tokens: int) -> float:
    """Scale c in L = c * sum_t sum_i exp(-|Y_ti|)  (reading of the loss step of Alg. 1)."""
    if reduce == "mean":
        return 1.0 / float(n_tokens)
    if reduce == "sum":
        return 1.0
    raise ValueError(f"unknown reduce mode {reduce!r}")


def householder_qr(Z):
    """Unblocked Householder QR, Alg. 2 (App. B.1), read as the textbook algorithm.

    Returns (Q, U0) with Z = Q @ U0, Q orthogonal, U0 upper triangular.  The signs of
    diag(U0) are whatever the reflections produce (they are fixed by ``qr_orth``).

    Step k of the reflector recurrence:  x = A[k:, k];  v = x + sign(x_1) ||x||_2 e_1 with
    sign(0) = +1;  v <- v / ||v||_2;  the reflection I - 2 v v^T is applied to the trailing
    block A[k:, k:] from the left and to the columns k.. of the accumulated orthogonal factor
    from the right.  A zero column below (and on) the diagonal is skipped (v would be 0).
    """
    A = _f64(Z)
    if A.ndim != 2 or A.shape[0] != A.shape[1]:
        raise ValueError("Z must be square")
    n = A.shape[0]
    Qacc = np.eye(n, dtype=np.float64)
    for k in range(n):
        x = A[k:, k].copy()
        norm_x = np.sqrt(np.sum(x * x))
        if norm_x == 0.0:
            continue
        sgn = 1.0 if x[0] >= 0.0 else -1.0
        v = x
        v[0] = v[0] + sgn * norm_x
        v = v / np.sqrt(np.sum(v * v))
        # reflect the trailing block of A
        w = v @ A[k:, k:]
        A[k:, k:] -= 2.0 * np.outer(v, w)
        # accumulate the orthogonal factor on the right, all rows
        q = Qacc[:, k:] @ v
        Qacc[:, k:] -= 2.0 * np.outer(q, v)
    U0 = np.triu(A)
    return Qacc, U0


def qr_orth(Z):
    """Z -> (R, U): orthogonal R, upper-triangular U with diag(U) >= 0, Z = R @ U.

    Sec. 4.3 (QR of the latent Z) followed by the sign normalisation
    s_i = +1 if U0[i,i] >= 0 else -1;  R = Q diag(s);  U = diag(s) U0.
    """
    Q, U0 = householder_qr(Z)
    s = np.where(np.diag(U0) >= 0.0, 1.0, -1.0)
    R = Q * s[None, :]
    U = U0 * s[:, None]
    return R, U


def hadamard_latent(signs) -> np.ndarray:
    """The initial latent of the paper's runs (App., hyper-parameter settings), read as diag(s) H_n / sqrt(n) with H_n
    built by Sylvester's doubling  H_1 = [1],  H_2m = [[H_m, H_m], [H_m, -H_m]];  n = len(s) a power of two."""
    s = _f64(signs)
    n = s.shape[0]
    if n < 1 or n & (n - 1):
        raise ValueError("n must be a power of two")
    H = np.array([[1.0]])
    while H.shape[0] < n:
        H = np.block([[H, H], [H, -H]])
    return (s[:, None] * H) / np.sqrt(float(n))


def outlier_count(Y, tau: float) -> int:
    """Sec. 4.1, Eq. 1 summed over the tokens of a block: how many entries have |y| > tau."""
    Y = np.asarray(Y)
    count = 0
    for row in Y.reshape(-1, Y.shape[-1]) if Y.ndim > 1 else [Y]:
        for y in row:
            if abs(float(y)) > tau:
                count += 1
    return count


def token_sampling(X, idx) -> np.ndarray:
    """The token-sampling step of Alg. 1: the activation rows named by idx, in that order (values untouched)."""
    X = np.asarray(X)
    idx = np.asarray(idx)
    if idx.ndim != 1:
        raise ValueError("idx must be a list of row numbers")
    out = np.empty((idx.shape[0],) + X.shape[1:], dtype=X.dtype)
    for t in range(idx.shape[0]):
        r = int(idx[t])
        if r < 0 or r >= X.shape[0]:
            raise IndexError(f"row {r} outside [0, {X.shape[0]})")
        out[t] = X[r]
    return out


def rotate(X, R):
    """O = X @ R  (the rotation step of Alg. 1; rows of X are tokens)."""
    return _f64(X) @ _f64(R)


def whip_loss(Y, reduce: str = "mean") -> float:
    """L = c * sum_t sum_i exp(-|Y_ti|)  (Eq. 4 summed over the token rows)."""
    Y = _f64(Y)
    c = _reduce_scale(reduce, Y.shape[0])
    return float(c * np.sum(np.exp(-np.abs(Y))))


def whip_grad(Y, reduce: str = "mean") -> np.ndarray:
    """dL/dY_ti = -c * sgn(Y_ti) * exp(-|Y_ti|), with sgn(0) = 0."""
    Y = _f64(Y)
    c = _reduce_scale(reduce, Y.shape[0])
    return -c * np.sign(Y) * np.exp(-np.abs(Y))


def variance_objective(Y, reduce: str = "mean"):
    """Per-token variance as the objective (Sec. 4.1 names it; formula: reading above).

    L = c * sum_t m2_t,  m2_t = (1/n) sum_i (Y_ti - mu_t)^2;   dL/dY_ti = c * (2/n) * (Y_ti - mu_t).
    Returns (loss, dY)."""
    Y = _f64(Y)
    T, n = Y.shape
    c = _reduce_scale(reduce, T)
    loss = 0.0
    dY = np.zeros_like(Y)
    for t in range(T):
        mu = np.sum(Y[t]) / n
        d = Y[t] - mu
        loss += np.sum(d * d) / n
        dY[t] = c * (2.0 / n) * d
    return float(c * loss), dY


def kurtosis_objective(Y, reduce: str = "mean"):
    """Per-token kurtosis as the objective (Sec. 4.1 names it; formula: reading above).

    kappa_t = m4 / m2^2 with central moments m_k = (1/n) sum_i d_i^k, d = Y_t - mu_t.  Since d m4 / d y_i =
    (4/n) (d_i^3 - m3) and d m2 / d y_i = (2/n) d_i,
        d kappa / d y_i = (4/n) * ( (d_i^3 - m3) / m2^2 - m4 * d_i / m2^3 ).
    A constant row (m2 = 0) contributes 0 and gets no gradient.  Returns (loss, dY)."""
    Y = _f64(Y)
    T, n = Y.shape
    c = _reduce_scale(reduce, T)
    loss = 0.0
    dY = np.zeros_like(Y)
    for t in range(T):
        mu = np.sum(Y[t]) / n
        d = Y[t] - mu
        m2 = np.sum(d ** 2) / n
        if m2 == 0.0:
            continue
        m3 = np.sum(d ** 3) / n
        m4 = np.sum(d ** 4) / n
        loss += m4 / (m2 * m2)
        dY[t] = c * (4.0 / n) * ((d ** 3 - m3) / (m2 * m2) - m4 * d / (m2 ** 3))
    return float(c * loss), dY


def quant_positions(Y, bits: int = 4) -> np.ndarray:
    """Position of every entry on its row's quantiser grid, u_i = (y_i - lo) / delta with lo / hi the row minimum /
    maximum and delta = (hi - lo) / (2^bits - 1): level k sits at u = k.  Rows without a range give zeros."""
    Y = _f64(Y)
    levels = (1 << int(bits)) - 1
    u = np.zeros_like(Y)
    for t in range(Y.shape[0]):
        lo, hi = np.min(Y[t]), np.max(Y[t])
        delta = (hi - lo) / levels
        if delta > 0:
            u[t] = (Y[t] - lo) / delta
    return u


def quant_objective(Y, bits: int = 4, reduce: str = "mean", codes=None):
    """Per-token asymmetric uniform quantisation error as the objective (Sec. 5 names the quantiser and the objective;
    formula: reading above).

    Per row: lo, hi = min, max;  delta = (hi - lo) / L with L = 2^bits - 1;  q_i = round((y_i - lo) / delta), ties to
    even;  yhat_i = lo + delta q_i = lo (1 - q_i / L) + hi q_i / L;  e_i = y_i - yhat_i;  loss_t = (1/n) sum_i e_i^2.
    With the codes held fixed,
        d loss_t / d y_j = (2/n) * ( e_j - [j = jmin] sum_i e_i (1 - q_i / L) - [j = jmax] sum_i e_i q_i / L ),
    jmin / jmax the first positions of the minimum / maximum.  ``codes`` (T x n integers in [0, L]) replaces the
    nearest-level decision by a given one (rows without a range ignore it).  Returns (loss, dY, codes)."""
    Y = _f64(Y)
    T, n = Y.shape
    levels = (1 << int(bits)) - 1
    c = _reduce_scale(reduce, T)
    u = quant_positions(Y, bits)
    loss = 0.0
    dY = np.zeros((T, n), dtype=np.float64)
    out_codes = np.zeros((T, n), dtype=np.int64)
    for t in range(T):
        y = Y[t]
        lo, hi = np.min(y), np.max(y)
        delta = (hi - lo) / levels
        if not delta > 0:
            continue
        if codes is None:
            q = np.rint(u[t])          # ties to even
        else:
            q = np.asarray(codes[t], dtype=np.float64)
            if np.any(q < 0) or np.any(q > levels) or np.any(q != np.rint(q)):
                raise ValueError("codes must be integers in [0, 2^bits - 1]")
        out_codes[t] = q.astype(np.int64)
        e = y - (lo + delta * q)
        loss += np.sum(e * e) / n
        g = e.copy()
        g[int(np.argmin(y))] -= np.sum(e * (1.0 - q / levels))
        g[int(np.argmax(y))] -= np.sum(e * (q / levels))
        dY[t] = c * (2.0 / n) * g
    return float(c * loss), dY, out_codes


def objective_loss_grad(Y, objective: str = "whip", reduce: str = "mean", bits: int = 4):
    """(loss, dY) of one of the four objectives the paper compares (Sec. 5, ablation of the optimisation objective)."""
    if objective == "whip":
        return whip_loss(Y, reduce), whip_grad(Y, reduce)
    if objective == "variance":
        return variance_objective(Y, reduce)
    if objective == "kurtosis":
        return kurtosis_objective(Y, reduce)
    if objective == "quant":
        loss, dY, _ = quant_objective(Y, bits, reduce)
        return loss, dY
    raise ValueError(f"unknown objective {objective!r}")


def grad_wrt_rotation(X, dY) -> np.ndarray:
    """G = dL/dR = X^T @ dY   (chain rule through O = X @ R)."""
    return _f64(X).T @ _f64(dY)


def _solve_right_upper_transposed(W, U) -> np.ndarray:
    """Solve M @ U^T = W for M (U upper triangular, so U^T is lower triangular).

    Column j of the product is  sum_{k >= j} M[:, k] * U[j, k], so the columns are
    found from the last to the first by substitution.
    """
    n = U.shape[0]
    M = np.zeros_like(W)
    for j in range(n - 1, -1, -1):
        acc = W[:, j].copy()
        if j + 1 < n:
            acc -= M[:, j + 1:] @ U[j, j + 1:]
        M[:, j] = acc / U[j, j]
    return M


def qr_backward(R, U, G) -> np.ndarray:
    """dL/dZ from G = dL/dR through Z = R U (diag(U) > 0), no gradient flowing into U.

    Derivation (not in the paper, which writes only dL/dZ in the last step of Alg. 1):
    dZ = dR U + R dU  =>  R^T dZ U^{-1} = Omega + dU U^{-1}, Omega = R^T dR skew,
    dU U^{-1} upper triangular  =>  Omega = Lo - Lo^T, Lo = strict_lower(R^T dZ U^{-1}).
    Then <G, R Omega> = <strict_lower(B - B^T), R^T dZ U^{-1}> with B = R^T G, hence
        dL/dZ = R @ strict_lower(B - B^T) @ U^{-T}.
    """
    R = _f64(R)
    U = _f64(U)
    G = _f64(G)
    if np.any(np.diag(U) == 0.0):
        raise ZeroDivisionError("U has a zero on its diagonal: Z is singular")
    B = R.T @ G
    P = np.tril(B - B.T, k=-1)
    M = _solve_right_upper_transposed(P, U)
    return R @ M


def sgd_update(Z, dZ, lr: float) -> np.ndarray:
    """Z <- Z - eta * dL/dZ  (the update step of Alg. 1; plain SGD, no momentum)."""
    return _f64(Z) - float(lr) * _f64(dZ)


def sgd_momentum_update(Z, dZ, buf, lr: float, mu: float):
    """SGD with momentum on the latent (Sec. 4.3: "any optimizer" may drive Z; the paper gives no formula, reading
    G11: heavy ball without dampening):  buf <- mu * buf + dL/dZ,  Z <- Z - eta * buf.   Returns (Z_new, buf_new)."""
    buf_new = float(mu) * _f64(buf) + _f64(dZ)
    return _f64(Z) - float(lr) * buf_new, buf_new


def adam_update(Z, dZ, m, v, step: int, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8):
    """Adam on the latent (Sec. 4.3 and Table 4 name Adam as an optimiser for Z and give no hyper-parameters,
    reading G10: the standard rule with bias correction and its usual defaults):

        m <- beta1 m + (1 - beta1) g,   v <- beta2 v + (1 - beta2) g^2,
        Z <- Z - eta * (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps),   t = step >= 1.

    Returns (Z_new, m_new, v_new)."""
    if int(step) < 1:
        raise ValueError("Adam's step counter starts at 1")
    g = _f64(dZ)
    m_new = float(beta1) * _f64(m) + (1.0 - float(beta1)) * g
    v_new = float(beta2) * _f64(v) + (1.0 - float(beta2)) * g * g
    m_hat = m_new / (1.0 - float(beta1) ** int(step))
    v_hat = v_new / (1.0 - float(beta2) ** int(step))
    return _f64(Z) - float(lr) * m_hat / (np.sqrt(v_hat) + float(eps)), m_new, v_new


def rotate_loss_grad(X, R, reduce: str = "mean", objective: str = "whip", bits: int = 4):
    """(loss, G, Y, dY) for a given rotation R  (Alg. 1, its rotation and loss steps, and dL/dR).  The quantisation objective decides
    its codes on Y rounded to float32 (the precision the GPU path holds Y in)."""
    Y = rotate(X, R)
    if objective == "quant":
        Y = Y.astype(np.float32).astype(np.float64)
    loss, dY = objective_loss_grad(Y, objective, reduce, bits)
    G = grad_wrt_rotation(X, dY)
    return loss, G, Y, dY


def calib_step(X, Z, lr: float, reduce: str = "mean", objective: str = "whip", bits: int = 4):
    """One pass of the loop body of Alg. 1.

    Returns a dict with the loss and rotation computed from the INPUT Z, the gradient
    dZ, and the updated latent Z_new.
    """
    Z = _f64(Z)
    R, U = qr_orth(Z)
    loss, G, Y, dY = rotate_loss_grad(X, R, reduce, objective, bits)
    dZ = qr_backward(R, U, G)
    Z_new = sgd_update(Z, dZ, lr)
    return {"loss": loss, "R": R, "U": U, "G": G, "dZ": dZ, "Z_new": Z_new}


def calib_step_adam(X, Z, m, v, step: int, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
                    reduce: str = "mean"):
    """The loop body of Alg. 1 with Adam in place of its SGD update."""
    Z = _f64(Z)
    R, U = qr_orth(Z)
    loss, G, Y, dY = rotate_loss_grad(X, R, reduce)
    dZ = qr_backward(R, U, G)
    Z_new, m_new, v_new = adam_update(Z, dZ, m, v, step, lr, beta1, beta2, eps)
    return {"loss": loss, "R": R, "U": U, "G": G, "dZ": dZ, "Z_new": Z_new, "m": m_new, "v": v_new}


def calibrate(X, Z0, steps: int, lr: float, reduce: str = "mean"):
    """Run ``steps`` passes of the loop of Alg. 1 from Z0.

    Returns (losses, Z_final, R_final) where losses[k] is the loss of the k-th input Z
    and R_final = qr_orth(Z_final)[0] is the calibrated rotation.
    """
    Z = _f64(Z0)
    losses = []
    for _ in range(int(steps)):
        out = calib_step(X, Z, lr, reduce)
        losses.append(out["loss"])
        Z = out["Z_new"]
    R_final, _ = qr_orth(Z)
    return np.array(losses), Z, R_final


def calibrate_batches(X_batches, Z0, steps: int, lr: float, reduce: str = "mean"):
    """The loop of Alg. 1 over mini-batches: step k runs the loop body on batch k mod len(X_batches),
    epoch after epoch in the given order.  Returns (losses, Z_final)."""
    Z = _f64(Z0)
    losses = []
    for k in range(int(steps)):
        out = calib_step(X_batches[k % len(X_batches)], Z, lr, reduce)
        losses.append(out["loss"])
        Z = out["Z_new"]
    return np.array(losses), Z


def cayley_sgd_update(R, G, M, lr: float, beta: float = 0.9, q: float = 0.5, s: int = 2, eps: float = 1e-8):
    """One update of Alg. 3 (App. B.2): Cayley SGD with momentum on an orthogonal matrix (the algorithm's X_k is the
    rotation R, its gradient G = dL/dR, its momentum buffer M, zero before the first step).

        M' = beta M - G
        W^ = M' R^T - (1/2) R (R^T M' R^T);   W = W^ - W^^T   (skew-symmetric)
        M_new = W R                              (the momentum, projected onto the tangent space at R)
        alpha = min(lr, 2 q / (||W||_F + eps))
        Y^0 = R + alpha M_new;   Y^i = R + (alpha / 2) W (R + Y^(i-1)),  i = 1 .. s;   R_new = Y^s
    The iteration is the fixed-point form of the Cayley transform (I - alpha/2 W)^-1 (I + alpha/2 W) R.
    Returns (R_new, M_new, alpha, W)."""
    R = _f64(R)
    Mp = float(beta) * _f64(M) - _f64(G)
    A = Mp @ R.T
    W_hat = A - 0.5 * (R @ (R.T @ A))
    W = W_hat - W_hat.T
    M_new = W @ R
    alpha = min(float(lr), 2.0 * float(q) / (float(np.sqrt(np.sum(W * W))) + float(eps)))
    Y = R + alpha * M_new
    for _ in range(int(s)):
        Y = R + (alpha / 2.0) * (W @ (R + Y))
    return Y, M_new, alpha, W


def cayley_step(X, R, M, lr: float, beta: float = 0.9, reduce: str = "mean", q: float = 0.5, s: int = 2,
                eps: float = 1e-8):
    """One calibration step with the optimiser of Alg. 3 in place of QR-Orth: loss and dL/dR at the INPUT rotation
    (Alg. 1, rotation and loss steps), then the Cayley update of R itself.  Returns a dict like ``calib_step``."""
    loss, G, Y, dY = rotate_loss_grad(X, R, reduce)
    R_new, M_new, alpha, W = cayley_sgd_update(R, G, M, lr, beta, q, s, eps)
    return {"loss": loss, "G": G, "R_new": R_new, "M_new": M_new, "alpha": alpha, "W": W}
