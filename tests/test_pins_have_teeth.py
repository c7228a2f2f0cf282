"""The pins of tests/test_oracle_pins.py must notice a wrong oracle.

Each case below plants one plausible mistake in the oracle module (a dropped term, a wrong sign, a transposed operand, a
missing normalisation, an off-by-one comparison), on the CPU and only for the duration of the case, and requires that
the named pin test then fails.  A pin that still passes against a broken oracle pins nothing.
"""

import numpy as np
import pytest

from oracle import dartqr_oracle as orc
try:                                    # pytest's default import mode puts tests/ itself on the path
    import test_oracle_pins as pins
except ImportError:                     # other import modes: through the repository root
    from tests import test_oracle_pins as pins


def _f64(a):
    return np.array(a, dtype=np.float64, copy=True)


# ---- mutants: the oracle's formula with one mistake each -------------------------------------------------

def whip_grad_wrong_sign(Y, reduce="mean"):
    Y = _f64(Y)
    return orc._reduce_scale(reduce, Y.shape[0]) * np.sign(Y) * np.exp(-np.abs(Y))


def whip_loss_no_abs(Y, reduce="mean"):
    Y = _f64(Y)
    return float(orc._reduce_scale(reduce, Y.shape[0]) * np.sum(np.exp(-Y)))


def rotate_column_convention(X, R):
    return _f64(X) @ _f64(R).T


def grad_wrt_rotation_transposed(X, dY):
    return (_f64(X).T @ _f64(dY)).T


def qr_orth_without_sign_fix(Z):
    return orc.householder_qr(Z)


def qr_backward_not_strict(R, U, G):
    R, U, G = _f64(R), _f64(U), _f64(G)
    B = R.T @ G
    return R @ orc._solve_right_upper_transposed(np.tril(B - B.T, k=0) + np.diag(np.diag(B)), U)


def qr_backward_symmetric_part(R, U, G):
    R, U, G = _f64(R), _f64(U), _f64(G)
    B = R.T @ G
    return R @ orc._solve_right_upper_transposed(np.tril(B + B.T, k=-1), U)


def qr_backward_untransposed_solve(R, U, G):
    R, U, G = _f64(R), _f64(U), _f64(G)
    B = R.T @ G
    return R @ (np.tril(B - B.T, k=-1) @ np.linalg.inv(U))


def solve_with_untransposed_factor(W, U):
    return _f64(W) @ np.linalg.inv(_f64(U))


def sgd_update_ascent(Z, dZ, lr):
    return _f64(Z) + float(lr) * _f64(dZ)


def adam_without_bias_correction(Z, dZ, m, v, step, lr, beta1=0.9, beta2=0.999, eps=1e-8):
    g = _f64(dZ)
    m_new = beta1 * _f64(m) + (1 - beta1) * g
    v_new = beta2 * _f64(v) + (1 - beta2) * g * g
    return _f64(Z) - lr * m_new / (np.sqrt(v_new) + eps), m_new, v_new


def momentum_with_dampening(Z, dZ, buf, lr, mu):
    buf_new = mu * _f64(buf) + (1 - mu) * _f64(dZ)
    return _f64(Z) - lr * buf_new, buf_new


def token_sampling_sorted(X, idx):
    return _ORIG["token_sampling"](X, sorted(int(i) for i in idx))


def outlier_count_inclusive(Y, tau):
    return int(np.sum(np.abs(np.asarray(Y, dtype=np.float64)) >= tau))


def hadamard_without_scale(signs):
    return _ORIG["hadamard_latent"](signs) * np.sqrt(float(len(signs)))


def hadamard_signs_on_columns(signs):
    H = _ORIG["hadamard_latent"](np.ones(len(signs)))
    return H * _f64(signs)[None, :]


def variance_grad_without_mean(Y, reduce="mean"):
    loss, _ = _ORIG["variance_objective"](Y, reduce)
    Y = _f64(Y)
    return loss, orc._reduce_scale(reduce, Y.shape[0]) * (2.0 / Y.shape[1]) * Y


def kurtosis_grad_without_third_moment(Y, reduce="mean"):
    Y = _f64(Y)
    T, n = Y.shape
    c = orc._reduce_scale(reduce, T)
    loss, dY = 0.0, np.zeros_like(Y)
    for t in range(T):
        d = Y[t] - Y[t].mean()
        m2, m4 = np.mean(d ** 2), np.mean(d ** 4)
        if m2 == 0.0:
            continue
        loss += m4 / m2 ** 2
        dY[t] = c * (4.0 / n) * (d ** 3 / m2 ** 2 - m4 * d / m2 ** 3)
    return float(c * loss), dY


def kurtosis_excess(Y, reduce="mean"):
    loss, dY = _ORIG["kurtosis_objective"](Y, reduce)
    Y = _f64(Y)
    return loss - 3.0 * orc._reduce_scale(reduce, Y.shape[0]) * Y.shape[0], dY


def quant_grad_without_range_terms(Y, bits=4, reduce="mean"):
    loss, dY, codes = _ORIG["quant_objective"](Y, bits, reduce)
    Y = np.asarray(Y, dtype=np.float64)
    L = (1 << bits) - 1
    c = orc._reduce_scale(reduce, Y.shape[0])
    out = np.zeros_like(dY)
    for t in range(Y.shape[0]):
        lo, hi = Y[t].min(), Y[t].max()
        if hi > lo:
            out[t] = c * (2.0 / Y.shape[1]) * (Y[t] - (lo + (hi - lo) * codes[t] / L))
    return loss, out, codes


def quant_round_half_up(Y, bits=4, reduce="mean"):
    Y32 = np.asarray(Y, dtype=np.float32)
    T, n = Y32.shape
    L = (1 << bits) - 1
    c = orc._reduce_scale(reduce, T)
    loss, dY, codes = 0.0, np.zeros((T, n)), np.zeros((T, n), dtype=np.int64)
    for t in range(T):
        y = Y32[t].astype(np.float64)
        lo, hi = y.min(), y.max()
        if not hi > lo:
            continue
        q = np.floor((y - lo) / ((hi - lo) / L) + 0.5)
        codes[t] = q.astype(np.int64)
        e = y - (lo + (hi - lo) * q / L)
        loss += np.sum(e * e) / n
    return float(c * loss), dY, codes


def calib_step_reports_updated_loss(X, Z, lr, reduce="mean", objective="whip", bits=4):
    out = _ORIG["calib_step"](X, Z, lr, reduce, objective, bits)
    out["loss"] = _ORIG["calib_step"](X, out["Z_new"], lr, reduce, objective, bits)["loss"]
    return out


def calibrate_batches_off_by_one(X_batches, Z0, steps, lr, reduce="mean"):
    return _ORIG["calibrate_batches"](list(X_batches[1:]) + list(X_batches[:1]), Z0, steps, lr, reduce)


def _cayley_variant(ascent=False, full_projection=False, symmetric=False, full_step_in_iteration=False,
                    momentum_before_projection=False):
    def f(R, G, M, lr, beta=0.9, q=0.5, s=2, eps=1e-8):
        R = _f64(R)
        Mp = float(beta) * _f64(M) + (_f64(G) if ascent else -_f64(G))
        A = Mp @ R.T
        W_hat = A - (1.0 if full_projection else 0.5) * (R @ (R.T @ A))
        W = W_hat + W_hat.T if symmetric else W_hat - W_hat.T
        M_new = Mp if momentum_before_projection else W @ R
        alpha = min(float(lr), 2.0 * float(q) / (float(np.sqrt(np.sum(W * W))) + float(eps)))
        Y = R + alpha * M_new
        for _ in range(int(s)):
            Y = R + (alpha if full_step_in_iteration else alpha / 2.0) * (W @ (R + Y))
        return Y, M_new, alpha, W
    return f


cayley_ascent = _cayley_variant(ascent=True)
cayley_ascent.__name__ = "cayley_ascent"
cayley_full_projection = _cayley_variant(full_projection=True)
cayley_full_projection.__name__ = "cayley_full_projection"
cayley_symmetric = _cayley_variant(symmetric=True)
cayley_symmetric.__name__ = "cayley_symmetric"
cayley_full_step_in_iteration = _cayley_variant(full_step_in_iteration=True)
cayley_full_step_in_iteration.__name__ = "cayley_full_step_in_iteration"
cayley_unprojected_momentum = _cayley_variant(momentum_before_projection=True)
cayley_unprojected_momentum.__name__ = "cayley_unprojected_momentum"


_ORIG = {name: getattr(orc, name) for name in orc.__all__}

CASES = [
    ("whip_grad", whip_grad_wrong_sign, lambda: pins.test_whip_grad_formula_and_finite_differences()),
    ("whip_loss", whip_loss_no_abs, lambda: pins.test_whip_brute_force()),
    ("rotate", rotate_column_convention, lambda: pins.test_rotate_is_row_vector_convention()),
    ("grad_wrt_rotation", grad_wrt_rotation_transposed, lambda: pins.test_grad_wrt_rotation_finite_differences()),
    ("qr_orth", qr_orth_without_sign_fix, lambda: [pins.test_qr_invariants(n) for n in (3, 8, 37)]),
    ("qr_backward", qr_backward_not_strict, lambda: pins.test_dZ_finite_differences_of_whole_map(4, 16, 32)),
    ("qr_backward", qr_backward_symmetric_part, lambda: pins.test_dZ_finite_differences_of_whole_map(4, 16, 32)),
    ("qr_backward", qr_backward_untransposed_solve, lambda: pins.test_dZ_structural_identities()),
    ("_solve_right_upper_transposed", solve_with_untransposed_factor,
     lambda: pins.test_triangular_solve_helper_against_library()),
    ("sgd_update", sgd_update_ascent, lambda: pins.test_sgd_step_norm_identity_and_update()),
    ("adam_update", adam_without_bias_correction, lambda: pins.test_adam_first_step_closed_form()),
    ("sgd_momentum_update", momentum_with_dampening, lambda: pins.test_momentum_zero_is_plain_sgd_and_geometric_sum()),
    ("token_sampling", token_sampling_sorted, lambda: pins.test_token_sampling_invariants()),
    ("outlier_count", outlier_count_inclusive, lambda: pins.test_outlier_count_pins()),
    ("hadamard_latent", hadamard_without_scale, lambda: pins.test_hadamard_latent_pins()),
    ("hadamard_latent", hadamard_signs_on_columns, lambda: pins.test_hadamard_latent_pins()),
    ("variance_objective", variance_grad_without_mean, lambda: pins.test_variance_objective_pins()),
    ("kurtosis_objective", kurtosis_grad_without_third_moment, lambda: pins.test_kurtosis_objective_pins()),
    ("kurtosis_objective", kurtosis_excess, lambda: pins.test_kurtosis_objective_pins()),
    ("quant_objective", quant_grad_without_range_terms, lambda: pins.test_quant_objective_pins(4)),
    ("quant_objective", quant_round_half_up, lambda: pins.test_quant_objective_closed_forms()),
    ("calib_step", calib_step_reports_updated_loss,
     lambda: pins.test_calibration_loop_decreases_loss_and_reports_input_loss()),
    ("calibrate_batches", calibrate_batches_off_by_one, lambda: pins.test_calibrate_batches_pins()),
    ("cayley_sgd_update", cayley_ascent, lambda: pins.test_cayley_update_descent_identities()),
    ("cayley_sgd_update", cayley_full_projection, lambda: pins.test_cayley_update_descent_identities()),
    ("cayley_sgd_update", cayley_symmetric,
     lambda: pins.test_cayley_update_is_the_cayley_transform_up_to_the_contraction_bound()),
    ("cayley_sgd_update", cayley_full_step_in_iteration,
     lambda: pins.test_cayley_update_is_the_cayley_transform_up_to_the_contraction_bound()),
    ("cayley_sgd_update", cayley_unprojected_momentum, lambda: pins.test_cayley_update_descent_identities()),
]


@pytest.mark.parametrize("name,mutant,pin", CASES, ids=[f"{c[0]}:{c[1].__name__}" for c in CASES])
def test_pin_fails_on_planted_mistake(monkeypatch, name, mutant, pin):
    pin()                                           # the pin passes on the oracle as it stands
    monkeypatch.setattr(orc, name, mutant)
    with pytest.raises((AssertionError, ValueError, ZeroDivisionError, FloatingPointError)):
        pin()
