"""Pins for the CPU oracle: it is checked against what the paper and the mathematics fix,
never against itself.  Every test here runs on the CPU in fp64.

Citations: Eq. 4 (Whip), Alg. 1 (calibration loop), Sec. 4.3 (Z = R U), Alg. 2
(Householder QR), the norm-invariance equation in the appendix on the Whip mechanism.
"""

import math

import numpy as np
import pytest

from oracle import dartqr_oracle as orc


def rng(seed):
    return np.random.Generator(np.random.Philox(seed))


# ----------------------------------------------------------------------------------
# QR-Orth: Z -> (R, U)
# ----------------------------------------------------------------------------------

def mgs_reorth(Z):
    """Independent route: modified Gram-Schmidt with one re-orthogonalisation pass.
    For nonsingular Z the factorisation with diag(U) > 0 is unique."""
    Z = np.asarray(Z, dtype=np.float64)
    n = Z.shape[0]
    Q = np.zeros((n, n))
    U = np.zeros((n, n))
    for j in range(n):
        v = Z[:, j].copy()
        for _pass in range(2):
            for i in range(j):
                h = Q[:, i] @ v
                v -= h * Q[:, i]
                U[i, j] += h
        U[j, j] = math.sqrt(v @ v)
        Q[:, j] = v / U[j, j]
    return Q, U


@pytest.mark.parametrize("n", [1, 2, 3, 8, 37, 96])
def test_qr_invariants(n):
    Z = rng(100 + n).standard_normal((n, n))
    R, U = orc.qr_orth(Z)
    assert np.max(np.abs(R.T @ R - np.eye(n))) < 1e-12
    assert np.max(np.abs(R @ R.T - np.eye(n))) < 1e-12
    assert np.max(np.abs(R @ U - Z)) < 1e-12 * max(1.0, np.abs(Z).max()) * n
    assert np.all(np.tril(U, -1) == 0.0)
    assert np.all(np.diag(U) > 0.0)


@pytest.mark.parametrize("n", [2, 5, 33, 64])
def test_qr_matches_gram_schmidt_route(n):
    Z = rng(200 + n).standard_normal((n, n))
    R, U = orc.qr_orth(Z)
    Q2, U2 = mgs_reorth(Z)
    assert np.max(np.abs(R - Q2)) < 1e-10
    assert np.max(np.abs(U - U2)) < 1e-10


@pytest.mark.parametrize("n", [4, 50])
def test_qr_matches_lapack_after_sign_fix(n):
    Z = rng(300 + n).standard_normal((n, n))
    R, U = orc.qr_orth(Z)
    Ql, Ul = np.linalg.qr(Z)
    s = np.sign(np.diag(Ul))
    assert np.max(np.abs(R - Ql * s[None, :])) < 1e-11
    assert np.max(np.abs(U - Ul * s[:, None])) < 1e-11


def test_householder_unnormalised_factors():
    Z = rng(7).standard_normal((20, 20))
    Q, U0 = orc.householder_qr(Z)
    assert np.max(np.abs(Q.T @ Q - np.eye(20))) < 1e-12
    assert np.max(np.abs(Q @ U0 - Z)) < 1e-12
    assert np.all(np.tril(U0, -1) == 0.0)


def _random_orthogonal(n, seed):
    # product of Givens rotations and a signed permutation: orthogonal by construction
    g = rng(seed)
    Q = np.eye(n)
    for _ in range(4 * n):
        i, j = g.choice(n, size=2, replace=False)
        th = g.uniform(0, 2 * math.pi)
        c, s = math.cos(th), math.sin(th)
        Gm = np.eye(n)
        Gm[i, i], Gm[j, j], Gm[i, j], Gm[j, i] = c, c, -s, s
        Q = Q @ Gm
    P = np.eye(n)[g.permutation(n)] * g.choice([-1.0, 1.0], size=n)[None, :]
    return Q @ P


def test_qr_closed_form_orthogonal_input():
    Zo = _random_orthogonal(12, 1)
    R, U = orc.qr_orth(Zo)
    assert np.max(np.abs(R - Zo)) < 1e-13
    assert np.max(np.abs(U - np.eye(12))) < 1e-13


def test_qr_closed_form_hadamard_input():
    # Sylvester Hadamard matrix / sqrt(n): the paper's initial latent is a Hadamard matrix
    H = np.array([[1.0]])
    for _ in range(4):
        H = np.block([[H, H], [H, -H]])
    H /= 4.0
    R, U = orc.qr_orth(H)
    assert np.max(np.abs(R - H)) < 1e-14
    assert np.max(np.abs(U - np.eye(16))) < 1e-14


def test_qr_closed_form_upper_triangular_input():
    g = rng(2)
    Zt = np.triu(g.standard_normal((9, 9)))
    Zt[np.arange(9), np.arange(9)] = np.abs(np.diag(Zt)) + 0.5
    R, U = orc.qr_orth(Zt)
    assert np.max(np.abs(R - np.eye(9))) < 1e-13
    assert np.max(np.abs(U - Zt)) < 1e-13


def test_qr_closed_form_diagonal_input():
    d = np.array([3.0, -2.0, 0.5, -7.0, 1.0])
    R, U = orc.qr_orth(np.diag(d))
    assert np.array_equal(R, np.diag(np.sign(d)))
    assert np.max(np.abs(U - np.diag(np.abs(d)))) < 1e-15


@pytest.mark.parametrize("z", [2.5, -0.3])
def test_qr_closed_form_n1(z):
    R, U = orc.qr_orth(np.array([[z]]))
    assert R[0, 0] == math.copysign(1.0, z)
    assert abs(U[0, 0] - abs(z)) < 1e-15


@pytest.mark.parametrize("Z", [np.array([[1.0, 2.0], [3.0, 4.0]]),
                               np.array([[-1.0, 0.5], [2.0, 3.0]]),
                               np.array([[0.3, -2.0], [-0.4, -0.1]])])
def test_qr_closed_form_n2(Z):
    a, c = Z[0, 0], Z[1, 0]
    r = math.hypot(a, c)
    s = math.copysign(1.0, np.linalg.det(Z))
    R_expected = np.array([[a / r, -s * c / r], [c / r, s * a / r]])
    R, U = orc.qr_orth(Z)
    assert np.max(np.abs(R - R_expected)) < 1e-14
    assert np.max(np.abs(R_expected.T @ Z - U)) < 1e-14


# ----------------------------------------------------------------------------------
# rotate
# ----------------------------------------------------------------------------------

def test_rotate_preserves_norms_and_identity():
    g = rng(11)
    X = g.standard_t(3.0, size=(40, 16))
    R, _ = orc.qr_orth(g.standard_normal((16, 16)))
    Y = orc.rotate(X, R)
    # norm invariance of a rotation (appendix, norm equation)
    assert np.max(np.abs(np.sum(Y * Y, axis=1) - np.sum(X * X, axis=1))) < 1e-10 * np.sum(X * X, axis=1).max()
    assert abs(np.linalg.norm(Y) - np.linalg.norm(X)) < 1e-11 * np.linalg.norm(X)
    assert np.array_equal(orc.rotate(X, np.eye(16)), X)


def test_rotate_is_row_vector_convention():
    # Y[t, i] = sum_c X[t, c] R[c, i]  (O = X @ R, the rotation step of Alg. 1), written as loops
    g = rng(12)
    X = g.standard_normal((3, 4))
    R = g.standard_normal((4, 4))
    Y = orc.rotate(X, R)
    for t in range(3):
        for i in range(4):
            acc = 0.0
            for c in range(4):
                acc += X[t, c] * R[c, i]
            assert abs(Y[t, i] - acc) < 1e-14


# ----------------------------------------------------------------------------------
# Whip loss (Eq. 4) and its gradient
# ----------------------------------------------------------------------------------

def brute_whip(Y, mean):
    total = 0.0
    for t in range(Y.shape[0]):
        per_token = 0.0
        for i in range(Y.shape[1]):
            per_token += math.exp(-abs(float(Y[t, i])))
        total += per_token
    return total / Y.shape[0] if mean else total


def test_whip_brute_force():
    Y = rng(21).standard_t(3.0, size=(13, 7)) * 2.0
    assert abs(orc.whip_loss(Y, "mean") - brute_whip(Y, True)) < 1e-13
    assert abs(orc.whip_loss(Y, "sum") - brute_whip(Y, False)) < 1e-12


def test_whip_closed_forms():
    n, T = 6, 5
    assert orc.whip_loss(np.zeros((T, n)), "mean") == pytest.approx(n, abs=1e-15)
    assert orc.whip_loss(np.zeros((T, n)), "sum") == pytest.approx(n * T, abs=1e-15)
    a = -1.7
    Y = np.zeros((1, n))
    Y[0, 0] = a
    assert orc.whip_loss(Y, "mean") == pytest.approx(math.exp(-abs(a)) + n - 1, abs=1e-15)
    # a single vector: Eq. 4 itself
    x = np.array([[0.5, -2.0, 3.0]])
    assert orc.whip_loss(x, "sum") == pytest.approx(math.exp(-0.5) + math.exp(-2.0) + math.exp(-3.0), abs=1e-15)


def test_whip_invariant_under_signed_permutation_of_rotation_columns():
    g = rng(22)
    X = g.standard_normal((30, 8))
    R, _ = orc.qr_orth(g.standard_normal((8, 8)))
    perm = g.permutation(8)
    signs = g.choice([-1.0, 1.0], size=8)
    R2 = R[:, perm] * signs[None, :]
    assert abs(orc.whip_loss(orc.rotate(X, R)) - orc.whip_loss(orc.rotate(X, R2))) < 1e-13


def test_whip_grad_formula_and_finite_differences():
    Y = rng(23).standard_normal((5, 4)) * 1.5
    Y[2, 1] = 0.0
    for mode, c in (("mean", 1.0 / 5), ("sum", 1.0)):
        dY = orc.whip_grad(Y, mode)
        assert dY[2, 1] == 0.0                       # reading: sgn(0) = 0
        h = 1e-6
        for t in range(5):
            for i in range(4):
                if Y[t, i] == 0.0:
                    continue
                # closed form: -c * sgn(y) * exp(-|y|): pushes small |y| away from zero
                assert dY[t, i] == pytest.approx(-c * math.copysign(1.0, Y[t, i]) * math.exp(-abs(Y[t, i])), abs=1e-15)
                Yp, Ym = Y.copy(), Y.copy()
                Yp[t, i] += h
                Ym[t, i] -= h
                fd = (orc.whip_loss(Yp, mode) - orc.whip_loss(Ym, mode)) / (2 * h)
                assert abs(fd - dY[t, i]) < 1e-8


def test_grad_wrt_rotation_finite_differences():
    g = rng(24)
    T, n = 12, 5
    X = g.standard_t(3.0, size=(T, n))
    R = g.standard_normal((n, n))          # entries treated as free variables
    loss, G, Y, dY = orc.rotate_loss_grad(X, R)
    assert loss == pytest.approx(brute_whip(X @ R, True), abs=1e-13)
    h = 1e-6
    for i in range(n):
        for j in range(n):
            Rp, Rm = R.copy(), R.copy()
            Rp[i, j] += h
            Rm[i, j] -= h
            fd = (orc.whip_loss(X @ Rp) - orc.whip_loss(X @ Rm)) / (2 * h)
            assert abs(fd - G[i, j]) < 2e-8 * max(1.0, abs(G[i, j]))


# ----------------------------------------------------------------------------------
# QR backward: dL/dZ
# ----------------------------------------------------------------------------------

def loss_of_Z(X, Z, mode="mean"):
    R, _ = orc.qr_orth(Z)
    return orc.whip_loss(orc.rotate(X, R), mode)


@pytest.mark.parametrize("n,T,seed", [(2, 9, 31), (4, 16, 32), (7, 20, 33)])
def test_dZ_finite_differences_of_whole_map(n, T, seed):
    g = rng(seed)
    X = g.standard_t(3.0, size=(T, n))
    Z = g.standard_normal((n, n))
    out = orc.calib_step(X, Z, lr=0.0)
    dZ = out["dZ"]
    h = 1e-6
    fd = np.zeros((n, n))
    for i in range(n):
        for j in range(n):
            Zp, Zm = Z.copy(), Z.copy()
            Zp[i, j] += h
            Zm[i, j] -= h
            fd[i, j] = (loss_of_Z(X, Zp) - loss_of_Z(X, Zm)) / (2 * h)
    assert np.max(np.abs(fd - dZ)) < 5e-8 * max(1.0, np.abs(dZ).max())


def test_dZ_structural_identities():
    g = rng(34)
    n, T = 24, 60
    X = g.standard_t(3.0, size=(T, n))
    Z = g.standard_normal((n, n))
    out = orc.calib_step(X, Z, lr=0.0)
    dZ = out["dZ"]
    scale = np.linalg.norm(Z) * np.linalg.norm(dZ)
    # Z -> Z (I + eps*Tu), Tu upper triangular, leaves R unchanged: triu(Z^T dZ) = 0
    assert np.max(np.abs(np.triu(Z.T @ dZ))) < 1e-12 * scale
    # scale invariance L(cZ) = L(Z): <Z, dZ> = 0
    assert abs(np.sum(Z * dZ)) < 1e-12 * scale
    # the last column of Z only fixes U[:, n-1]: its gradient vanishes
    assert np.max(np.abs(dZ[:, -1])) < 1e-13 * np.abs(dZ).max()
    # column j of dZ is orthogonal to columns 0..j of Z
    for j in range(n):
        assert np.max(np.abs(Z[:, : j + 1].T @ dZ[:, j])) < 1e-11 * scale


def test_dZ_n1_is_zero():
    X = rng(35).standard_normal((5, 1))
    out = orc.calib_step(X, np.array([[-0.7]]), lr=0.0)
    assert out["dZ"][0, 0] == 0.0


@pytest.mark.parametrize("Z", [np.array([[1.0, 2.0], [3.0, 4.0]]), np.array([[-1.5, 0.5], [0.7, 3.0]])])
def test_dZ_closed_form_n2_angle_parametrisation(Z):
    # R = [[cos, -s sin], [sin, s cos]], theta = atan2(c, a), s = sign(det Z).
    X = rng(36).standard_t(3.0, size=(11, 2))
    T = X.shape[0]
    a, c = Z[0, 0], Z[1, 0]
    r2 = a * a + c * c
    th = math.atan2(c, a)
    s = math.copysign(1.0, np.linalg.det(Z))
    dL_dth = 0.0
    for t in range(T):
        y1 = X[t, 0] * math.cos(th) + X[t, 1] * math.sin(th)
        y2 = s * (-X[t, 0] * math.sin(th) + X[t, 1] * math.cos(th))
        dy1 = -X[t, 0] * math.sin(th) + X[t, 1] * math.cos(th)
        dy2 = s * (-X[t, 0] * math.cos(th) - X[t, 1] * math.sin(th))
        dL_dth += -math.copysign(1.0, y1) * math.exp(-abs(y1)) * dy1
        dL_dth += -math.copysign(1.0, y2) * math.exp(-abs(y2)) * dy2
    dL_dth /= T
    expected = np.array([[-c / r2 * dL_dth, 0.0], [a / r2 * dL_dth, 0.0]])
    dZ = orc.calib_step(X, Z, lr=0.0)["dZ"]
    assert np.max(np.abs(dZ - expected)) < 1e-13


def test_dZ_matches_library_autograd_route():
    torch = pytest.importorskip("torch")
    g = rng(37)
    n, T = 10, 40
    X = g.standard_t(3.0, size=(T, n))
    Z = g.standard_normal((n, n))
    Zt = torch.tensor(Z, dtype=torch.float64, requires_grad=True)
    Q, Rt = torch.linalg.qr(Zt)
    Y = torch.tensor(X, dtype=torch.float64) @ Q
    L = torch.exp(-Y.abs()).sum() / T
    L.backward()
    out = orc.calib_step(X, Z, lr=0.0)
    assert abs(out["loss"] - L.item()) < 1e-13
    assert np.max(np.abs(out["dZ"] - Zt.grad.numpy())) < 1e-12


def test_qr_backward_rejects_singular():
    Z = np.array([[1.0, 2.0], [2.0, 4.0]])
    R, U = orc.qr_orth(Z)
    U[1, 1] = 0.0
    with pytest.raises(ZeroDivisionError):
        orc.qr_backward(R, U, np.ones((2, 2)))


def test_triangular_solve_helper_against_library():
    g = rng(38)
    U = np.triu(g.standard_normal((9, 9))) + 3 * np.eye(9)
    W = g.standard_normal((6, 9))
    M = orc._solve_right_upper_transposed(W, U)
    assert np.max(np.abs(M @ U.T - W)) < 1e-12
    assert np.max(np.abs(M - np.linalg.solve(U, W.T).T)) < 1e-12


# ----------------------------------------------------------------------------------
# SGD step and the loop
# ----------------------------------------------------------------------------------

def test_sgd_step_norm_identity_and_update():
    g = rng(41)
    n, T = 16, 64
    X = g.standard_t(3.0, size=(T, n))
    Z = g.standard_normal((n, n))
    lr = 0.05
    out = orc.calib_step(X, Z, lr)
    assert np.array_equal(out["Z_new"], Z - lr * out["dZ"])
    lhs = np.linalg.norm(out["Z_new"]) ** 2
    rhs = np.linalg.norm(Z) ** 2 + lr ** 2 * np.linalg.norm(out["dZ"]) ** 2
    assert abs(lhs - rhs) < 1e-11 * rhs


def test_calibration_loop_decreases_loss_and_reports_input_loss():
    g = rng(42)
    n, T = 16, 256
    X = g.standard_normal((T, n))
    X[:, [3, 9]] *= 30.0
    Z0 = g.standard_normal((n, n))
    losses, Zf, Rf = orc.calibrate(X, Z0, steps=8, lr=0.001)
    assert len(losses) == 8
    assert losses[0] == pytest.approx(loss_of_Z(X, Z0), abs=1e-14)
    assert np.all(np.diff(losses) < 0.0)          # small step: monotone decrease
    assert np.max(np.abs(Rf.T @ Rf - np.eye(n))) < 1e-12
    assert np.max(np.abs(Rf - orc.qr_orth(Zf)[0])) == 0.0


def test_loss_independent_of_qr_sign_convention():
    g = rng(43)
    n, T = 9, 30
    X = g.standard_t(3.0, size=(T, n))
    Z = g.standard_normal((n, n))
    Q, U0 = orc.householder_qr(Z)            # raw signs
    R, U = orc.qr_orth(Z)                    # normalised signs
    l_raw, G_raw, _, _ = orc.rotate_loss_grad(X, Q)
    l_nrm, G_nrm, _, _ = orc.rotate_loss_grad(X, R)
    assert abs(l_raw - l_nrm) < 1e-13
    dZ_raw = orc.qr_backward(Q, U0, G_raw)
    dZ_nrm = orc.qr_backward(R, U, G_nrm)
    assert np.max(np.abs(dZ_raw - dZ_nrm)) < 1e-12


# ----------------------------------------------------------------------------------- optimisers other than plain SGD
# (Sec. 4.3 / Table 4: the latent may be driven by SGD or Adam; the rules themselves are the standard ones)


def test_adam_first_step_closed_form():
    # from m = v = 0 the bias-corrected moments are g and g^2: the first update is lr * g / (|g| + eps)
    g = rng(900).standard_normal((6, 6))
    Z = rng(901).standard_normal((6, 6))
    Zn, m, v = orc.adam_update(Z, g, np.zeros_like(Z), np.zeros_like(Z), 1, 0.01, 0.9, 0.999, 1e-8)
    assert np.allclose(Zn, Z - 0.01 * g / (np.abs(g) + 1e-8), rtol=1e-13, atol=0)
    assert np.allclose(m, 0.1 * g) and np.allclose(v, 0.001 * g * g)


def test_adam_constant_gradient_walks_at_unit_speed():
    # with a constant gradient and eps = 0 every bias-corrected step is exactly lr * sign(g)
    g = rng(902).standard_normal((5, 5))
    Z = np.zeros((5, 5)); m = np.zeros_like(Z); v = np.zeros_like(Z)
    for t in range(1, 8):
        Z, m, v = orc.adam_update(Z, g, m, v, t, 0.05, 0.9, 0.999, 0.0)
    assert np.allclose(Z, -7 * 0.05 * np.sign(g), rtol=1e-12, atol=0)


def test_adam_is_invariant_to_gradient_scale():
    g1 = rng(903).standard_normal((4, 4)); g2 = rng(904).standard_normal((4, 4))
    def run(c):
        Z = np.ones((4, 4)); m = np.zeros_like(Z); v = np.zeros_like(Z)
        for t, g in enumerate((g1, g2, g1), start=1):
            Z, m, v = orc.adam_update(Z, c * g, m, v, t, 0.01, 0.9, 0.999, 0.0)
        return Z
    assert np.allclose(run(1.0), run(37.5), rtol=1e-12, atol=1e-15)


def test_adam_matches_library_optimiser():
    torch = pytest.importorskip("torch")
    gs = [rng(910 + i).standard_normal((5, 3)) for i in range(6)]
    Z0 = rng(920).standard_normal((5, 3))
    p = torch.nn.Parameter(torch.tensor(Z0, dtype=torch.float64))
    opt = torch.optim.Adam([p], lr=0.02, betas=(0.8, 0.95), eps=1e-6)
    Z = Z0.copy(); m = np.zeros_like(Z); v = np.zeros_like(Z)
    for t, g in enumerate(gs, start=1):
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        Z, m, v = orc.adam_update(Z, g, m, v, t, 0.02, 0.8, 0.95, 1e-6)
        assert np.allclose(Z, p.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_adam_rejects_step_zero():
    with pytest.raises(ValueError):
        orc.adam_update(np.zeros((2, 2)), np.zeros((2, 2)), np.zeros((2, 2)), np.zeros((2, 2)), 0, 0.1)


def test_momentum_zero_is_plain_sgd_and_geometric_sum():
    g = rng(930).standard_normal((4, 4)); Z = rng(931).standard_normal((4, 4))
    Zn, buf = orc.sgd_momentum_update(Z, g, np.zeros_like(Z), 0.1, 0.0)
    assert np.array_equal(Zn, orc.sgd_update(Z, g, 0.1)) and np.array_equal(buf, g)
    # constant gradient: buf_k = g (1 - mu^k) / (1 - mu)
    mu = 0.8; buf = np.zeros_like(Z); Zk = Z.copy(); total = np.zeros_like(Z)
    for k in range(1, 6):
        Zk, buf = orc.sgd_momentum_update(Zk, g, buf, 0.1, mu)
        assert np.allclose(buf, g * (1 - mu ** k) / (1 - mu), rtol=1e-13)
        total += buf
    assert np.allclose(Zk, Z - 0.1 * total, rtol=1e-13)


def test_momentum_matches_library_optimiser():
    torch = pytest.importorskip("torch")
    gs = [rng(940 + i).standard_normal((3, 4)) for i in range(5)]
    Z0 = rng(950).standard_normal((3, 4))
    p = torch.nn.Parameter(torch.tensor(Z0, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=0.05, momentum=0.9)
    Z = Z0.copy(); buf = np.zeros_like(Z)
    for g in gs:
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        Z, buf = orc.sgd_momentum_update(Z, g, buf, 0.05, 0.9)
        assert np.allclose(Z, p.detach().numpy(), rtol=1e-13, atol=1e-15)


def test_calib_step_adam_composes_the_pieces():
    n, T = 12, 40
    X = rng(960).standard_normal((T, n)); Z = rng(961).standard_normal((n, n))
    m = 0.01 * rng(962).standard_normal((n, n)); v = np.abs(rng(963).standard_normal((n, n))) * 1e-4
    out = orc.calib_step_adam(X, Z, m, v, 3, 0.01)
    ref = orc.calib_step(X, Z, 0.0)
    assert np.array_equal(out["dZ"], ref["dZ"]) and out["loss"] == ref["loss"]
    Zn, mn, vn = orc.adam_update(Z, ref["dZ"], m, v, 3, 0.01)
    assert np.array_equal(out["Z_new"], Zn) and np.array_equal(out["m"], mn) and np.array_equal(out["v"], vn)


# ----------------------------------------------------------------------------------- token sampling (Alg. 1)
def test_token_sampling_invariants():
    g = np.random.Generator(np.random.Philox(901))
    T, n = 57, 12
    X = g.standard_normal((T, n))
    R, _ = orc.qr_orth(g.standard_normal((n, n)))
    idx = g.integers(0, T, 23)
    Xs = orc.token_sampling(X, idx)
    assert Xs.shape == (23, n) and Xs.dtype == X.dtype
    # the rows are the named ones, bit for bit, repeats included
    assert all(np.array_equal(Xs[t], X[idx[t]]) for t in range(23))
    assert np.array_equal(orc.token_sampling(X, np.arange(T)), X)
    assert np.array_equal(orc.token_sampling(X, np.arange(T)[::-1]), X[::-1])
    # selecting rows commutes with everything the loop does row by row: the rotation ...
    assert np.array_equal(orc.rotate(Xs, R), orc.token_sampling(orc.rotate(X, R), idx))
    # ... and the summed loss of the sample is the sum of the per-token Whip values of the chosen tokens
    per_token = np.array([orc.whip_loss(orc.rotate(X[t:t + 1], R), "sum") for t in range(T)])
    assert orc.whip_loss(orc.rotate(Xs, R), "sum") == pytest.approx(per_token[idx].sum(), rel=1e-14)
    # a full permutation leaves the mean loss and G = X^T dY unchanged
    perm = g.permutation(T)
    l0, G0, _, _ = orc.rotate_loss_grad(X, R)
    l1, G1, _, _ = orc.rotate_loss_grad(orc.token_sampling(X, perm), R)
    assert l1 == pytest.approx(l0, rel=1e-14) and np.allclose(G1, G0, rtol=0, atol=1e-14)
    with pytest.raises(IndexError):
        orc.token_sampling(X, [0, T])
    with pytest.raises(IndexError):
        orc.token_sampling(X, [-1])


# ----------------------------------------------------------------------------------- outlier count (Sec. 4.1, Eq. 1)
def test_outlier_count_pins():
    g = np.random.Generator(np.random.Philox(902))
    Y = g.standard_normal((37, 11))
    # hand-made case
    assert orc.outlier_count(np.array([[0.0, -3.0, 2.0], [2.5, -2.5, 7.0]]), 2.5) == 2      # strictly greater
    # against the vectorised definition, and its elementary properties
    for tau in (0.0, 0.5, 1.0, 2.0, 10.0):
        assert orc.outlier_count(Y, tau) == int(np.sum(np.abs(Y) > tau))
    assert orc.outlier_count(Y, 0.0) == Y.size
    assert orc.outlier_count(Y, np.abs(Y).max()) == 0
    counts = [orc.outlier_count(Y, t) for t in (0.1, 0.5, 1.0, 2.0)]
    assert counts == sorted(counts, reverse=True)
    assert orc.outlier_count(-Y[::-1, ::-1], 1.0) == orc.outlier_count(Y, 1.0)
    # a per-token sum: the count of a block is the sum of the counts of its rows
    assert orc.outlier_count(Y, 1.0) == sum(orc.outlier_count(Y[t], 1.0) for t in range(Y.shape[0]))
    # the reason the paper rotates at all: a vector with one massive entry has an outlier, its image under a
    # rotation that spreads it evenly (a normalised Hadamard matrix) has none at the same threshold
    H = np.array([[1.0]])
    for _ in range(3):
        H = np.block([[H, H], [H, -H]])
    H /= np.sqrt(8.0)
    x = np.zeros((1, 8)); x[0, 3] = 8.0
    assert orc.outlier_count(x, 3.0) == 1 and orc.outlier_count(orc.rotate(x, H), 3.0) == 0


# ----------------------------------------------------------------------------------- Hadamard initial latent
def test_hadamard_latent_pins():
    g = np.random.Generator(np.random.Philox(903))
    for n in (1, 2, 8, 64):
        s = g.choice([-1.0, 1.0], n)
        Z = orc.hadamard_latent(s)
        assert Z.shape == (n, n)
        assert np.allclose(Z.T @ Z, np.eye(n), atol=1e-14) and np.allclose(Z @ Z.T, np.eye(n), atol=1e-14)
        assert np.allclose(np.abs(Z), 1.0 / np.sqrt(n), rtol=1e-15)
        # entries by the bit-count form, H[r][c] = (-1)^popcount(r & c)
        r, c = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
        par = np.array([[bin(int(a) & int(b)).count("1") & 1 for b in range(n)] for a in range(n)])
        assert np.array_equal(np.sign(Z), s[:, None] * np.where(par == 1, -1.0, 1.0))
        # Kronecker power of H_2
        K = np.array([[1.0]])
        for _ in range(int(np.log2(n))):
            K = np.kron(np.array([[1.0, 1.0], [1.0, -1.0]]), K)
        assert np.allclose(Z, s[:, None] * K / np.sqrt(n), rtol=1e-15)
    # an orthogonal latent is its own rotation up to the sign normalisation: R = Z diag(sign of the first ... ) and U = I
    Z = orc.hadamard_latent(g.choice([-1.0, 1.0], 16))
    R, U = orc.qr_orth(Z)
    assert np.allclose(U, np.eye(16), atol=1e-13) and np.allclose(R, Z, atol=1e-13)
    with pytest.raises(ValueError):
        orc.hadamard_latent(np.ones(12))


# ------------------------------------------------------------------------------------------------
# Alternative objectives (Sec. 4.1 and the objective ablation of Sec. 5 name them, no formulas printed)

def _fd_grad(f, Y, h=1e-6):
    g = np.zeros_like(Y)
    for idx in np.ndindex(*Y.shape):
        Yp, Ym = Y.copy(), Y.copy()
        Yp[idx] += h
        Ym[idx] -= h
        g[idx] = (f(Yp) - f(Ym)) / (2 * h)
    return g


def test_variance_objective_pins():
    rng = np.random.default_rng(301)
    Y = rng.standard_normal((5, 12)) * rng.uniform(0.5, 3.0, (5, 1)) + rng.standard_normal((5, 1))
    for reduce, c in (("mean", 1.0 / 5), ("sum", 1.0)):
        loss, dY = orc.variance_objective(Y, reduce)
        # library route: numpy's population variance, row by row
        assert loss == pytest.approx(c * sum(np.var(Y[t]) for t in range(5)), rel=1e-13)
        np.testing.assert_allclose(dY, _fd_grad(lambda A: orc.variance_objective(A, reduce)[0], Y), atol=1e-8)
        # shifting a row changes nothing: the gradient of every row sums to zero
        np.testing.assert_allclose(dY.sum(axis=1), 0.0, atol=1e-14)
    # n * (variance + mean^2) of a row is its squared norm, which no rotation changes (the paper's reason for
    # rejecting the objective, Sec. 4.1)
    X = rng.standard_normal((7, 16))
    Q, _ = np.linalg.qr(rng.standard_normal((16, 16)))
    for A in (X, X @ Q):
        loss, _ = orc.variance_objective(A, "sum")
        mu = A.mean(axis=1)
        assert 16 * (loss + np.sum(mu * mu)) == pytest.approx(np.sum(X * X), rel=1e-12)
    # closed form: the row (0, 2) has mean 1 and variance 1
    assert orc.variance_objective(np.array([[0.0, 2.0]]), "sum")[0] == pytest.approx(1.0)
    assert orc.variance_objective(np.full((2, 6), 3.5), "sum")[0] == 0.0


def test_kurtosis_objective_pins():
    from scipy import stats
    rng = np.random.default_rng(302)
    Y = rng.standard_t(4.0, size=(4, 20)) + rng.standard_normal((4, 1))
    for reduce, c in (("mean", 0.25), ("sum", 1.0)):
        loss, dY = orc.kurtosis_objective(Y, reduce)
        assert loss == pytest.approx(c * sum(stats.kurtosis(Y[t], fisher=False, bias=True) for t in range(4)), rel=1e-12)
        np.testing.assert_allclose(dY, _fd_grad(lambda A: orc.kurtosis_objective(A, reduce)[0], Y), atol=2e-7)
        # kurtosis ignores shift and scale of a row: the gradient is orthogonal to 1 and to the row itself
        np.testing.assert_allclose(dY.sum(axis=1), 0.0, atol=1e-13)
        np.testing.assert_allclose(np.sum(dY * Y, axis=1), 0.0, atol=1e-12)
    a, b = orc.kurtosis_objective(Y, "sum")[0], orc.kurtosis_objective(-3.0 * Y + 7.0, "sum")[0]
    assert a == pytest.approx(b, rel=1e-12)
    # closed forms: two equally likely values -> 1; a large Gaussian sample -> 3; uniform grid -> 9/5 in the limit
    assert orc.kurtosis_objective(np.array([[1.0, -1.0, 1.0, -1.0]]), "sum")[0] == pytest.approx(1.0)
    big = np.random.default_rng(5).standard_normal((1, 400000))
    assert orc.kurtosis_objective(big, "sum")[0] == pytest.approx(3.0, abs=0.03)
    grid = np.linspace(-1, 1, 20001)[None, :]
    assert orc.kurtosis_objective(grid, "sum")[0] == pytest.approx(1.8, abs=1e-3)
    # two values always give 1 and three values always 3/2, so their gradients vanish
    for k, val in ((2, 1.0), (3, 1.5)):
        loss, dY = orc.kurtosis_objective(rng.standard_normal((5, k)) * 3.0 + 1.0, "sum")
        assert loss == pytest.approx(5 * val, rel=1e-12) and np.abs(dY).max() < 1e-12
    # a constant row counts as zero and gets no gradient
    loss, dY = orc.kurtosis_objective(np.vstack([np.full(6, 2.0), Y[0, :6]]), "sum")
    assert loss == pytest.approx(stats.kurtosis(Y[0, :6], fisher=False)) and not dY[0].any()


def _nearest_level_error(y, bits):
    """Brute force: squared distance of every value to the nearest of the 2^bits levels between min and max."""
    y = y.astype(np.float64)
    lo, hi = y.min(), y.max()
    lev = lo + (hi - lo) * np.arange(1 << bits) / ((1 << bits) - 1)
    return np.min((y[:, None] - lev[None, :]) ** 2, axis=1)


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_quant_objective_pins(bits):
    rng = np.random.default_rng(303 + bits)
    Y = (rng.standard_t(3.0, size=(6, 40)) * 2.0).astype(np.float32)
    L = (1 << bits) - 1
    loss, dY, codes = orc.quant_objective(Y, bits, "sum")
    assert codes.min() == 0 and codes.max() == L
    # every code is the nearest level (brute force over all levels)
    ref = sum(_nearest_level_error(Y[t], bits).sum() / 40 for t in range(6))
    assert loss == pytest.approx(ref, rel=1e-12)
    # error bound of a uniform quantiser: |e| <= delta / 2
    for t in range(6):
        y = Y[t].astype(np.float64)
        delta = (y.max() - y.min()) / L
        e = y - (y.min() + delta * codes[t])
        assert np.max(np.abs(e)) <= delta / 2 * (1 + 1e-12)
        assert codes[t][np.argmin(y)] == 0 and codes[t][np.argmax(y)] == L
    # mean over tokens is the sum divided by T
    assert orc.quant_objective(Y, bits, "mean")[0] == pytest.approx(loss / 6, rel=1e-14)
    # finite differences with the codes held fixed (the stated reading of the derivative): the piecewise-quadratic loss
    # written out for given codes
    def fixed_code_loss(A):
        tot = 0.0
        for t in range(6):
            lo, hi = A[t].min(), A[t].max()
            yhat = lo + (hi - lo) * codes[t] / L
            tot += np.sum((A[t] - yhat) ** 2) / 40
        return tot
    np.testing.assert_allclose(dY, _fd_grad(fixed_code_loss, Y.astype(np.float64)), atol=2e-6)
    # and the true loss agrees with it for steps that cross no rounding boundary
    t, i = 2, int(np.argsort(Y[2])[20])
    frac = ((Y[t, i] - Y[t].min()) / ((Y[t].max() - Y[t].min()) / L)) % 1.0
    h = np.float32(2.0 ** -12)
    if 0.05 < frac < 0.45 or 0.55 < frac < 0.95:
        Yp, Ym = Y.copy(), Y.copy()
        Yp[t, i] += h
        Ym[t, i] -= h
        fd = (orc.quant_objective(Yp, bits, "sum")[0] - orc.quant_objective(Ym, bits, "sum")[0]) / (
            float(Yp[t, i]) - float(Ym[t, i]))
        assert fd == pytest.approx(dY[t, i], rel=1e-3, abs=1e-7)


def test_quant_objective_closed_forms():
    # values on the grid quantise without error; the midpoint of two levels has error delta / 2
    row = np.array([[0.0, 1.0, 2.0, 3.0]], dtype=np.float32)
    loss, dY, codes = orc.quant_objective(row, 2, "sum")
    assert loss == 0.0 and not dY.any() and codes.tolist() == [[0, 1, 2, 3]]
    row = np.array([[0.0, 3.0, 1.25]], dtype=np.float32)       # delta = 1, 1.25 -> level 1, error 0.25
    loss, dY, codes = orc.quant_objective(row, 2, "sum")
    assert codes.tolist() == [[0, 3, 1]] and loss == pytest.approx(0.25 ** 2 / 3)
    # d/dy of the middle value: (2/3) e; the minimum carries -(2/3) e (1 - 1/3), the maximum -(2/3) e / 3
    np.testing.assert_allclose(dY[0], (2.0 / 3) * 0.25 * np.array([-(2.0 / 3), -(1.0 / 3), 1.0]), rtol=1e-12)
    # ties round to even: 0.5 -> 0, 1.5 -> 2, 2.5 -> 2
    row = np.array([[0.0, 3.0, 0.5, 1.5, 2.5]], dtype=np.float32)
    assert orc.quant_objective(row, 2, "sum")[2].tolist() == [[0, 3, 0, 2, 2]]
    # a constant row has no range: zero loss, zero gradient
    loss, dY, _ = orc.quant_objective(np.full((2, 5), 1.5, dtype=np.float32), 4, "sum")
    assert loss == 0.0 and not dY.any()
    # grid positions: level k sits at u = k; a constant row has none
    u = orc.quant_positions(np.array([[0.0, 3.0, 1.25], [2.0, 2.0, 2.0]]), 2)
    np.testing.assert_allclose(u, [[0.0, 3.0, 1.25], [0.0, 0.0, 0.0]], rtol=0, atol=1e-15)
    # given codes replace the decision: the other neighbour of a tie has the same error, any other code a larger one
    row = np.array([[0.0, 3.0, 1.5]])
    l_even, _, c_even = orc.quant_objective(row, 2, "sum")
    l_odd, dY_odd, c_odd = orc.quant_objective(row, 2, "sum", codes=[[0, 3, 1]])
    assert c_even.tolist() == [[0, 3, 2]] and c_odd.tolist() == [[0, 3, 1]] and l_odd == pytest.approx(l_even)
    assert dY_odd[0, 2] == pytest.approx((2.0 / 3) * 0.5)
    assert orc.quant_objective(row, 2, "sum", codes=[[0, 3, 0]])[0] > l_even
    with pytest.raises(ValueError):
        orc.quant_objective(row, 2, "sum", codes=[[0, 4, 1]])


def test_objective_dispatch_and_step():
    rng = np.random.default_rng(304)
    Y = rng.standard_normal((3, 8)).astype(np.float32).astype(np.float64)
    assert orc.objective_loss_grad(Y, "whip")[0] == orc.whip_loss(Y)
    assert orc.objective_loss_grad(Y, "variance", "sum")[0] == orc.variance_objective(Y, "sum")[0]
    assert orc.objective_loss_grad(Y, "kurtosis")[0] == orc.kurtosis_objective(Y)[0]
    assert orc.objective_loss_grad(Y, "quant", bits=3)[0] == orc.quant_objective(Y, 3)[0]
    with pytest.raises(ValueError):
        orc.objective_loss_grad(Y, "entropy")
    # a kurtosis-driven step lowers the kurtosis of a heavy-tailed block (small step, exact gradient)
    X = rng.standard_t(3.0, size=(64, 8))
    Z = rng.standard_normal((8, 8))
    out = orc.calib_step(X, Z, 1e-3, "mean", "kurtosis")
    after = orc.calib_step(X, out["Z_new"], 1e-3, "mean", "kurtosis")["loss"]
    assert after < out["loss"]
    # the variance objective is blind to the rotation up to the row means: G pairs to zero with every skew direction
    # only through the mean term
    Xc = X - X.mean(axis=1, keepdims=True)
    R, _ = orc.qr_orth(Z)
    l1 = orc.rotate_loss_grad(Xc, R, "sum", "variance")[0]
    assert l1 + np.sum((Xc @ R).mean(axis=1) ** 2) == pytest.approx(np.sum(Xc * Xc) / 8, rel=1e-12)


def test_calibrate_batches_pins():
    rng = np.random.default_rng(401)
    Xs = [rng.standard_normal((24, 6)) for _ in range(3)]
    Z0 = rng.standard_normal((6, 6))
    # one batch: the plain loop
    l1, Z1 = orc.calibrate_batches(Xs[:1], Z0, 4, 1e-2)
    l2, Z2, _ = orc.calibrate(Xs[0], Z0, 4, 1e-2)
    assert np.array_equal(l1, l2) and np.array_equal(Z1, Z2)
    # three batches, five steps: batch order 0 1 2 0 1, written out
    losses, Z = orc.calibrate_batches(Xs, Z0, 5, 1e-2)
    Zm = Z0.copy()
    for k, j in enumerate([0, 1, 2, 0, 1]):
        out = orc.calib_step(Xs[j], Zm, 1e-2)
        assert out["loss"] == losses[k]
        Zm = out["Z_new"]
    assert np.array_equal(Z, Zm)
    # with the sum reduction, one step on the stacked batches is the sum of the per-batch gradients at the same Z
    g_all = orc.calib_step(np.vstack(Xs), Z0, 1.0, "sum")["dZ"]
    g_sum = sum(orc.calib_step(x, Z0, 1.0, "sum")["dZ"] for x in Xs)
    np.testing.assert_allclose(g_all, g_sum, rtol=1e-10, atol=1e-12)


# ----------------------------------------------------------------------------------- Cayley SGD (Alg. 3, App. B.2)
def _random_rotation(rng, n):
    Q, Rf = np.linalg.qr(rng.standard_normal((n, n)))
    return Q * np.sign(np.diag(Rf))[None, :]


def test_cayley_update_is_the_cayley_transform_up_to_the_contraction_bound():
    rng = np.random.default_rng(401)
    n = 12
    R = _random_rotation(rng, n)
    G = rng.standard_normal((n, n))
    M = 0.3 * rng.standard_normal((n, n))
    for lr in (1e-3, 5e-2, 10.0):                    # the last one is cut by the 2 q / ||W|| rule
        for s in (1, 2, 5):
            Rn, Mn, alpha, W = orc.cayley_sgd_update(R, G, M, lr, beta=0.9, q=0.5, s=s)
            np.testing.assert_allclose(W, -W.T, atol=1e-14)
            assert alpha == pytest.approx(min(lr, 1.0 / (np.linalg.norm(W) + 1e-8)), rel=1e-14)
            # exact transform by a linear solve (library routine)
            I = np.eye(n)
            exact = np.linalg.solve(I - 0.5 * alpha * W, (I + 0.5 * alpha * W) @ R)
            np.testing.assert_allclose(exact.T @ exact, I, atol=1e-12)        # skew W: the transform is orthogonal
            rho = 0.5 * alpha * np.linalg.norm(W, 2)
            assert rho <= 0.5 + 1e-12
            y0 = R + alpha * (W @ R)
            # the iteration contracts towards the transform at rate rho per pass
            assert np.linalg.norm(Rn - exact, 2) <= rho ** s * np.linalg.norm(y0 - exact, 2) * (1 + 1e-9) + 1e-14
            # so the result is orthogonal to that accuracy
            assert np.abs(Rn.T @ Rn - I).max() <= 3 * rho ** s * np.linalg.norm(y0 - exact, 2) + 1e-13
    # many passes: the transform itself
    Rn, _, alpha, W = orc.cayley_sgd_update(R, G, M, 5e-2, s=60)
    np.testing.assert_allclose(Rn, np.linalg.solve(np.eye(n) - 0.5 * alpha * W, (np.eye(n) + 0.5 * alpha * W) @ R),
                               atol=1e-13)


def test_cayley_update_descent_identities():
    """Without momentum and at an orthogonal R:  W = (A - A^T) / 2 with A = -G R^T, the new momentum W R is tangent
    (R^T (W R) is skew-symmetric), and <G, W R> = -||W||_F^2: the first-order change of the loss along the step."""
    rng = np.random.default_rng(402)
    n = 9
    R = _random_rotation(rng, n)
    G = rng.standard_normal((n, n))
    Rn, Mn, alpha, W = orc.cayley_sgd_update(R, G, np.zeros((n, n)), 1e-4, beta=0.0)
    A = -G @ R.T
    np.testing.assert_allclose(W, 0.5 * (A - A.T), atol=1e-13)
    np.testing.assert_allclose(Mn, W @ R, atol=1e-14)
    np.testing.assert_allclose(R.T @ Mn, -(R.T @ Mn).T, atol=1e-13)
    assert np.sum(G * Mn) == pytest.approx(-np.sum(W * W), rel=1e-12)
    # first order in alpha: R_new = R + alpha W R + O(alpha^2)
    assert np.linalg.norm(Rn - (R + alpha * Mn)) <= 0.6 * alpha ** 2 * np.linalg.norm(W, 2) ** 2 * np.linalg.norm(R)
    # the momentum enters linearly before the projection: beta M - G
    M = rng.standard_normal((n, n))
    _, _, _, W2 = orc.cayley_sgd_update(R, G, M, 1e-4, beta=0.7)
    _, _, _, W3 = orc.cayley_sgd_update(R, G - 0.7 * M, np.zeros((n, n)), 1e-4, beta=0.0)
    np.testing.assert_allclose(W2, W3, atol=1e-13)


def test_cayley_update_two_by_two_closed_form():
    """n = 2: rotations are unit complex numbers and W = w J; two passes of the iteration give
    R (1 + i a - a^2 / 2 - i a^3 / 4) with a = alpha w."""
    theta, lr = 0.7, 0.3
    R = np.array([[np.cos(theta), -np.sin(theta)], [np.sin(theta), np.cos(theta)]])
    G = np.array([[0.3, -1.1], [0.4, 0.2]])
    Rn, Mn, alpha, W = orc.cayley_sgd_update(R, G, np.zeros((2, 2)), lr, beta=0.0, s=2)
    A = -G @ R.T
    w = 0.5 * (A[1, 0] - A[0, 1])                    # W = [[0, -w], [w, 0]]
    np.testing.assert_allclose(W, [[0.0, -w], [w, 0.0]], atol=1e-15)
    assert alpha == pytest.approx(min(lr, 1.0 / (np.sqrt(2.0) * abs(w) + 1e-8)), rel=1e-14)
    a = alpha * w
    z = np.exp(1j * theta) * (1 + 1j * a - a * a / 2 - 1j * a ** 3 / 4)
    np.testing.assert_allclose(Rn, [[z.real, -z.imag], [z.imag, z.real]], atol=1e-14)


def test_cayley_step_lowers_the_loss_and_reports_the_input_rotation():
    rng = np.random.default_rng(403)
    n, T = 8, 96
    X = rng.standard_t(3.0, size=(T, n))
    R = _random_rotation(rng, n)
    M = np.zeros((n, n))
    losses = []
    for _ in range(8):
        out = orc.cayley_step(X, R, M, 0.5, beta=0.5)
        assert out["loss"] == pytest.approx(orc.whip_loss(orc.rotate(X, R)), rel=1e-14)
        losses.append(out["loss"])
        R, M = out["R_new"], out["M_new"]
    assert losses[-1] < losses[0]
    assert np.abs(R.T @ R - np.eye(n)).max() < 1e-2        # the two-pass iteration drifts slowly off the manifold
