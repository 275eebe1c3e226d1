"""CPU-only pins for the fp64 oracle: what the paper and the mathematics fix.

Each test holds the oracle to something other than itself: an explicit matrix
inverse, a closed form, a textbook special case, an invariant stated in the
paper, a value the paper prints, or brute-force finite differences.
"""
import os

import numpy as np
import pytest

import oracle
import vla_inputs

RNG = np.random.default_rng


def unit(x):
    return x / np.linalg.norm(x, axis=-1, keepdims=True)


def read_golden(golden_dir):
    out = {}
    with open(os.path.join(golden_dir, "paper_values.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, value, tol = [s.strip() for s in line.split("|")[:3]]
            out[name] = (float(value), float(tol))
    return out


def alpha_hat_probe(k, A0, lambda0, u=None, eps=1e-4):
    """Read alpha^_1 out of the oracle: with S_0 = 0 and v = e_0 the first row of S_1 is alpha^_1."""
    d = k.shape[-1]
    v = np.zeros((1, 1, 1, d)); v[..., 0] = 1.0
    r = oracle.forward(np.zeros((1, 1, 1, d)), k.reshape(1, 1, 1, d), v, None,
                       None if A0 is None else A0.reshape(1, 1, d, d), lambda0=lambda0, eps=eps,
                       u=None if u is None else u.reshape(1, 1, 1, d))
    return r["S_T"][0, 0, 0, :], r["A_T"][0, 0]


# ---------------------------------------------------------------- P1: A_T = M_T^{-1}
@pytest.mark.parametrize("d,T,lambda0", [(4, 9, 1.0), (16, 64, 0.1), (64, 1000, 0.1)])
def test_sherman_morrison_equals_explicit_inverse_key_penalty(d, T, lambda0):
    """eq. (penalty) + eq. (sm), and the whitening-view identity of Section 7.1:
    A_T = (lambda0 I + sum u u^T)^{-1} with u = k^."""
    q, k, v = vla_inputs.gaussian_qkv(2, 2, T, d, seed=11)
    r = oracle.forward(q, k, v, lambda0=lambda0)
    kh = unit(k.astype(np.float64))
    for b in range(2):
        for h in range(2):
            M = lambda0 * np.eye(d) + kh[b, h].T @ kh[b, h]
            ref = np.linalg.inv(M)
            err = np.abs(r["A_T"][b, h] - ref).max() / np.abs(ref).max()
            assert err < 1e-10, err


@pytest.mark.parametrize("u_scale", [1.0, 0.25])
def test_sherman_morrison_equals_explicit_inverse_supplied_u(u_scale):
    """General penalty directions (eq. (penalty)): unit-normalised, optionally scaled
    (Algorithm 1 divides by sqrt(d_h)); non-identity SPD A_0."""
    d, T = 8, 40
    rng = RNG(5)
    q, k, v = vla_inputs.gaussian_qkv(1, 3, T, d, seed=12)
    u = rng.standard_normal((1, 3, T, d))
    W = rng.standard_normal((1, 3, d, d))
    M0 = W @ np.swapaxes(W, -1, -2) + 0.5 * np.eye(d)
    A0 = np.linalg.inv(M0)
    r = oracle.forward(q, k, v, None, A0, u=u, u_scale=u_scale)
    un = u_scale * unit(u)
    for h in range(3):
        ref = np.linalg.inv(M0[0, h] + un[0, h].T @ un[0, h])
        assert np.abs(r["A_T"][0, h] - ref).max() / np.abs(ref).max() < 1e-10


# ---------------------------------------------------------------- P2/P3: SPD, delta >= 1, printed ||A_0||
def test_A_stays_symmetric_positive_definite_and_delta_at_least_one():
    d, T = 32, 600
    q, k, v = vla_inputs.gaussian_qkv(1, 4, T, d, seed=13)
    r = oracle.forward(q, k, v, lambda0=0.1, trace=True)
    A = r["A_T"]
    assert np.abs(A - np.swapaxes(A, -1, -2)).max() <= 1e-14 * np.abs(A).max()
    for h in range(4):
        assert np.linalg.eigvalsh(0.5 * (A[0, h] + A[0, h].T)).min() > 0
    tr = r["trace"]
    assert (tr[..., 2] >= 1.0 - 1e-12).all()          # delta_t >= 1 (Section 3.3)
    assert (tr[..., 7] == tr[..., 2]).all()           # so the clamp never acts
    normA = tr[0, :, :, 1]
    assert (np.diff(normA, axis=-1) <= 1e-12).all()    # A_t <= A_{t-1} in the PSD order
    assert (normA[:, 0] < np.sqrt(d) / 0.1).all()


def test_printed_initial_A_norm_and_diagonal(golden_dir):
    g = read_golden(golden_dir)
    d = 32
    z = np.zeros((1, 1, 0, d))
    r = oracle.forward(z, z, z, lambda0=0.1)
    val, tol = g["normA0_dh32_lambda0_0p1"]
    assert abs(np.linalg.norm(r["A_T"][0, 0]) - val) <= tol
    assert abs(np.linalg.norm(r["A_T"][0, 0]) - np.sqrt(d) / 0.1) < 1e-12
    dval, dtol = g["A0_diagonal_lambda0_0p1"]
    assert np.abs(np.diag(r["A_T"][0, 0]) - dval).max() <= dtol + 1e-15
    assert np.count_nonzero(r["A_T"][0, 0] - np.diag(np.diag(r["A_T"][0, 0]))) == 0
    assert np.count_nonzero(r["S_T"]) == 0             # S_0 = 0


def test_isotropic_keys_A_norm_estimate():
    """For isotropic unit keys M_T ~ (lambda0 + T/d) I, so ||A_T||_F ~ sqrt(d)/(lambda0 + T/d)."""
    d, T, lam = 64, 1000, 0.1
    q, k, v = vla_inputs.gaussian_qkv(1, 2, T, d, seed=14)
    r = oracle.forward(q, k, v, lambda0=lam)
    est = np.sqrt(d) / (lam + T / d)
    got = np.linalg.norm(r["A_T"][0, 0])
    assert 0.9 * est < got < 1.3 * est


# ---------------------------------------------------------------- P4: unit vectors, Prop. 1
def test_unit_vectors_and_bounded_state_inequality():
    d, T = 16, 300
    q, k, v = vla_inputs.gaussian_qkv(2, 2, T, d, seed=15)
    r = oracle.forward(q, k, v, lambda0=0.1, trace=True)
    tr = r["trace"]
    assert np.abs(tr[..., 5] - 1).max() < 1e-14      # ||k^|| = 1
    assert np.abs(tr[..., 6] - 1).max() < 1e-14      # ||alpha^|| = 1
    normS, norme = tr[..., 0], tr[..., 3]
    prev = np.concatenate([np.zeros_like(normS[..., :1]), normS[..., :-1]], axis=-1)
    assert (normS <= prev + norme + 1e-12).all()      # Prop. 1, one step
    assert (normS <= np.cumsum(norme, axis=-1) + 1e-9).all()   # Prop. 1, telescoped
    assert ((tr[..., 4] > 0) & (tr[..., 4] <= 1 + 1e-14)).all()  # c = k^.alpha^ in (0,1] since A > 0


def test_update_has_frobenius_norm_of_the_residual():
    """||S_t - S_{t-1}||_F = ||e_t|| (proof of Prop. 1), via single-token calls with carried state."""
    d, T = 8, 12
    q, k, v = vla_inputs.gaussian_qkv(1, 1, T, d, seed=16)
    S = np.zeros((1, 1, d, d)); A = np.eye(d).reshape(1, 1, d, d) / 0.1
    for t in range(T):
        r = oracle.forward(q[:, :, t:t + 1], k[:, :, t:t + 1], v[:, :, t:t + 1], S, A, trace=True)
        assert abs(np.linalg.norm(r["S_T"] - S) - r["trace"][0, 0, 0, 3]) < 1e-13
        assert np.linalg.matrix_rank(r["S_T"][0, 0] - S[0, 0], tol=1e-10) == 1
        S, A = r["S_T"], r["A_T"]


# ---------------------------------------------------------------- P5: Jacobian by finite differences
@pytest.mark.parametrize("d_k,d_v,seed", [(3, 3, 0), (8, 8, 1), (6, 4, 2)])
def test_jacobian_structure_by_finite_differences(d_k, d_v, seed):
    """Prop. 2 (Section 4.2) where it holds and its correction.

    vec(S_{t-1}) -> vec(S_t) (row by row) has Jacobian I_{d_v} (x) (I - k^ alpha^^T)^T: every row of
    S is right-multiplied by (I - k^ alpha^^T).  Eigenvalues: 1 (d_k - 1 times) and 1 - c with
    c = k^.alpha^ (stated in the proof of Prop. 2); the largest singular value is
    sqrt(((3 - 2c) + sqrt(5 - 4c)) / 2) >= 1 with equality iff c = 1, so 'spectral norm 1' is
    exact only when alpha^ = k^.
    """
    rng = RNG(seed)
    k = rng.standard_normal(d_k); q = rng.standard_normal(d_k); v = rng.standard_normal(d_v)
    W = rng.standard_normal((d_k, d_k)); A0 = np.linalg.inv(W @ W.T + 0.3 * np.eye(d_k))
    S0 = rng.standard_normal((d_v, d_k))

    def step(S):
        r = oracle.forward(q.reshape(1, 1, 1, -1), k.reshape(1, 1, 1, -1), v.reshape(1, 1, 1, -1),
                           S.reshape(1, 1, d_v, d_k), A0.reshape(1, 1, d_k, d_k))
        return r["S_T"][0, 0]

    n = d_v * d_k
    J = np.zeros((n, n))
    h = 1e-3  # the map is affine in S, so central differences are exact up to rounding
    for a in range(n):
        dS = np.zeros(n); dS[a] = h
        J[:, a] = (step(S0 + dS.reshape(d_v, d_k)) - step(S0 - dS.reshape(d_v, d_k))).ravel() / (2 * h)

    # independent construction of k^, alpha^ from the definitions (explicit inverse, no Sherman-Morrison)
    kh = k / np.linalg.norm(k)
    A1 = np.linalg.inv(np.linalg.inv(A0) + np.outer(kh, kh))
    al = A1 @ kh; al /= np.linalg.norm(al)
    block = (np.eye(d_k) - np.outer(kh, al)).T          # d S_t[i,b] / d S_{t-1}[i,a] = delta_ab - k^_a alpha^_b
    assert np.abs(J - np.kron(np.eye(d_v), block)).max() < 1e-9
    c = kh @ al
    ev = np.sort(np.linalg.eigvals(J).real)
    expect = np.sort(np.concatenate([np.ones((d_k - 1) * d_v), np.full(d_v, 1 - c)]))
    assert np.abs(ev - expect).max() < 1e-6
    assert abs(np.abs(np.linalg.eigvals(J)).max() - 1.0) < 1e-6     # spectral radius 1
    smax = np.linalg.svd(J, compute_uv=False).max()
    assert abs(smax - np.sqrt(((3 - 2 * c) + np.sqrt(5 - 4 * c)) / 2)) < 1e-9
    assert smax >= 1 - 1e-12


@pytest.mark.parametrize("d", [32, 64, 96, 128])
def test_jacobian_unit_spectral_norm_where_prop2_holds(d, golden_dir):
    """First step from A_0 = I/lambda0 with u = k^ gives alpha^_1 = k^_1, hence sigma_max = 1.000
    (the 'normalised' column of the Jacobian table, Section 4.2)."""
    val, tol = read_golden(golden_dir)["jacobian_sigma_max_normalised"]
    k = RNG(d).standard_normal(d)
    al, _ = alpha_hat_probe(k, None, 0.1)
    kh = k / np.linalg.norm(k)
    assert np.abs(al - kh).max() < 1e-14
    J = np.eye(d) - np.outer(al, kh)
    assert abs(np.linalg.svd(J, compute_uv=False).max() - val) <= tol


# ---------------------------------------------------------------- P6: u = k^ identity
def test_key_penalty_identity_alpha_parallel_to_pre_update_A_k():
    """With u = k^:  A_t k^_t = z_t / delta_t, so alpha^_t is parallel to A_{t-1} k^_t."""
    d = 8
    rng = RNG(21)
    W = rng.standard_normal((d, d)); A0 = np.linalg.inv(W @ W.T + 0.2 * np.eye(d))
    k = rng.standard_normal(d)
    al, A1 = alpha_hat_probe(k, A0, 0.1)
    kh = k / np.linalg.norm(k)
    z = A0 @ kh
    assert np.abs(al - z / np.linalg.norm(z)).max() < 1e-13
    assert np.abs(A1 @ kh - z / (1 + kh @ z)).max() < 1e-13


def test_write_direction_uses_post_update_A_when_u_differs_from_k():
    """With u != k^ the pre- and post-update A give different directions; the paper uses A_t
    (Appendix A, 'Why post-update A_t')."""
    d = 6
    rng = RNG(22)
    k = rng.standard_normal(d); u = rng.standard_normal(d)
    al, _ = alpha_hat_probe(k, None, 0.5, u=u)
    kh = k / np.linalg.norm(k); uh = u / np.linalg.norm(u)
    A1 = np.linalg.inv(0.5 * np.eye(d) + np.outer(uh, uh))
    post = A1 @ kh; post /= np.linalg.norm(post)
    pre = kh.copy()                                        # A_0 k^ is parallel to k^
    assert np.abs(al - post).max() < 1e-13
    assert np.abs(al - pre).max() > 1e-3


# ---------------------------------------------------------------- P7: orthonormal keys, exact recall
@pytest.mark.parametrize("d_k,d_v,n", [(16, 16, 16), (12, 5, 7)])
def test_orthonormal_keys_exact_recall_and_closed_form_A(d_k, d_v, n):
    """Prop. 3 in the form its footnote states (orthogonal keys): S_n k_i = v_i, read out through
    o = S q at zero-key query tokens; and A_n = I/l - (1/l - 1/(l+1)) sum k_i k_i^T."""
    lam = 0.1
    rng = RNG(23)
    Q, _ = np.linalg.qr(rng.standard_normal((d_k, d_k)))
    keys = Q[:, :n].T * rng.uniform(0.5, 3.0, size=(n, 1))      # any positive scale: k is normalised
    vals = rng.standard_normal((n, d_v))
    T = 2 * n
    k = np.zeros((1, 1, T, d_k)); v = np.zeros((1, 1, T, d_v)); q = np.zeros((1, 1, T, d_k))
    k[0, 0, :n] = keys; v[0, 0, :n] = vals
    q[0, 0, n:] = unit(keys)
    r = oracle.forward(q, k, v, lambda0=lam)
    assert np.abs(r["o"][0, 0, n:] - vals).max() < 1e-12
    kh = unit(keys)
    A_ref = np.eye(d_k) / lam - (1 / lam - 1 / (lam + 1)) * kh.T @ kh
    assert np.abs(r["A_T"][0, 0] - A_ref).max() < 1e-12
    assert np.abs(r["S_T"][0, 0] - vals.T @ kh).max() < 1e-12


# ---------------------------------------------------------------- P8: two correlated keys
@pytest.mark.parametrize("lam", [0.1, 1.0, 1e-6])
def test_two_correlated_keys_write_direction(lam):
    """Section 7.2: the write direction for k^_2 removes its overlap with k^_1:
    alpha^_2 is parallel to k^_2 - rho/(1+lambda0) k^_1 (the paper's k^_2 - rho k^_1 as lambda0 -> 0)."""
    d = 10
    rng = RNG(24)
    k1 = unit(rng.standard_normal(d)); k2 = unit(rng.standard_normal(d) + 0.8 * k1)
    rho = k1 @ k2
    _, A1 = alpha_hat_probe(k1, None, lam)
    al2, _ = alpha_hat_probe(k2, A1, lam)
    ref = k2 - rho / (1 + lam) * k1
    ref /= np.linalg.norm(ref)
    assert np.abs(al2 - ref).max() < 1e-9
    if lam == 1e-6:
        assert abs(al2 @ k1) < 1e-5        # orthogonal to the stored key in the limit


# ---------------------------------------------------------------- P9: zero key is a no-op write
def test_zero_key_token_is_a_noop_write_but_still_reads():
    d = 8
    q, k, v = vla_inputs.gaussian_qkv(1, 1, 20, d, seed=25)
    r0 = oracle.forward(q[:, :, :10], k[:, :, :10], v[:, :, :10])
    k2 = k.copy(); k2[:, :, 10:] = 0.0
    r = oracle.forward(q, k2, v)
    assert np.array_equal(r["S_T"], r0["S_T"]) and np.array_equal(r["A_T"], r0["A_T"])
    ref_o = np.einsum("ij,tj->ti", r0["S_T"][0, 0], q[0, 0, 10:].astype(np.float64))
    assert np.abs(r["o"][0, 0, 10:] - ref_o).max() < 1e-13
    assert np.isfinite(r["o"]).all()


# ---------------------------------------------------------------- P10: state carry
def test_state_carry_is_bitwise():
    d, T, T1 = 16, 50, 17
    q, k, v = vla_inputs.gaussian_qkv(2, 1, T, d, seed=26)
    full = oracle.forward(q, k, v, lambda0=0.1)
    a = oracle.forward(q[:, :, :T1], k[:, :, :T1], v[:, :, :T1], lambda0=0.1)
    b = oracle.forward(q[:, :, T1:], k[:, :, T1:], v[:, :, T1:], a["S_T"], a["A_T"])
    assert np.array_equal(np.concatenate([a["o"], b["o"]], axis=2), full["o"])
    assert np.array_equal(b["S_T"], full["S_T"]) and np.array_equal(b["A_T"], full["A_T"])


# ---------------------------------------------------------------- P11: u = 0 -> normalised delta rule
def test_zero_penalty_reduces_to_normalised_delta_rule():
    """Remark of Section 4.4: u_t = 0 keeps A = I/lambda0, alpha^ = k^, and the update becomes the
    textbook normalised-LMS / Kaczmarz step S += (v - S k^) k^^T."""
    d_k, d_v, T = 7, 5, 30
    rng = RNG(27)
    q = rng.standard_normal((1, 1, T, d_k)); k = rng.standard_normal((1, 1, T, d_k))
    v = rng.standard_normal((1, 1, T, d_v))
    r = oracle.forward(q, k, v, lambda0=0.1, u=np.zeros_like(k))
    S = np.zeros((d_v, d_k)); o = []
    for t in range(T):
        kh = k[0, 0, t] / np.linalg.norm(k[0, 0, t])
        S = S + np.outer(v[0, 0, t] - S @ kh, kh)
        o.append(S @ q[0, 0, t])
    assert np.abs(r["S_T"][0, 0] - S).max() < 1e-12
    assert np.abs(r["o"][0, 0] - np.array(o)).max() < 1e-12
    assert np.array_equal(r["A_T"][0, 0], np.eye(d_k) / 0.1)


# ---------------------------------------------------------------- P12: independence and causality
def test_head_independence_and_causality():
    d, T = 8, 40
    q, k, v = vla_inputs.gaussian_qkv(2, 3, T, d, seed=28)
    r = oracle.forward(q, k, v)
    perm = np.array([4, 2, 5, 0, 3, 1])
    fl = lambda x: x.reshape(1, 6, *x.shape[2:])[:, perm]
    rp = oracle.forward(fl(q), fl(k), fl(v))
    assert np.array_equal(rp["o"], fl(r["o"])) and np.array_equal(rp["S_T"], fl(r["S_T"]))
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    q2[:, :, 25:] += 1; k2[:, :, 25:] *= -2; v2[:, :, 25:] = 7
    r2 = oracle.forward(q2, k2, v2)
    assert np.array_equal(r2["o"][:, :, :25], r["o"][:, :, :25])
    assert not np.array_equal(r2["o"][:, :, 25:], r["o"][:, :, 25:])


# ---------------------------------------------------------------- P13: invariances
def test_key_scale_invariance_and_linearity():
    d, T = 8, 40
    rng = RNG(29)
    q, k, v = [x.astype(np.float64) for x in vla_inputs.gaussian_qkv(1, 2, T, d, seed=29)]
    S0 = rng.standard_normal((1, 2, d, d))
    r = oracle.forward(q, k, v, S0)
    scale = rng.uniform(0.1, 10, size=(1, 2, T, 1))
    rs = oracle.forward(q, k * scale, v, S0)
    assert np.abs(rs["o"] - r["o"]).max() < 1e-11 and np.abs(rs["A_T"] - r["A_T"]).max() < 1e-12
    r3 = oracle.forward(3 * q, k, v, S0)
    assert np.abs(r3["o"] - 3 * r["o"]).max() < 1e-11        # o linear in q
    v2 = rng.standard_normal(v.shape); S02 = rng.standard_normal(S0.shape)
    rb = oracle.forward(q, k, v2, S02)
    rc = oracle.forward(q, k, 2 * v - v2, 2 * S0 - S02)
    assert np.abs(rc["o"] - (2 * r["o"] - rb["o"])).max() < 1e-10      # (o, S_T) linear in (v, S_0)
    assert np.abs(rc["S_T"] - (2 * r["S_T"] - rb["S_T"])).max() < 1e-10


# ---------------------------------------------------------------- step-by-step re-derivation with explicit inverses
def test_against_definition_with_explicit_inverses_tiny():
    """Every step from the definitions, A_t by inverting M_t afresh (no rank-1 recursion),
    d_k != d_v so a transposed S or a q/k mix-up cannot pass."""
    d_k, d_v, T, lam = 4, 3, 7, 0.3
    rng = RNG(30)
    q = rng.standard_normal((T, d_k)); k = rng.standard_normal((T, d_k))
    v = rng.standard_normal((T, d_v)); u = rng.standard_normal((T, d_k))
    r = oracle.forward(q[None, None], k[None, None], v[None, None], lambda0=lam, u=u[None, None])
    M = lam * np.eye(d_k); S = np.zeros((d_v, d_k))
    for t in range(T):
        kh = k[t] / np.linalg.norm(k[t]); uh = u[t] / np.linalg.norm(u[t])
        M = M + np.outer(uh, uh)
        a = np.linalg.solve(M, kh); a /= np.linalg.norm(a)
        S = S + np.outer(v[t] - S @ kh, a)
        assert np.abs(r["o"][0, 0, t] - S @ q[t]).max() < 1e-12
    assert np.abs(r["S_T"][0, 0] - S).max() < 1e-12
    assert np.abs(r["A_T"][0, 0] - np.linalg.inv(M)).max() < 1e-12


# ---------------------------------------------------------------- P14: bounded vs growing state norm
def test_norm_growth_gap_vs_linear_attention():
    """Section 6.2 / Prop. 1, qualitatively: VLA's ||S_t||_F plateaus (about d for N(0,1) inputs)
    while additive linear attention keeps growing (d*sqrt(T) for zero-mean inputs).  The paper's
    absolute values (<15 vs ~1630) come from its trained model's features and are not reproduced."""
    c = vla_inputs.CONFIGS["norm_growth"]
    q, k, v = vla_inputs.gaussian_qkv(c["B"], c["H"], c["T"], c["d"], c["seed"], c["std"])
    r = oracle.forward(q, k, v, lambda0=c["lambda0"], trace=True)
    lin = oracle.linear_attention(q, k, v)
    normS = r["trace"][..., 0]
    d, T = c["d"], c["T"]
    assert normS.max() <= 1.2 * d
    assert normS[..., T // 2:].min() >= 0.5 * d                 # a plateau, not decay to zero
    ratio = lin["normS"][..., -1] / normS[..., -1]
    assert ratio.min() >= 10
    growth = lin["normS"][..., -1].mean() / (d * np.sqrt(T))
    assert 0.9 < growth < 1.1
    # additive baseline pinned to its closed form S_T = V^T K
    ref = np.einsum("bhti,bhtj->bhij", v.astype(np.float64), k.astype(np.float64))
    assert np.abs(lin["S_T"] - ref).max() < 1e-9


# ---------------------------------------------------------------- P15: synthetic recall
def test_synthetic_recall_retrieves_stored_values():
    """Bare-recurrence stand-in for the MQAR task (Section 5.2): n <= d random unit keys written
    once, queried later through zero-key tokens.  Retrieval by nearest stored value is perfect;
    cosine to the stored value degrades gracefully with load (Section 7.2)."""
    c = vla_inputs.CONFIGS["recall"]
    B, H, T, d = 8, c["H"], c["T"], c["d"]
    q, k, v, meta = vla_inputs.recall_task(B, H, T, d, c["seed"], c["n_pairs"])
    r = oracle.forward(q, k, v, lambda0=c["lambda0"])
    cos_by_n = {}
    for (b, h), qpos in meta["query_pos"].items():
        vals = meta["values"][(b, h)].astype(np.float64)
        got = r["o"][b, h, qpos]
        sim = unit(got) @ unit(vals).T
        assert (sim.argmax(axis=1) == meta["sigma"][(b, h)]).all()
        cos_by_n.setdefault(int(meta["n"][b, h]), []).append(
            sim[np.arange(len(qpos)), meta["sigma"][(b, h)]].mean())
    means = {n: float(np.mean(x)) for n, x in cos_by_n.items()}
    assert means[16] > 0.99 and means[32] > 0.97 and means[48] > 0.93 and means[64] > 0.85
    assert means[16] > means[32] > means[48] > means[64]
    # filler tokens (all-zero) read nothing and write nothing
    filler = (np.abs(q).sum(-1) == 0) & (np.abs(k).sum(-1) == 0)
    assert np.count_nonzero(r["o"][filler]) == 0


# ---------------------------------------------------------------- the other lines of Algorithm 1 (switches)
def test_identity_refresh_against_explicit_inverses():
    """Algorithm 1's periodic refresh: A <- A + eta I after the rank-1 update of every `period`-th step.
    A_t is recomputed here from scratch with matrix inverses (no rank-1 recursion)."""
    d, T, lam, period, eta = 5, 23, 0.2, 4, 1e-2
    rng = RNG(40)
    q = rng.standard_normal((T, d)); k = rng.standard_normal((T, d)); v = rng.standard_normal((T, d))
    r = oracle.forward(q[None, None], k[None, None], v[None, None], lambda0=lam,
                       refresh_period=period, refresh_eta=eta)
    A = np.eye(d) / lam; S = np.zeros((d, d))
    for t in range(T):
        kh = k[t] / np.linalg.norm(k[t])
        A = np.linalg.inv(np.linalg.inv(A) + np.outer(kh, kh))
        if (t + 1) % period == 0:
            A = A + eta * np.eye(d)
        a = A @ kh; a /= np.linalg.norm(a)
        S = S + np.outer(v[t] - S @ kh, a)
        assert np.abs(r["o"][0, 0, t] - S @ q[t]).max() < 1e-11
    assert np.abs(r["A_T"][0, 0] - A).max() < 1e-11
    # and it really differs from the run without refresh
    r0 = oracle.forward(q[None, None], k[None, None], v[None, None], lambda0=lam)
    assert np.abs(r0["A_T"] - r["A_T"]).max() > 1e-3


def test_output_normaliser_and_key_accumulator():
    """eq. (output): o_t = S_t q_t / max(q_t . zkey_t, eps), zkey_t = sum_{s<=t} k_s; the denominator
    here comes from numpy's cumsum, the numerator from the un-normalised run."""
    d, T = 6, 40
    rng = RNG(41)
    q = np.abs(rng.standard_normal((1, 2, T, d))) + 0.1
    k = np.abs(rng.standard_normal((1, 2, T, d))) + 0.1
    v = rng.standard_normal((1, 2, T, d))
    z0 = np.abs(rng.standard_normal((1, 2, d)))
    plain = oracle.forward(q, k, v)
    norm = oracle.forward(q, k, v, normalise_output=True, zkey0=z0)
    zk = z0[:, :, None, :] + np.cumsum(k, axis=2)
    den = np.maximum(np.einsum("bhtd,bhtd->bht", zk, q), 1e-4)
    assert np.abs(norm["o"] - plain["o"] / den[..., None]).max() < 1e-12
    assert np.abs(norm["zkey_T"] - zk[:, :, -1]).max() < 1e-12
    assert np.array_equal(norm["S_T"], plain["S_T"]) and np.array_equal(norm["A_T"], plain["A_T"])
    # the floor: a query orthogonal to every key gives den = eps
    q2 = q.copy(); q2[0, 0, 5] = 0.0
    n2 = oracle.forward(q2, k, v, normalise_output=True)
    assert np.count_nonzero(n2["o"][0, 0, 5]) == 0
    # carry of the accumulator across calls
    a = oracle.forward(q[:, :, :15], k[:, :, :15], v[:, :, :15], normalise_output=True, zkey0=z0)
    b = oracle.forward(q[:, :, 15:], k[:, :, 15:], v[:, :, 15:], a["S_T"], a["A_T"],
                       normalise_output=True, zkey0=a["zkey_T"])
    assert np.array_equal(np.concatenate([a["o"], b["o"]], axis=2), norm["o"])


def test_elu_plus_one_feature_map():
    """phi(x) = ELU(x) + 1 (Section 3.3): printed values phi(0) = 1, phi(1) = 2, phi(-1) = 1/e, positivity,
    and equivalence with transforming q and k beforehand."""
    d, T = 4, 12
    rng = RNG(42)
    q = rng.standard_normal((1, 1, T, d)); k = rng.standard_normal((1, 1, T, d)); v = rng.standard_normal((1, 1, T, d))
    phi = lambda x: np.where(x > 0, x + 1.0, np.exp(np.minimum(x, 0.0)))
    assert phi(np.array([0.0, 1.0, -1.0])).tolist() == [1.0, 2.0, float(np.exp(-1.0))]
    r = oracle.forward(q, k, v, feature_map=True, normalise_output=True)
    ref = oracle.forward(phi(q), phi(k), v, normalise_output=True)
    for name in ("o", "S_T", "A_T", "zkey_T"):
        assert np.abs(r[name] - ref[name]).max() < 1e-14
    # probe phi itself through the accumulator: one token, k = (0, 1, -1, 5)
    kk = np.array([0.0, 1.0, -1.0, 5.0]).reshape(1, 1, 1, 4)
    z = oracle.forward(np.ones((1, 1, 1, 4)), kk, np.zeros((1, 1, 1, 4)), feature_map=True)["zkey_T"][0, 0]
    assert np.abs(z - np.array([1.0, 2.0, np.exp(-1.0), 6.0])).max() < 1e-15


def test_full_algorithm1_tiny_with_every_switch():
    """All lines of Algorithm 1 together (feature map, supplied u scaled by 1/sqrt(d_h), refresh every 3
    steps, normalised read-out), re-derived with fresh inverses at d_k != d_v."""
    d_k, d_v, T, lam, eta, period = 4, 3, 10, 0.1, 1e-3, 3
    rng = RNG(43)
    q = rng.standard_normal((T, d_k)); k = rng.standard_normal((T, d_k)); v = rng.standard_normal((T, d_v))
    u = rng.standard_normal((T, d_k))
    r = oracle.forward(q[None, None], k[None, None], v[None, None], lambda0=lam, u=u[None, None],
                       u_scale=d_k ** -0.5, refresh_period=period, refresh_eta=eta,
                       normalise_output=True, feature_map=True)
    phi = lambda x: np.where(x > 0, x + 1.0, np.exp(np.minimum(x, 0.0)))
    A = np.eye(d_k) / lam; S = np.zeros((d_v, d_k)); z = np.zeros(d_k)
    for t in range(T):
        kf, qf = phi(k[t]), phi(q[t])
        kh = kf / np.linalg.norm(kf)
        uu = u[t] / np.linalg.norm(u[t]) / np.sqrt(d_k)
        A = np.linalg.inv(np.linalg.inv(A) + np.outer(uu, uu))
        if (t + 1) % period == 0:
            A = A + eta * np.eye(d_k)
        a = A @ kh; a /= np.linalg.norm(a)
        S = S + np.outer(v[t] - S @ kh, a)
        z = z + kf
        assert np.abs(r["o"][0, 0, t] - S @ qf / max(z @ qf, 1e-4)).max() < 1e-11
    assert np.abs(r["A_T"][0, 0] - A).max() < 1e-10 and np.abs(r["S_T"][0, 0] - S).max() < 1e-11


# ---------------------------------------------------------------- the refresh schedule across split calls
# Algorithm 1 refreshes when the 1-based step count is a multiple of the period.  For period 4 and a call of
# 11 tokens that starts after `offset` earlier tokens (its tokens are steps offset + 1 ... offset + 11), the
# local 0-based indices that refresh, counted out by hand:
REFRESH_STEPS_PERIOD4_T11 = {
    0: [3, 7],          # steps 1..11:  4, 8
    1: [2, 6, 10],      # steps 2..12:  4, 8, 12
    2: [1, 5, 9],       # steps 3..13:  4, 8, 12
    3: [0, 4, 8],       # steps 4..14:  4, 8, 12
    4: [3, 7],          # steps 5..15:  8, 12
    7: [0, 4, 8],       # steps 8..18:  8, 12, 16
    18: [1, 5, 9],      # steps 19..29: 20, 24, 28
}


@pytest.mark.parametrize("offset", sorted(REFRESH_STEPS_PERIOD4_T11))
def test_step_offset_shifts_the_refresh_schedule(offset):
    """A call with step_offset = k refreshes at the steps of the table above; A_t is recomputed with
    fresh inverses (no rank-1 recursion), eta I added at exactly the listed tokens."""
    d, T, lam, period, eta = 4, 11, 0.25, 4, 5e-2
    refresh_at = REFRESH_STEPS_PERIOD4_T11[offset]
    rng = RNG(50 + offset)
    q = rng.standard_normal((T, d)); k = rng.standard_normal((T, d)); v = rng.standard_normal((T, d))
    r = oracle.forward(q[None, None], k[None, None], v[None, None], lambda0=lam, refresh_period=period,
                       refresh_eta=eta, step_offset=offset)
    A = np.eye(d) / lam; S = np.zeros((d, d))
    for t in range(T):
        kh = k[t] / np.linalg.norm(k[t])
        A = np.linalg.inv(np.linalg.inv(A) + np.outer(kh, kh))
        if t in refresh_at:
            A = A + eta * np.eye(d)
        a = A @ kh; a /= np.linalg.norm(a)
        S = S + np.outer(v[t] - S @ kh, a)
        assert np.abs(r["o"][0, 0, t] - S @ q[t]).max() < 1e-11, t
    assert np.abs(r["A_T"][0, 0] - A).max() < 1e-11 and np.abs(r["S_T"][0, 0] - S).max() < 1e-11
    # a schedule shifted by one token is a different result (so the comparison above can tell them apart)
    other = oracle.forward(q[None, None], k[None, None], v[None, None], lambda0=lam, refresh_period=period,
                           refresh_eta=eta, step_offset=offset + 1)
    assert np.abs(other["A_T"] - r["A_T"]).max() > 1e-4


@pytest.mark.parametrize("T1", [5, 8, 13, 1, 19])
def test_split_call_with_refresh_reproduces_one_call_bitwise(T1):
    """Running [0, T1) and then [T1, T) with step_offset = T1 and the carried S, A and key sum is the single
    call over [0, T), bit for bit, whether or not T1 is a multiple of the period (period 4), with every option
    on; without the offset the second half refreshes at the wrong steps."""
    d_k, d_v, T, period = 6, 5, 20, 4
    rng = RNG(60)
    q = rng.standard_normal((2, 1, T, d_k)); k = rng.standard_normal((2, 1, T, d_k))
    v = rng.standard_normal((2, 1, T, d_v)); u = rng.standard_normal((2, 1, T, d_k))
    opt = dict(lambda0=0.2, refresh_period=period, refresh_eta=1e-2, normalise_output=True, feature_map=True,
               u_scale=0.5)
    full = oracle.forward(q, k, v, u=u, **opt)
    a = oracle.forward(q[:, :, :T1], k[:, :, :T1], v[:, :, :T1], u=u[:, :, :T1], **opt)
    b = oracle.forward(q[:, :, T1:], k[:, :, T1:], v[:, :, T1:], a["S_T"], a["A_T"], u=u[:, :, T1:],
                       step_offset=T1, zkey0=a["zkey_T"], **opt)
    assert np.array_equal(np.concatenate([a["o"], b["o"]], axis=2), full["o"])
    for name in ("S_T", "A_T", "zkey_T"):
        assert np.array_equal(b[name], full[name]), name
    if T1 % period:
        wrong = oracle.forward(q[:, :, T1:], k[:, :, T1:], v[:, :, T1:], a["S_T"], a["A_T"], u=u[:, :, T1:],
                               zkey0=a["zkey_T"], **opt)
        assert np.abs(wrong["A_T"] - full["A_T"]).max() > 1e-4
