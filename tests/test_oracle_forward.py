"""Pins for the fp64 oracle's forward pass (CPU only).

Nothing here compares the oracle with itself alone: each test ties it to a
brute-force evaluation with explicit loops, to a library routine (scipy's
softmax, torch's elu), to a closed form, or to an invariant of the method.
"""
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle import flurka_oracle as fo

PHIS = [fo.PHI_PERFORMER, fo.PHI_ELU1]


def tiny(seed, B=2, H=2, n=7, d=4, k=3, m=5, phi=fo.PHI_PERFORMER, scale=0.6):
    rng = np.random.default_rng(seed)
    Q = rng.standard_normal((B, H, n, d)) * scale
    K = rng.standard_normal((B, H, n, d)) * scale
    V = rng.standard_normal((B, H, n, d))
    E = rng.standard_normal((k, n)) / math.sqrt(k)
    F = rng.standard_normal((k, n)) / math.sqrt(k)
    omega = rng.standard_normal((H, m, d)) if phi == fo.PHI_PERFORMER else None
    return Q, K, V, E, F, omega


def brute_force_head(Q, K, V, E, F, omega, phi):
    """Materialise the n x k attention matrix with plain loops, normalise its
    rows, multiply by V' (App. D: entries phi(x_i).phi(y_j) / sum_k phi(x_i).phi(y_k))."""
    n, d, k = len(Q), len(Q[0]), len(E)
    Kp = [[sum(E[r][i] * K[i][t] for i in range(n)) for t in range(d)] for r in range(k)]
    Vp = [[sum(F[r][i] * V[i][t] for i in range(n)) for t in range(d)] for r in range(k)]

    def feat(x):
        if phi == fo.PHI_PERFORMER:
            m = len(omega)
            half = 0.5 * sum(v * v for v in x)
            return [math.exp(sum(omega[j][t] * x[t] for t in range(d)) - half) / math.sqrt(m)
                    for j in range(m)]
        return [v + 1.0 if v > 0 else math.exp(v) for v in x]

    fq = [feat(Q[i]) for i in range(n)]
    fk = [feat(Kp[r]) for r in range(k)]
    out = np.zeros((n, d))
    for i in range(n):
        a = [sum(x * y for x, y in zip(fq[i], fk[r])) for r in range(k)]
        tot = sum(a)
        for t in range(d):
            out[i, t] = sum(a[r] / tot * Vp[r][t] for r in range(k))
    return out


@pytest.mark.parametrize("phi", PHIS)
def test_matches_bruteforce_attention_matrix(phi):
    Q, K, V, E, F, omega = tiny(1, phi=phi)
    got_def = fo.flurka_attention_definition(Q, K, V, E, F, omega, phi)
    got_safe = fo.flurka_attention(Q, K, V, E, F, omega, phi)
    for b in range(Q.shape[0]):
        for h in range(Q.shape[1]):
            om = None if omega is None else omega[h].tolist()
            ref = brute_force_head(Q[b, h].tolist(), K[b, h].tolist(), V[b, h].tolist(),
                                   E.tolist(), F.tolist(), om, phi)
            assert np.max(np.abs(got_def[b, h] - ref)) < 1e-12
            assert np.max(np.abs(got_safe[b, h] - ref)) < 1e-12


def test_projection_matches_loops_and_is_not_transposed():
    rng = np.random.default_rng(2)
    n, d, k = 5, 3, 2
    E = rng.standard_normal((k, n))
    X = rng.standard_normal((n, d))
    got = fo.sequence_projection(E, X)
    assert got.shape == (k, d)
    for r in range(k):
        for t in range(d):
            assert abs(got[r, t] - sum(E[r, i] * X[i, t] for i in range(n))) < 1e-13


def test_positive_random_features_estimate_the_softmax_kernel():
    """E[psi(x) psi(y)] = exp(x.y) (Sec. 2; Thm. 1): phi(x).phi(y) -> exp(x.y)."""
    rng = np.random.default_rng(3)
    d, m = 4, 1 << 18
    omega = rng.standard_normal((m, d))
    x = np.array([0.5, -0.3, 0.2, 0.4])
    y = np.array([-0.2, 0.6, 0.1, 0.3])
    fx = fo.phi_performer(x[None], omega)[0]
    fy = fo.phi_performer(y[None], omega)[0]
    assert np.all(fx > 0) and np.all(fy > 0)
    est = float(fx @ fy)
    exact = math.exp(float(x @ y))
    # psi(x)psi(y) = exp(w.(x+y) - (|x|^2+|y|^2)/2); its variance is
    # exp(2 x.y) (exp(|x+y|^2) - 1); allow five standard errors.
    s = x + y
    sd = math.sqrt(math.exp(2 * float(x @ y)) * (math.exp(float(s @ s)) - 1.0) / m)
    assert abs(est - exact) < 5 * sd
    assert 5 * sd < 0.02 * exact          # the test is sharp enough to see a wrong term
    # same vector: phi(x).phi(x) -> exp(|x|^2) pins the -|x|^2/2 and the 1/sqrt(m)
    sdx = math.sqrt(math.exp(2 * float(x @ x)) * (math.exp(4 * float(x @ x)) - 1.0) / m)
    assert abs(float(fx @ fx) - math.exp(float(x @ x))) < 5 * sdx


def test_many_features_limit_is_linformer_softmax_attention():
    """Proof sketch of Thm. 1: as m grows, phi(x).phi(y) -> exp(x.y), so the
    output tends to softmax(Q K'^T) V' with K' = E K, V' = F V."""
    rng = np.random.default_rng(4)
    B, H, n, d, k, m = 1, 2, 6, 4, 4, 1 << 18
    Q = rng.standard_normal((B, H, n, d)) * 0.4
    K = rng.standard_normal((B, H, n, d)) * 0.2
    # unequal key norms, so that dropping |k'|^2/2 would visibly skew the weights
    K[:, :, ::2] *= 2.5
    V = rng.standard_normal((B, H, n, d))
    E = rng.standard_normal((k, n)) / math.sqrt(k)
    F = rng.standard_normal((k, n)) / math.sqrt(k)
    omega = rng.standard_normal((H, m, d))
    got = fo.flurka_attention(Q, K, V, E, F, omega, fo.PHI_PERFORMER)
    Kp = np.matmul(E, K)
    Vp = np.matmul(F, V)
    W = scipy.special.softmax(np.matmul(Q, np.swapaxes(Kp, -1, -2)), axis=-1)
    ref = np.matmul(W, Vp)
    assert fo.rel_l2(got, ref) < 1.5e-2
    # the same limit without the norm term is far away: the pin can tell
    norms = 0.5 * np.sum(Kp * Kp, axis=-1)[:, :, None, :]
    W_bad = scipy.special.softmax(np.matmul(Q, np.swapaxes(Kp, -1, -2)) + norms, axis=-1)
    assert fo.rel_l2(np.matmul(W_bad, Vp), ref) > 0.1


def test_identity_projection_elu_is_plain_linear_attention():
    """E = F = I, k = n: Eq. 2 collapses to the kernel method of Sec. 2."""
    rng = np.random.default_rng(5)
    B, H, n, d = 1, 2, 9, 4
    Q = rng.standard_normal((B, H, n, d))
    K = rng.standard_normal((B, H, n, d))
    V = rng.standard_normal((B, H, n, d))
    I = np.eye(n)
    got = fo.flurka_attention(Q, K, V, I, I, None, fo.PHI_ELU1)
    fq = torch.nn.functional.elu(torch.from_numpy(Q)) + 1.0
    fk = torch.nn.functional.elu(torch.from_numpy(K)) + 1.0
    A = fq @ fk.transpose(-1, -2)
    ref = ((A / A.sum(-1, keepdim=True)) @ torch.from_numpy(V)).numpy()
    assert np.max(np.abs(got - ref)) < 1e-12


def test_identity_projection_performer_tends_to_full_softmax_attention():
    rng = np.random.default_rng(6)
    B, H, n, d, m = 1, 1, 8, 4, 1 << 17
    Q = rng.standard_normal((B, H, n, d)) * 0.5
    K = rng.standard_normal((B, H, n, d)) * 0.5
    V = rng.standard_normal((B, H, n, d))
    omega = rng.standard_normal((H, m, d))
    I = np.eye(n)
    got = fo.flurka_attention(Q, K, V, I, I, omega, fo.PHI_PERFORMER)
    ref = np.matmul(scipy.special.softmax(np.matmul(Q, np.swapaxes(K, -1, -2)), axis=-1), V)
    assert fo.rel_l2(got, ref) < 2e-2


def test_elu_feature_map_is_textbook_elu_plus_one():
    x = np.array([-50.0, -3.0, -1e-9, 0.0, 1e-9, 0.5, 7.0])
    got = fo.phi_elu1(x)
    ref = (torch.nn.functional.elu(torch.from_numpy(x)) + 1.0).numpy()
    assert np.allclose(got, ref, rtol=0, atol=1e-15)
    assert got[3] == 1.0 and got[-1] == 8.0 and 0.0 < got[0] < 1e-20
    assert np.all(got > 0)


@pytest.mark.parametrize("phi", PHIS)
def test_rows_of_implicit_attention_sum_to_one(phi):
    """The weights are a normalised ratio (App. D), so constant V' rows pass
    through unchanged and a shift of V' shifts the output by the same amount."""
    Q, K, V, E, F, omega = tiny(7, phi=phi)
    F = np.abs(F)
    F /= F.sum(axis=1, keepdims=True)           # rows of F sum to 1
    const = np.array([1.5, -2.0, 0.25, 3.0])
    Vc = np.broadcast_to(const, V.shape).copy()  # then every row of V' = F V is `const`
    out = fo.flurka_attention(Q, K, Vc, E, F, omega, phi)
    assert np.max(np.abs(out - const)) < 1e-12
    base = fo.flurka_attention(Q, K, V, E, F, omega, phi)
    shifted = fo.flurka_attention(Q, K, V + const, E, F, omega, phi)
    assert np.max(np.abs(shifted - base - const)) < 1e-12


@pytest.mark.parametrize("phi", PHIS)
def test_output_rows_are_convex_combinations_of_projected_values(phi):
    Q, K, V, E, F, omega = tiny(8, n=33, k=6, phi=phi, scale=2.5)   # large norms
    out = fo.flurka_attention(Q, K, V, E, F, omega, phi)
    Vp = np.matmul(F, V)
    lo = Vp.min(axis=2, keepdims=True) - 1e-12
    hi = Vp.max(axis=2, keepdims=True) + 1e-12
    assert np.all(np.isfinite(out))
    assert np.all(out >= lo) and np.all(out <= hi)


def test_single_projected_key_returns_its_value():
    """k = 1: the only weight is 1, so out_i = V'_0 for every query."""
    for phi in PHIS:
        Q, K, V, E, F, omega = tiny(9, k=1, phi=phi)
        out = fo.flurka_attention(Q, K, V, E, F, omega, phi)
        Vp = np.matmul(F, V)                       # (B,H,1,d)
        assert np.max(np.abs(out - Vp)) < 1e-12


def test_single_feature_output_is_constant_over_queries():
    """m = 1 (performer): phi(q_i) is a scalar that cancels, so every query
    gets out = sum_r w_r V'_r with w_r proportional to exp(omega.k'_r - |k'_r|^2/2)."""
    Q, K, V, E, F, omega = tiny(10, m=1)
    out = fo.flurka_attention(Q, K, V, E, F, omega, fo.PHI_PERFORMER)
    Kp = np.matmul(E, K)
    Vp = np.matmul(F, V)
    for b in range(Q.shape[0]):
        for h in range(Q.shape[1]):
            w = np.array([math.exp(float(omega[h, 0] @ kp) - 0.5 * float(kp @ kp)) for kp in Kp[b, h]])
            ref = (w[:, None] * Vp[b, h]).sum(0) / w.sum()
            assert np.max(np.abs(out[b, h] - ref[None, :])) < 1e-12


def test_closed_form_two_keys_scalar_case():
    """d = 1, m = 1, k = 2, E = F = I: out = (a V_0 + b V_1)/(a + b) with
    a = exp(w K_0 - K_0^2/2), b = exp(w K_1 - K_1^2/2)."""
    w, k0, k1, v0, v1 = 0.7, 0.4, -1.1, 2.0, -3.0
    a = math.exp(w * k0 - 0.5 * k0 * k0)
    b = math.exp(w * k1 - 0.5 * k1 * k1)
    ref = (a * v0 + b * v1) / (a + b)
    Q = np.array([[[[0.3], [-0.9]]]])
    K = np.array([[[[k0], [k1]]]])
    V = np.array([[[[v0], [v1]]]])
    out = fo.flurka_attention(Q, K, V, np.eye(2), np.eye(2), np.array([[[w]]]), fo.PHI_PERFORMER)
    assert np.max(np.abs(out - ref)) < 1e-14


@pytest.mark.parametrize("phi", PHIS)
def test_permutation_symmetries(phi):
    Q, K, V, E, F, omega = tiny(11, n=8, k=4, phi=phi)
    base = fo.flurka_attention(Q, K, V, E, F, omega, phi)
    rng = np.random.default_rng(0)
    # sequence positions of keys/values, with the matching columns of E and F
    p = rng.permutation(Q.shape[2])
    out = fo.flurka_attention(Q, K[:, :, p], V[:, :, p], E[:, p], F[:, p], omega, phi)
    assert np.max(np.abs(out - base)) < 1e-12
    # query rows
    out = fo.flurka_attention(Q[:, :, p], K, V, E, F, omega, phi)
    assert np.max(np.abs(out - base[:, :, p])) < 1e-12
    # projected slots (rows of E and F together)
    r = rng.permutation(E.shape[0])
    out = fo.flurka_attention(Q, K, V, E[r], F[r], omega, phi)
    assert np.max(np.abs(out - base)) < 1e-12
    # rows of E alone DO change the pairing of keys with values
    out = fo.flurka_attention(Q, K, V, E[np.roll(np.arange(E.shape[0]), 1)], F, omega, phi)
    assert np.max(np.abs(out - base)) > 1e-3
    if phi == fo.PHI_PERFORMER:
        j = rng.permutation(omega.shape[1])
        out = fo.flurka_attention(Q, K, V, E, F, omega[:, j], phi)
        assert np.max(np.abs(out - base)) < 1e-12
        # one shared omega == the same omega given per head
        shared = omega[:1]
        a = fo.flurka_attention(Q, K, V, E, F, shared, phi)
        b = fo.flurka_attention(Q, K, V, E, F, np.repeat(shared, Q.shape[1], axis=0), phi)
        assert np.array_equal(a, b)


@pytest.mark.parametrize("phi", PHIS)
def test_range_safe_form_equals_definition_and_survives_long_sequence_scales(phi):
    Q, K, V, E, F, omega = tiny(12, n=16, k=5, phi=phi, scale=0.4)
    a = fo.flurka_attention_definition(Q, K, V, E, F, omega, phi)
    b = fo.flurka_attention(Q, K, V, E, F, omega, phi)
    assert np.max(np.abs(a - b)) < 1e-12
    # |k'|^2/2 of several hundred, as in the long-sequence workload: the plain
    # definition underflows to 0/0, the shifted evaluation must stay finite.
    rng = np.random.default_rng(12)
    n, d, k, m = 64, 128, 4, 8
    Qb = rng.standard_normal((1, 1, n, d)) * d ** -0.25
    Kb = rng.standard_normal((1, 1, n, d)) * 4.0
    Vb = rng.standard_normal((1, 1, n, d))
    Eb = rng.standard_normal((k, n))
    om = rng.standard_normal((1, m, d)) if phi == fo.PHI_PERFORMER else None
    out = fo.flurka_attention(Qb, Kb, Vb, Eb, Eb, om, phi)
    assert np.all(np.isfinite(out))
    if phi == fo.PHI_PERFORMER:
        with np.errstate(all="ignore"):
            raw = fo.flurka_attention_definition(Qb, Kb, Vb, Eb, Eb, om, phi)
        assert not np.all(np.isfinite(raw))


def test_rows_argument_selects_query_rows():
    Q, K, V, E, F, omega = tiny(13, n=12)
    full = fo.flurka_attention(Q, K, V, E, F, omega, fo.PHI_PERFORMER)
    rows = np.array([0, 5, 11])
    part = fo.flurka_attention(Q, K, V, E, F, omega, fo.PHI_PERFORMER, rows=rows)
    assert np.array_equal(part, full[:, :, rows])


def test_rel_l2_metric():
    ref = np.array([3.0, 4.0])
    assert fo.rel_l2(ref, ref) == 0.0
    assert abs(fo.rel_l2(ref + np.array([0.3, 0.4]), ref) - 0.1) < 1e-15


# --- the products in the order Eq. 2 prints them ------------------------------------------------
def _paper_order_case(phi, seed=40, B=2, H=3, n=11, d=4, k=5, m=6, dm=7):
    rng = np.random.default_rng(seed)
    Q = rng.standard_normal((B, H, n, d)) * 0.6
    XK = rng.standard_normal((B, n, dm))
    XV = rng.standard_normal((B, n, dm))
    E = rng.standard_normal((k, n)) / np.sqrt(k)
    F = rng.standard_normal((k, n)) / np.sqrt(k)
    WK = rng.standard_normal((H, d, dm)) * 0.3
    WV = rng.standard_normal((H, d, dm)) * 0.3
    om = rng.standard_normal((H, m, d)) if phi == fo.PHI_PERFORMER else None
    return Q, XK, XV, E, F, WK, WV, om


@pytest.mark.parametrize("phi", [fo.PHI_PERFORMER, fo.PHI_ELU1])
def test_paper_order_equals_transform_first(phi):
    """(E X) W = E (X W): projecting the layer input first and transforming its k rows gives the same
    attention as transforming all n positions first (the order the other entry point assumes)."""
    Q, XK, XV, E, F, WK, WV, om = _paper_order_case(phi)
    got = fo.flurka_attention_paper_order(Q, XK, XV, E, F, WK, WV, om, phi)
    K = np.einsum("bnc,hdc->bhnd", XK, WK)
    V = np.einsum("bnc,hdc->bhnd", XV, WV)
    ref = fo.flurka_attention_definition(Q, K, V, E, F, om, phi)
    assert np.max(np.abs(got - ref)) < 1e-12


def test_paper_order_projected_keys_by_explicit_loops():
    """K'[r, t] = sum_c (sum_i E[r, i] X[i, c]) W[t, c] with W stored (d, dm): a transposed transform, or
    E applied on the wrong axis, changes the result."""
    Q, XK, XV, E, F, WK, WV, om = _paper_order_case(fo.PHI_ELU1, B=1, H=2, n=6, d=3, k=4, dm=5)
    k, n = E.shape
    H, d, dm = WK.shape
    out = np.empty_like(Q)
    for h in range(H):
        Kp = np.zeros((k, d)); Vp = np.zeros((k, d))
        for r in range(k):
            for t in range(d):
                for c in range(dm):
                    yk = sum(E[r, i] * XK[0, i, c] for i in range(n))
                    yv = sum(F[r, i] * XV[0, i, c] for i in range(n))
                    Kp[r, t] += yk * WK[h, t, c]
                    Vp[r, t] += yv * WV[h, t, c]
        PQ, PK = fo.phi_elu1(Q[0, h]), fo.phi_elu1(Kp)
        A = PQ @ PK.T
        out[0, h] = (A / A.sum(axis=1, keepdims=True)) @ Vp
    got = fo.flurka_attention_paper_order(Q, XK, XV, E, F, WK, WV, None, fo.PHI_ELU1)
    assert np.max(np.abs(got - out)) < 1e-12


def test_paper_order_with_selector_transforms_is_plain_attention():
    """W_h that picks d coordinates of the layer input: the paper-order forward is the plain forward on
    those coordinates as per-head K, V."""
    Q, XK, XV, E, F, _, _, om = _paper_order_case(fo.PHI_PERFORMER, H=2, d=3, dm=6)
    H, d, dm = 2, 3, 6
    W = np.zeros((H, d, dm))
    for h in range(H):
        for t in range(d):
            W[h, t, h * d + t] = 1.0
    got = fo.flurka_attention_paper_order(Q, XK, XV, E, F, W, W, om, fo.PHI_PERFORMER)
    K = np.stack([XK[:, :, h * d:(h + 1) * d] for h in range(H)], axis=1)
    V = np.stack([XV[:, :, h * d:(h + 1) * d] for h in range(H)], axis=1)
    ref = fo.flurka_attention(Q, K, V, E, F, om, fo.PHI_PERFORMER)
    assert np.max(np.abs(got - ref)) < 1e-12


# --- the constituents used as comparison baselines ------------------------------------------------
@pytest.mark.parametrize("phi", [fo.PHI_PERFORMER, fo.PHI_ELU1])
def test_kernel_attention_is_the_method_with_identity_projections(phi):
    rng = np.random.default_rng(50)
    B, H, n, d, m = 2, 2, 9, 4, 5
    Q, K, V = (rng.standard_normal((B, H, n, d)) * 0.7 for _ in range(3))
    om = rng.standard_normal((H, m, d)) if phi == fo.PHI_PERFORMER else None
    got = fo.kernel_attention(Q, K, V, om, phi)
    ref = fo.flurka_attention_definition(Q, K, V, np.eye(n), np.eye(n), om, phi)
    assert np.max(np.abs(got - ref)) < 1e-12
    # and the n x n matrix written out, one head
    pq = fo.phi_elu1(Q[0, 1]) if phi == fo.PHI_ELU1 else fo.phi_performer(Q[0, 1], om[1])
    pk = fo.phi_elu1(K[0, 1]) if phi == fo.PHI_ELU1 else fo.phi_performer(K[0, 1], om[1])
    A = np.array([[sum(pq[i, j] * pk[r, j] for j in range(pq.shape[1])) for r in range(n)] for i in range(n)])
    assert np.max(np.abs(got[0, 1] - (A / A.sum(axis=1, keepdims=True)) @ V[0, 1])) < 1e-12


def test_linformer_attention_against_library_softmax():
    rng = np.random.default_rng(51)
    B, H, n, d, k = 1, 2, 10, 4, 3
    Q, K, V = (rng.standard_normal((B, H, n, d)) for _ in range(3))
    E, F = rng.standard_normal((k, n)), rng.standard_normal((k, n))
    got = fo.linformer_attention(Q, K, V, E, F)
    for h in range(H):
        Kp = np.array([[sum(E[r, i] * K[0, h, i, t] for i in range(n)) for t in range(d)] for r in range(k)])
        Vp = np.array([[sum(F[r, i] * V[0, h, i, t] for i in range(n)) for t in range(d)] for r in range(k)])
        w = scipy.special.softmax(Q[0, h] @ Kp.T, axis=1)
        assert np.max(np.abs(got[0, h] - w @ Vp)) < 1e-12
    # k = 1: every row is the one projected value; shifting all scores of a row changes nothing
    one = fo.linformer_attention(Q, K, V, E[:1], F[:1])
    assert np.max(np.abs(one - (F[:1] @ V)[:, :, :1, :].repeat(n, axis=2))) < 1e-12
