"""Pins for the fp64 oracle's backward pass (CPU only).

The paper prints no backward; the oracle's is the chain rule of its forward.
It is pinned by central finite differences of the (separately pinned)
forward, by adjoint identities that hold exactly because the output is
linear in V and in F, and by structural identities (gradients of shared
parameters add over heads, permutation equivariance).
"""
import math

import numpy as np
import pytest

from oracle import flurka_oracle as fo

PHIS = [fo.PHI_PERFORMER, fo.PHI_ELU1]


def tiny(seed, B=2, H=2, n=6, d=3, k=3, m=4, phi=fo.PHI_PERFORMER):
    rng = np.random.default_rng(seed)
    Q = rng.standard_normal((B, H, n, d)) * 0.7
    K = rng.standard_normal((B, H, n, d)) * 0.7
    V = rng.standard_normal((B, H, n, d))
    E = rng.standard_normal((k, n)) / math.sqrt(k)
    F = rng.standard_normal((k, n)) / math.sqrt(k)
    omega = rng.standard_normal((H, m, d)) if phi == fo.PHI_PERFORMER else None
    G = rng.standard_normal((B, H, n, d))
    return dict(Q=Q, K=K, V=V, E=E, F=F), omega, G


def loss(t, omega, G, phi):
    return float(np.sum(fo.flurka_attention(t["Q"], t["K"], t["V"], t["E"], t["F"], omega, phi) * G))


def central_difference(t, omega, G, phi, name, h=1e-6):
    base = t[name]
    g = np.zeros_like(base)
    it = np.nditer(base, flags=["multi_index"])
    for _ in it:
        idx = it.multi_index
        keep = base[idx]
        base[idx] = keep + h
        up = loss(t, omega, G, phi)
        base[idx] = keep - h
        dn = loss(t, omega, G, phi)
        base[idx] = keep
        g[idx] = (up - dn) / (2 * h)
    return g


@pytest.mark.parametrize("phi", PHIS)
def test_all_gradients_match_central_differences(phi):
    t, omega, G = tiny(21, phi=phi)
    got = dict(zip(["Q", "K", "V", "E", "F"],
                   fo.flurka_attention_bwd(t["Q"], t["K"], t["V"], t["E"], t["F"], omega, G, phi)))
    for name in ["Q", "K", "V", "E", "F"]:
        fd = central_difference(t, omega, G, phi, name)
        assert fo.rel_l2(got[name], fd) < 2e-7, name


def test_elu_gradient_across_the_kink():
    """elu(x)+1 has slope 1 above zero and exp(x) below; entries on both sides
    of zero (also in K') are present, and the finite difference still agrees."""
    t, omega, G = tiny(22, phi=fo.PHI_ELU1)
    assert (t["Q"] > 0).any() and (t["Q"] < 0).any()
    Kp = np.matmul(t["E"], t["K"])
    assert (Kp > 0).any() and (Kp < 0).any()
    dQ = fo.flurka_attention_bwd(t["Q"], t["K"], t["V"], t["E"], t["F"], None, G, fo.PHI_ELU1)[0]
    fd = central_difference(t, None, G, fo.PHI_ELU1, "Q")
    assert fo.rel_l2(dQ, fd) < 2e-7


@pytest.mark.parametrize("phi", PHIS)
def test_adjoint_identities_for_linear_arguments(phi):
    """out is linear in V and in F (out = W F V with W independent of both), so
    <dV, V2> = <G, out(V2)> and <dF, F2> = <G, out(F2)> hold to rounding."""
    t, omega, G = tiny(23, phi=phi)
    _, _, dV, _, dF = fo.flurka_attention_bwd(t["Q"], t["K"], t["V"], t["E"], t["F"], omega, G, phi)
    rng = np.random.default_rng(5)
    V2 = rng.standard_normal(t["V"].shape)
    F2 = rng.standard_normal(t["F"].shape)
    lhs = float(np.sum(dV * V2))
    rhs = float(np.sum(G * fo.flurka_attention(t["Q"], t["K"], V2, t["E"], t["F"], omega, phi)))
    assert abs(lhs - rhs) < 1e-11 * max(1.0, abs(rhs))
    lhs = float(np.sum(dF * F2))
    rhs = float(np.sum(G * fo.flurka_attention(t["Q"], t["K"], t["V"], t["E"], F2, omega, phi)))
    assert abs(lhs - rhs) < 1e-11 * max(1.0, abs(rhs))


def test_performer_query_gradient_is_free_of_the_norm_term():
    """phi(q) enters only through a ratio that is invariant to any positive
    rescaling of the row, so d out / d(log scale of row i) = 0.  For the
    positive random features that means dQ_i = dU_i omega exactly, i.e. the
    -rowsum(dU) q_i term vanishes; equivalently the loss does not change when
    the |q|^2/2 term is present or absent.  Checked through the forward:
    moving q_i along any direction v changes the loss by dQ_i.v, and the
    finite difference of a forward that omits the norm term agrees."""
    t, omega, G = tiny(24)
    dQ = fo.flurka_attention_bwd(t["Q"], t["K"], t["V"], t["E"], t["F"], omega, G, fo.PHI_PERFORMER)[0]

    def loss_without_query_norm(Qx):
        tot = 0.0
        for b in range(Qx.shape[0]):
            for h in range(Qx.shape[1]):
                Kp = t["E"] @ t["K"][b, h]
                Vp = t["F"] @ t["V"][b, h]
                fk = fo.phi_performer(Kp, omega[h])
                fq = np.exp(Qx[b, h] @ omega[h].T)          # no -|q|^2/2, no 1/sqrt(m)
                out = (fq @ (fk.T @ Vp)) / (fq @ fk.sum(0))[:, None]
                tot += float(np.sum(out * G[b, h]))
        return tot

    rng = np.random.default_rng(6)
    v = rng.standard_normal(t["Q"].shape)
    h = 1e-6
    fd = (loss_without_query_norm(t["Q"] + h * v) - loss_without_query_norm(t["Q"] - h * v)) / (2 * h)
    assert abs(fd - float(np.sum(dQ * v))) < 1e-7 * max(1.0, abs(fd))


@pytest.mark.parametrize("phi", PHIS)
def test_shared_projection_gradients_add_over_batch_and_heads(phi):
    """E and F are one pair shared by every (batch, head): replicating one head
    B*H times multiplies dE and dF by B*H and leaves per-head gradients alone."""
    t, omega, G = tiny(25, B=1, H=1, phi=phi)
    one = fo.flurka_attention_bwd(t["Q"], t["K"], t["V"], t["E"], t["F"], omega, G, phi)
    rep = lambda x: np.tile(x, (2, 3, 1, 1))
    om = None if omega is None else np.tile(omega, (3, 1, 1))
    many = fo.flurka_attention_bwd(rep(t["Q"]), rep(t["K"]), rep(t["V"]), t["E"], t["F"], om, rep(G), phi)
    for a, b in zip(one[:3], many[:3]):
        assert np.max(np.abs(rep(a) - b)) < 1e-13
    for a, b in zip(one[3:], many[3:]):
        assert fo.rel_l2(b, 6 * a) < 1e-13


@pytest.mark.parametrize("phi", PHIS)
def test_value_gradient_columns_sum_rule(phi):
    """Weights of every query sum to 1.  With every row of F equal to one
    vector f, all projected values coincide (V'_r = f^T V), so out_i = f^T V
    for every query and the loss is (sum_i G_i).(V^T f): dV = f (sum_i G_i)^T."""
    t, omega, G = tiny(26, B=1, H=1, phi=phi)
    k, n = t["F"].shape
    f = np.random.default_rng(7).standard_normal(n)
    Fc = np.tile(f[None, :], (k, 1))
    dV = fo.flurka_attention_bwd(t["Q"], t["K"], t["V"], t["E"], Fc, omega, G, phi)[2]
    ref = np.outer(f, G[0, 0].sum(axis=0))
    assert np.max(np.abs(dV[0, 0] - ref)) < 1e-12


@pytest.mark.parametrize("phi", PHIS)
def test_backward_permutation_equivariance(phi):
    t, omega, G = tiny(27, phi=phi)
    base = fo.flurka_attention_bwd(t["Q"], t["K"], t["V"], t["E"], t["F"], omega, G, phi)
    p = np.random.default_rng(8).permutation(t["Q"].shape[2])
    perm = fo.flurka_attention_bwd(t["Q"], t["K"][:, :, p], t["V"][:, :, p],
                                   t["E"][:, p], t["F"][:, p], omega, G, phi)
    assert np.max(np.abs(perm[0] - base[0])) < 1e-12            # dQ unchanged
    assert np.max(np.abs(perm[1] - base[1][:, :, p])) < 1e-12   # dK rows follow
    assert np.max(np.abs(perm[2] - base[2][:, :, p])) < 1e-12
    assert np.max(np.abs(perm[3] - base[3][:, p])) < 1e-12      # dE columns follow
    assert np.max(np.abs(perm[4] - base[4][:, p])) < 1e-12


# --- variants: per-head projection pairs, gradient for omega --------------------------------------
def _variant_case(seed=70, B=2, H=3, n=7, d=3, k=4, m=5):
    rng = np.random.default_rng(seed)
    Q, K, V, G = (rng.standard_normal((B, H, n, d)) * 0.6 for _ in range(4))
    E = rng.standard_normal((H, k, n)) / np.sqrt(k)
    F = rng.standard_normal((H, k, n)) / np.sqrt(k)
    om = rng.standard_normal((H, m, d))
    return Q, K, V, E, F, om, G


def test_per_head_pairs_reduce_to_the_shared_pair():
    """H copies of one (E, F) pair give the shared-pair forward and backward; the per-head dE, dF then
    add up to the shared ones (which are sums over batch AND heads)."""
    Q, K, V, E, F, om, G = _variant_case()
    H = Q.shape[1]
    Ec, Fc = np.repeat(E[:1], H, axis=0), np.repeat(F[:1], H, axis=0)
    for phi, w in ((fo.PHI_PERFORMER, om), (fo.PHI_ELU1, None)):
        assert np.max(np.abs(fo.flurka_attention_per_head(Q, K, V, Ec, Fc, w, phi)
                             - fo.flurka_attention(Q, K, V, E[0], F[0], w, phi))) < 1e-13
        a = fo.flurka_attention_per_head_bwd(Q, K, V, Ec, Fc, w, G, phi)
        b = fo.flurka_attention_bwd(Q, K, V, E[0], F[0], w, G, phi)
        for x, y in zip(a[:3], b[:3]):
            assert np.max(np.abs(x - y)) < 1e-12
        assert np.max(np.abs(a[3].sum(axis=0) - b[3])) < 1e-12
        assert np.max(np.abs(a[4].sum(axis=0) - b[4])) < 1e-12


def test_per_head_pairs_by_central_differences():
    """Different pairs per head: dE[h], dF[h] against central differences of sum(out * G)."""
    Q, K, V, E, F, om, G = _variant_case(seed=71)
    phi = fo.PHI_PERFORMER
    g = fo.flurka_attention_per_head_bwd(Q, K, V, E, F, om, G, phi)
    loss = lambda E_, F_: float(np.sum(fo.flurka_attention_per_head(Q, K, V, E_, F_, om, phi) * G))
    rng = np.random.default_rng(1)
    h_ = 1e-6
    for _ in range(12):
        idx = tuple(rng.integers(0, s) for s in E.shape)
        for which, grad in ((0, g[3]), (1, g[4])):
            Ep, Em, Fp, Fm = E.copy(), E.copy(), F.copy(), F.copy()
            (Ep if which == 0 else Fp)[idx] += h_
            (Em if which == 0 else Fm)[idx] -= h_
            num = (loss(Ep, Fp) - loss(Em, Fm)) / (2 * h_)
            assert abs(num - grad[idx]) <= 2e-7 * max(1.0, abs(grad[idx])), (which, idx, num, grad[idx])


@pytest.mark.parametrize("shared", [False, True])
def test_omega_gradient_by_central_differences(shared):
    """Every entry of d omega against central differences; with one omega for all heads the gradient is
    the sum of the per-head ones."""
    Q, K, V, E, F, om, G = _variant_case(seed=72, B=2, H=2, n=6, d=3, k=3, m=4)
    if shared:
        om = om[:1]
    E0, F0 = E[0], F[0]
    dW = fo.flurka_attention_bwd_omega(Q, K, V, E0, F0, om, G)
    assert dW.shape == om.shape
    loss = lambda w: float(np.sum(fo.flurka_attention(Q, K, V, E0, F0, w, fo.PHI_PERFORMER) * G))
    h_ = 1e-6
    for idx in np.ndindex(*om.shape):
        wp, wm = om.copy(), om.copy()
        wp[idx] += h_
        wm[idx] -= h_
        num = (loss(wp) - loss(wm)) / (2 * h_)
        assert abs(num - dW[idx]) <= 2e-7 * max(1.0, abs(dW[idx])), (idx, num, dW[idx])
    if shared:
        per = fo.flurka_attention_bwd_omega(Q, K, V, E0, F0, np.repeat(om, Q.shape[1], axis=0), G)
        assert np.max(np.abs(per.sum(axis=0, keepdims=True) - dW)) < 1e-12
