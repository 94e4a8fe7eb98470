"""fp64 CPU oracle for FLuRKA attention -- TEST INFRASTRUCTURE ONLY.

Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may
import this module.  It shares no code with the HIP library and never calls
it; the library never calls this.

What it computes (one attention head; B and H are plain batch axes):

    K' = E K,  V' = F V                      sequence projection n -> k
    out = phi(Q) (phi(K')^T V')  /  phi(Q) (phi(K')^T 1)

Structure: Eq. 2 (optimised unification: project the keys and values along
the sequence first, then kernelise).  E, F in R^{k x n} as in Sec. 2,
"Low-rank Methods" (there d_k x N).  The product order phi(Q)(phi(K)^T V)
is the one of Sec. 2, "Kernel Methods".  Eq. 2 as printed leaves out the
transpose and the row normaliser; the normalised ratio is the form the
accuracy proof works with (App. D, where each attention entry is
phi(x_i)^T phi(y_j) / sum_k phi(x_i)^T phi(y_k)), and it is what is
implemented here.

Feature maps (Sec. 2, "Kernel Methods"):
  * random-feature map phi(x) = m^{-1/2} [psi_1(x) .. psi_m(x)] with
    E[psi_j(x) psi_j(y)] = exp(x.y).  The paper states only this property;
    the concrete positive random features used here are
    psi_j(x) = exp(omega_j.x - |x|^2/2) with omega_j ~ N(0, I_d), which has
    exactly that expectation (pinned by a Monte-Carlo test and by the
    m -> infinity limit of Thm. 1's proof sketch).
  * the non-random map of the RNN variant: phi(x) = elu(x) + 1 elementwise.

The method reaches an exactly defined result (re-associating the product
changes cost, not value), so `flurka_attention_definition` is that
definition written out.  `flurka_attention` evaluates the same ratio with
the exponents shifted (one constant per head on the key side, one per query
row on the query side).  Both shifts cancel in the ratio; they only keep
exp() inside the fp64 range for the long-sequence workloads, where
|k'|^2/2 reaches several hundred.

The backward pass is not printed in the paper; it is the chain rule applied
to the forward above, and is pinned by central finite differences.

Parity pins for every function here live in tests/test_oracle_*.py.
"""
from __future__ import annotations

import numpy as np

PHI_PERFORMER = "performer"
PHI_ELU1 = "elu1"


# --------------------------------------------------------------------------
# building blocks
# --------------------------------------------------------------------------
def sequence_projection(E: np.ndarray, X: np.ndarray) -> np.ndarray:
    """(E_1 K) resp. (E_2 V) of Eq. 2: contract the sequence axis n -> k.

    E: (k, n); X: (..., n, d) -> (..., k, d).
    """
    return np.matmul(np.asarray(E, np.float64), np.asarray(X, np.float64))


def phi_performer(X: np.ndarray, omega: np.ndarray) -> np.ndarray:
    """Positive random features (Sec. 2, "Kernel Methods"; Thm. 1 statement).

    X: (..., d); omega: (m, d) -> (..., m), every entry > 0.
    """
    X = np.asarray(X, np.float64)
    omega = np.asarray(omega, np.float64)
    m = omega.shape[0]
    sq = 0.5 * np.sum(X * X, axis=-1, keepdims=True)
    return np.exp(X @ omega.T - sq) / np.sqrt(m)


def phi_elu1(X: np.ndarray) -> np.ndarray:
    """elu(x) + 1, alpha = 1, elementwise (the RNN variant's kernel, Sec. 2)."""
    X = np.asarray(X, np.float64)
    return np.where(X > 0.0, X + 1.0, np.exp(np.minimum(X, 0.0)))


def _phi_elu1_grad(X: np.ndarray) -> np.ndarray:
    X = np.asarray(X, np.float64)
    return np.where(X > 0.0, 1.0, np.exp(np.minimum(X, 0.0)))


def _head_omega(omega, h):
    """omega is (H, m, d) (one draw per head) or (1, m, d) (shared)."""
    if omega is None:
        return None
    omega = np.asarray(omega, np.float64)
    if omega.ndim == 2:
        return omega
    return omega[h if omega.shape[0] > 1 else 0]


# --------------------------------------------------------------------------
# forward: the definition
# --------------------------------------------------------------------------
def flurka_head_definition(Q, K, V, E, F, omega, phi):
    """One head, straight from the definition (no exponent shifting).

    Q, K, V: (n, d); E, F: (k, n); omega: (m, d) or None -> out (n, d).
    """
    Kp = sequence_projection(E, K)
    Vp = sequence_projection(F, V)
    if phi == PHI_PERFORMER:
        PQ = phi_performer(Q, omega)
        PK = phi_performer(Kp, omega)
    elif phi == PHI_ELU1:
        PQ = phi_elu1(Q)
        PK = phi_elu1(Kp)
    else:
        raise ValueError(phi)
    S = PK.T @ Vp                      # (m, d)   phi(K')^T V'
    z = PK.sum(axis=0)                 # (m,)     phi(K')^T 1
    return (PQ @ S) / (PQ @ z)[:, None]


def flurka_attention_definition(Q, K, V, E, F, omega, phi):
    """All heads of `flurka_head_definition`.  Q, K, V: (B, H, n, d)."""
    Q = np.asarray(Q, np.float64)
    B, H = Q.shape[:2]
    out = np.empty_like(Q)
    for b in range(B):
        for h in range(H):
            out[b, h] = flurka_head_definition(Q[b, h], K[b, h], V[b, h], E, F,
                                               _head_omega(omega, h), phi)
    return out


# --------------------------------------------------------------------------
# forward: same value, exponents shifted into range
# --------------------------------------------------------------------------
def key_state(Kp, Vp, omega, phi):
    """Key-side state of one head.

    Returns (PhiK, S, z, c): PhiK (k, m) = phi(K') up to the positive factor
    exp(-c)/sqrt(m) (performer) or exactly phi(K') with c = 0 (elu1);
    S = PhiK^T V' (m, d); z = PhiK^T 1 (m,).
    """
    Kp = np.asarray(Kp, np.float64)
    Vp = np.asarray(Vp, np.float64)
    if phi == PHI_PERFORMER:
        e = Kp @ omega.T - 0.5 * np.sum(Kp * Kp, axis=1, keepdims=True)
        c = float(e.max())
        PhiK = np.exp(e - c)
    elif phi == PHI_ELU1:
        c = 0.0
        PhiK = phi_elu1(Kp)
    else:
        raise ValueError(phi)
    return PhiK, PhiK.T @ Vp, PhiK.sum(axis=0), c


def query_features(Q, omega, phi):
    """phi(Q) of one head up to a positive factor per row (performer) or exactly (elu1)."""
    Q = np.asarray(Q, np.float64)
    if phi == PHI_PERFORMER:
        u = Q @ omega.T
        return np.exp(u - u.max(axis=1, keepdims=True))
    if phi == PHI_ELU1:
        return phi_elu1(Q)
    raise ValueError(phi)


def flurka_head(Q, K, V, E, F, omega, phi, rows=None):
    """One head, range-safe.  `rows` optionally restricts the query rows."""
    Kp = sequence_projection(E, K)
    Vp = sequence_projection(F, V)
    _, S, z, _ = key_state(Kp, Vp, omega, phi)
    Qs = np.asarray(Q, np.float64)
    if rows is not None:
        Qs = Qs[rows]
    P = query_features(Qs, omega, phi)
    return (P @ S) / (P @ z)[:, None]


def flurka_attention(Q, K, V, E, F, omega, phi, rows=None):
    """FLuRKA attention forward for all heads.

    Q, K, V: (B, H, n, d); E, F: (k, n); omega: (H|1, m, d) or None.
    Returns out (B, H, n, d), or (B, H, len(rows), d) when `rows` (an index
    array into the query axis) is given.
    """
    Q = np.asarray(Q, np.float64)
    B, H, n, d = Q.shape
    nr = n if rows is None else len(rows)
    out = np.empty((B, H, nr, d), np.float64)
    for b in range(B):
        for h in range(H):
            out[b, h] = flurka_head(Q[b, h], K[b, h], V[b, h], E, F,
                                    _head_omega(omega, h), phi, rows)
    return out


# --------------------------------------------------------------------------
# forward with the linear transforms in the order Eq. 2 prints them
# --------------------------------------------------------------------------
def flurka_attention_paper_order(Q, XK, XV, E, F, WK, WV, omega, phi):
    """Eq. 2 read literally: phi(Q W^Q) (phi((E_1 K) W^K)^T ((E_2 V) W^V)), row-normalised.

    The sequence projection acts on the model-wide layer inputs, the per-head
    transform on the k projected rows (App. B lists the steps in this order:
    "low-rank downsampling products E_1 K & E_2 V", then the linear
    transformations).  Q: (B, H, n, d), already transformed; XK, XV: (B, n, dm);
    WK, WV: (H, d, dm), head h's (dm x d) transform stored transposed;
    E, F: (k, n).  Returns out (B, H, n, d).
    """
    Q = np.asarray(Q, np.float64)
    B, H, n, d = Q.shape
    out = np.empty_like(Q)
    for b in range(B):
        YK = sequence_projection(E, XK[b])          # (k, dm)
        YV = sequence_projection(F, XV[b])
        for h in range(H):
            Kp = YK @ np.asarray(WK[h], np.float64).T    # (k, d)
            Vp = YV @ np.asarray(WV[h], np.float64).T
            om = _head_omega(omega, h)
            _, S, z, _ = key_state(Kp, Vp, om, phi)
            P = query_features(Q[b, h], om, phi)
            out[b, h] = (P @ S) / (P @ z)[:, None]
    return out


# --------------------------------------------------------------------------
# the two constituents (comparison baselines)
# --------------------------------------------------------------------------
def kernel_attention(Q, K, V, omega, phi):
    """Kernel attention of Sec. 2, "Kernel Methods": phi(Q) (phi(K)^T V), each row divided by
    phi(Q) (phi(K)^T 1) -- the method without a sequence projection.  Q, K, V: (B, H, n, d)."""
    Q = np.asarray(Q, np.float64)
    B, H = Q.shape[:2]
    out = np.empty_like(Q)
    for b in range(B):
        for h in range(H):
            om = _head_omega(omega, h)
            _, S, z, _ = key_state(K[b, h], V[b, h], om, phi)
            P = query_features(Q[b, h], om, phi)
            out[b, h] = (P @ S) / (P @ z)[:, None]
    return out


def linformer_attention(Q, K, V, E, F):
    """Low-rank attention of Sec. 2, "Low-rank Methods": softmax(Q (E K)^T) (F V), the softmax taken
    over the k projected keys, no temperature.  Q, K, V: (B, H, n, d); E, F: (k, n)."""
    Q = np.asarray(Q, np.float64)
    B, H = Q.shape[:2]
    out = np.empty_like(Q)
    for b in range(B):
        for h in range(H):
            Kp = sequence_projection(E, K[b, h])
            Vp = sequence_projection(F, V[b, h])
            s = Q[b, h] @ Kp.T
            a = np.exp(s - s.max(axis=1, keepdims=True))
            out[b, h] = (a / a.sum(axis=1, keepdims=True)) @ Vp
    return out


# --------------------------------------------------------------------------
# backward (chain rule of the forward above)
# --------------------------------------------------------------------------
def flurka_head_bwd(Q, K, V, E, F, omega, G, phi):
    """Gradients of sum(out * G) for one head.

    Returns dQ, dK, dV (n, d) and this head's contribution dE_h, dF_h (k, n).
    With N = P S, D = P z, out = N / D (P, S, z from the range-safe forward;
    the shifts are constants whose true derivative is zero because `out` does
    not depend on them):
        dN = G / D                 dD = -(G . out) / D        (row-wise)
        dP = dN S^T + dD z^T       dS = P^T dN                dz = P^T dD
        dPhiK = V' dS^T + 1 dz^T   dV' = PhiK dS
      performer: with U = x omega^T - |x|^2/2 feeding exp,
        dU = dphi * phi,  dx = dU omega - rowsum(dU) x
      elu1:  dx = dphi * phi'(x)
        dK = E^T dK'   dV = F^T dV'   dE_h = dK' K^T   dF_h = dV' V^T
    """
    Q = np.asarray(Q, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    E = np.asarray(E, np.float64)
    F = np.asarray(F, np.float64)
    G = np.asarray(G, np.float64)
    Kp = sequence_projection(E, K)
    Vp = sequence_projection(F, V)
    PhiK, S, z, _ = key_state(Kp, Vp, omega, phi)
    P = query_features(Q, omega, phi)
    D = P @ z
    out = (P @ S) / D[:, None]

    dN = G / D[:, None]
    dD = -np.sum(G * out, axis=1) / D
    dP = dN @ S.T + np.outer(dD, z)
    dS = P.T @ dN
    dz = P.T @ dD
    dPhiK = Vp @ dS.T + dz[None, :]
    dVp = PhiK @ dS

    if phi == PHI_PERFORMER:
        dUq = dP * P
        dQ = dUq @ omega - dUq.sum(axis=1, keepdims=True) * Q
        dUk = dPhiK * PhiK
        dKp = dUk @ omega - dUk.sum(axis=1, keepdims=True) * Kp
    elif phi == PHI_ELU1:
        dQ = dP * _phi_elu1_grad(Q)
        dKp = dPhiK * _phi_elu1_grad(Kp)
    else:
        raise ValueError(phi)

    dK = E.T @ dKp
    dV = F.T @ dVp
    dE = dKp @ K.T
    dF = dVp @ V.T
    return dQ, dK, dV, dE, dF


def flurka_attention_bwd(Q, K, V, E, F, omega, dOut, phi):
    """Backward for all heads.  dE, dF are summed over batch and heads
    because one (E, F) pair is shared by all of them."""
    Q = np.asarray(Q, np.float64)
    B, H, n, d = Q.shape
    k = np.asarray(E).shape[0]
    dQ = np.empty_like(Q)
    dK = np.empty_like(Q)
    dV = np.empty_like(Q)
    dE = np.zeros((k, n), np.float64)
    dF = np.zeros((k, n), np.float64)
    for b in range(B):
        for h in range(H):
            g = flurka_head_bwd(Q[b, h], K[b, h], V[b, h], E, F,
                                _head_omega(omega, h), dOut[b, h], phi)
            dQ[b, h], dK[b, h], dV[b, h] = g[0], g[1], g[2]
            dE += g[3]
            dF += g[4]
    return dQ, dK, dV, dE, dF


# --------------------------------------------------------------------------
# variants: one projection pair per head (Thm. 1 writes E_i, F_i), gradient for omega
# --------------------------------------------------------------------------
def flurka_attention_per_head(Q, K, V, E, F, omega, phi):
    """Forward with E, F of shape (H, k, n): head h projects with its own pair E[h], F[h]."""
    Q = np.asarray(Q, np.float64)
    B, H = Q.shape[:2]
    out = np.empty_like(Q)
    for b in range(B):
        for h in range(H):
            out[b, h] = flurka_head(Q[b, h], K[b, h], V[b, h], E[h], F[h], _head_omega(omega, h), phi)
    return out


def flurka_attention_per_head_bwd(Q, K, V, E, F, omega, dOut, phi):
    """Backward of `flurka_attention_per_head`: dE, dF are (H, k, n), summed over the batch only."""
    Q = np.asarray(Q, np.float64)
    B, H = Q.shape[:2]
    dQ, dK, dV = np.empty_like(Q), np.empty_like(Q), np.empty_like(Q)
    dE = np.zeros(np.asarray(E).shape, np.float64)
    dF = np.zeros(np.asarray(F).shape, np.float64)
    for b in range(B):
        for h in range(H):
            g = flurka_head_bwd(Q[b, h], K[b, h], V[b, h], E[h], F[h], _head_omega(omega, h), dOut[b, h], phi)
            dQ[b, h], dK[b, h], dV[b, h] = g[0], g[1], g[2]
            dE[h] += g[3]
            dF[h] += g[4]
    return dQ, dK, dV, dE, dF


def flurka_head_bwd_omega(Q, K, V, E, F, omega, G):
    """d sum(out * G) / d omega for one head of the random-feature map, (m, d).

    omega enters through the exponents u_ij = omega_j . q_i - |q_i|^2/2 of phi(Q) and
    e_rj = omega_j . k'_r - |k'_r|^2/2 of phi(K'):  d omega_j = sum_i dU^Q_ij q_i + sum_r dU^K_rj k'_r,
    with dU = dphi * phi on either side (notation of `flurka_head_bwd`)."""
    Q = np.asarray(Q, np.float64)
    G = np.asarray(G, np.float64)
    omega = np.asarray(omega, np.float64)
    Kp = sequence_projection(E, K)
    Vp = sequence_projection(F, V)
    PhiK, S, z, _ = key_state(Kp, Vp, omega, PHI_PERFORMER)
    P = query_features(Q, omega, PHI_PERFORMER)
    D = P @ z
    out = (P @ S) / D[:, None]
    dN = G / D[:, None]
    dD = -np.sum(G * out, axis=1) / D
    dUq = (dN @ S.T + np.outer(dD, z)) * P
    dS = P.T @ dN
    dz = P.T @ dD
    dUk = (Vp @ dS.T + dz[None, :]) * PhiK
    return dUq.T @ Q + dUk.T @ Kp


def flurka_attention_bwd_omega(Q, K, V, E, F, omega, dOut):
    """Gradient for omega over all heads: (H, m, d), or (1, m, d) summed over heads when omega is shared.
    E, F: (k, n) shared or (H, k, n) per head."""
    Q = np.asarray(Q, np.float64)
    B, H = Q.shape[:2]
    omega = np.asarray(omega, np.float64)
    per_head_ef = np.asarray(E).ndim == 3
    dW = np.zeros_like(omega)
    for b in range(B):
        for h in range(H):
            Eh, Fh = (E[h], F[h]) if per_head_ef else (E, F)
            g = flurka_head_bwd_omega(Q[b, h], K[b, h], V[b, h], Eh, Fh, _head_omega(omega, h), dOut[b, h])
            dW[h if omega.shape[0] > 1 else 0] += g
    return dW


# --------------------------------------------------------------------------
# error metric
# --------------------------------------------------------------------------
def rel_l2(x, ref) -> float:
    """|x - ref|_F / |ref|_F over the whole tensor, in fp64."""
    x = np.asarray(x, np.float64)
    ref = np.asarray(ref, np.float64)
    den = float(np.linalg.norm(ref.ravel()))
    num = float(np.linalg.norm((x - ref).ravel()))
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / den
