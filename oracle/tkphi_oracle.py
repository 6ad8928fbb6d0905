"""CPU float64 oracle for Top-K+phi residual-mass decoding.  TEST INFRASTRUCTURE.

This file is the reference the HIP kernels are checked against.  It is plain
numpy in float64, written from the paper's definitions in the paper's order
and notation; it shares no code with the GPU path and must never be imported
by the product (only tests, the smoke check and the bench's CPU-baseline leg
use it).  There is no blocking, fusion or reordering here: each function is
the printed definition, with a library matmul / sort as a step.

Conventions
  * One layer at a time.  K, V are [Hkv][L][d]; q is [Hq][d]; query head g
    reads KV head g // G with G = Hq // Hkv (consecutive query heads share a
    KV head, the Llama grouping; the paper's "fixed head grouping",
    Sec. "Positive feature maps and summary states").
  * Summaries are stored feature-major: S[h][j][c] = sum_i phi_k(k_i)[j] v_i[c]
    (the transpose of the paper's d_v x d_phi S in eq. (natural_cache)),
    u[h][j] = sum_i phi_k(k_i)[j].
  * The feature map has the positive-random-feature form
        phi(x) = exp(a * W x - c * |x|^2 + b)
    (exponentiated affine output as in the paper's final layer
    phi = exp(W_o g + b_o), App. "Head-wise phi architecture", plus the norm
    term of positive random features).  W, b are per head; a, c are scalars.
  * exp(s_i) is written unshifted, exactly as the paper prints it
    (eq. (full_attention), eq. (exact_terms)); in float64 this is safe for
    |s| < ~700, far beyond any test input.

Parity pins (tests/test_oracle_pins.py): dense limit against an independent
softmax, subtraction against brute force over unretrieved tokens, positivity,
brute-force Top-K with ties, subset-bias identity, exact-subtraction identity,
partition sums, constant-feature closed form, q = 0 special case, random
feature convergence to exp(q.k/sqrt d), the paper's K = 21/144/636 worked
example, K = 0; entropy / mass-recovery diagnostics against closed forms; the residual
denominator share rho_res, the residual log-partition error and the boundary gap against the
constant-feature closed form (Z_R^ = |R|) and scalar loops over the token classes, with and
without generated tokens; the MLP feature map against the printed per-head parameter counts,
its alpha = 0 and W1 = 0 reductions and GeLU's defining values.  Parity unpinned: nothing in this file; the *quality* of the
estimate for the synthetic random-feature phi has no published value and is
reported as a diagnostic only.
"""
from __future__ import annotations

import math

import numpy as np

F64 = np.float64


# ---------------------------------------------------------------------------
# budgets
# ---------------------------------------------------------------------------
def budget_paper(L: int, r_bp: int, n_sink: int, n_tail: int) -> int:
    """K = max(0, ceil(r L) - |A|): anchors count toward the total exact-support
    budget r (Sec. "Models, tasks, and protocol").  r is given in basis points
    so the ceiling is taken in exact integer arithmetic."""
    n_anchor = min(L, n_sink + n_tail)
    ceil_rL = -((-r_bp * L) // 10000)
    return max(0, ceil_rL - n_anchor)


def budget_mid(L: int, r_bp: int, n_sink: int, n_tail: int) -> int:
    """K = floor(r |M|): budget as a fraction of the mid-region (the synthetic
    workloads' convention, e.g. 1 % of 4028 mid tokens -> 40)."""
    n_mid = max(0, L - n_sink - n_tail)
    return (r_bp * n_mid) // 10000


# ---------------------------------------------------------------------------
# index sets, eq. (partition)
# ---------------------------------------------------------------------------
def partition(L: int, n_sink: int, n_tail: int):
    """A = {0..n_sink-1} U {L-n_tail..L-1},  M = {n_sink..L-n_tail-1}.
    If the two anchor ranges would overlap, every token is an anchor."""
    if n_sink + n_tail >= L:
        return np.arange(L, dtype=np.int64), np.zeros(0, dtype=np.int64)
    A = np.concatenate([np.arange(0, n_sink), np.arange(L - n_tail, L)]).astype(np.int64)
    M = np.arange(n_sink, L - n_tail, dtype=np.int64)
    return A, M


# ---------------------------------------------------------------------------
# feature map
# ---------------------------------------------------------------------------
def phi(x, W, b, a, c):
    """phi(x) = exp(a W x - c |x|^2 + b) for rows x [n][d]; W [dphi][d], b [dphi].
    Returns [n][dphi], strictly positive."""
    x = np.atleast_2d(np.asarray(x, dtype=F64))
    W = np.asarray(W, dtype=F64)
    b = np.asarray(b, dtype=F64)
    sq = np.sum(x * x, axis=1, keepdims=True)
    return np.exp(F64(a) * (x @ W.T) - F64(c) * sq + b[None, :])


def gelu(x):
    """GeLU(x) = x Phi(x) with the exact Gaussian cdf, Phi(x) = (1 + erf(x / sqrt 2)) / 2."""
    from scipy.special import erf
    x = np.asarray(x, dtype=F64)
    return 0.5 * x * (1.0 + erf(x / math.sqrt(2.0)))


def phi_mlp(x, P):
    """The head-wise one-block ReZero MLP feature map (App. "Head-wise phi architecture"):
        g0 = Ws x + bs;  Delta = W2 GeLU(W1 g0 + b1) + b2;  g1 = g0 + alpha Delta;
        phi(x) = exp(Wo g1 + bo)
    for rows x [n][d]; P holds one head's Ws [E][d], bs [E], W1, W2 [E][E], b1, b2 [E],
    alpha (scalar), Wo [dphi][E], bo [dphi].  Returns [n][dphi], strictly positive."""
    x = np.atleast_2d(np.asarray(x, dtype=F64))
    g0 = x @ np.asarray(P["Ws"], dtype=F64).T + np.asarray(P["bs"], dtype=F64)
    hid = gelu(g0 @ np.asarray(P["W1"], dtype=F64).T + np.asarray(P["b1"], dtype=F64))
    delta = hid @ np.asarray(P["W2"], dtype=F64).T + np.asarray(P["b2"], dtype=F64)
    g1 = g0 + F64(P["alpha"]) * delta
    return np.exp(g1 @ np.asarray(P["Wo"], dtype=F64).T + np.asarray(P["bo"], dtype=F64))


def mlp_param_count(d, d_emb, dphi):
    """Parameters of one head's map as printed in the architecture equations: the four affine
    layers and the scalar alpha."""
    return (d_emb * d + d_emb) + 2 * (d_emb * d_emb + d_emb) + (dphi * d_emb + dphi) + 1


# ---------------------------------------------------------------------------
# prefill: summary states, eq. (natural_cache)
# ---------------------------------------------------------------------------
def build_summaries(K, V, Wk, bk, a, c, n_sink, n_tail, phi_k_fns=None, n_gen=0):
    """S_M[h] = sum_{i in M} phi_k(k_i) v_i^T  ([dphi][d]),  u_M[h] = sum_{i in M} phi_k(k_i).
    phi_k_fns: optional list of per-KV-head feature maps (rows -> features) used instead of
    the exp-affine map (Wk, bk, a, c).  n_gen: the last n_gen rows of K, V are generated tokens,
    not part of the prefill segment the partition is defined on."""
    K = np.asarray(K, dtype=F64)
    V = np.asarray(V, dtype=F64)
    Hkv, L, d = K.shape
    L -= int(n_gen)
    _, M = partition(L, n_sink, n_tail)
    feat = (lambda h, x: phi(x, Wk[h], bk[h], a, c)) if phi_k_fns is None else (lambda h, x: phi_k_fns[h](x))
    dphi = feat(0, K[0, :1]).shape[1]
    S = np.zeros((Hkv, dphi, d), dtype=F64)
    u = np.zeros((Hkv, dphi), dtype=F64)
    for h in range(Hkv):
        if M.size == 0:
            continue
        f = feat(h, K[h, M])                          # [|M|][dphi]
        S[h] = f.T @ V[h, M]
        u[h] = f.sum(axis=0)
    return S, u


# ---------------------------------------------------------------------------
# decode
# ---------------------------------------------------------------------------
def scores(q_g, K_h, scale):
    """s_i = q^T k_i / sqrt(d_h) for every prefill token (eq. (full_attention));
    `scale` is the float32-valued 1/sqrt(d_h) both implementations are given."""
    return F64(scale) * (np.asarray(K_h, dtype=F64) @ np.asarray(q_g, dtype=F64))


def topk_mid(s, M, k):
    """Exhaustive Top-K over the mid-region: the k highest-scoring tokens of M
    (Sec. "Models, tasks, and protocol").  Ties go to the lower token index.
    A full sort, no selection trick.  Returns indices ordered best-first."""
    k = min(int(k), M.size)
    if k <= 0:
        return np.zeros(0, dtype=np.int64)
    order = np.lexsort((M, -s[M]))        # primary key: score descending; then index ascending
    return M[order[:k]]


def full_attention(q_g, K_h, V_h, scale):
    """y_full = sum_i exp(s_i) v_i / sum_i exp(s_i), eq. (full_attention)."""
    s = scores(q_g, K_h, scale)
    w = np.exp(s)
    return (w @ np.asarray(V_h, dtype=F64)) / w.sum()


def decode_head(q_g, K_h, V_h, S_M, u_M, Wq_g, bq_g, Wk_h, bk_h, a, c, scale,
                n_sink, n_tail, k, retrieved=None, phi_q_fn=None, phi_k_fn=None, n_gen=0):
    """One query head.  Returns a dict with the Top-K+phi output `y`, every
    intermediate of the method and the paper's comparison estimators.

    `retrieved`: optional explicit retrieved set (token indices in M) to use
    instead of the Top-K selection (for accounting checks under a fixed set,
    Sec. "Analysis: validating residual accounting").
    `phi_q_fn`, `phi_k_fn`: optional feature maps (rows -> features) of this query head / its KV
    head, used instead of the exp-affine maps (Wq_g, bq_g) / (Wk_h, bk_h).
    `n_gen`: the last n_gen rows of K_h, V_h are the generated-token prefix G: exact, outside the
    partition of the prefill segment, added to the same numerator and denominator
    (eq. (implemented_decode)); with n_gen = 0 every output is that of eq. (hybrid_merge).
    """
    K_h = np.asarray(K_h, dtype=F64)
    V_h = np.asarray(V_h, dtype=F64)
    n_gen = int(n_gen)
    L = K_h.shape[0] - n_gen                           # prefill segment
    A, M = partition(L, n_sink, n_tail)
    Gset = np.arange(L, L + n_gen, dtype=np.int64)

    s = scores(q_g, K_h, scale)
    if retrieved is None:
        Kset = topk_mid(s, M, k)
    else:
        Kset = np.asarray(retrieved, dtype=np.int64)
    inK = np.zeros(L + n_gen, dtype=bool)
    inK[Kset] = True
    Rset = M[~inK[M]]                                  # R = M \ K
    Eset = np.concatenate([A, Kset])                   # E = A U K

    e = np.exp(s)
    # exact-support terms, eq. (exact_terms)
    nu_E = e[Eset] @ V_h[Eset]
    Z_E = e[Eset].sum()

    # feature maps: query, and retrieved keys recomputed (Sec. "Retrieved-token subtraction")
    fq = (lambda x: phi(x, Wq_g, bq_g, a, c)) if phi_q_fn is None else phi_q_fn
    fk = (lambda x: phi(x, Wk_h, bk_h, a, c)) if phi_k_fn is None else phi_k_fn
    p = fq(q_g)[0]                                     # phi_q(q)  [dphi]
    f_K = fk(K_h[Kset]) if Kset.size else np.zeros((0, p.size))

    # subtraction, eq. (subtraction), materialised
    S_R = np.asarray(S_M, dtype=F64) - f_K.T @ V_h[Kset]
    u_R = np.asarray(u_M, dtype=F64) - f_K.sum(axis=0)

    # residual completion and single-normalisation merge, eq. (hybrid_merge)
    nu_R_hat = S_R.T @ p
    Z_R_hat = p @ u_R
    # generated tokens: another exact branch under the same normalisation, eq. (implemented_decode)
    nu_G, Z_G = e[Gset] @ V_h[Gset], e[Gset].sum()
    y = (nu_E + nu_R_hat + nu_G) / (Z_E + Z_R_hat + Z_G)

    # ---- comparison estimators and diagnostics --------------------------
    nu_M_hat = np.asarray(S_M, dtype=F64).T @ p        # un-subtracted mid estimates
    Z_M_hat = p @ np.asarray(u_M, dtype=F64)
    nu_A, Z_A = e[A] @ V_h[A], e[A].sum()
    nu_K, Z_K = e[Kset] @ V_h[Kset], e[Kset].sum()
    nu_R, Z_R = e[Rset] @ V_h[Rset], e[Rset].sum()
    nu_M, Z_M = e[M] @ V_h[M], e[M].sum()
    y_full = (e @ V_h) / e.sum()
    out = {
        "y": y, "idx": Kset, "s": s,
        "nu_E": nu_E, "Z_E": Z_E, "nu_G": nu_G, "Z_G": Z_G, "p": p, "f_K": f_K,
        "S_R": S_R, "u_R": u_R, "nu_R_hat": nu_R_hat, "Z_R_hat": Z_R_hat,
        "nu_M_hat": nu_M_hat, "Z_M_hat": Z_M_hat,
        "nu_A": nu_A, "Z_A": Z_A, "nu_K": nu_K, "Z_K": Z_K,
        "nu_R": nu_R, "Z_R": Z_R, "nu_M": nu_M, "Z_M": Z_M,
        "y_full": y_full,
        "y_topk": (nu_E + nu_G) / (Z_E + Z_G),                           # selection-only Top-K
        "y_nosub": (nu_E + nu_M_hat + nu_G) / (Z_E + Z_M_hat + Z_G),     # NoSub ablation
        "y_exactsub": (nu_E + nu_R + nu_G) / (Z_E + Z_R + Z_G),          # eq. (exact_sub_oracle)
        "y_exactnosub": (nu_E + nu_M + nu_G) / (Z_E + Z_M + Z_G),        # eq. (exact_nosub_oracle)
        "rho_res": Z_R_hat / (Z_E + Z_G + Z_R_hat),                      # residual denominator share
        "log_Z_err": (math.log(Z_R_hat) - math.log(Z_R)) if (Z_R_hat > 0 and Z_R > 0) else float("nan"),
    }
    # entropy / mass-recovery diagnostics (Sec. "Analysis: entropy and completion gains";
    # App. "Entropy, mass recovery, and residual-denominator diagnostics")
    if M.size > 0:
        p_mid = e[M] / Z_M                                               # mid-normalised distribution
        ent = -float(np.sum(p_mid * np.log(p_mid)))
        out["H_mid"] = ent / math.log(M.size) if M.size > 1 else 0.0     # normalised entropy
        out["C_mid"] = Z_K / Z_M                                         # mid mass recovered by Top-K
        out["rho_res_star"] = Z_R / (Z_A + Z_M + Z_G)                    # true residual share
    if Kset.size < M.size and Kset.size > 0 and retrieved is None:
        srt = np.sort(s[M])[::-1]
        out["boundary_gap"] = srt[Kset.size - 1] - srt[Kset.size]
    return out


def rel_l1(y_hat, y_ref):
    """|y_hat - y_ref|_1 / (|y_ref|_1 + 1e-12), the paper's attention-output error
    (Sec. "Analysis: entropy and completion gains")."""
    y_hat = np.asarray(y_hat, dtype=F64)
    y_ref = np.asarray(y_ref, dtype=F64)
    return np.abs(y_hat - y_ref).sum() / (np.abs(y_ref).sum() + 1e-12)


def decode_layer(q, K, V, S, u, Wq, bq, Wk, bk, a, c, scale, n_sink, n_tail, k,
                 heads=None, retrieved=None, phi_q_fns=None, phi_k_fns=None, n_gen=0):
    """All (or the listed) query heads of one layer; returns a list of per-head dicts."""
    Hq = np.asarray(q).shape[0]
    Hkv = np.asarray(K).shape[0]
    G = Hq // Hkv
    res = []
    for g in (range(Hq) if heads is None else heads):
        h = g // G
        res.append(decode_head(q[g], K[h], V[h], S[h], u[h],
                               None if Wq is None else Wq[g], None if bq is None else bq[g],
                               None if Wk is None else Wk[h], None if bk is None else bk[h],
                               a, c, scale, n_sink, n_tail, k,
                               retrieved=None if retrieved is None else retrieved[g],
                               phi_q_fn=None if phi_q_fns is None else phi_q_fns[g],
                               phi_k_fn=None if phi_k_fns is None else phi_k_fns[h], n_gen=n_gen))
    return res
