"""Comparison of the HIP path's results with the CPU oracle, element by element.

Tolerances (the bar the path is held to):
  * scores            |gpu - oracle| <= 1e-5 * max(1, |oracle|)
  * Top-K index sets  identical, except that tokens may be exchanged across the selection
                      boundary when their oracle scores lie within 1e-5 * max(1, |s_K|) of
                      the K-th score s_K; when that happens the output (and the unnormalised
                      terms) are checked against the oracle re-run on the GPU's set
  * outputs y         max-abs <= 2e-3 and relative l1 <= 1e-2 per query head
  * summaries S, u    fp32 storage: relative Frobenius error <= 2e-5.  bf16 storage (matrix-core
                      path, features carried as a bf16 hi + lo pair): element-wise
                      |dS[j][c]| <= eps * sum_i phi_ij |v_ic|, |du[j]| <= eps * u[j],
                      eps = 2^-16 + 2^-17 (see check_summaries)
"""
from __future__ import annotations

import numpy as np

from oracle import tkphi_oracle as orc
from paper_2604_05438_amd import inputs as I

Y_MAX_ABS = 2e-3
Y_REL_L1 = 1e-2
SCORE_TOL = 1e-5
SWAP_TOL = 1e-5


def oracle_inputs(P: dict) -> dict:
    """float64 copies of a layer's tensors; K, V cut to the rows the problem uses (prefill length P["L"] plus
    P["n_gen"] generated tokens: the buffers may hold rows of later steps)."""
    O = {k: I.to_f64(P[k]) for k in ("q", "K", "V", "Wq", "Wk", "bq", "bk")}
    rows = int(P["L"]) + int(P.get("n_gen", 0))
    O["K"], O["V"] = O["K"][:, :rows], O["V"][:, :rows]
    return O


def mlp_feature_fns(P: dict):
    """(phi_q_fns, phi_k_fns) of a layer that carries MLP feature maps under P["mlp"]
    (inputs.make_mlp_phi), else (None, None): the exp-affine map of Wq / Wk applies."""
    if "mlp" not in P:
        return None, None

    def head_fns(side):
        T = {k: I.to_f64(v) for k, v in P["mlp"][side].items()}
        return [(lambda x, hh=hh: orc.phi_mlp(x, {k: v[hh] for k, v in T.items()})) for hh in range(T["alpha"].shape[0])]

    return head_fns("q"), head_fns("k")


def oracle_layer(w, P, k, heads=None, S=None, u=None, retrieved=None):
    O = oracle_inputs(P)
    fq, fk = mlp_feature_fns(P)
    O["phi_k_fns"] = fk
    O["n_gen"] = int(P.get("n_gen", 0))
    n_gen = int(P.get("n_gen", 0))                     # generated tokens: the last n_gen rows of K, V
    if S is None:
        S, u = orc.build_summaries(O["K"], O["V"], O["Wk"], O["bk"], w.phi_in_scale, w.phi_norm_coef,
                                   w.n_sink, w.n_tail, phi_k_fns=fk, n_gen=n_gen)
    res = orc.decode_layer(O["q"], O["K"], O["V"], S, u, O["Wq"], O["bq"], O["Wk"], O["bk"],
                           w.phi_in_scale, w.phi_norm_coef, w.score_scale, w.n_sink, w.n_tail, k,
                           heads=heads, retrieved=retrieved, phi_q_fns=fq, phi_k_fns=fk, n_gen=n_gen)
    return res, S, u, O


def check_scores(gpu_scores_row: np.ndarray, r: dict, n_sink: int, n_mid: int):
    s_or = r["s"][n_sink:n_sink + n_mid]
    err = np.abs(gpu_scores_row[:n_mid].astype(np.float64) - s_or)
    tol = SCORE_TOL * np.maximum(1.0, np.abs(s_or))
    assert (err <= tol).all(), f"score mismatch: max err {err.max():.3e} (tol {tol.min():.1e})"


def check_index_set(gpu_idx: np.ndarray, r: dict, n_sink: int, n_mid: int) -> bool:
    """Returns True if the set equals the oracle's exactly, False if it differs only by
    admissible boundary swaps; asserts otherwise."""
    k = r["idx"].size
    got = np.asarray(gpu_idx[:k], dtype=np.int64)
    assert (got >= n_sink).all() and (got < n_sink + n_mid).all(), "index outside the mid-region"
    assert np.unique(got).size == k, "duplicate retrieved index"
    assert (np.diff(got) > 0).all(), "retrieved indices not ascending"
    want = np.sort(r["idx"])
    if np.array_equal(got, want):
        return True
    s = r["s"]
    s_k = s[r["idx"][-1]]                      # K-th best oracle score
    tol = SWAP_TOL * max(1.0, abs(s_k))
    only_gpu = np.setdiff1d(got, want)
    only_or = np.setdiff1d(want, got)
    assert only_gpu.size == only_or.size
    assert (np.abs(s[only_gpu] - s_k) <= tol).all() and (np.abs(s[only_or] - s_k) <= tol).all(), \
        f"index sets differ beyond boundary swaps: gpu-only {only_gpu[:8]}, oracle-only {only_or[:8]}"
    return False


def check_output(y_gpu: np.ndarray, y_or: np.ndarray, what="y"):
    y_gpu = y_gpu.astype(np.float64)
    assert np.isfinite(y_gpu).all(), f"{what}: non-finite output"
    max_abs = np.abs(y_gpu - y_or).max()
    rel = orc.rel_l1(y_gpu, y_or)
    assert max_abs <= Y_MAX_ABS and rel <= Y_REL_L1, f"{what}: max-abs {max_abs:.3e}, rel-l1 {rel:.3e}"
    return max_abs, rel


MLP_FEATURE_EPS = 2.0 ** -12


def check_summaries(S_gpu, u_gpu, S_or, u_or, tol, w=None, O=None, eps=None):
    """fp32 storage: relative Frobenius error <= tol.
    bf16 storage (w, O given): the kernel keeps every feature phi_k(k_i)[j] as a bf16 hi + lo
    pair before the contraction (16 significant bits: unit roundoff 2^-16 per term; the fp32
    exponent adds ~2^-20), so element-wise
        |S_gpu - S|[j][c] <= eps * sum_i phi_ij |v_ic|   and   |u_gpu - u|[j] <= eps * u[j]
    with eps = 2^-16 + 2^-17, the second term covering fp32 accumulation over the tokens.
    MLP feature maps (eps = MLP_FEATURE_EPS): the logit of a feature passes three contractions over
    d_emb terms whose left operands carry 2^-17 relative error (bf16 hi + lo) and whose sums are
    fp32; by Cauchy-Schwarz each adds at most 2^-17 |g|_2 |w|_2 ~ 2^-17 * 27 to the logit for unit-norm
    weight rows and O(1) activations, so 2^-12 bounds the relative error of exp(logit) with margin."""
    eps = 2.0 ** -16 + 2.0 ** -17 if eps is None else eps
    for h in range(S_or.shape[0]):
        dS = np.abs(S_gpu[h].astype(np.float64) - S_or[h])
        du = np.abs(u_gpu[h].astype(np.float64) - u_or[h])
        eS = np.linalg.norm(dS) / max(np.linalg.norm(S_or[h]), 1e-300)
        eu = np.linalg.norm(du) / max(np.linalg.norm(u_or[h]), 1e-300)
        if w is None:
            assert eS <= tol and eu <= tol, f"head {h}: S rel-F {eS:.3e}, u rel {eu:.3e} (tol {tol:.1e})"
        else:
            L = O["K"].shape[1] - int(O.get("n_gen", 0))
            _, M = orc.partition(L, w.n_sink, w.n_tail)
            if O.get("phi_k_fns") is not None:
                F = O["phi_k_fns"][h](O["K"][h, M])
            else:
                F = orc.phi(O["K"][h, M], O["Wk"][h], O["bk"][h], w.phi_in_scale, w.phi_norm_coef)
            bound = eps * (F.T @ np.abs(O["V"][h, M]))
            assert (dS <= bound + 1e-30).all(), \
                f"head {h}: S error exceeds the bf16-feature bound by x{(dS / (bound + 1e-300)).max():.3f} (rel-F {eS:.3e})"
            assert (du <= eps * u_or[h]).all(), f"head {h}: u rel {eu:.3e}"


def check_layer(w, P, k, batch, i, heads=None, sum_tol=None, mode="sub", check_aux=True, summaries=None):
    """Full comparison of problem i of `batch` (already built + decoded, debug outputs on).
    `summaries` = (S, u) from an earlier oracle build of the same cache skips both the oracle's
    rebuild and the summary comparison (the caller has done it once)."""
    L = int(P["L"])
    n_mid = max(0, L - w.n_sink - w.n_tail)
    Hq = w.n_q_heads
    heads = list(range(Hq)) if heads is None else list(heads)
    if summaries is None:
        res, S_or, u_or, O = oracle_layer(w, P, k, heads=heads)
    else:
        res, S_or, u_or, O = oracle_layer(w, P, k, heads=heads, S=summaries[0], u=summaries[1])
    if sum_tol is None:
        sum_tol = 2e-3 if w.dtype == "bf16" else 2e-5
    if n_mid > 0 and summaries is None:
        rounded_features = (w.dtype == "bf16" and w.d_phi == w.d_head) or "mlp" in P   # the matrix-core paths
        check_summaries(batch.result(i, "S"), batch.result(i, "u"), S_or, u_or, sum_tol,
                        w=w if rounded_features else None, O=O, eps=MLP_FEATURE_EPS if "mlp" in P else None)
    y = batch.result(i, "out")
    idx = batch.result(i, "topk_idx")
    sc = batch.result(i, "scores")
    aux = batch.result(i, "aux")
    key = {"sub": "y", "nosub": "y_nosub", "topk": "y_topk"}[mode]
    worst = (0.0, 0.0)
    n_swapped = 0
    d = w.d_head
    for g, r in zip(heads, res):
        if n_mid > 0:
            check_scores(sc[g], r, w.n_sink, n_mid)
        exact = check_index_set(idx[g], r, w.n_sink, n_mid)
        if not exact:
            # admissible swaps of (near-)tied tokens at the selection boundary: both sets are correct
            # selections; the output is unique only given the set, so it is compared with the oracle
            # run on the GPU's set (tied tokens can carry large weights, e.g. planted needles at K = 1)
            n_swapped += 1
            forced = {g: idx[g][: r["idx"].size].astype(np.int64)}
            r = oracle_layer(w, P, k, heads=[g], S=S_or, u=u_or, retrieved=forced)[0][0]
        a, b = check_output(y[g], r[key], f"head {g} {key}" + ("" if exact else " (oracle on the GPU's set)"))
        worst = (max(worst[0], a), max(worst[1], b))
        if check_aux:
            m = float(aux[g, 0])
            n_gen = int(P.get("n_gen", 0))            # generated tokens count with the exact support
            E = np.concatenate([orc.partition(L, w.n_sink, w.n_tail)[0], r["idx"], np.arange(L, L + n_gen)])
            m_or = r["s"][E].max() if E.size else 0.0
            assert abs(m - m_or) <= 1e-5 * max(1.0, abs(m_or)), f"head {g}: shift {m} vs {m_or}"
            Z_or = (r["Z_E"] + r["Z_G"]) * np.exp(-m_or)
            assert abs(aux[g, 1] - Z_or) <= 1e-4 * Z_or + 1e-30, f"head {g}: Z_E {aux[g, 1]} vs {Z_or}"
            nu_or = (r["nu_E"] + r["nu_G"]) * np.exp(-m_or)
            assert np.abs(aux[g, 4:4 + d] - nu_or).max() <= 1e-4 * max(np.abs(nu_or).max(), 1e-30) + 1e-6
            # the numerical clamp (residual denominator <= 0 after the subtraction) may only fire where the
            # true remainder is below the rounding of the two fp32 sums it is the difference of
            clamped = aux[g, 3] != 0.0
            assert not clamped or (mode == "sub" and r["Z_R_hat"] <= 1e-5 * r["Z_M_hat"]), \
                f"head {g}: residual clamp fired (Z_R_hat {r['Z_R_hat']}, Z_M_hat {r['Z_M_hat']})"
            if mode == "sub" and n_mid > r["idx"].size and not clamped:
                # the residual denominator (unshifted) against the oracle's
                # (a difference of two fp32 sums of size Z_M_hat: with nearly every mid token retrieved the
                # small remainder carries their rounding, ~1e-6 Z_M_hat)
                assert abs(aux[g, 2] - r["Z_R_hat"]) <= 5e-3 * r["Z_R_hat"] + 1e-5 * r["Z_M_hat"], \
                    f"head {g}: Z_R_hat {aux[g, 2]} vs {r['Z_R_hat']} (Z_M_hat {r['Z_M_hat']})"
    return {"max_abs": worst[0], "rel_l1": worst[1], "swapped_heads": n_swapped}
