"""Pins for the CPU oracle: it is checked against what the paper and the
mathematics fix, by routes that do not go through the oracle's own formulas
(hand-written loops, scipy's softmax, closed forms, the paper's printed
worked example)."""
import math
import os

import numpy as np
import pytest
import scipy.special

from oracle import tkphi_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_problem(rng, L=200, d=16, dphi=24, Hq=4, Hkv=2, wscale=0.4, kscale=0.7):
    q = rng.standard_normal((Hq, d))
    K = kscale * rng.standard_normal((Hkv, L, d))
    V = rng.standard_normal((Hkv, L, d))
    Wk = wscale * rng.standard_normal((Hkv, dphi, d))
    Wq = wscale * rng.standard_normal((Hq, dphi, d))       # phi_q != phi_k allowed
    bk = 0.1 * rng.standard_normal((Hkv, dphi))
    bq = 0.1 * rng.standard_normal((Hq, dphi))
    return dict(q=q, K=K, V=V, Wk=Wk, Wq=Wq, bk=bk, bq=bq, a=0.5, c=0.125,
                scale=1.0 / math.sqrt(d), n_sink=3, n_tail=7)


def _run(P, k, **kw):
    S, u = orc.build_summaries(P["K"], P["V"], P["Wk"], P["bk"], P["a"], P["c"],
                               P["n_sink"], P["n_tail"])
    return orc.decode_layer(P["q"], P["K"], P["V"], S, u, P["Wq"], P["bq"], P["Wk"], P["bk"],
                            P["a"], P["c"], P["scale"], P["n_sink"], P["n_tail"], k, **kw), S, u


def _dense_softmax_attention(q, K, V, scale):
    # independent route: scipy's max-shifted softmax
    w = scipy.special.softmax(scale * (K @ q))
    return w @ V


# --- worked example printed in the paper -----------------------------------
def test_budget_rule_matches_paper_worked_example():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "budget_rule.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for L, bp, ns, nt, K in rows:
        assert orc.budget_paper(int(L), int(bp), int(ns), int(nt)) == int(K)
    # the max{0, .} branch: 68 anchors exceed 1 % of 4096
    assert orc.budget_paper(4096, 100, 4, 64) == 0
    # the synthetic workloads' convention: 1 % of the 4028 mid tokens -> 40
    assert orc.budget_mid(4096, 100, 4, 64) == 40
    assert orc.budget_mid(32768, 100, 4, 64) == 327
    assert [orc.budget_mid(131072, bp, 4, 64) for bp in (50, 100, 200, 400)] == [655, 1310, 2620, 5240]


def test_summary_state_size_matches_paper():
    row = [l.split() for l in open(os.path.join(GOLDEN, "summary_state_size.txt"))
           if l.strip() and not l.startswith("#")][0]
    Hkv, d, dphi, nl, eb = (int(x) for x in row[:5])
    P = _rand_problem(np.random.default_rng(0), L=40, d=d, dphi=dphi, Hq=Hkv, Hkv=Hkv)
    S, u = orc.build_summaries(P["K"], P["V"], P["Wk"], P["bk"], P["a"], P["c"], 3, 7)
    per_layer = (S.size + u.size) * eb
    assert per_layer == 66560
    assert abs(per_layer / 1024 - float(row[5])) / float(row[5]) < 0.03
    assert abs(per_layer * nl / 2 ** 20 - float(row[6])) / float(row[6]) < 0.03


# --- partition -----------------------------------------------------------------
def test_partition_sets():
    A, M = orc.partition(10, 2, 3)
    assert A.tolist() == [0, 1, 7, 8, 9] and M.tolist() == [2, 3, 4, 5, 6]
    A, M = orc.partition(5, 2, 3)
    assert A.tolist() == [0, 1, 2, 3, 4] and M.size == 0
    A, M = orc.partition(4, 4, 64)
    assert A.tolist() == [0, 1, 2, 3] and M.size == 0
    A, M = orc.partition(6, 0, 0)
    assert A.size == 0 and M.tolist() == list(range(6))


# --- Top-K: brute force, with ties ---------------------------------------------
def test_topk_equals_bruteforce_with_ties():
    rng = np.random.default_rng(1)
    for trial in range(50):
        L = int(rng.integers(12, 200))
        ns, nt = int(rng.integers(0, 4)), int(rng.integers(0, 6))
        _, M = orc.partition(L, ns, nt)
        # few distinct values -> many exact ties
        s = rng.integers(-3, 4, size=L).astype(np.float64) * 0.25
        k = int(rng.integers(0, M.size + 3))
        got = orc.topk_mid(s, M, k)
        brute = sorted(M.tolist(), key=lambda i: (-s[i], i))[:min(k, M.size)]
        assert got.tolist() == brute
        assert all(ns <= i < L - nt for i in got)


def test_topk_never_returns_anchor_even_if_anchor_scores_highest():
    s = np.array([9.0, 8.0, 0.1, 0.3, 0.2, 7.0])
    _, M = orc.partition(6, 2, 1)
    assert orc.topk_mid(s, M, 2).tolist() == [3, 4]


# --- scores / GQA map / orientation --------------------------------------------
def test_scores_and_gqa_mapping_by_hand():
    rng = np.random.default_rng(2)
    P = _rand_problem(rng, L=30, d=8, dphi=5, Hq=6, Hkv=2)
    res, S, u = _run(P, 4)
    G = 3
    for g in range(6):
        h = g // G
        for i in (0, 7, 29):
            s_hand = sum(P["q"][g][c] * P["K"][h][i][c] for c in range(8)) / math.sqrt(8)
            assert abs(res[g]["s"][i] - s_hand) < 1e-13


def test_summary_orientation_and_phi_formula_by_hand():
    # one mid token: S must be the outer product phi(k) v^T, feature-major
    rng = np.random.default_rng(3)
    d, dphi = 4, 3
    K = rng.standard_normal((1, 3, d))
    V = rng.standard_normal((1, 3, d))
    W = rng.standard_normal((1, dphi, d))
    b = rng.standard_normal((1, dphi))
    a, c = 0.7, 0.3
    S, u = orc.build_summaries(K, V, W, b, a, c, 1, 1)      # M = {1}
    k, v = K[0, 1], V[0, 1]
    for j in range(dphi):
        f_j = math.exp(a * sum(W[0, j, t] * k[t] for t in range(d)) - c * sum(x * x for x in k) + b[0, j])
        assert abs(u[0, j] - f_j) < 1e-13 * max(1, f_j)
        for ch in range(d):
            assert abs(S[0, j, ch] - f_j * v[ch]) < 1e-13 * max(1, abs(f_j * v[ch]))


# --- P1: dense limit -------------------------------------------------------------
def test_dense_limit_full_support_equals_softmax_attention():
    rng = np.random.default_rng(4)
    P = _rand_problem(rng)
    n_mid = 200 - 10
    res, _, _ = _run(P, n_mid)
    for g, r in enumerate(res):
        ref = _dense_softmax_attention(P["q"][g], P["K"][g // 2], P["V"][g // 2], P["scale"])
        assert orc.rel_l1(r["y"], ref) < 1e-12
        assert orc.rel_l1(r["y_full"], ref) < 1e-13
        assert orc.rel_l1(orc.full_attention(P["q"][g], P["K"][g // 2], P["V"][g // 2], P["scale"]), ref) < 1e-13
        # with everything retrieved the residual summaries vanish
        assert np.abs(r["S_R"]).max() < 1e-11 * np.abs(r["nu_M_hat"]).max() + 1e-12
    # K larger than |M| is clipped
    res2, _, _ = _run(P, n_mid + 50)
    assert all(r2["idx"].size == n_mid for r2 in res2)


# --- P2 / P3: subtraction equals brute force over unretrieved tokens; positivity -------
def test_subtracted_summaries_equal_bruteforce_over_unretrieved():
    rng = np.random.default_rng(5)
    P = _rand_problem(rng, L=120)
    res, S, u = _run(P, 11)
    for g, r in enumerate(res):
        h = g // 2
        retrieved = set(r["idx"].tolist())
        assert len(retrieved) == 11
        S_bf = np.zeros_like(S[h])
        u_bf = np.zeros_like(u[h])
        for i in range(P["n_sink"], 120 - P["n_tail"]):
            if i in retrieved:
                continue
            k = P["K"][h][i]
            f = np.array([math.exp(P["a"] * float(P["Wk"][h][j] @ k) - P["c"] * float(k @ k) + P["bk"][h][j])
                          for j in range(S.shape[1])])
            S_bf += np.outer(f, P["V"][h][i])
            u_bf += f
        assert np.abs(r["S_R"] - S_bf).max() <= 1e-12 * np.abs(S[h]).max()
        assert np.abs(r["u_R"] - u_bf).max() <= 1e-12 * np.abs(u[h]).max()
        # positivity: features, residual denominator, merged denominator
        assert (r["p"] > 0).all() and (r["f_K"] > 0).all() and (u_bf > 0).all()
        Z_R_bf = float(r["p"] @ u_bf)
        assert Z_R_bf > 0 and r["Z_R_hat"] > 0 and r["Z_E"] + r["Z_R_hat"] > 0
        assert abs(r["Z_R_hat"] - Z_R_bf) <= 1e-12 * float(r["p"] @ u[h])
        # and the output follows from the brute-forced residual summaries
        y_bf = (r["nu_E"] + S_bf.T @ r["p"]) / (r["Z_E"] + Z_R_bf)
        assert orc.rel_l1(r["y"], y_bf) < 1e-11


# --- P5: subset-renormalisation bias identity --------------------------------------
def test_subset_bias_identity():
    rng = np.random.default_rng(6)
    P = _rand_problem(rng)
    res, _, _ = _run(P, 9)
    for r in res:
        y_R = r["nu_R"] / r["Z_R"]
        lhs = r["y_full"] - r["y_topk"]
        rhs = r["Z_R"] / (r["Z_E"] + r["Z_R"]) * (y_R - r["y_topk"])
        assert np.abs(lhs - rhs).max() < 1e-12


# --- P6 / P7: exact-residual estimators and partition sums --------------------------
def test_exact_sub_recovers_full_and_nosub_double_counts():
    rng = np.random.default_rng(7)
    P = _rand_problem(rng)
    res, _, _ = _run(P, 13)
    for g, r in enumerate(res):
        ref = _dense_softmax_attention(P["q"][g], P["K"][g // 2], P["V"][g // 2], P["scale"])
        assert orc.rel_l1(r["y_exactsub"], ref) < 1e-12
        assert orc.rel_l1(r["y_exactnosub"], ref) > 1e-6          # double counting is visible
        assert np.allclose(r["nu_E"], r["nu_A"] + r["nu_K"], rtol=1e-12, atol=0)
        assert np.allclose(r["nu_M"], r["nu_K"] + r["nu_R"], rtol=1e-12, atol=1e-13)
        assert abs(r["Z_E"] - (r["Z_A"] + r["Z_K"])) < 1e-12 * r["Z_E"]
        assert abs(r["Z_M"] - (r["Z_K"] + r["Z_R"])) < 1e-12 * r["Z_M"]
        # selection-only output is the exact-support ratio
        E = np.concatenate([np.arange(3), np.arange(193, 200), r["idx"]])
        w = np.exp(r["s"][E])
        assert orc.rel_l1(r["y_topk"], (w @ P["V"][g // 2][E]) / w.sum()) < 1e-12


# --- P8: closed form with constant features -------------------------------------------
def test_constant_feature_closed_form():
    rng = np.random.default_rng(8)
    P = _rand_problem(rng, dphi=16)
    dphi = 16
    P["Wk"][:] = 0.0
    P["Wq"][:] = 0.0
    P["c"] = 0.0
    P["bk"][:] = -0.5 * math.log(dphi)
    P["bq"][:] = -0.5 * math.log(dphi)
    res, _, _ = _run(P, 17)                      # z(q,k) == 1 for every pair
    for g, r in enumerate(res):
        h = g // 2
        R = [i for i in range(3, 193) if i not in set(r["idx"].tolist())]
        y_closed = (r["nu_E"] + P["V"][h][R].sum(axis=0)) / (r["Z_E"] + len(R))
        assert orc.rel_l1(r["y"], y_closed) < 1e-12
        assert abs(r["Z_R_hat"] - len(R)) < 1e-10


# --- P9: q = 0 makes the factorisation exact --------------------------------------------
def test_zero_query_exact_factorisation_gives_mean_value():
    rng = np.random.default_rng(9)
    P = _rand_problem(rng, dphi=16)
    P["Wk"][:] = 0.0
    P["Wq"][:] = 0.0
    P["c"] = 0.0
    P["bk"][:] = -0.5 * math.log(16)
    P["bq"][:] = -0.5 * math.log(16)
    P["q"][:] = 0.0                               # exp(s_i) = 1 = z(q,k_i)
    for k in (0, 5, 60, 190):
        res, _, _ = _run(P, k)
        for g, r in enumerate(res):
            mean_v = P["V"][g // 2].mean(axis=0)
            assert np.abs(r["y"] - mean_v).max() < 1e-12
            assert np.abs(r["y_full"] - mean_v).max() < 1e-12


# --- P10: positive random features converge to the softmax kernel ----------------------
def test_random_feature_estimate_converges_to_exp_kernel():
    # E_w exp(w.x - |x|^2/2) exp(w.y - |y|^2/2) = exp(x.y), w ~ N(0, I), with
    # x = q d^(-1/4), y = k d^(-1/4); b = -ln(dphi)/2 on both maps averages the
    # dphi features.  A dropped norm term, a wrong sign or a misplaced scale
    # breaks the convergence.
    rng = np.random.default_rng(10)
    d, L = 8, 64
    q = 0.6 * rng.standard_normal(d)
    K = 0.6 * rng.standard_normal((L, d))
    a, c = d ** -0.25, 1.0 / (2.0 * math.sqrt(d))
    target = np.exp(K @ q / math.sqrt(d))
    errs = []
    for dphi in (2 ** 8, 2 ** 12, 2 ** 16):
        W = rng.standard_normal((dphi, d))
        b = np.full(dphi, -0.5 * math.log(dphi))
        z = orc.phi(K, W, b, a, c) @ orc.phi(q, W, b, a, c)[0]
        errs.append(np.abs(z / target - 1).mean())
    assert errs[2] < 0.02
    assert errs[2] < errs[1] < errs[0]
    assert errs[0] / errs[2] > 6          # ~ sqrt(256) = 16 expected


def test_ideal_factorisation_recovers_full_attention_any_k():
    # With 2^16 random features on a short sequence the kernel estimate is nearly
    # exact, so the Top-K+phi output approaches full attention for every K
    # (Sec. "Single-normalization merge"), and far better than selection-only Top-K.
    rng = np.random.default_rng(11)
    d, L, dphi = 8, 96, 2 ** 16
    q = 0.6 * rng.standard_normal((1, d))
    K = 0.6 * rng.standard_normal((1, L, d))
    V = rng.standard_normal((1, L, d))
    W = rng.standard_normal((1, dphi, d))
    b = np.full((1, dphi), -0.5 * math.log(dphi))
    a, c, sc = d ** -0.25, 1.0 / (2.0 * math.sqrt(d)), 1.0 / math.sqrt(d)
    S, u = orc.build_summaries(K, V, W, b, a, c, 2, 4)
    ref = _dense_softmax_attention(q[0], K[0], V[0], sc)
    for k in (0, 8, 40):
        r = orc.decode_layer(q, K, V, S, u, W, b, W, b, a, c, sc, 2, 4, k)[0]
        assert orc.rel_l1(r["y"], ref) < 0.05
        assert orc.rel_l1(r["y"], ref) < 0.5 * orc.rel_l1(r["y_topk"], ref)


# --- P12: K = 0 -----------------------------------------------------------------------
def test_zero_budget_is_anchors_plus_unsubtracted_summaries():
    rng = np.random.default_rng(12)
    P = _rand_problem(rng)
    res, S, u = _run(P, 0)
    for g, r in enumerate(res):
        h = g // 2
        assert r["idx"].size == 0
        A = list(range(3)) + list(range(193, 200))
        w = np.exp(r["s"][A])
        y0 = (w @ P["V"][h][A] + S[h].T @ r["p"]) / (w.sum() + r["p"] @ u[h])
        assert orc.rel_l1(r["y"], y0) < 1e-12
        assert orc.rel_l1(r["y"], r["y_nosub"]) < 1e-12


def test_no_mid_region_reduces_to_dense_attention():
    rng = np.random.default_rng(13)
    P = _rand_problem(rng, L=9)            # 3 sink + 7 tail >= 9
    res, S, u = _run(P, 5)
    assert np.all(S == 0) and np.all(u == 0)
    for g, r in enumerate(res):
        ref = _dense_softmax_attention(P["q"][g], P["K"][g // 2], P["V"][g // 2], P["scale"])
        assert orc.rel_l1(r["y"], ref) < 1e-12


def test_fixed_retrieved_set_is_honoured():
    rng = np.random.default_rng(14)
    P = _rand_problem(rng)
    forced = [np.array([5, 50, 100]) for _ in range(4)]
    res, _, _ = _run(P, 3, retrieved=forced)
    for r in res:
        assert r["idx"].tolist() == [5, 50, 100]
        assert orc.rel_l1(r["y_exactsub"], r["y_full"]) < 1e-12


def test_rel_l1_definition():
    assert abs(orc.rel_l1([1.0, -2.0], [1.5, -1.0]) - (0.5 + 1.0) / (2.5 + 1e-12)) < 1e-15
    assert orc.rel_l1([0.0], [0.0]) == 0.0


def test_entropy_and_mass_recovery_closed_forms():
    """Diagnostics of the entropy / mass-recovery analysis against closed forms: with q = 0 every
    score is 0, so the mid-normalised distribution is uniform (normalised entropy 1), Top-K
    recovers K/|M| of the mid mass and the true residual share is (|M|-K)/(|A|+|M|); with one
    dominant key the entropy tends to 0 and Top-1 recovers (almost) all of the mass."""
    rng = np.random.default_rng(5)
    L, d, dphi, n_sink, n_tail, k = 200, 8, 16, 3, 5, 17
    K = rng.standard_normal((L, d)); V = rng.standard_normal((L, d))
    W = rng.standard_normal((dphi, d)); b = np.zeros(dphi)
    S, u = orc.build_summaries(K[None], V[None], W[None], b[None], 0.5, 0.1, n_sink, n_tail)
    r = orc.decode_head(np.zeros(d), K, V, S[0], u[0], W, b, W, b, 0.5, 0.1, 0.35, n_sink, n_tail, k)
    n_mid = L - n_sink - n_tail
    assert abs(r["H_mid"] - 1.0) < 1e-12
    assert abs(r["C_mid"] - k / n_mid) < 1e-12
    assert abs(r["rho_res_star"] - (n_mid - k) / (n_sink + n_tail + n_mid)) < 1e-12
    # one dominant key in the mid-region
    q = rng.standard_normal(d)
    K2 = 0.01 * K
    K2[50] = 40.0 * q / np.linalg.norm(q)
    r2 = orc.decode_head(q, K2, V, S[0], u[0], W, b, W, b, 0.5, 0.1, 1.0, n_sink, n_tail, 1)
    assert r2["idx"][0] == 50
    assert r2["H_mid"] < 1e-6 and r2["C_mid"] > 1 - 1e-9
    # entropy from its definition on a small random case, by explicit loops
    r3 = orc.decode_head(q, K, V, S[0], u[0], W, b, W, b, 0.5, 0.1, 0.35, n_sink, n_tail, k)
    s = [0.35 * float(np.dot(q, K[i])) for i in range(n_sink, L - n_tail)]
    z = sum(np.exp(x) for x in s)
    h = -sum((np.exp(x) / z) * np.log(np.exp(x) / z) for x in s) / np.log(n_mid)
    assert abs(r3["H_mid"] - h) < 1e-12
    top = sorted(s, reverse=True)[:k]
    assert abs(r3["C_mid"] - sum(np.exp(x) for x in top) / z) < 1e-12


def test_mlp_feature_map_shapes_and_reductions():
    """The one-block ReZero MLP feature map: (1) the layer shapes reproduce the paper's per-head
    parameter counts (the printed equations account for all but one scalar in every row);
    (2) alpha = 0 reduces the map to an exponentiated affine map, which must agree with `phi`
    for the composed weights; (3) W1 = 0 makes the residual update the constant
    W2 GeLU(b1) + b2; (4) GeLU's defining values; (5) positivity."""
    import os
    rows = [l.split() for l in open(os.path.join(os.path.dirname(__file__), "golden", "phi_param_counts.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for d, dphi, demb, count in rows:
        assert orc.mlp_param_count(int(d), int(demb), int(dphi)) + 1 == int(count)
    rng = np.random.default_rng(11)
    d, E, dphi, n = 8, 32, 16, 5
    P = {"Ws": rng.standard_normal((E, d)), "bs": rng.standard_normal(E), "W1": rng.standard_normal((E, E)) / 6,
         "b1": rng.standard_normal(E), "W2": rng.standard_normal((E, E)) / 6, "b2": rng.standard_normal(E),
         "alpha": 0.7, "Wo": rng.standard_normal((dphi, E)) / 6, "bo": rng.standard_normal(dphi)}
    x = rng.standard_normal((n, d))
    f = orc.phi_mlp(x, P)
    assert f.shape == (n, dphi) and (f > 0).all()
    # (2) alpha = 0: exp(Wo (Ws x + bs) + bo) = phi(x; W = Wo Ws, b = Wo bs + bo, a = 1, c = 0)
    P0 = dict(P, alpha=0.0)
    ref = orc.phi(x, P["Wo"] @ P["Ws"], P["Wo"] @ P["bs"] + P["bo"], 1.0, 0.0)
    assert np.abs(orc.phi_mlp(x, P0) / ref - 1).max() < 1e-12
    # (3) W1 = 0: Delta is the constant W2 GeLU(b1) + b2, written out with scalar loops
    Pz = dict(P, W1=np.zeros((E, E)))
    import math
    gb = np.array([0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in P["b1"]])
    delta = np.array([sum(P["W2"][i, j] * gb[j] for j in range(E)) + P["b2"][i] for i in range(E)])
    for r in range(n):
        g1 = P["Ws"] @ x[r] + P["bs"] + 0.7 * delta
        assert np.abs(orc.phi_mlp(x[r], Pz)[0] / np.exp(P["Wo"] @ g1 + P["bo"]) - 1).max() < 1e-12
    # (4) GeLU(0) = 0, GeLU(x) -> x and GeLU(-x) -> 0 for large x, GeLU(x) - GeLU(-x) = x
    assert orc.gelu(0.0) == 0.0
    assert abs(orc.gelu(12.0) - 12.0) < 1e-12 and abs(orc.gelu(-12.0)) < 1e-12
    t = rng.standard_normal(50)
    assert np.abs(orc.gelu(t) - orc.gelu(-t) - t).max() < 1e-14
    assert abs(orc.gelu(1.0) - 0.8413447460685429) < 1e-15          # = Phi(1), the standard normal cdf at 1
    # the method with MLP maps still satisfies the dense limit (exact support = every token)
    L, n_sink, n_tail = 60, 2, 3
    K = rng.standard_normal((1, L, d)); V = rng.standard_normal((1, L, d)); q = rng.standard_normal((1, d))
    fk = [lambda z: orc.phi_mlp(z, P)]; fq = [lambda z: orc.phi_mlp(z, P0)]
    S, u = orc.build_summaries(K, V, None, None, 0, 0, n_sink, n_tail, phi_k_fns=fk)
    r = orc.decode_layer(q, K, V, S, u, None, None, None, None, 0, 0, 0.3, n_sink, n_tail, L, phi_q_fns=fq, phi_k_fns=fk)[0]
    # (the subtracted summaries cancel to rounding relative to |S|, which these unscaled random
    # maps make large next to Z_E)
    assert orc.rel_l1(r["y"], r["y_full"]) < 1e-7
    r = orc.decode_layer(q, K, V, S, u, None, None, None, None, 0, 0, 0.3, n_sink, n_tail, 7, phi_q_fns=fq, phi_k_fns=fk)[0]
    # subtraction = brute force over the unretrieved tokens, with the MLP features
    _, M = orc.partition(L, n_sink, n_tail)
    rest = np.setdiff1d(M, r["idx"])
    fr = orc.phi_mlp(K[0, rest], P)
    assert np.abs(r["S_R"] - fr.T @ V[0, rest]).max() < 1e-10 * np.abs(S).max()


# --- generated tokens: eq. (implemented_decode) ----------------------------------------
def test_generated_tokens_are_one_more_exact_branch():
    """The generated-token prefix G is exact and outside the prefill partition.  Pinned by routes
    that do not use the branch's own formula: (a) G appended to the tail anchors of a longer
    "prefill" gives the same mid-region, hence the same summaries, selection and output;
    (b) with every mid token retrieved the output is dense softmax attention over prefill + G
    (scipy); (c) a brute-force loop over the token classes; (d) n_gen = 0 changes nothing."""
    rng = np.random.default_rng(21)
    P = _rand_problem(rng, L=230)
    n_gen, k = 9, 17
    L = 230 - n_gen
    kw = dict(a=P["a"], c=P["c"], n_sink=P["n_sink"])
    S, u = orc.build_summaries(P["K"], P["V"], P["Wk"], P["bk"], n_tail=P["n_tail"], n_gen=n_gen, **kw)
    S2, u2 = orc.build_summaries(P["K"], P["V"], P["Wk"], P["bk"], n_tail=P["n_tail"] + n_gen, **kw)
    assert np.array_equal(S, S2) and np.array_equal(u, u2)
    args = (P["q"], P["K"], P["V"], S, u, P["Wq"], P["bq"], P["Wk"], P["bk"], P["a"], P["c"], P["scale"], P["n_sink"])
    res = orc.decode_layer(*args, P["n_tail"], k, n_gen=n_gen)
    res2 = orc.decode_layer(*args, P["n_tail"] + n_gen, k)                       # (a)
    for g, (r, r2) in enumerate(zip(res, res2)):
        h = g // 2
        assert np.array_equal(r["idx"], r2["idx"])
        assert orc.rel_l1(r["y"], r2["y"]) < 1e-13
        assert orc.rel_l1(r["y_topk"], r2["y_topk"]) < 1e-13 and orc.rel_l1(r["y_nosub"], r2["y_nosub"]) < 1e-13
        assert abs(r["Z_E"] + r["Z_G"] - r2["Z_E"]) < 1e-12 * r2["Z_E"]
        # (c) brute force: exact weights on sink, tail, retrieved and generated tokens; feature estimate elsewhere
        q, Kh, Vh = P["q"][g], P["K"][h], P["V"][h]
        num, den = np.zeros(Kh.shape[1]), 0.0
        pq = orc.phi(q, P["Wq"][g], P["bq"][g], P["a"], P["c"])[0]
        sel = set(r["idx"].tolist())
        for i in range(L + n_gen):
            exact = i < P["n_sink"] or i >= L - P["n_tail"] or i in sel
            w = math.exp(P["scale"] * float(Kh[i] @ q)) if exact else \
                float(pq @ orc.phi(Kh[i], P["Wk"][h], P["bk"][h], P["a"], P["c"])[0])
            num += w * Vh[i]
            den += w
        assert orc.rel_l1(r["y"], num / den) < 1e-11
        assert all(L - P["n_tail"] > i >= P["n_sink"] for i in sel)              # G is never retrieved
    n_mid = L - P["n_sink"] - P["n_tail"]
    for g, r in enumerate(orc.decode_layer(*args, P["n_tail"], n_mid, n_gen=n_gen)):     # (b)
        ref = _dense_softmax_attention(P["q"][g], P["K"][g // 2], P["V"][g // 2], P["scale"])
        assert orc.rel_l1(r["y"], ref) < 1e-12 and orc.rel_l1(r["y_full"], ref) < 1e-13
    Pz = _rand_problem(np.random.default_rng(22))
    rz, _, _ = _run(Pz, 11)
    rz0, _, _ = _run(Pz, 11, n_gen=0)                                             # (d)
    assert all(np.array_equal(x["y"], y["y"]) and x["Z_G"] == 0.0 for x, y in zip(rz0, rz))


# --- residual-denominator share and residual log-partition error ------------------------------
def test_residual_share_and_log_partition_error_closed_forms():
    """rho_res = Z_R^ / (Z_E + Z_R^) (App. "Entropy, mass recovery, and residual-denominator
    diagnostics") and the residual log-partition error log Z_R^ - log Z_R (Sec. "Analysis: validating
    residual accounting"), pinned by routes that do not use the oracle's expressions:
    (a) the constant feature map (W = 0, c = 0, b = -0.5 ln d_phi, so z = 1 for every pair) makes
        Z_R^ = |R| exactly; with q = 0 every exp(s_i) = 1, so Z_E = |A| + K, Z_G = n_gen, Z_R = |R|:
        rho_res = |R| / (|A| + K + n_gen + |R|) and the log error is 0, with and without generated tokens;
    (b) the same map with a random query: Z_R^ = |R| still, the exact masses come from explicit loops;
    (c) a general random problem with n_gen > 0, every term by scalar loops over the token classes;
    (d) the boundary gap is the difference between the K-th and (K+1)-th largest mid score."""
    rng = np.random.default_rng(33)
    d, dphi, n_sink, n_tail = 8, 16, 3, 5
    W0 = np.zeros((dphi, d)); b0 = np.full(dphi, -0.5 * math.log(dphi))
    for n_gen in (0, 6):
        L, k = 150, 13
        K = rng.standard_normal((L + n_gen, d)); V = rng.standard_normal((L + n_gen, d))
        S, u = orc.build_summaries(K[None], V[None], W0[None], b0[None], 0.5, 0.0, n_sink, n_tail, n_gen=n_gen)
        n_mid = L - n_sink - n_tail
        nR = n_mid - k
        # (a) q = 0
        r = orc.decode_head(np.zeros(d), K, V, S[0], u[0], W0, b0, W0, b0, 0.5, 0.0, 0.35, n_sink, n_tail, k, n_gen=n_gen)
        assert abs(r["rho_res"] - nR / (n_sink + n_tail + k + n_gen + nR)) < 1e-13
        assert abs(r["log_Z_err"]) < 1e-12
        # (b) random q: the estimate stays |R|, the exact side by loops
        q = rng.standard_normal(d)
        r = orc.decode_head(q, K, V, S[0], u[0], W0, b0, W0, b0, 0.5, 0.0, 0.35, n_sink, n_tail, k, n_gen=n_gen)
        s = [0.35 * float(np.dot(q, K[i])) for i in range(L + n_gen)]
        mid = list(range(n_sink, L - n_tail))
        sel = sorted(mid, key=lambda i: (-s[i], i))[:k]
        Z_exact = sum(math.exp(s[i]) for i in range(L + n_gen) if i < n_sink or i >= L - n_tail or i in sel)
        Z_R = sum(math.exp(s[i]) for i in mid if i not in sel)
        assert abs(r["rho_res"] - nR / (Z_exact + nR)) < 1e-12
        assert abs(r["log_Z_err"] - (math.log(nR) - math.log(Z_R))) < 1e-12
    # (c) general maps, generated tokens, scalar loops
    P = _rand_problem(np.random.default_rng(34), L=120)
    n_gen, k = 7, 9
    L = 120 - n_gen
    S, u = orc.build_summaries(P["K"], P["V"], P["Wk"], P["bk"], P["a"], P["c"], P["n_sink"], P["n_tail"], n_gen=n_gen)
    res = orc.decode_layer(P["q"], P["K"], P["V"], S, u, P["Wq"], P["bq"], P["Wk"], P["bk"], P["a"], P["c"], P["scale"],
                           P["n_sink"], P["n_tail"], k, n_gen=n_gen)
    for g, r in enumerate(res):
        h = g // 2
        q, Kh = P["q"][g], P["K"][h]
        s = [P["scale"] * float(np.dot(q, Kh[i])) for i in range(L + n_gen)]
        mid = list(range(P["n_sink"], L - P["n_tail"]))
        sel = set(r["idx"].tolist())
        pq = orc.phi(q, P["Wq"][g], P["bq"][g], P["a"], P["c"])[0]
        Z_hat = 0.0                                    # estimate over the unretrieved mid tokens, one token at a time
        Z_true = 0.0
        for i in mid:
            if i in sel:
                continue
            Z_hat += float(pq @ orc.phi(Kh[i], P["Wk"][h], P["bk"][h], P["a"], P["c"])[0])
            Z_true += math.exp(s[i])
        Z_exact = sum(math.exp(s[i]) for i in range(L + n_gen) if i not in mid or i in sel)
        assert abs(r["rho_res"] - Z_hat / (Z_exact + Z_hat)) < 1e-12
        assert abs(r["log_Z_err"] - (math.log(Z_hat) - math.log(Z_true))) < 1e-11
        # (d)
        ranked = sorted((s[i] for i in mid), reverse=True)
        assert abs(r["boundary_gap"] - (ranked[k - 1] - ranked[k])) < 1e-15
        assert r["boundary_gap"] >= 0.0
