"""GPU parity at the full sizes of the synthetic workloads, in the launch configuration
bench.py times (single problem per call for the single-layer shapes).  The oracle computes
whole heads one by one; for the larger shapes a sample of query heads is checked."""
import numpy as np
import pytest

from paper_2604_05438_amd import inputs as I

pytestmark = pytest.mark.gpu


def test_l1b_32k_full_layer():
    # 32q/8kv, head_dim 64, L 32768, K = 327 (1 % of the mid-region): every query head
    import parity_utils as PU
    from paper_2604_05438_amd import harness as H
    w = I.WORKLOADS["l1b_32k"]
    k = I.mid_budget(w.L, w.budget_bp, w.n_sink, w.n_tail)
    assert k == 327
    P = I.make_layer(w)
    b = H.Batch(H.config_of(w), [P], [k], debug=True)
    b.build(); b.decode()
    assert b.status() == 0
    rep = PU.check_layer(w, P, k, b, 0)
    print("l1b_32k", rep)


def test_l3b_128k_budget_sweep():
    # 24q/8kv, head_dim 128, L 131072; budgets 0.5 / 1 / 2 / 4 % of the mid-region
    import parity_utils as PU
    from paper_2604_05438_amd import harness as H
    w = I.WORKLOADS["l3b_128k"]
    P = I.make_layer(w)
    ks = [I.mid_budget(w.L, bp, w.n_sink, w.n_tail) for bp in (50, 100, 200, 400)]
    assert ks == [655, 1310, 2620, 5240]
    b = H.Batch(H.config_of(w), [P], [ks[-1]], debug=True)
    b.build()
    O = PU.oracle_inputs(P)
    from oracle import tkphi_oracle as orc
    S_or, u_or = orc.build_summaries(O["K"], O["V"], O["Wk"], O["bk"], w.phi_in_scale, w.phi_norm_coef,
                                     w.n_sink, w.n_tail)
    PU.check_summaries(b.result(0, "S"), b.result(0, "u"), S_or, u_or, 2e-3, w=w, O=O)
    heads = [0, 4, 8, 11, 17, 23]
    n_mid = w.L - w.n_sink - w.n_tail
    for k in ks:
        b.set_topk(0, k)
        b.decode()
        assert b.status() == 0
        y = b.result(0, "out"); idx = b.result(0, "topk_idx"); sc = b.result(0, "scores")
        res = orc.decode_layer(O["q"], O["K"], O["V"], S_or, u_or, O["Wq"], O["bq"], O["Wk"], O["bk"],
                               w.phi_in_scale, w.phi_norm_coef, w.score_scale, w.n_sink, w.n_tail, k, heads=heads)
        worst = 0.0
        for g, r in zip(heads, res):
            PU.check_scores(sc[g], r, w.n_sink, n_mid)
            exact = PU.check_index_set(idx[g], r, w.n_sink, n_mid)
            if exact:
                a, _ = PU.check_output(y[g], r["y"], f"K={k} head {g}")
            else:
                r2 = orc.decode_layer(O["q"], O["K"], O["V"], S_or, u_or, O["Wq"], O["bq"], O["Wk"], O["bk"],
                                      w.phi_in_scale, w.phi_norm_coef, w.score_scale, w.n_sink, w.n_tail, k,
                                      heads=[g], retrieved={g: idx[g][:k].astype(np.int64)})[0]
                a, _ = PU.check_output(y[g], r2["y"], f"K={k} head {g} (GPU's set)")
            worst = max(worst, a)
        print("l3b_128k K", k, "max_abs", worst)


def test_million_token_context():
    """One KV head with two query heads over 2^20 tokens (1024 score chunks: the select plan's
    many-chunk path; K = 10485 retrieved tokens, 164 gather tiles; a boundary bin with thousands of
    candidates: the radix paths of the resolve step)."""
    import dataclasses
    import parity_utils as PU
    from paper_2604_05438_amd import harness as H
    w = dataclasses.replace(I.WORKLOADS["l1b_32k"], name="long_1m", n_q_heads=2, n_kv_heads=1, L=1 << 20,
                            n_needles=32, seed=31337)
    k = I.mid_budget(w.L, w.budget_bp, w.n_sink, w.n_tail)
    assert k == 10485
    P = I.make_layer(w)
    b = H.Batch(H.config_of(w), [P], [k], debug=True)
    b.build(); b.decode()
    assert b.status() == 0
    rep = PU.check_layer(w, P, k, b, 0)
    print("1M tokens", rep)


def test_l3b_128k_mlp_feature_maps():
    """The 128K / 1 % layer with the one-block ReZero MLP maps of width 512, as `bench.py
    --mlp-d-emb 512` runs it (32 token blocks of 4096 through the GEMM chain): summaries against
    the oracle's build, stored features on a sample of tokens of every KV head, outputs and index
    sets of a sample of query heads."""
    import parity_utils as PU
    from oracle import tkphi_oracle as orc
    from paper_2604_05438_amd import harness as H
    w = I.WORKLOADS["l3b_128k"]
    k = I.mid_budget(w.L, w.budget_bp, w.n_sink, w.n_tail)
    assert k == 1310
    P = I.make_layer(w)
    P["mlp"] = I.make_mlp_phi(w, d_emb=512)
    b = H.Batch(H.config_of(w, d_emb=512), [P], [k], debug=True)
    b.build(); b.decode()
    assert b.status() == 0
    rep = PU.check_layer(w, P, k, b, 0, heads=[0, 10, 23])
    print("l3b_128k mlp", rep, flush=True)
    O = PU.oracle_inputs(P)
    _, fk = PU.mlp_feature_fns(P)
    n_mid = w.L - w.n_sink - w.n_tail
    rng = np.random.default_rng(11)
    sample = np.unique(np.concatenate([rng.integers(0, n_mid, size=1500), [0, 4095, 4096, n_mid - 1]]))
    C = b.result(0, "phi_cache")
    worst = 0.0
    for h in range(w.n_kv_heads):
        F = fk[h](O["K"][h, w.n_sink + sample])
        worst = max(worst, float((np.abs(C[h, sample].astype(np.float64) - F) / F).max()))
    print(f"l3b_128k mlp: stored features (sample), worst relative error {worst:.3e}", flush=True)
    assert worst <= PU.MLP_FEATURE_EPS
