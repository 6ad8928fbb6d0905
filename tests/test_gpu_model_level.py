"""GPU parity for the two model-level workloads, in the launch shape they would run in:

  * ragged batch: one decode step for every (sequence, layer) pair of a 1B-shaped model,
    16 sequences x 16 layers = 256 problems of different lengths in ONE build call and ONE
    decode call;
  * build + 64 queries: all 28 layers of a 3B-shaped model at 128K in one problem table,
    summaries built once, then 64 consecutive decode calls against the fixed cache.

The oracle checks a sample of (problem, head, query) triples element by element; every
problem is also checked through properties that hold at any size (device status, finite
outputs, the retrieved set is valid and is a Top-K set of the kernel's own scores)."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

from paper_2604_05438_amd import inputs as I

pytestmark = pytest.mark.gpu

N_GEN_THREADS = 8


def _upload(P):
    from paper_2604_05438_amd import harness as H
    out = {name: H.to_device(P[name]) for name in ("q", "K", "V", "Wq", "bq", "Wk", "bk")}
    out["L"] = int(P["L"])
    return out


def _check_topk_property(w, L, k, idx_row, score_row):
    """The retrieved set against the kernel's own scores: in range, distinct, ascending, and no
    unretrieved mid token scores above the lowest retrieved one."""
    n_mid = max(0, L - w.n_sink - w.n_tail)
    k = min(k, n_mid)
    if k == 0:
        return
    got = idx_row[:k].astype(np.int64)
    assert (got >= w.n_sink).all() and (got < w.n_sink + n_mid).all()
    assert (np.diff(got) > 0).all()
    s = score_row[:n_mid]
    sel = np.zeros(n_mid, dtype=bool)
    sel[got - w.n_sink] = True
    if k < n_mid:
        assert s[sel].min() >= s[~sel].max()


def test_ragged_batch_all_layers():
    import parity_utils as PU
    from paper_2604_05438_amd import harness as H
    w = I.WORKLOADS["l1b_ragged"]
    lens = I.ragged_lengths(w)
    assert lens.size == 16 and lens.min() >= 16384 and lens.max() <= 65536
    pairs = [(layer, seq) for layer in range(w.n_layers) for seq in range(w.n_seqs)]
    ks = [I.mid_budget(int(lens[seq]), w.budget_bp, w.n_sink, w.n_tail) for _, seq in pairs]
    # oracle sample: the shortest and the longest sequence, first / middle / last layer
    s_lo, s_hi = int(np.argmin(lens)), int(np.argmax(lens))
    sample = {(0, s_lo), (0, s_hi), (7, s_hi), (15, s_lo), (15, (s_lo + 5) % 16), (9, 3)}
    kept = {}
    layers = []
    with ThreadPoolExecutor(N_GEN_THREADS) as ex:
        gen = ex.map(lambda p: I.make_layer(w, layer=p[0], seq=p[1], L=int(lens[p[1]])), pairs)
        for p, P in zip(pairs, gen):
            layers.append(_upload(P))
            if p in sample:
                kept[p] = P
    b = H.Batch(H.config_of(w), layers, ks, debug=True)
    assert b.n == 256
    b.build()
    b.decode()
    assert b.status() == 0
    for i, p in enumerate(pairs):
        L = int(lens[p[1]])
        y = b.result(i, "out")
        assert np.isfinite(y).all(), f"problem {p}: non-finite output"
        if p[0] in (0, 5, 15):
            idx = b.result(i, "topk_idx"); sc = b.result(i, "scores")
            for g in (0, 13, 31):
                _check_topk_property(w, L, ks[i], idx[g], sc[g])
    worst = 0.0
    for p, P in kept.items():
        i = pairs.index(p)
        rep = PU.check_layer(w, P, ks[i], b, i, heads=[0, 5, 18, 31])
        worst = max(worst, rep["max_abs"])
    print("ragged 256 problems: worst max_abs", worst)


def test_model_build_then_64_queries():
    import parity_utils as PU
    from oracle import tkphi_oracle as orc
    from paper_2604_05438_amd import harness as H
    w = I.WORKLOADS["l3b_128k_model"]
    k = I.mid_budget(w.L, w.budget_bp, w.n_sink, w.n_tail)
    assert k == 1310 and w.n_layers == 28
    sample_layers = (0, 13, 27)
    sample_queries = (0, 1, 37, 63)
    kept = {}
    layers = []
    with ThreadPoolExecutor(N_GEN_THREADS) as ex:
        gen = ex.map(lambda l: I.make_layer(w, layer=l), range(w.n_layers))
        for l, P in enumerate(gen):
            layers.append(_upload(P))
            if l in sample_layers:
                kept[l] = P
    b = H.Batch(H.config_of(w), layers, [k] * w.n_layers, debug=True)
    b.build()
    assert b.status() == 0
    summ = {}
    for l, P in kept.items():
        O = PU.oracle_inputs(P)
        S_or, u_or = orc.build_summaries(O["K"], O["V"], O["Wk"], O["bk"], w.phi_in_scale, w.phi_norm_coef,
                                         w.n_sink, w.n_tail)
        PU.check_summaries(b.result(l, "S"), b.result(l, "u"), S_or, u_or, 2e-3, w=w, O=O)
        summ[l] = (S_or, u_or)
    worst = 0.0
    for j in range(64):
        qs = [I.make_layer(w, layer=l, query_index=j, with_kv=False)["q"] for l in range(w.n_layers)]
        for l, q in enumerate(qs):
            b.set_query(l, q)
        b.decode()
        assert b.status() == 0, f"query {j}"
        for l in range(w.n_layers):
            assert np.isfinite(b.result(l, "out")).all(), f"layer {l} query {j}"
        if j in sample_queries:
            for l, P in kept.items():
                Pj = dict(P, q=qs[l])
                heads = [(3 * j + 7 * l) % w.n_q_heads, (11 + j + l) % w.n_q_heads]
                rep = PU.check_layer(w, Pj, k, b, l, heads=heads, summaries=summ[l])
                worst = max(worst, rep["max_abs"])
            lp = (5 * j + 2) % w.n_layers
            idx = b.result(lp, "topk_idx"); sc = b.result(lp, "scores")
            for g in (1, 22):
                _check_topk_property(w, w.L, k, idx[g], sc[g])
    print("model-level: 28 layers x 64 queries, worst sampled max_abs", worst)


def test_decode_loop_with_growing_generated_prefix():
    """A decode loop as a caller runs it: summaries built once over the prefill, then eight steps,
    each with a new query and one more generated token after the prefill rows (the rows are in
    the K/V buffers from the start; only n_gen in the problem table and q change).  Every step is
    compared with the oracle's eq. (implemented_decode) on the same rows."""
    import parity_utils as PU
    from paper_2604_05438_amd import harness as H
    w = I.WORKLOADS["l1b_32k"]
    L, steps, k = 6000, 8, 59
    P = I.make_layer(w, L=L + steps)
    P["L"], P["n_gen"] = L, 0
    b = H.Batch(H.config_of(w, max_gen=steps), [P], [k], debug=True)
    b.build()
    S0, u0 = b.result(0, "S").copy(), b.result(0, "u").copy()
    summaries = None
    for t in range(steps + 1):
        q = I.make_layer(w, L=L + steps, query_index=t, with_kv=False)["q"]
        P["q"], P["n_gen"] = q, t
        b.set_query(0, q)
        b.set_n_gen(0, t)
        b.decode()
        assert b.status() == 0
        if summaries is None:
            _, S_or, u_or, _ = PU.oracle_layer(w, P, k, heads=[0])
            summaries = (S_or, u_or)
            PU.check_layer(w, P, k, b, 0, heads=[0, 17, 31])                    # also checks S, u once
        else:
            PU.check_layer(w, P, k, b, 0, heads=[0, 17, 31], summaries=summaries)
    assert np.array_equal(S0, b.result(0, "S")) and np.array_equal(u0, b.result(0, "u"))   # decode never writes them
