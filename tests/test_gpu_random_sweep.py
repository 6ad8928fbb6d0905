"""GPU parity on seeded random configurations: shapes, anchor sizes, ragged batches, budgets from 0
to the whole mid-region, accounting modes, the feature cache, the MLP maps and generated
tokens in random combination.  Complements the hand-picked cases of the other GPU tests."""
import dataclasses

import numpy as np
import pytest

from paper_2604_05438_amd import inputs as I

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_random_configurations(seed):
    import parity_utils as PU
    from paper_2604_05438_amd import binding as B
    from paper_2604_05438_amd import harness as H
    rng = np.random.default_rng(seed)
    modes = {"sub": B.TKPHI_MODE_SUB, "nosub": B.TKPHI_MODE_NOSUB, "topk": B.TKPHI_MODE_TOPK_ONLY}
    for case in range(25):
        w = I.WORKLOADS[str(rng.choice(["l1b_32k", "l3b_128k", "tiny_f32"]))]
        if rng.random() < 0.3:
            w = dataclasses.replace(w, n_sink=int(rng.integers(0, 9)), n_tail=int(rng.integers(0, 130)), name=w.name + "_a")
        if seed % 2 == 0 and rng.random() < 0.6:        # feature widths and GQA ratios off the tuned shapes
            w = dataclasses.replace(w, d_phi=int(rng.choice([16, 48, 64, 96, 128, 192, 256])), name=w.name + "_p",
                                    n_q_heads=int(w.n_kv_heads * rng.choice([1, 2, 4])) if w.n_kv_heads > 1 else w.n_q_heads)
        cache = bool(rng.random() < 0.3)
        max_gen = int(rng.choice([0, 0, 17, 100]))
        d_emb = int(rng.choice([0, 0, 0, 128] if seed % 2 else [0, 0, 64, 128, 256])) if w.dtype == "bf16" else 0
        if d_emb and not (d_emb in (128, 256, 512) and w.d_phi <= 256):
            cache = True                                     # (without a cache the MLP maps need a width of the one-launch chain)
        layers, ks = [], []
        for i in range(int(rng.integers(1, 5))):
            L = int(rng.choice([rng.integers(1, 200), rng.integers(200, 3000), rng.integers(3000, 12000),
                                rng.integers(12000, 40000)], p=[0.3, 0.4, 0.25, 0.05]))
            ng = int(rng.integers(0, max_gen + 1)) if max_gen else 0
            n_mid = max(0, L - w.n_sink - w.n_tail)
            k = int(rng.choice([0, 1, rng.integers(0, max(2, n_mid // 50 + 2)), rng.integers(0, max(2, n_mid // 8 + 2)),
                                rng.integers(0, n_mid + 10), n_mid], p=[0.2, 0.2, 0.3, 0.2, 0.05, 0.05]))
            P = I.make_layer(w, L=L + ng, seq=i, layer=int(rng.integers(0, 100)))
            P["L"], P["n_gen"] = L, ng
            if d_emb:
                P["mlp"] = I.make_mlp_phi(w, layer=i, d_emb=d_emb)
            layers.append(P)
            ks.append(k)
        mode = str(rng.choice(["sub", "sub", "nosub", "topk"]))
        print(f"seed {seed} case {case}: {w.name} Hq={w.n_q_heads} d_phi={w.d_phi} sink={w.n_sink} tail={w.n_tail} cache={cache} d_emb={d_emb} "
              f"max_gen={max_gen} mode={mode} " + " ".join(f"(L={int(P['L'])},g={P['n_gen']},k={k})" for P, k in zip(layers, ks)),
              flush=True)
        b = H.Batch(H.config_of(w, cache_features=cache, d_emb=d_emb, max_gen=max_gen), layers, ks, debug=True)
        b.build()
        b.decode(modes[mode])
        st = b.status()
        assert st in (0, B.TKPHI_DEV_CLAMPED)               # (a clamp is checked per head by check_layer)
        if st == B.TKPHI_DEV_CLAMPED:
            print(f"seed {seed} case {case}: residual clamp fired", flush=True)
        for i, (P, k) in enumerate(zip(layers, ks)):
            heads = sorted(set(int(x) for x in rng.integers(0, w.n_q_heads, size=2)))
            PU.check_layer(w, P, k, b, i, heads=heads, mode=mode)
