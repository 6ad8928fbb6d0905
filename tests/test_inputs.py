"""The seeded generators: storage rounding is exact RNE, draws are reproducible,
needles sit in the mid-region with the stated geometry."""
import math

import numpy as np
import torch

from paper_2604_05438_amd import inputs as I


def test_bf16_rounding_matches_torch_rne():
    x = np.random.default_rng(0).standard_normal(200000).astype(np.float32)
    x[:4] = [0.0, -0.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8]      # exact ties
    bits = I.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).bfloat16().view(torch.int16).numpy().view(np.uint16)
    assert (bits == ref).all()
    back = I.bf16_bits_to_f32(bits)
    assert (back == torch.from_numpy(x).bfloat16().float().numpy()).all()
    assert I.to_f64(bits).dtype == np.float64 and (I.to_f64(bits) == back.astype(np.float64)).all()


def test_layer_is_reproducible_and_shaped():
    w = I.WORKLOADS["l1b_32k"]
    a = I.make_layer(w, L=1000)
    b = I.make_layer(w, L=1000)
    for k in ("q", "K", "V", "Wq", "Wk", "bq", "bk"):
        assert (a[k] == b[k]).all()
    assert a["K"].shape == (8, 1000, 64) and a["K"].dtype == np.uint16
    assert a["q"].shape == (32, 64) and a["Wq"].shape == (32, 64, 64)
    # queries of a group share their KV head's W
    assert (a["Wq"][5] == a["Wk"][1]).all()
    # a new query index changes q only
    c = I.make_layer(w, L=1000, query_index=3)
    assert (c["K"] == a["K"]).all() and (c["V"] == a["V"]).all() and not (c["q"] == a["q"]).all()
    # another layer is a different draw
    d = I.make_layer(w, L=1000, layer=1)
    assert not (d["K"] == a["K"]).all()


def test_needles_are_in_mid_region_with_cosine_0p8():
    w = I.WORKLOADS["tiny_f32"]
    P = I.make_layer(w)
    pos = P["needle_pos"][0]
    assert len(set(pos.tolist())) == 8 and pos.min() >= w.n_sink and pos.max() < w.L - w.n_tail
    q = P["q"][0].astype(np.float64)
    for p in pos:
        k = P["K"][0, p].astype(np.float64)
        cos = k @ q / np.linalg.norm(k) / np.linalg.norm(q)
        assert abs(cos - 0.8) < 1e-4 and abs(np.linalg.norm(k) - math.sqrt(64)) < 1e-3


def test_ragged_lengths_and_budget():
    w = I.WORKLOADS["l1b_ragged"]
    Ls = I.ragged_lengths(w)
    assert Ls.shape == (16,) and Ls.min() >= 16384 and Ls.max() <= 65536
    assert (Ls == I.ragged_lengths(w)).all()
    assert I.mid_budget(4096, 100, 4, 64) == 40
    assert I.mid_budget(50, 100, 4, 64) == 0
