"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol that
include/tkphi.h declares, and its pure-host entry points validate arguments."""
import ctypes as C
import os
import re

import pytest

from paper_2604_05438_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "tkphi.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tkphi_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    names = _declared_symbols()
    assert set(names) == set(B.EXPORTS), names
    for n in names:
        assert getattr(lib, n) is not None


def test_budget_rules_match_paper_example():
    # K = max(0, ceil(r L) - |A|): 21 / 144 / 636 at 4k / 16k / 64k, 1 %, 20 anchors
    assert [B.tkphi_budget_paper(L, 100, 4, 16) for L in (4096, 16384, 65536)] == [21, 144, 636]
    assert B.tkphi_budget_paper(4096, 100, 4, 64) == 0
    assert B.tkphi_budget_mid(4096, 100, 4, 64) == 40
    assert [B.tkphi_budget_mid(131072, bp, 4, 64) for bp in (50, 100, 200, 400)] == [655, 1310, 2620, 5240]


def _cfg(**kw):
    base = dict(n_q_heads=32, n_kv_heads=8, d_head=64, d_phi=64, n_sink=4, n_tail=64, dtype="bf16",
                score_scale=0.125, phi_in_scale=0.35, phi_norm_coef=0.0625)
    base.update(kw)
    return B.make_config(**base)


def test_workspace_query_and_config_validation():
    assert B.tkphi_workspace_bytes(_cfg(), 1, 32768, 327) > 32 * 32700 * 4
    assert B.tkphi_workspace_bytes(_cfg(), 4, 32768, 327) > 4 * 32 * 32700 * 4
    for bad in (dict(d_head=96), dict(n_q_heads=30), dict(d_phi=20), dict(n_q_heads=128), dict(dtype=7),
                dict(n_sink=-1)):
        assert B.tkphi_workspace_bytes(_cfg(**bad), 1, 4096, 40) == 0
        assert B.tkphi_last_error() != ""
    assert B.tkphi_workspace_bytes(_cfg(), 1, 0, 0) == 0


def test_tuning_overrides_are_validated_and_change_the_geometry():
    base = B.tkphi_workspace_bytes(_cfg(), 1, 32768, 327)
    assert B.tkphi_workspace_bytes(_cfg(tuning={"build_chunk": 64}), 1, 32768, 327) > base   # more chunk partials
    for bad in ({"scan_chunk": -1}, {"scan_chunk": 1 << 20}, {"interleave": 3}, {"force_generic": 2}, {"mlp_mode": 5},
                {"build_chunk": -64}, {"select_mode": 3}, {"select_test": -1}):
        assert B.tkphi_workspace_bytes(_cfg(tuning=bad), 1, 32768, 327) == 0
        assert "tuning" in B.tkphi_last_error()
    cfg = _cfg()
    cfg.tuning.reserved[2] = 1
    assert B.tkphi_workspace_bytes(cfg, 1, 32768, 327) == 0


def test_mlp_feature_map_config_validation():
    mlp = dict(phi_kind=B.TKPHI_PHI_MLP, cache_features=1, d_emb=512)
    base = B.tkphi_workspace_bytes(_cfg(cache_features=1), 1, 32768, 327)
    with_mlp = B.tkphi_workspace_bytes(_cfg(**mlp), 1, 32768, 327)
    assert with_mlp > base > 0                     # activation block + packed weights of the MLP build
    # without a feature cache the build holds the features of a group of problems in the workspace
    assert B.tkphi_workspace_bytes(_cfg(**dict(mlp, cache_features=0)), 1, 32768, 327) > with_mlp
    assert B.tkphi_workspace_bytes(_cfg(**dict(mlp, cache_features=0, d_emb=64)), 1, 4096, 40) == 0   # (not a width that fuses)
    for bad in (dict(mlp, d_emb=96), dict(mlp, d_emb=32), dict(mlp, d_emb=2048), dict(mlp, dtype="f32"), dict(phi_kind=7)):
        assert B.tkphi_workspace_bytes(_cfg(**bad), 1, 4096, 40) == 0
        assert B.tkphi_last_error() != ""
    # the problem table must carry the MLP tables instead of Wq / Wk
    cfg = _cfg(**mlp)
    p = B.tkphi_problem(K=4096, V=8192, stride_head=1000 * 64, stride_tok=64, Wq=0, bq=0, Wk=0, bk=0, S=4096, u=4096,
                        q=4096, out=4096, topk_idx=0, aux=0, scores=0, phi_cache=4096, mlp_q=4096, mlp_k=4096,
                        L=1000, topk=9)
    B.tkphi_check_problems(cfg, (B.tkphi_problem * 1)(p), 1, 1000, 9, True)
    for field in ("mlp_q", "mlp_k", "phi_cache"):
        q = B.tkphi_problem.from_buffer_copy(p)
        setattr(q, field, 0)
        with pytest.raises(B.TkphiError):
            B.tkphi_check_problems(cfg, (B.tkphi_problem * 1)(q), 1, 1000, 9, True)
    # ... and no cache where the configuration has none
    q = B.tkphi_problem.from_buffer_copy(p)
    q.phi_cache = 0
    B.tkphi_check_problems(_cfg(**dict(mlp, cache_features=0)), (B.tkphi_problem * 1)(q), 1, 1000, 9, True)


def test_generated_token_bounds_are_validated():
    assert B.tkphi_workspace_bytes(_cfg(max_gen=64), 1, 4096, 40) >= B.tkphi_workspace_bytes(_cfg(), 1, 4096, 40) > 0
    assert B.tkphi_workspace_bytes(_cfg(max_gen=-1), 1, 4096, 40) == 0
    cfg = _cfg(max_gen=32)
    p = B.tkphi_problem(K=4096, V=8192, stride_head=1100 * 64, stride_tok=64, Wq=4096, bq=4096, Wk=4096, bk=4096,
                        S=4096, u=4096, q=4096, out=4096, L=1000, topk=9, n_gen=32)
    B.tkphi_check_problems(cfg, (B.tkphi_problem * 1)(p), 1, 1000, 9, True)
    for bad in (33, -1):
        q = B.tkphi_problem.from_buffer_copy(p)
        q.n_gen = bad
        with pytest.raises(B.TkphiError) as e:
            B.tkphi_check_problems(cfg, (B.tkphi_problem * 1)(q), 1, 1000, 9, True)
        assert e.value.status == B.TKPHI_ESHAPE


def test_status_strings():
    seen = {B.tkphi_status_string(s) for s in range(-6, 1)}
    assert len(seen) == 7 and B.tkphi_status_string(-99) == "unknown status"


def test_check_problems_rejects_bad_tables():
    cfg = _cfg()
    good = B.tkphi_problem(K=4096, V=8192, stride_head=1000 * 64, stride_tok=64, Wq=4096, bq=4096, Wk=4096,
                           bk=4096, S=4096, u=4096, q=4096, out=4096, topk_idx=0, aux=0, scores=0, L=1000, topk=9)
    arr = (B.tkphi_problem * 1)(good)
    B.tkphi_check_problems(cfg, arr, 1, 1000, 9, True)

    def expect(status, **kw):
        p = B.tkphi_problem.from_buffer_copy(good)
        for k, v in kw.items():
            setattr(p, k, v)
        with pytest.raises(B.TkphiError) as e:
            B.tkphi_check_problems(cfg, (B.tkphi_problem * 1)(p), 1, 1000, 9, True)
        assert e.value.status == status, e.value

    expect(B.TKPHI_EINVAL, K=0)
    expect(B.TKPHI_EINVAL, out=0)
    expect(B.TKPHI_EALIGN, V=8200)
    expect(B.TKPHI_EALIGN, stride_tok=65)
    expect(B.TKPHI_EALIGN, stride_tok=32)
    expect(B.TKPHI_ESHAPE, L=1001)
    expect(B.TKPHI_ESHAPE, L=0)
    expect(B.TKPHI_ESHAPE, topk=10)
    expect(B.TKPHI_ESHAPE, topk=-1)


def test_calls_reject_bad_arguments_before_any_launch():
    cfg = _cfg()
    lib = B.lib()
    nbytes = B.tkphi_workspace_bytes(cfg, 1, 1000, 9)
    # null workspace / too small / misaligned / bad mode / null table: all fail on the host
    assert lib.tkphi_decode(C.byref(cfg), 4096, 1, 1000, 9, 0, None, nbytes, None) == B.TKPHI_EWORKSPACE
    assert lib.tkphi_decode(C.byref(cfg), 4096, 1, 1000, 9, 0, 4096, nbytes - 1, None) == B.TKPHI_EWORKSPACE
    assert lib.tkphi_decode(C.byref(cfg), 4096, 1, 1000, 9, 0, 4100, nbytes, None) == B.TKPHI_EWORKSPACE
    assert lib.tkphi_decode(C.byref(cfg), 4096, 1, 1000, 9, 5, 4096, nbytes, None) == B.TKPHI_EINVAL
    assert lib.tkphi_decode(C.byref(cfg), None, 1, 1000, 9, 0, 4096, nbytes, None) == B.TKPHI_EINVAL
    assert lib.tkphi_build_summaries(C.byref(cfg), None, 1, 1000, 4096, nbytes, None) == B.TKPHI_EINVAL
    assert lib.tkphi_build_summaries(None, 4096, 1, 1000, 4096, nbytes, None) == B.TKPHI_EINVAL
    assert "null" in B.tkphi_last_error()
    # zero problems is a no-op
    assert lib.tkphi_decode(C.byref(cfg), None, 0, 1000, 9, 0, 4096, nbytes, None) == B.TKPHI_OK
