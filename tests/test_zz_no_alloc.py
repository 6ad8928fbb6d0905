"""tkphi_decode_static: the decode entry point that allocates nothing (its scratch memory is a static
device array inside the library), against tkphi_decode on the same problems, through the C ABI.
Two calls in a row, the second on a smaller input; results must be bit-identical to the
workspace-based entry point (same kernels, deterministic summation order); oversized requests and
the MLP maps are refused without enqueueing anything."""
import numpy as np
import pytest

from paper_2604_05438_amd import inputs as I

pytestmark = pytest.mark.gpu


def _decode_both(w, L, k, mode=0):
    import torch
    from paper_2604_05438_amd import binding as B
    from paper_2604_05438_amd import harness as H
    P = I.make_layer(w, L=L)
    b = H.Batch(H.config_of(w), [P], [k], debug=True)
    b.build()
    b.decode(mode)
    torch.cuda.synchronize()
    ref = {n: b.result(0, n).copy() for n in ("out", "topk_idx", "aux")}
    for n in ("out", "topk_idx", "aux"):
        b.dev[0][n].fill_(-5)
    mem0 = torch.cuda.memory_allocated()
    B.tkphi_decode_static(b.cfg, b.table.data_ptr(), b.n, b.max_L, b.max_K, mode, B.current_stream_ptr())
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == mem0
    got = {n: b.result(0, n).copy() for n in ("out", "topk_idx", "aux")}
    return ref, got, b, P


def test_static_scratch_decode_matches_workspace_decode():
    import parity_utils as PU
    from paper_2604_05438_amd import binding as B
    from paper_2604_05438_amd import harness as H
    w = I.WORKLOADS["l3b_128k"]
    # first call: a long layer; second call right after it: a smaller one (the array keeps the first call's contents)
    for L, k in ((40000, 399), (3001, 29)):
        ref, got, b, P = _decode_both(w, L, k)
        for n in ref:
            assert np.array_equal(ref[n], got[n]), f"L={L}: {n} differs between tkphi_decode and tkphi_decode_static"
        rep = PU.check_layer(w, P, k, b, 0, heads=[0, 11, 23])      # and both match the oracle
        print("static", L, k, rep, flush=True)
    # another shape and accounting mode through the same array
    w1 = I.WORKLOADS["l1b_32k"]
    ref, got, b, P = _decode_both(w1, 5000, 49, mode=B.TKPHI_MODE_NOSUB)
    for n in ref:
        assert np.array_equal(ref[n], got[n])
    # requests that do not fit, or that the entry point does not serve, are refused before any launch
    big = H.config_of(I.WORKLOADS["l1b_ragged"])
    with pytest.raises(B.TkphiError) as e:
        B.tkphi_decode_static(big, b.table.data_ptr(), 16, 65536, 654, 0, B.current_stream_ptr())
    assert e.value.status == B.TKPHI_EWORKSPACE
    with pytest.raises(B.TkphiError) as e:
        B.tkphi_decode_static(H.config_of(w1, d_emb=128), b.table.data_ptr(), 1, 5000, 49, 0, B.current_stream_ptr())
    assert e.value.status == B.TKPHI_EUNSUPPORTED
