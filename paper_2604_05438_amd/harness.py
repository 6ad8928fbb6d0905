"""Device-side plumbing shared by the tests, the smoke check and bench.py: uploads the
seeded host tensors, builds the problem table, and calls the C ABI through the binding.
No arithmetic of the method happens here."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from .inputs import Workload


def to_device(a: np.ndarray, device="cuda") -> torch.Tensor:
    """float32 stays float32; uint16 arrays are bf16 bit patterns."""
    t = torch.from_numpy(np.ascontiguousarray(a))
    if a.dtype == np.uint16:
        return t.view(torch.int16).to(device).view(torch.bfloat16)
    return t.to(device)


def config_of(w: Workload, cache_features: bool | None = None, d_emb: int = 0, max_gen: int = 0,
              tuning: dict | None = None) -> B.tkphi_config:
    """d_emb > 0 selects the MLP feature maps; cache_features None: the feature cache is on for the MLP maps and
    off for the exp-affine ones; max_gen bounds the generated tokens a problem may append after its prefill
    rows; tuning: tkphi_tuning fields."""
    cache = (d_emb > 0) if cache_features is None else bool(cache_features)
    return B.make_config(w.n_q_heads, w.n_kv_heads, w.d_head, w.d_phi, w.n_sink, w.n_tail, w.dtype,
                         w.score_scale, w.phi_in_scale, w.phi_norm_coef, int(cache),
                         B.TKPHI_PHI_MLP if d_emb > 0 else B.TKPHI_PHI_EXP_AFFINE, d_emb, max_gen, tuning=tuning)


class Batch:
    """A set of (sequence, layer) problems resident on the GPU, with outputs and workspace."""

    def __init__(self, cfg: B.tkphi_config, layers: list[dict], topk: list[int], debug: bool = False,
                 device="cuda", max_L: int | None = None, max_K: int | None = None, diag: bool = False):
        self.cfg = cfg
        self.device = device
        self.n = len(layers)
        Hq, Hkv, d, dphi = cfg.n_q_heads, cfg.n_kv_heads, cfg.d_head, cfg.d_phi
        self.max_L = int(max_L if max_L is not None else max(int(l["L"]) for l in layers))
        self.max_K = int(max_K if max_K is not None else max([int(k) for k in topk] + [0]))
        self.dev: list[dict] = []
        probs = []
        for lay, k in zip(layers, topk):
            t = {name: (lay[name] if isinstance(lay[name], torch.Tensor) else to_device(lay[name], device))
                 for name in ("q", "K", "V", "Wq", "bq", "Wk", "bk")}
            if cfg.phi_kind == B.TKPHI_PHI_MLP:        # lay["mlp"] = inputs.make_mlp_phi(...)
                for side in ("q", "k"):
                    t["mlp_" + side + "_w"] = {kk: (vv if kk == "alpha" else to_device(vv, device))
                                               for kk, vv in lay["mlp"][side].items()}
                    t["mlp_" + side] = B.upload_mlp(t["mlp_" + side + "_w"], device)
            L = int(lay["L"])                      # prefill length; K, V hold L + lay["n_gen"] rows
            n_mid = max(0, L - cfg.n_sink - cfg.n_tail)
            t["S"] = torch.empty((Hkv, dphi, d), dtype=torch.float32, device=device)
            t["u"] = torch.empty((Hkv, dphi), dtype=torch.float32, device=device)
            t["out"] = torch.empty((Hq, d), dtype=torch.float32, device=device)
            if debug:
                t["topk_idx"] = torch.full((Hq, max(self.max_K, 1)), -1, dtype=torch.int32, device=device)
                t["aux"] = torch.zeros((Hq, B.aux_stride(d)), dtype=torch.float32, device=device)
                t["scores"] = torch.zeros((Hq, max(n_mid, 1)), dtype=torch.float32, device=device)
            if cfg.cache_features:
                t["phi_cache"] = torch.empty((Hkv, max(n_mid, 1), dphi), dtype=torch.float32, device=device)
            if debug or diag:
                t["diag"] = torch.full((Hq, B.TKPHI_DIAG_STRIDE), -7.0, dtype=torch.float32, device=device)
            self.dev.append(t)
            probs.append(B.make_problem(t["K"], t["V"], t["Wq"], t["bq"], t["Wk"], t["bk"], t["S"], t["u"],
                                        q=t["q"], out=t["out"], topk_idx=t.get("topk_idx"), aux=t.get("aux"),
                                        scores=t.get("scores"), L=L, topk=int(k), diag=t.get("diag"), phi_cache=t.get("phi_cache"),
                                        mlp_q=t.get("mlp_q"), mlp_k=t.get("mlp_k"), n_gen=int(lay.get("n_gen", 0))))
        self.host_table, self.table = B.upload_problems(probs, device)
        B.tkphi_check_problems(cfg, self.host_table, self.n, self.max_L, self.max_K, True)
        self.ws_bytes = B.tkphi_workspace_bytes(cfg, self.n, self.max_L, self.max_K)
        if self.ws_bytes == 0:
            raise B.TkphiError(B.TKPHI_ESHAPE, B.tkphi_last_error())
        self.ws = B.alloc_workspace(self.ws_bytes, device)

    def build(self) -> None:
        B.tkphi_build_summaries(self.cfg, self.table.data_ptr(), self.n, self.max_L, self.ws.data_ptr(),
                                self.ws_bytes, B.current_stream_ptr())

    def decode(self, mode: int = B.TKPHI_MODE_SUB) -> None:
        B.tkphi_decode(self.cfg, self.table.data_ptr(), self.n, self.max_L, self.max_K, mode,
                       self.ws.data_ptr(), self.ws_bytes, B.current_stream_ptr())

    def decode_stage_times(self, mode: int = B.TKPHI_MODE_SUB) -> list:
        return B.tkphi_decode_stage_times(self.cfg, self.table.data_ptr(), self.n, self.max_L, self.max_K, mode,
                                          self.ws.data_ptr(), self.ws_bytes, B.current_stream_ptr())

    def status(self) -> int:
        return B.tkphi_read_device_status(self.ws.data_ptr(), B.current_stream_ptr())

    def set_topk(self, i: int, k: int) -> None:
        """Changes problem i's budget (<= max_K) and re-uploads the table."""
        assert 0 <= k <= self.max_K
        self.host_table[i].topk = int(k)
        raw = bytearray(bytes(memoryview(self.host_table).cast("B")))
        self.table.copy_(torch.frombuffer(raw, dtype=torch.uint8))

    def set_n_gen(self, i: int, n_gen: int) -> None:
        """Changes the number of generated tokens of problem i (<= cfg.max_gen; the rows must already be
        in its K, V buffers) and re-uploads the table."""
        assert 0 <= n_gen <= self.cfg.max_gen
        self.host_table[i].n_gen = int(n_gen)
        raw = bytearray(bytes(memoryview(self.host_table).cast("B")))
        self.table.copy_(torch.frombuffer(raw, dtype=torch.uint8))

    def set_query(self, i: int, q: np.ndarray) -> None:
        self.dev[i]["q"].copy_(to_device(q, self.device))

    def result(self, i: int, name: str) -> np.ndarray:
        t = self.dev[i][name]
        if t.dtype == torch.bfloat16:
            return t.view(torch.int16).cpu().numpy().view(np.uint16)
        return t.cpu().numpy()
