"""Shared plumbing for the GPU parity tests: move synthetic inputs to the device, call the
C ABI through the binding, run the oracle on the same inputs."""
from __future__ import annotations

import math

import numpy as np
import torch

from oracle import lukv_oracle as O
from paper_2602_08585_amd import lukv, synth


def dev(x: np.ndarray, bf16: bool = False) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x))
    if x.dtype == np.uint16:
        t = t.view(torch.bfloat16)
    return t.cuda()


def host_bits(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> numpy, bf16 as uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.uint16).numpy()
    return t.numpy()


class Problem:
    """A workload's inputs on host and device, plus its lukv Config and workspace."""

    def __init__(self, wl: synth.Workload, layers=None, data=None, alloc=None, workers=1):
        self.wl = wl
        self.data = synth.make_qkv(wl, layers, workers=workers) if data is None else data
        self.alloc = synth.make_allocation_inputs(wl) if alloc is None else alloc
        self.q = dev(self.data["q_win"])
        self.k = dev(self.data["k"])
        self.v = dev(self.data["v"])
        self.cfg = lukv.Config.for_tensors(self.q, self.k, wl.window, wl.cu_seqlens.tolist(),
                                           wl.pool_kernel, wl.n_sink)
        self.curves = dev(self.alloc["curves"])
        self.knots = dev(self.alloc["knots"])
        self.b_min = dev(self.alloc["b_min"])
        self.b_max = dev(self.alloc["b_max"])
        self.B = [int(x) for x in self.alloc["B"]]
        self.ws = lukv.alloc_workspace(lukv.lukv_workspace_bytes(self.cfg, wl.n_grid))
        self.n_hi = self.cfg.n_heads_total

    # ---- outputs ----
    def new_outputs(self, rows=None):
        rows = sum(self.B) if rows is None else rows
        wl = self.wl
        tdt = self.k.dtype
        out = {
            "budgets": torch.full((self.n_hi,), -7, dtype=torch.int32, device="cuda"),
            "offsets": torch.full((self.n_hi + 1,), -7, dtype=torch.int64, device="cuda"),
            "kept_idx": torch.full((max(rows, 1),), -7, dtype=torch.int32, device="cuda"),
            "k_out": torch.zeros((max(rows, 1), wl.head_dim), dtype=tdt, device="cuda"),
            "v_out": torch.zeros((max(rows, 1), wl.head_dim), dtype=tdt, device="cuda"),
            "pooled": torch.full((self.k.shape[0], wl.n_kv_heads, wl.total_len), float("nan"),
                                 dtype=torch.float32, device="cuda"),
            "status": torch.full((wl.n_seqs + 1,), -7, dtype=torch.int32, device="cuda"),
        }
        return out

    def evict(self, out=None, with_pooled=True):
        out = self.new_outputs() if out is None else out
        lukv.lukv_evict(self.cfg, self.q, self.k, self.v, self.wl.n_grid, self.curves, self.knots,
                        self.b_min, self.b_max, self.B, out["budgets"], out["offsets"],
                        out["kept_idx"], out["k_out"], out["v_out"],
                        out["pooled"] if with_pooled else None, out["status"], self.ws)
        torch.cuda.synchronize()
        return out

    def oracle(self, layers=None, lse=None):
        wl, a = self.wl, self.alloc
        return O.evict(self.data["q_win"], self.data["k"], self.data["v"], wl.cu_seqlens,
                       wl.n_kv_heads, wl.window, wl.pool_kernel, wl.n_sink, a["curves"], a["knots"],
                       a["b_min"], a["b_max"], a["B"], layers=layers, lse=lse)

    def oracle_lse(self):
        """The window rows' log-sum-exp as the oracle computes it (fp64, rounded to fp32):
        [NL, H_q, n_seqs*w], the extra INPUT of the lse variants."""
        wl = self.wl
        q, k = self.data["q_win"], self.data["k"]
        out = np.zeros((q.shape[0], wl.n_q_heads, wl.n_seqs * wl.window), np.float32)
        cu = wl.cu_seqlens
        for l in range(q.shape[0]):
            for s in range(wl.n_seqs):
                sl = slice(s * wl.window, (s + 1) * wl.window)
                out[l, :, sl] = O.window_lse(O.decode(q[l, :, sl, :]), O.decode(k[l, :, cu[s]:cu[s + 1], :]),
                                             wl.n_kv_heads)
        return out

    def evict_lse(self, lse, out=None, with_pooled=True):
        out = self.new_outputs() if out is None else out
        lukv.lukv_evict_lse(self.cfg, self.q, self.k, self.v, lse, self.wl.n_grid, self.curves,
                            self.knots, self.b_min, self.b_max, self.B, out["budgets"], out["offsets"],
                            out["kept_idx"], out["k_out"], out["v_out"],
                            out["pooled"] if with_pooled else None, out["status"], self.ws)
        torch.cuda.synchronize()
        return out


def assert_scores_close(got: np.ndarray, want: np.ndarray, rtol=1e-3):
    """|g - o| <= rtol*|o| + 1e-12 on finite entries; infinities must coincide."""
    assert got.shape == want.shape
    assert np.array_equal(np.isinf(want), np.isinf(got)), "forced (+inf) positions differ"
    assert not np.isnan(got).any()
    fin = np.isfinite(want)
    err = np.abs(got[fin].astype(np.float64) - want[fin].astype(np.float64))
    bound = rtol * np.abs(want[fin].astype(np.float64)) + 1e-12
    worst = float((err / bound).max()) if err.size else 0.0
    assert worst <= 1.0, "score error %.3g x tolerance" % worst
    return worst


def check_band(kept_gpu: np.ndarray, kept_orc: np.ndarray, scores_orc: np.ndarray, band: float):
    """Fused-path rule: the two kept sets have equal size and may differ only at positions
    whose oracle score lies within `band` (relative) of the oracle's k-th score."""
    assert kept_gpu.size == kept_orc.size
    assert np.all(np.diff(kept_gpu) > 0), "kept positions not strictly ascending"
    if np.array_equal(kept_gpu, kept_orc):
        return 0
    k = kept_orc.size
    thr = np.sort(scores_orc.astype(np.float64))[::-1][k - 1]
    diff = np.setxor1d(kept_gpu, kept_orc)
    s = scores_orc[diff].astype(np.float64)
    assert np.all(np.abs(s - thr) <= band * abs(thr)), "kept sets differ outside the tolerance band"
    return int(diff.size)
