"""lukv_evict_static (the entry point that allocates nothing, scratch inside the library) against
lukv_evict on the same inputs: every output bit for bit, on two calls in a row, the second with a
smaller input, so that whatever the first call left in the library's scratch is seen to be harmless."""
import numpy as np
import pytest
import torch

from paper_2602_08585_amd import lukv, synth
from tests.helpers import Problem

pytestmark = pytest.mark.gpu


def _both(p):
    want = p.evict()
    got = p.new_outputs()
    wl = p.wl
    lukv.lukv_evict_static(p.cfg, p.q, p.k, p.v, wl.n_grid, p.curves, p.knots, p.b_min, p.b_max, p.B,
                           got["budgets"], got["offsets"], got["kept_idx"], got["k_out"], got["v_out"],
                           got["pooled"], got["status"])
    torch.cuda.synchronize()
    for key in ("budgets", "offsets", "kept_idx", "k_out", "v_out", "status"):
        assert torch.equal(got[key], want[key]), (wl.name, key)
    assert torch.equal(got["pooled"].view(torch.int32), want["pooled"].view(torch.int32)), wl.name
    assert int(got["status"].abs().sum()) == 0
    return got


def test_static_scratch_entry_point_matches_lukv_evict_twice_in_a_row():
    print("case lukv_evict_static: 8b_32k, then a smaller ragged problem", flush=True)
    big = Problem(synth.workload("8b_32k"))
    assert lukv.lukv_workspace_bytes(big.cfg, big.wl.n_grid) <= lukv.LUKV_STATIC_SCRATCH_BYTES
    _both(big)
    small = Problem(synth.Workload(name="static_small", n_layers=2, n_q_heads=8, n_kv_heads=4, head_dim=128,
                                   seq_lens=[700, 1300, 2049], window=32, pool_kernel=7, n_sink=4,
                                   dtype=synth.BF16, keep_ratio=0.2, n_grid=16, heavy_frac=0.02, seed=1234,
                                   q_gain=128.0))
    _both(small)
    _both(Problem(synth.workload("tiny")))
    # a configuration that does not fit is refused, nothing enqueued
    cfg = lukv.Config(1, 8, 8, 64, 16, 7, 4, lukv.LUKV_BF16, [0, 200000], 8 * 200000 * 64, 200000 * 64, 64,
                      8 * 16 * 64, 16 * 64, 64)
    assert lukv.lukv_workspace_bytes(cfg, 8) > lukv.LUKV_STATIC_SCRATCH_BYTES
    out = small.new_outputs()
    with pytest.raises(lukv.LukvError) as e:
        lukv.lukv_evict_static(cfg, small.q, small.k, small.v, 8, small.curves, small.knots, small.b_min,
                               small.b_max, [100], out["budgets"], out["offsets"], out["kept_idx"],
                               out["k_out"], out["v_out"], None, out["status"])
    assert e.value.code == lukv.LUKV_EWORKSPACE
    torch.cuda.synchronize()
    assert int(out["budgets"][0]) == -7
