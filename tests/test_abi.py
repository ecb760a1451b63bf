"""Host-only checks of the C-ABI library: it loads without a GPU, exports every function
include/lukv.h declares, and refuses bad configurations on the host (no compute calls)."""
import ctypes
import os
import re

import pytest

from paper_2602_08585_amd import lukv, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lukv_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = lukv.load_library()
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["lukv.h", "lukv_bench.h"]
    assert set(_declared("lukv.h")) == set(lukv.EXPORTS)
    assert set(_declared("lukv_bench.h")) == set(lukv.BENCH_EXPORTS)
    for n in lukv.EXPORTS + lukv.BENCH_EXPORTS:
        assert hasattr(lib, n), n


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    """lukv_evict_static: a configuration whose workspace exceeds the built-in scratch is refused on
    the host before anything touches a device."""
    lib = lukv.load_library()
    fake = ctypes.c_void_p(256)       # never dereferenced
    B = (ctypes.c_int64 * 1)(1000)
    big = _cfg(cu_seqlens=[0, 131072], stride_head=131072 * 128, stride_layer=8 * 131072 * 128)
    assert lukv.lukv_workspace_bytes(big, 64) > lukv.LUKV_STATIC_SCRATCH_BYTES
    assert lukv.lukv_workspace_bytes(_cfg(), 64) <= lukv.LUKV_STATIC_SCRATCH_BYTES
    rc = lib.lukv_evict_static(ctypes.byref(big.to_c()), fake, fake, fake, 64, fake, fake, fake, fake, B,
                               fake, fake, fake, fake, fake, None, fake, None)
    assert rc == lukv.LUKV_EWORKSPACE


def test_strerror_covers_codes():
    for code in (0, -1, -2, -3, -4, -5):
        assert "unknown" not in lukv.strerror(code)
    assert "unknown" in lukv.strerror(-99)


def _cfg(**kw):
    base = dict(n_layers=1, n_q_heads=32, n_kv_heads=8, head_dim=128, window=32, pool_kernel=7,
                n_sink=4, dtype=lukv.LUKV_BF16, cu_seqlens=[0, 32768], stride_layer=8 * 32768 * 128,
                stride_head=32768 * 128, stride_tok=128, qstride_layer=32 * 32 * 128,
                qstride_head=32 * 128, qstride_tok=128)
    base.update(kw)
    return lukv.Config(**base)


def test_workspace_bytes_is_pure_and_monotone():
    a = lukv.lukv_workspace_bytes(_cfg(), 64)
    assert a == lukv.lukv_workspace_bytes(_cfg(), 64) and a > 2 * 8 * 32768 * 4
    assert lukv.lukv_workspace_bytes(_cfg(cu_seqlens=[0, 65536]), 64) > a
    assert lukv.lukv_allocate_workspace_bytes(1, 8, 64) <= a


@pytest.mark.parametrize("kw,code", [
    (dict(n_kv_heads=5), lukv.LUKV_EINVAL),             # G not integral
    (dict(head_dim=96), lukv.LUKV_EDTYPE),
    (dict(dtype=7), lukv.LUKV_EDTYPE),
    (dict(pool_kernel=4), lukv.LUKV_EINVAL),            # even kernel
    (dict(cu_seqlens=[0, 32]), lukv.LUKV_EINVAL),       # context not longer than the window
    (dict(cu_seqlens=[0, 34]), lukv.LUKV_EINVAL),       # n_sink > L - w
    (dict(cu_seqlens=[1, 4096]), lukv.LUKV_EINVAL),
    (dict(stride_tok=100), lukv.LUKV_EINVAL),           # rows not 16-byte aligned / < head_dim
    (dict(window=256), lukv.LUKV_EINVAL),               # G*w > 512
    (dict(cu_seqlens=list(range(0, 66 * 64, 64))), lukv.LUKV_EINVAL),   # > LUKV_MAX_SEQS
    (dict(softmax_scale=-1.0), lukv.LUKV_EINVAL),
])
def test_bad_configurations_are_refused(kw, code):
    with pytest.raises(lukv.LukvError) as e:
        lukv.lukv_workspace_bytes(_cfg(**kw), 64)
    assert e.value.code == code


def test_named_workloads_are_accepted():
    for name in ("tiny", "8b_32k", "8b_full_20", "long_128k", "batched"):
        wl = synth.workload(name)
        T, d = wl.total_len, wl.head_dim
        cfg = lukv.Config(wl.n_layers, wl.n_q_heads, wl.n_kv_heads, d, wl.window, wl.pool_kernel,
                          wl.n_sink, lukv.LUKV_F32 if wl.dtype == synth.F32 else lukv.LUKV_BF16,
                          wl.cu_seqlens.tolist(), wl.n_kv_heads * T * d, T * d, d,
                          wl.n_q_heads * wl.n_seqs * wl.window * d, wl.n_seqs * wl.window * d, d)
        assert lukv.lukv_workspace_bytes(cfg, wl.n_grid) > 0


def test_synth_budgets_match_named_configs():
    assert synth.workload("tiny").budget_total(0) == 819
    assert synth.workload("8b_32k").budget_total(0) == 52428
    assert synth.workload("8b_full_20").budget_total(0) == 1677721
    assert synth.workload("8b_full_10").budget_total(0) == 838860
    assert synth.workload("long_128k").budget_total(0) == 1677721


def test_host_refusals_of_the_profile_and_lse_entry_points():
    """Nothing here reaches a kernel: bad dimensions, null pointers and unordered grids are
    refused on the host."""
    lib = lukv.load_library()
    out = ctypes.c_int64(0)
    assert lib.lukv_profile_workspace_bytes(0, 8, 64, ctypes.byref(out)) == lukv.LUKV_EINVAL
    assert lib.lukv_profile_workspace_bytes(65, 8, 64, ctypes.byref(out)) == lukv.LUKV_EINVAL
    assert lib.lukv_profile_workspace_bytes(3, 8, 64, ctypes.byref(out)) == lukv.LUKV_OK and out.value > 0
    rho_bad = (ctypes.c_double * 3)(0.0, 0.5, 0.5)
    rho_ok = (ctypes.c_double * 3)(0.0, 0.5, 1.0)
    fake = ctypes.c_void_p(256)       # never dereferenced: the calls below are refused first
    assert lib.lukv_profile_build(3, 8, 64, fake, fake, fake, fake, 4096, 3, rho_bad, fake, fake, 1 << 30,
                                  None) == lukv.LUKV_EINVAL
    assert lib.lukv_profile_build(3, 8, 64, fake, fake, fake, fake, 4096, 3, rho_ok, fake, fake, 16,
                                  None) == lukv.LUKV_EWORKSPACE
    assert lib.lukv_budgets_from_profile(8, 3, rho_bad, fake, 0.5, 4096, fake, fake, fake, fake,
                                         None) == lukv.LUKV_EINVAL
    assert lib.lukv_budgets_from_profile(8, 3, rho_ok, None, 0.5, 4096, fake, fake, fake, fake,
                                         None) == lukv.LUKV_EINVAL
    assert lib.lukv_budgets_from_profile(8, 3, rho_ok, fake, float("nan"), 4096, fake, fake, fake, fake,
                                         None) == lukv.LUKV_EINVAL
    c = _cfg().to_c()
    assert lib.lukv_score_lse(ctypes.byref(c), fake, fake, None, fake, fake, 1 << 40, None) == lukv.LUKV_EINVAL
    assert lib.lukv_evict_budgets(ctypes.byref(c), fake, fake, fake, None, None, fake, 10, fake, fake, fake,
                                  None, fake, fake, 1 << 40, None) == lukv.LUKV_EINVAL


def test_host_refusals_of_the_topk_allocation():
    lib = lukv.load_library()
    fake = ctypes.c_void_p(256)       # never dereferenced
    c = _cfg().to_c()
    B = (ctypes.c_int64 * 1)(1000)
    neg = (ctypes.c_int64 * 1)(-1)
    args = lambda Bp, floor, ws_bytes: (ctypes.byref(c), fake, Bp, floor, fake, fake, fake, fake, ws_bytes, None)
    assert lib.lukv_allocate_topk(*args(B, -1, 1 << 40)) == lukv.LUKV_EINVAL
    assert lib.lukv_allocate_topk(*args(neg, 0, 1 << 40)) == lukv.LUKV_EINFEASIBLE
    assert lib.lukv_allocate_topk(*args(B, 0, 16)) == lukv.LUKV_EWORKSPACE
    assert lib.lukv_allocate_topk(ctypes.byref(c), None, B, 0, fake, fake, fake, fake, 1 << 40, None) == lukv.LUKV_EINVAL
    many = _cfg(n_layers=600, n_q_heads=8, n_kv_heads=8, qstride_layer=8 * 32 * 128, qstride_head=32 * 128).to_c()
    assert lib.lukv_allocate_topk(ctypes.byref(many), fake, B, 0, fake, fake, fake, fake, 1 << 50, None) == lukv.LUKV_EINVAL


def test_sequences_longer_than_the_limit_are_refused():
    with pytest.raises(lukv.LukvError):
        lukv.lukv_workspace_bytes(_cfg(cu_seqlens=[0, (1 << 20) + 1], stride_head=((1 << 20) + 1) * 128,
                                       stride_layer=8 * ((1 << 20) + 1) * 128), 64)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_synthetic_inputs_are_seeded_and_bf16_rounding_is_nearest_even():
    import numpy as np
    import torch
    wl = synth.workload("tiny")
    a, b = synth.make_qkv(wl), synth.make_qkv(wl)
    for key in ("q_win", "k", "v"):
        assert np.array_equal(a[key], b[key])
    c = synth.make_qkv(__import__("dataclasses").replace(wl, seed=wl.seed + 1))
    assert not np.array_equal(a["k"], c["k"])
    x = np.random.default_rng(0).standard_normal(4096).astype(np.float32)
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 3.0e38]          # exact ties (to even) and a large value
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.uint16).numpy()
    assert np.array_equal(synth.f32_to_bf16_bits(x), want)
    al = synth.make_allocation_inputs(wl)
    assert int(al["B"][0]) == 819 and al["curves"].shape == (1, 4, 32) and np.all(al["knots"][..., 0] == 0)
    assert np.all(np.diff(al["knots"], axis=-1) > 0) and np.all(np.diff(al["curves"], axis=-1) >= 0)
