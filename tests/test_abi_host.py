"""CPU-only checks of the C-ABI library: it loads, exports every function include/ppmoe.h declares,
and its host-side logic (capacity, row bounds, workspace layout, argument validation) is right.
No kernel is launched here."""

import ctypes
import os
import re

import pytest

from oracle import ppmoe_oracle as O
from paper_2304_11414_amd import binding as B
from paper_2304_11414_amd import build as build_mod
from paper_2304_11414_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        build_mod.build_library()
    return B.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ppmoe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_function_is_exported_and_bound(lib):
    names = declared_functions()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), f"{n} declared in ppmoe.h but not exported"
    assert sorted(B.EXPORTED_SYMBOLS) == names       # the Python binding carries the same names


def test_config_struct_matches_header():
    assert ctypes.sizeof(B.MoeConfig) == 11 * 4
    assert [f[0] for f in B.MoeConfig._fields_] == [
        "T", "d", "F", "E", "top_k", "local_begin", "local_count", "capacity_factor", "renorm_topk",
        "in_dtype", "out_dtype"]


def test_capacity_and_row_bounds_match_oracle(lib):
    for lc in synth.CONFIGS:
        cfg = B.config_from(lc)
        cap = O.capacity(lc.capacity_factor, lc.top_k, lc.T, lc.E)
        assert B.moe_capacity(cfg) == (-1 if cap is None else cap)
    assert B.moe_capacity(B.config_from(synth.CONFIGS[2])) == 2560
    assert B.moe_capacity(B.make_config(20, 64, 64, 4, 1, capacity_factor=1.2)) == 7   # float32(1.2) > 1.2
    for cf, k, T, E in [(1.0, 1, 10, 4), (0.5, 2, 1001, 7), (1.25, 2, 16384, 16), (2.0, 1, 5, 8),
                        (1.1, 1, 1000, 10), (1.2, 1, 20, 4), (0.7, 1, 30, 3), (1.3, 2, 12345, 7),
                        (0.9, 1, 70000, 9), (1.1, 2, 65536, 11)]:
        cfg = B.make_config(T, 64, 64, E, k, capacity_factor=cf)
        assert B.moe_capacity(cfg) == O.capacity(cf, k, T, E)
    # packed-row bound: k*T without capacity; min(k*T, N*min(C, T)) with one
    assert B.moe_max_rows(B.config_from(synth.CONFIGS[1])) == 8192
    assert B.moe_max_rows(B.config_from(synth.CONFIGS[2])) == 32768          # 16 * 2560 > 2 * 16384
    assert B.moe_max_rows(B.config_from(synth.CONFIGS[3])) == 16384
    assert B.moe_max_rows(B.make_config(1000, 64, 64, 8, 2, 0, 2, capacity_factor=0.5)) == 250
    assert B.moe_max_rows(B.make_config(1000, 64, 64, 8, 2, 0, 1)) == 1000   # one expert: at most T


def test_workspace_layout_is_disjoint_and_aligned(lib):
    for lc in synth.CONFIGS:
        cfg = B.config_from(lc)
        total = B.moe_workspace_bytes(cfg)
        L = B.moe_workspace_offsets(cfg)
        rows, tk = B.moe_max_rows(cfg), lc.T * lc.top_k
        eb = 2 if lc.in_dtype == "bf16" else 4
        sizes = dict(scratch=B.moe_dispatch_workspace_bytes(cfg), expert_idx=tk * 4, gate_w=tk * 4,
                     counts=lc.n_local * 4, offsets=(lc.n_local + 1) * 4, perm=rows * 4,
                     inv_perm=tk * 4, x_sliced=rows * lc.d * eb, H=rows * lc.F * eb,
                     y_sliced=rows * lc.d * eb, gemm=B.moe_ffn_workspace_bytes(cfg),
                     logits=lc.T * lc.E * 4, aux=B.moe_aux_workspace_bytes(cfg))
        spans = sorted((getattr(L, n), getattr(L, n) + s) for n, s in sizes.items())
        for (a0, a1), (b0, b1) in zip(spans, spans[1:]):
            assert a1 <= b0
        assert all(a0 % 256 == 0 for a0, _ in spans) and spans[-1][1] <= total
        assert B.moe_dispatch_workspace_bytes(cfg) <= total


def test_invalid_arguments_are_rejected_before_any_launch(lib):
    ok = B.make_config(64, 64, 64, 4, 1)
    bad_shapes = [dict(T=-1), dict(d=12), dict(F=0), dict(E=0), dict(E=257), dict(top_k=0),
                  dict(top_k=5), dict(local_begin=3, local_count=2), dict(local_count=0)]
    for kw in bad_shapes:
        args = dict(T=64, d=64, F=64, E=4, top_k=1, local_begin=0, local_count=4)
        args.update(kw)
        cfg = B.make_config(**args)
        assert B.moe_workspace_bytes(cfg) == 0, kw
        assert lib.moe_gate(ctypes.byref(cfg), *([None] * 8)) == -2, kw
    cfg = B.make_config(64, 64, 64, 4, 1, in_dtype="f32", out_dtype="bf16")
    assert lib.moe_gate(ctypes.byref(cfg), *([None] * 8)) == -3
    assert lib.moe_gate(ctypes.byref(ok), *([None] * 8)) == -1                  # NULL outputs
    p = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    assert lib.moe_gate(ctypes.byref(ok), odd, p, None, None, None, p, p, None) == -4
    assert lib.moe_combine(ctypes.byref(ok), p, p, p, None, None) == -1
    assert lib.moe_slice_dispatch(ctypes.byref(ok), p, p, p, p, p, p, p, p, 0, None) == -5
    assert lib.moe_layer_forward(ctypes.byref(ok), p, p, None, p, p, p, p, 16, None, None) == -5
    assert lib.moe_layer_forward(None, p, p, None, p, p, p, p, 16, None, None) == -1
    assert lib.moe_status_string(-5) == b"workspace too small"
    assert lib.moe_status_string(0) == b"ok"
    with pytest.raises(B.MoeError):
        B._check(-2, "x")


def test_missing_library_is_a_loud_error(tmp_path, monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    with pytest.raises(B.MoeError):
        B.load_library(str(tmp_path / "libppmoe.so"))


def test_skew_recipe_of_the_wide_config():
    """The Zipf(1.5) router bias of the skewed workload puts about 45 % of the assignments on the
    heaviest expert (checked on a 1/8 sample of its tokens)."""
    import numpy as np
    lc = synth.CONFIGS[4].scaled(T=4096)
    inp = synth.make_inputs(lc, parts=("x", "Wg_t", "bias"))
    _, idx, _ = O.gate(inp["x"], inp["Wg_t"].T, inp["bias"], lc.top_k, lc.renorm_topk)
    share = np.bincount(idx.reshape(-1), minlength=lc.E) / idx.size
    assert abs(share[0] - 0.45) < 0.015 and np.all(np.diff(share) < 0)


def test_set_option_validates_on_the_host(lib):
    with pytest.raises(B.MoeError):
        B.moe_set_option(99, 1)
    with pytest.raises(B.MoeError):
        B.moe_set_option(B.MOE_OPT_HANDOVER_SPIN_LIMIT, -1)
    B.moe_set_option(B.MOE_OPT_HANDOVER_DEVICE_SCOPE, 0)
    B.moe_set_option(B.MOE_OPT_HANDOVER_SPIN_LIMIT, 1 << 17)
