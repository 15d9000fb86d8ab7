"""Thin ctypes binding over libppmoe.so: the same entry points as include/ppmoe.h, taking torch
tensors (device memory) and passing their pointers.  Argument marshalling only -- every step of the
path runs in the HIP kernels.  There is no fallback: a missing library is an error."""

from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, byref, c_char_p, c_double, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libppmoe.so")

MOE_F32, MOE_BF16, MOE_F16 = 0, 1, 2
MOE_NUM_STAGES = 6
STAGE_NAMES = ("gate", "permute", "slice", "ffn_up", "ffn_down", "combine")


class MoeConfig(Structure):
    _fields_ = [("T", c_int32), ("d", c_int32), ("F", c_int32), ("E", c_int32), ("top_k", c_int32),
                ("local_begin", c_int32), ("local_count", c_int32), ("capacity_factor", c_float),
                ("renorm_topk", c_int32), ("in_dtype", c_int32), ("out_dtype", c_int32)]


class MoeWorkspaceLayout(Structure):
    _fields_ = [(n, c_size_t) for n in ("expert_idx", "gate_w", "counts", "offsets", "perm",
                                        "inv_perm", "x_sliced", "H", "y_sliced", "scratch", "gemm",
                                        "logits", "aux")]


class MoeError(RuntimeError):
    pass


_PROTOTYPES = {
    "moe_status_string": (c_char_p, [c_int]),
    "moe_init": (c_int, [c_void_p]),
    "moe_set_option": (c_int, [c_int, c_int64]),
    "moe_capacity": (c_int64, [POINTER(MoeConfig)]),
    "moe_max_rows": (c_int64, [POINTER(MoeConfig)]),
    "moe_workspace_bytes": (c_size_t, [POINTER(MoeConfig)]),
    "moe_dispatch_workspace_bytes": (c_size_t, [POINTER(MoeConfig)]),
    "moe_workspace_offsets": (c_int, [POINTER(MoeConfig), POINTER(MoeWorkspaceLayout)]),
    "moe_gate": (c_int, [POINTER(MoeConfig)] + [c_void_p] * 8),
    "moe_aux_workspace_bytes": (c_size_t, [POINTER(MoeConfig)]),
    "moe_aux_loss": (c_int, [POINTER(MoeConfig)] + [c_void_p] * 6 + [c_size_t, c_void_p]),
    "moe_slice_dispatch": (c_int, [POINTER(MoeConfig)] + [c_void_p] * 8 + [c_size_t, c_void_p]),
    "moe_slice_dispatch_static": (c_int, [POINTER(MoeConfig)] + [c_void_p] * 8),
    "moe_slice_rows": (c_int, [POINTER(MoeConfig)] + [c_void_p] * 5),
    "moe_ffn_workspace_bytes": (c_size_t, [POINTER(MoeConfig)]),
    "moe_expert_ffn_up": (c_int, [POINTER(MoeConfig)] + [c_void_p] * 5 + [c_size_t, c_void_p]),
    "moe_expert_ffn_down": (c_int, [POINTER(MoeConfig)] + [c_void_p] * 5 + [c_size_t, c_void_p]),
    "moe_expert_ffn": (c_int, [POINTER(MoeConfig)] + [c_void_p] * 7 + [c_size_t, c_void_p]),
    "moe_ffn_backward_workspace_bytes": (c_size_t, [POINTER(MoeConfig)]),
    "moe_expert_ffn_backward": (c_int, [POINTER(MoeConfig)] + [c_void_p] * 9 + [c_size_t, c_void_p]),
    "moe_layer_backward_workspace_bytes": (c_size_t, [POINTER(MoeConfig)]),
    "moe_layer_backward": (c_int, [POINTER(MoeConfig)] + [c_void_p] * 12 + [c_size_t, c_void_p]),
    "moe_layer_saved_bytes": (c_size_t, [POINTER(MoeConfig)]),
    "moe_layer_forward_train": (c_int, [POINTER(MoeConfig)] + [c_void_p] * 10 + [c_size_t, c_void_p, c_size_t, c_void_p]),
    "moe_layer_backward_saved": (c_int, [POINTER(MoeConfig)] + [c_void_p] * 6 + [c_size_t] + [c_void_p] * 6 +
                                 [c_size_t, c_void_p]),
    "moe_ffn_check": (c_int, [POINTER(MoeConfig), c_void_p, c_int, POINTER(c_int32), c_void_p]),
    "moe_ffn_clock": (c_int, [POINTER(MoeConfig), c_void_p, c_int, POINTER(c_double), POINTER(c_double), c_void_p]),
    "moe_combine": (c_int, [POINTER(MoeConfig)] + [c_void_p] * 5),
    "moe_layer_forward": (c_int, [POINTER(MoeConfig)] + [c_void_p] * 7 + [c_size_t, POINTER(c_void_p), c_void_p]),
    "moe_layer_forward_aux": (c_int, [POINTER(MoeConfig)] + [c_void_p] * 10 + [c_size_t, POINTER(c_void_p), c_void_p]),
    "moe_layer_fuses": (c_int, [POINTER(MoeConfig)]),
    "moe_copy_bytes": (c_int, [c_void_p, c_void_p, c_size_t, c_void_p]),
    "moe_mfma_probe": (c_int, [c_int64, c_int, c_void_p, POINTER(c_double), c_void_p]),
    "moe_event_create": (c_int, [POINTER(c_void_p)]),
    "moe_event_destroy": (c_int, [c_void_p]),
    "moe_event_record": (c_int, [c_void_p, c_void_p]),
    "moe_event_elapsed_ms": (c_int, [c_void_p, c_void_p, POINTER(c_float)]),
}
EXPORTED_SYMBOLS = tuple(_PROTOTYPES)

_lib = None


def load_library(path: str = LIB_PATH):
    """Load libppmoe.so (built in-tree by paper_2304_11414_amd.build).  Raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(path):
        raise MoeError(f"{path} is missing: build it with `python -m paper_2304_11414_amd.build` "
                       "(there is no CPU or PyTorch fallback)")
    lib = ctypes.CDLL(path)
    for name, (res, args) in _PROTOTYPES.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def _check(status: int, what: str):
    if status != 0:
        msg = load_library().moe_status_string(status).decode()
        raise MoeError(f"{what} failed: {msg} ({status})")


def _ptr(t):
    return None if t is None else c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return c_void_p(s.cuda_stream)


def make_config(T, d, F, E, top_k, local_begin=0, local_count=None, capacity_factor=0.0,
                renorm_topk=False, in_dtype="bf16", out_dtype="bf16") -> MoeConfig:
    code = {"f32": MOE_F32, "bf16": MOE_BF16, "f16": MOE_F16}
    return MoeConfig(T, d, F, E, top_k, local_begin, E if local_count in (None, -1) else local_count,
                     float(capacity_factor), int(bool(renorm_topk)), code[in_dtype], code[out_dtype])


def config_from(layer_cfg) -> MoeConfig:
    """From a synth.LayerConfig."""
    return make_config(layer_cfg.T, layer_cfg.d, layer_cfg.F, layer_cfg.E, layer_cfg.top_k,
                       layer_cfg.local_begin, layer_cfg.n_local, layer_cfg.capacity_factor,
                       layer_cfg.renorm_topk, layer_cfg.in_dtype, layer_cfg.out_dtype)


MOE_OPT_HANDOVER_DEVICE_SCOPE, MOE_OPT_HANDOVER_SPIN_LIMIT = 1, 2


def moe_init(stream=None):
    """One-time set-up of the current device (synchronises the stream; not under capture)."""
    _check(load_library().moe_init(_stream(stream)), "moe_init")


def moe_set_option(option: int, value: int):
    _check(load_library().moe_set_option(int(option), int(value)), "moe_set_option")


def moe_capacity(cfg) -> int:
    return load_library().moe_capacity(byref(cfg))


def moe_max_rows(cfg) -> int:
    return load_library().moe_max_rows(byref(cfg))


def moe_workspace_bytes(cfg) -> int:
    return load_library().moe_workspace_bytes(byref(cfg))


def moe_dispatch_workspace_bytes(cfg) -> int:
    return load_library().moe_dispatch_workspace_bytes(byref(cfg))


def moe_workspace_offsets(cfg) -> MoeWorkspaceLayout:
    L = MoeWorkspaceLayout()
    _check(load_library().moe_workspace_offsets(byref(cfg), byref(L)), "moe_workspace_offsets")
    return L


def moe_gate(cfg, x, Wg, bias, logits_in, logits_out, expert_idx, gate_w, stream=None):
    _check(load_library().moe_gate(byref(cfg), _ptr(x), _ptr(Wg), _ptr(bias), _ptr(logits_in),
                                   _ptr(logits_out), _ptr(expert_idx), _ptr(gate_w), _stream(stream)),
           "moe_gate")


def moe_aux_workspace_bytes(cfg) -> int:
    return load_library().moe_aux_workspace_bytes(byref(cfg))


def moe_aux_loss(cfg, logits, expert_idx, l_aux, mean_prob, first_counts, workspace, stream=None):
    _check(load_library().moe_aux_loss(byref(cfg), _ptr(logits), _ptr(expert_idx), _ptr(l_aux),
                                       _ptr(mean_prob), _ptr(first_counts), _ptr(workspace),
                                       _nbytes(workspace), _stream(stream)), "moe_aux_loss")


def moe_slice_dispatch(cfg, x, expert_idx, counts, offsets, perm, inv_perm, x_sliced, workspace,
                       stream=None):
    _check(load_library().moe_slice_dispatch(
        byref(cfg), _ptr(x), _ptr(expert_idx), _ptr(counts), _ptr(offsets), _ptr(perm),
        _ptr(inv_perm), _ptr(x_sliced), _ptr(workspace), workspace.numel() * workspace.element_size(),
        _stream(stream)), "moe_slice_dispatch")


MOE_STATIC_SCRATCH_BYTES = 4 << 20


def moe_slice_dispatch_static(cfg, x, expert_idx, counts, offsets, perm, inv_perm, x_sliced, stream=None):
    """moe_slice_dispatch without a workspace argument: nothing is allocated anywhere on the way."""
    _check(load_library().moe_slice_dispatch_static(
        byref(cfg), _ptr(x), _ptr(expert_idx), _ptr(counts), _ptr(offsets), _ptr(perm),
        _ptr(inv_perm), _ptr(x_sliced), _stream(stream)), "moe_slice_dispatch_static")


def moe_slice_rows(cfg, x, perm, offsets, x_sliced, stream=None):
    _check(load_library().moe_slice_rows(byref(cfg), _ptr(x), _ptr(perm), _ptr(offsets), _ptr(x_sliced),
                                         _stream(stream)), "moe_slice_rows")


def moe_ffn_workspace_bytes(cfg) -> int:
    return load_library().moe_ffn_workspace_bytes(byref(cfg))


def _nbytes(t):
    return t.numel() * t.element_size()


def moe_expert_ffn_up(cfg, x_sliced, offsets, W1, H, workspace, stream=None):
    _check(load_library().moe_expert_ffn_up(byref(cfg), _ptr(x_sliced), _ptr(offsets), _ptr(W1),
                                            _ptr(H), _ptr(workspace), _nbytes(workspace),
                                            _stream(stream)), "moe_expert_ffn_up")


def moe_expert_ffn_down(cfg, H, offsets, W2, y_sliced, workspace, stream=None):
    _check(load_library().moe_expert_ffn_down(byref(cfg), _ptr(H), _ptr(offsets), _ptr(W2),
                                              _ptr(y_sliced), _ptr(workspace), _nbytes(workspace),
                                              _stream(stream)), "moe_expert_ffn_down")


def moe_expert_ffn(cfg, x_sliced, offsets, W1, W2, H, y_sliced, workspace, stream=None):
    _check(load_library().moe_expert_ffn(byref(cfg), _ptr(x_sliced), _ptr(offsets), _ptr(W1),
                                         _ptr(W2), _ptr(H), _ptr(y_sliced), _ptr(workspace),
                                         _nbytes(workspace), _stream(stream)), "moe_expert_ffn")


def moe_ffn_backward_workspace_bytes(cfg) -> int:
    return load_library().moe_ffn_backward_workspace_bytes(byref(cfg))


def moe_expert_ffn_backward(cfg, x_sliced, offsets, W1, W2, dY, dX_sliced, dW1, dW2, workspace, stream=None):
    _check(load_library().moe_expert_ffn_backward(
        byref(cfg), _ptr(x_sliced), _ptr(offsets), _ptr(W1), _ptr(W2), _ptr(dY), _ptr(dX_sliced), _ptr(dW1),
        _ptr(dW2), _ptr(workspace), _nbytes(workspace), _stream(stream)), "moe_expert_ffn_backward")


def moe_layer_backward_workspace_bytes(cfg) -> int:
    return load_library().moe_layer_backward_workspace_bytes(byref(cfg))


def moe_layer_backward(cfg, x, Wg, bias, W1, W2, d_out, dx, dWg, dbias, dW1, dW2, workspace, stream=None):
    _check(load_library().moe_layer_backward(
        byref(cfg), _ptr(x), _ptr(Wg), _ptr(bias), _ptr(W1), _ptr(W2), _ptr(d_out), _ptr(dx), _ptr(dWg),
        _ptr(dbias), _ptr(dW1), _ptr(dW2), _ptr(workspace), _nbytes(workspace), _stream(stream)),
        "moe_layer_backward")


def moe_layer_saved_bytes(cfg) -> int:
    return load_library().moe_layer_saved_bytes(byref(cfg))


def moe_layer_forward_train(cfg, x, Wg, bias, W1, W2, out, l_aux, mean_prob, first_counts, saved, workspace,
                            stream=None):
    """The layer's forward that keeps in `saved` what moe_layer_backward_saved reads (l_aux, mean_prob,
    first_counts may be None)."""
    _check(load_library().moe_layer_forward_train(
        byref(cfg), _ptr(x), _ptr(Wg), _ptr(bias), _ptr(W1), _ptr(W2), _ptr(out), _ptr(l_aux),
        _ptr(mean_prob), _ptr(first_counts), _ptr(saved), _nbytes(saved), _ptr(workspace), _nbytes(workspace),
        _stream(stream)), "moe_layer_forward_train")


def moe_layer_backward_saved(cfg, x, Wg, W1, W2, d_out, saved, dx, dWg, dbias, dW1, dW2, workspace, stream=None):
    _check(load_library().moe_layer_backward_saved(
        byref(cfg), _ptr(x), _ptr(Wg), _ptr(W1), _ptr(W2), _ptr(d_out), _ptr(saved), _nbytes(saved), _ptr(dx),
        _ptr(dWg), _ptr(dbias), _ptr(dW1), _ptr(dW2), _ptr(workspace), _nbytes(workspace), _stream(stream)),
        "moe_layer_backward_saved")


def moe_ffn_check(cfg, workspace, layer_workspace, stream=None) -> int:
    """0 when every hand-over of partial sums since the last check went through (synchronises)."""
    status = c_int32(-1)
    _check(load_library().moe_ffn_check(byref(cfg), _ptr(workspace), int(bool(layer_workspace)),
                                        byref(status), _stream(stream)), "moe_ffn_check")
    return status.value


def moe_ffn_clock(cfg, workspace, layer_workspace, stream=None):
    """(shader clock in GHz, lifetime in microseconds) of the first block of the last fast-path GEMM
    launch on `workspace` (synchronises); (0, 0) if there was none."""
    ghz, us = c_double(0.0), c_double(0.0)
    _check(load_library().moe_ffn_clock(byref(cfg), _ptr(workspace), int(bool(layer_workspace)),
                                        byref(ghz), byref(us), _stream(stream)), "moe_ffn_clock")
    return ghz.value, us.value


def moe_combine(cfg, y_sliced, inv_perm, gate_w, out, stream=None):
    _check(load_library().moe_combine(byref(cfg), _ptr(y_sliced), _ptr(inv_perm), _ptr(gate_w),
                                      _ptr(out), _stream(stream)), "moe_combine")


def moe_layer_forward(cfg, x, Wg, bias, W1, W2, out, workspace, stage_events=None, stream=None):
    ev = None
    if stage_events is not None:
        assert len(stage_events) == MOE_NUM_STAGES + 1
        ev = (c_void_p * (MOE_NUM_STAGES + 1))(*stage_events)
    _check(load_library().moe_layer_forward(
        byref(cfg), _ptr(x), _ptr(Wg), _ptr(bias), _ptr(W1), _ptr(W2), _ptr(out), _ptr(workspace),
        workspace.numel() * workspace.element_size(), ev, _stream(stream)), "moe_layer_forward")


def moe_layer_forward_aux(cfg, x, Wg, bias, W1, W2, out, l_aux, mean_prob, first_counts, workspace,
                          stage_events=None, stream=None):
    """The layer plus Algorithm 1's second return value (device tensors l_aux[1], mean_prob[E],
    first_counts[E]; the last two may be None)."""
    ev = None
    if stage_events is not None:
        assert len(stage_events) == MOE_NUM_STAGES + 1
        ev = (c_void_p * (MOE_NUM_STAGES + 1))(*stage_events)
    _check(load_library().moe_layer_forward_aux(
        byref(cfg), _ptr(x), _ptr(Wg), _ptr(bias), _ptr(W1), _ptr(W2), _ptr(out), _ptr(l_aux),
        _ptr(mean_prob), _ptr(first_counts), _ptr(workspace), _nbytes(workspace), ev, _stream(stream)),
        "moe_layer_forward_aux")


MOE_FUSE_SLICE, MOE_FUSE_COMBINE = 1, 2


def moe_layer_fuses(cfg) -> int:
    """Mask of MOE_FUSE_SLICE / MOE_FUSE_COMBINE: the stages moe_layer_forward folds into the GEMMs."""
    return load_library().moe_layer_fuses(byref(cfg))


def moe_copy_bytes(src, dst, stream=None):
    _check(load_library().moe_copy_bytes(_ptr(src), _ptr(dst), _nbytes(src), _stream(stream)),
           "moe_copy_bytes")


def moe_mfma_probe(iters, random_operands, sink, stream=None) -> float:
    """Launches the probe; returns the flop count of the launch."""
    fl = c_double()
    _check(load_library().moe_mfma_probe(int(iters), int(bool(random_operands)), _ptr(sink), byref(fl),
                                         _stream(stream)), "moe_mfma_probe")
    return fl.value


def moe_event_create() -> int:
    ev = c_void_p()
    _check(load_library().moe_event_create(byref(ev)), "moe_event_create")
    return ev.value


def moe_event_destroy(ev):
    _check(load_library().moe_event_destroy(c_void_p(ev)), "moe_event_destroy")


def moe_event_record(ev, stream=None):
    _check(load_library().moe_event_record(c_void_p(ev), _stream(stream)), "moe_event_record")


def moe_event_elapsed_ms(start, stop) -> float:
    ms = c_float()
    _check(load_library().moe_event_elapsed_ms(c_void_p(start), c_void_p(stop), byref(ms)),
           "moe_event_elapsed_ms")
    return ms.value


def workspace_views(cfg, workspace):
    """Typed views of the intermediates moe_layer_forward left in `workspace` (a uint8 tensor)."""
    import torch
    L = moe_workspace_offsets(cfg)
    tk = cfg.T * cfg.top_k
    rows = moe_max_rows(cfg)
    n = cfg.local_count
    et = {MOE_BF16: torch.bfloat16, MOE_F16: torch.float16, MOE_F32: torch.float32}[cfg.in_dtype]
    eb = 4 if cfg.in_dtype == MOE_F32 else 2

    def view(off, count, dtype, size):
        return workspace[off:off + count * size].view(dtype)

    return dict(
        expert_idx=view(L.expert_idx, tk, torch.int32, 4).view(cfg.T, cfg.top_k),
        gate_w=view(L.gate_w, tk, torch.float32, 4).view(cfg.T, cfg.top_k),
        counts=view(L.counts, n, torch.int32, 4),
        offsets=view(L.offsets, n + 1, torch.int32, 4),
        perm=view(L.perm, rows, torch.int32, 4),
        inv_perm=view(L.inv_perm, tk, torch.int32, 4).view(cfg.T, cfg.top_k),
        x_sliced=view(L.x_sliced, rows * cfg.d, et, eb).view(rows, cfg.d),
        H=view(L.H, rows * cfg.F, et, eb).view(rows, cfg.F),
        y_sliced=view(L.y_sliced, rows * cfg.d, et, eb).view(rows, cfg.d),
    )
