"""Helpers for the GPU parity tests: moving seeded NumPy inputs to the device, running the C-ABI
stages, and the error measures the tolerances are written in."""

from __future__ import annotations

import numpy as np

from paper_2304_11414_amd import binding as B


def torch_dtype(name):
    import torch
    return {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[name]


def to_dev(a, dtype_name=None):
    """NumPy array -> cuda tensor.  float arrays that hold bf16-representable values convert exactly."""
    import torch
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    if dtype_name is not None:
        t = t.to(torch_dtype(dtype_name))
    return t.contiguous()


def to_np(t):
    import torch
    if t.dtype in (torch.bfloat16, torch.float16):
        t = t.float()
    return t.detach().cpu().numpy()


def max_rel_err(got, ref):
    """max |got - ref| / max |ref| over the compared tensor (the measure the 2e-2 / 1e-5 bars use;
    a purely elementwise relative error is undefined on the exactly-zero rows)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    scale = np.max(np.abs(ref)) if ref.size else 0.0
    if scale == 0.0:
        return float(np.max(np.abs(got))) if got.size else 0.0
    return float(np.max(np.abs(got - ref)) / scale)


def assert_close(got, ref, tol, what="", elem_tol=None):
    """The max-relative-error bar, plus an elementwise bound |got-ref| <= elem_tol*(rms(ref) + |ref|)
    (elem_tol = tol unless given), the rms taken over the non-zero elements of ref (exact-zero rows
    would dilute it)."""
    elem_tol = tol if elem_tol is None else elem_tol
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    if ref.size == 0:
        return
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    err = max_rel_err(got, ref)
    assert err <= tol, f"{what}: max rel err {err:.3e} > {tol:.1e}"
    nz = ref != 0.0
    rms = float(np.sqrt(np.mean(ref[nz] ** 2))) if nz.any() else 0.0
    bad = np.abs(got - ref) > elem_tol * (rms + np.abs(ref))
    assert not bad.any(), f"{what}: {int(bad.sum())} elements outside tol*(rms+|ref|), tol={elem_tol:.1e}"


# f16 (not named by the benchmark spec): the same error model as bf16 with 11 instead of 8 significant
# bits, i.e. an eighth of the bf16 bar.
TOL = {"bf16": 2e-2, "f16": 2.5e-3, "f32": 1e-5}
# Gradients: a weight-gradient element is a sum over an expert's rows of products of two factors that
# were each rounded to the 16-bit type, one of them (H) from a rounded pre-activation: three roundings
# of relative standard deviation 2^-8 / sqrt(3) per term, random in sign, give an error of standard
# deviation ~0.4 % of the tensor's rms per element whatever the number of rows; over the ~10^6 elements
# of a gradient tensor the largest is ~6 sigma = 2.4 %.  The elementwise bound of the gradient tests is
# therefore 1.5 x the forward's; the max-relative-error bar stays the forward's.
GRAD_ELEM_FACTOR = 1.5


class DeviceLayer:
    """Device copies of one layer's inputs plus the scratch the stage calls need."""

    def __init__(self, lc, inp):
        import torch
        self.lc = lc
        self.cfg = B.config_from(lc)
        self.x = to_dev(inp.get("x"), lc.in_dtype)
        self.Wg = to_dev(inp.get("Wg_t"), lc.in_dtype)
        self.bias = to_dev(inp.get("bias"))
        self.W1 = to_dev(inp.get("W1_t"), lc.in_dtype)
        self.W2 = to_dev(inp.get("W2_t"), lc.in_dtype)
        self.rows = B.moe_max_rows(self.cfg)
        self.torch = torch

    def empty(self, shape, dtype):
        return self.torch.empty(shape, dtype=dtype, device="cuda")

    def workspace(self, fill=None):
        n = B.moe_workspace_bytes(self.cfg)
        ws = self.empty((max(n, 16),), self.torch.uint8)
        if fill is not None:
            ws.fill_(fill)
        return ws

    def run_gate(self, logits_in=None, want_logits=True):
        t, c = self.torch, self.cfg
        idx = self.empty((c.T, c.top_k), t.int32)
        w = self.empty((c.T, c.top_k), t.float32)
        lo = self.empty((c.T, c.E), t.float32) if want_logits else None
        li = to_dev(logits_in) if logits_in is not None else None
        B.moe_gate(c, self.x, self.Wg, self.bias, li, lo, idx, w)
        t.cuda.synchronize()
        return (to_np(lo) if lo is not None else None), to_np(idx), to_np(w)

    def run_dispatch(self, expert_idx, with_rows=True):
        t, c = self.torch, self.cfg
        idx = to_dev(np.asarray(expert_idx, dtype=np.int32))
        counts = self.empty((c.local_count,), t.int32)
        offsets = self.empty((c.local_count + 1,), t.int32)
        perm = t.full((max(self.rows, 1),), -7, dtype=t.int32, device="cuda")
        inv = self.empty((c.T, c.top_k), t.int32)
        xs = self.empty((max(self.rows, 1), c.d), torch_dtype(self.lc.in_dtype)) if with_rows else None
        ws = self.empty((max(B.moe_dispatch_workspace_bytes(c), 16),), t.uint8)
        B.moe_slice_dispatch(c, self.x, idx, counts, offsets, perm, inv, xs, ws)
        t.cuda.synchronize()
        return (to_np(counts), to_np(offsets), to_np(perm), to_np(inv),
                to_np(xs) if xs is not None else None)

    def run_ffn(self, x_sliced, offsets, want_status=False):
        t, c = self.torch, self.cfg
        et = torch_dtype(self.lc.in_dtype)
        xs = self.empty((max(self.rows, 1), c.d), et)
        xs.zero_()
        n = x_sliced.shape[0]
        if n:
            xs[:n] = to_dev(np.asarray(x_sliced, dtype=np.float32), self.lc.in_dtype)
        off = to_dev(np.asarray(offsets, dtype=np.int32))
        H = self.empty((max(self.rows, 1), c.F), et)
        y = self.empty((max(self.rows, 1), c.d), et)
        ws = self.empty((B.moe_ffn_workspace_bytes(c),), t.uint8)
        B.moe_expert_ffn(c, xs, off, self.W1, self.W2, H, y, ws)
        status = B.moe_ffn_check(c, ws, False)
        t.cuda.synchronize()
        if want_status:
            return to_np(H[:n]), to_np(y[:n]), status
        assert status == 0, "a hand-over of partial sums did not arrive"
        return to_np(H[:n]), to_np(y[:n])

    def run_ffn_backward(self, x_sliced, offsets, dY):
        """moe_expert_ffn_backward on packed rows; returns (dX[:n], dW1 [N,F,d], dW2 [N,d,F]) as NumPy."""
        t, c = self.torch, self.cfg
        et = torch_dtype(self.lc.in_dtype)
        rows = max(self.rows, 1)
        xs = self.empty((rows, c.d), et)
        dy = self.empty((rows, c.d), et)
        xs.fill_(float("nan"))                     # rows past the last packed row must not be read
        dy.fill_(float("nan"))
        n = x_sliced.shape[0]
        if n:
            xs[:n] = to_dev(np.asarray(x_sliced, dtype=np.float32), self.lc.in_dtype)
            dy[:n] = to_dev(np.asarray(dY, dtype=np.float32), self.lc.in_dtype)
        off = to_dev(np.asarray(offsets, dtype=np.int32))
        dX = self.empty((rows, c.d), et)
        dX.fill_(5.0)
        dW1 = t.full((c.local_count, c.F, c.d), 7.0, dtype=t.float32, device="cuda")
        dW2 = t.full((c.local_count, c.d, c.F), 7.0, dtype=t.float32, device="cuda")
        ws = self.empty((B.moe_ffn_backward_workspace_bytes(c),), t.uint8)
        ws.fill_(0xFF)
        B.moe_expert_ffn_backward(c, xs, off, self.W1, self.W2, dy, dX, dW1, dW2, ws)
        t.cuda.synchronize()
        assert bool((dX[n:] == 5.0).all()), "rows past the last packed row were written"
        return to_np(dX[:n]), to_np(dW1), to_np(dW2)

    def run_layer_backward(self, d_out):
        """moe_layer_backward; returns dict(dx, dWg, dbias, dW1, dW2) as NumPy (library layouts)."""
        t, c = self.torch, self.cfg
        do = to_dev(np.asarray(d_out, dtype=np.float32), self.lc.out_dtype)
        dx = self.empty((c.T, c.d), torch_dtype(self.lc.in_dtype))
        dWg = t.full((c.E, c.d), 7.0, dtype=t.float32, device="cuda")
        dbias = t.full((c.E,), 7.0, dtype=t.float32, device="cuda")
        dW1 = t.full((c.local_count, c.F, c.d), 7.0, dtype=t.float32, device="cuda")
        dW2 = t.full((c.local_count, c.d, c.F), 7.0, dtype=t.float32, device="cuda")
        ws = self.empty((B.moe_layer_backward_workspace_bytes(c),), t.uint8)
        ws.fill_(0xAB)
        B.moe_layer_backward(c, self.x, self.Wg, self.bias, self.W1, self.W2, do, dx, dWg, dbias, dW1, dW2, ws)
        t.cuda.synchronize()
        return dict(dx=to_np(dx), dWg=to_np(dWg), dbias=to_np(dbias), dW1=to_np(dW1), dW2=to_np(dW2))

    def run_train_step(self, d_out):
        """moe_layer_forward_train, then moe_layer_backward_saved on what it kept; returns (out, l_aux,
        gradients as run_layer_backward, True if the backward left `saved` as it was)."""
        t, c = self.torch, self.cfg
        ws = self.workspace(fill=0xAB)
        saved = self.empty((B.moe_layer_saved_bytes(c),), t.uint8)
        saved.fill_(0xCD)
        out = self.empty((c.T, c.d), torch_dtype(self.lc.out_dtype))
        out.fill_(7.0)
        l_aux = t.full((1,), -1.0, dtype=t.float32, device="cuda")
        B.moe_layer_forward_train(c, self.x, self.Wg, self.bias, self.W1, self.W2, out, l_aux, None, None, saved, ws)
        assert B.moe_ffn_check(c, ws, True) == 0, "a hand-over of partial sums did not arrive"
        before = saved.clone()
        do = to_dev(np.asarray(d_out, dtype=np.float32), self.lc.out_dtype)
        dx = self.empty((c.T, c.d), torch_dtype(self.lc.in_dtype))
        dWg = t.full((c.E, c.d), 7.0, dtype=t.float32, device="cuda")
        dbias = t.full((c.E,), 7.0, dtype=t.float32, device="cuda")
        dW1 = t.full((c.local_count, c.F, c.d), 7.0, dtype=t.float32, device="cuda")
        dW2 = t.full((c.local_count, c.d, c.F), 7.0, dtype=t.float32, device="cuda")
        bws = self.empty((B.moe_layer_backward_workspace_bytes(c),), t.uint8)
        bws.fill_(0xAB)
        B.moe_layer_backward_saved(c, self.x, self.Wg, self.W1, self.W2, do, saved, dx, dWg, dbias, dW1, dW2, bws)
        t.cuda.synchronize()
        untouched = bool(t.equal(saved, before))
        grads = dict(dx=to_np(dx), dWg=to_np(dWg), dbias=to_np(dbias), dW1=to_np(dW1), dW2=to_np(dW2))
        return to_np(out), float(l_aux.item()), grads, untouched

    def run_combine(self, y_sliced, inv_perm, gate_w):
        t, c = self.torch, self.cfg
        y = self.empty((max(self.rows, 1), c.d), torch_dtype(self.lc.in_dtype))
        n = y_sliced.shape[0]
        if n:
            y[:n] = to_dev(np.asarray(y_sliced, dtype=np.float32), self.lc.in_dtype)
        inv = to_dev(np.asarray(inv_perm, dtype=np.int32))
        w = to_dev(np.asarray(gate_w, dtype=np.float32))
        out = self.empty((c.T, c.d), torch_dtype(self.lc.out_dtype))
        out.fill_(7.0)
        B.moe_combine(c, y, inv, w, out)
        t.cuda.synchronize()
        return to_np(out)

    def run_layer(self, ws_fill=0xAB, aux=False):
        """One fused layer call.  aux=True: through moe_layer_forward_aux; the views then also hold
        l_aux (float), mean_prob [E] and first_counts [E] as NumPy arrays."""
        t, c = self.torch, self.cfg
        ws = self.workspace(fill=ws_fill)
        out = self.empty((c.T, c.d), torch_dtype(self.lc.out_dtype))
        out.fill_(7.0)
        if aux:
            l_aux = t.full((1,), -1.0, dtype=t.float32, device="cuda")
            mean_prob = t.full((c.E,), -1.0, dtype=t.float32, device="cuda")
            first = t.full((c.E,), -1, dtype=t.int32, device="cuda")
            B.moe_layer_forward_aux(c, self.x, self.Wg, self.bias, self.W1, self.W2, out, l_aux, mean_prob,
                                    first, ws)
        else:
            B.moe_layer_forward(c, self.x, self.Wg, self.bias, self.W1, self.W2, out, ws)
        assert B.moe_ffn_check(c, ws, True) == 0, "a hand-over of partial sums did not arrive"
        t.cuda.synchronize()
        views = B.workspace_views(c, ws)
        if aux:
            views.update(l_aux=float(l_aux.item()), mean_prob=to_np(mean_prob), first_counts=to_np(first))
        return out, views
