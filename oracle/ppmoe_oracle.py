"""CPU fp64 oracle for the Pipeline-MoE (PPMoE) MoE-layer forward on one device's share.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is the plain, slow definition the HIP
library is checked against.  Only the tests, the smoke check and the benchmark's CPU-baseline leg
may call it.  It shares no code, table, constant generator or helper with the HIP path and never
imports it; every input is passed in as an array, no value it consumes is produced by the GPU.

What it follows
---------------
Algorithm 1 of the paper (forward of the expert-parallel MoE layer), step by step and in the
paper's order: gating linear map -> softmax -> gating schedule (top-k) -> per-local-expert
index selection -> the local experts' FFNs one after another -> zero-initialised output with the
expert outputs placed back at their token rows.  The closing all-reduce over the tensor-parallel
group is outside this oracle: the value returned is the partial sum one device would contribute.
The dispatching-order bookkeeping follows the worked example of Section 3.3.3 (8 tokens, 4 experts).
The expert is the FFN of Section 3.1.3, GeLU(X A) B, without the Dropout (which the paper applies
after the all-reduce, Section 3.3.4).

Arithmetic is float64 throughout, except that the gating module's logits are rounded to float32
before softmax / top-k when ``logits_dtype`` says so (the paper runs the gating module in float32,
Section 4.1), so that both sides take the integer top-k decision on the same numbers.

Readings of points the paper leaves open:
  * the gate weight returned by the gating function IS applied to the expert output
    (Section 3.1.4 describes scores per token; Algorithm 1 returns ``weights`` but never uses it);
  * placing expert outputs back is an accumulation (a token picked by two local experts under top-2
    gets the sum), not an overwrite;
  * top-k is taken on the logits (softmax is strictly monotone), equal logits -> lower expert index;
    picks are listed in descending-logit order;
  * gate weight = softmax probability of the pick, optionally renormalised over the k picks
    (renormalisation happens before any capacity drop);
  * a device holds a contiguous block of experts [local_begin, local_begin + local_count);
  * GeLU is the tanh form; the FFN has no bias.

Parity unpinned by the paper (builder's stated definitions, pinned only by brute force and
invariants in the tests):
  * the capacity limit (PPMoE abandons it, Section 4.1): C = ceil(cf * k * T / E); an assignment is
    kept iff fewer than C earlier assignments (ascending t*k + j) chose the same expert;
  * the top-1 gate-weight convention (raw softmax probability vs renormalised to 1);
  * the auxiliary balance loss ``l_aux`` that Algorithm 1 returns: the paper only says it follows
    GShard (Section 4.1) and prints no formula.  ``aux_loss`` below is the GShard form; it is pinned
    by closed forms and a scalar-loop restatement, not by anything the paper prints.

The backward functions at the end (expert_ffn_backward, gate_backward, layer_backward) are the
derivative of this forward by the chain rule (the paper prints no backward algorithm); they are
pinned by central finite differences of the forward in the tests.
"""

from __future__ import annotations

import math

import numpy as np

F64 = np.float64


# ----------------------------------------------------------------------------------------------
# Gating module  (Section 3.3.3: linear mapping, softmax score function, gating schedule;
#                 Algorithm 1: logits = wg(h); scores = softmax(logits); gate_function(scores))
# ----------------------------------------------------------------------------------------------

def router_logits(x, Wg, bias=None):
    """logits[t, e] = sum_i x[t, i] * Wg[i, e] (+ bias[e]).  Wg has the paper's shape h x E
    (Section 3.3.4).  float64."""
    logits = np.asarray(x, dtype=F64) @ np.asarray(Wg, dtype=F64)
    if bias is not None:
        logits = logits + np.asarray(bias, dtype=F64)[None, :]
    return logits


def softmax_rows(logits):
    """Softmax over all E (global) experts of each token, max-subtracted, float64."""
    z = np.asarray(logits, dtype=F64)
    z = z - z.max(axis=1, keepdims=True)
    p = np.exp(z)
    return p / p.sum(axis=1, keepdims=True)


def top_k_picks(logits, k):
    """Gating schedule: k times over, take the largest logit not yet taken; among equal logits the
    lower expert index wins.  Returns int32 [T, k], picks in the order taken."""
    work = np.array(logits, dtype=F64, copy=True)
    T, E = work.shape
    assert 1 <= k <= E
    picks = np.empty((T, k), dtype=np.int32)
    rows = np.arange(T)
    for j in range(k):
        e = np.argmax(work, axis=1)          # first occurrence of the maximum = lowest index
        picks[:, j] = e
        work[rows, e] = -np.inf
    return picks


def gate(x, Wg, bias, k, renorm, logits_in=None, logits_dtype=np.float32):
    """The gating module.  Returns (logits, expert_idx[T,k] int32, gate_w[T,k] float64).

    If ``logits_in`` is given it is used verbatim (this is how "given identical router logits" is
    tested); otherwise the logits are computed in float64 and, if ``logits_dtype`` is float32,
    rounded once to float32 -- the precision the paper's gating module works in (Section 4.1)."""
    if logits_in is not None:
        logits = np.asarray(logits_in)
    else:
        logits = router_logits(x, Wg, bias)
        if logits_dtype is not None:
            logits = logits.astype(logits_dtype)
    logits64 = logits.astype(F64)            # exact for float32 input
    scores = softmax_rows(logits64)
    expert_idx = top_k_picks(logits64, k)
    gate_w = np.take_along_axis(scores, expert_idx.astype(np.int64), axis=1)
    if renorm:
        gate_w = gate_w / gate_w.sum(axis=1, keepdims=True)
    return logits, expert_idx, gate_w


def aux_loss(logits, expert_idx):
    """Auxiliary load-balance loss returned by Algorithm 1 next to the output ("l_aux"); the paper
    names GShard as its source (Section 4.1) and gives no formula, so this is the GShard form:

        l_aux = E * sum_e  mean_prob[e] * first_fraction[e]

    mean_prob[e]      = mean over tokens of the softmax probability of expert e,
    first_fraction[e] = share of the tokens whose FIRST pick is expert e (also under top-2 gating,
                        and before any capacity drop).
    Returns dict(l_aux, mean_prob[E] float64, first_counts[E] int64).  Parity unpinned by the paper."""
    logits = np.asarray(logits)
    T, E = logits.shape
    scores = softmax_rows(logits.astype(F64))
    first = np.asarray(expert_idx).reshape(T, -1)[:, 0].astype(np.int64)
    first_counts = np.bincount(first, minlength=E).astype(np.int64)
    if T == 0:
        return dict(l_aux=0.0, mean_prob=np.zeros(E, dtype=F64), first_counts=first_counts)
    mean_prob = scores.sum(axis=0) / T
    l_aux = float(E * np.sum(mean_prob * (first_counts / T)))
    return dict(l_aux=l_aux, mean_prob=mean_prob, first_counts=first_counts)


# ----------------------------------------------------------------------------------------------
# Dispatching order -> per-expert index lists (Section 3.3.3 worked example; Algorithm 1's
# ``indices``), optional capacity limit (builder's definition, see header).
# ----------------------------------------------------------------------------------------------

def capacity(capacity_factor, k, T, E):
    """Per-expert queue limit, or None for "no limit" (what PPMoE does, Section 4.1).

    The factor is a single-precision number (the field of the layer's configuration record is a
    float32), so it is rounded to float32 first; the product is then formed left to right in
    float64.  With a factor that float32 cannot hold this decides whether a queue keeps one
    assignment more: float32(1.2) = 1.2000000476837158203125, so 1.2 * 20 / 4 gives 7, not 6."""
    if capacity_factor is None or capacity_factor <= 0:
        return None
    cf = float(np.float32(capacity_factor))
    return int(math.ceil(cf * k * T / E))


def dispatch(expert_idx, E, local_begin, local_count, cap=None):
    """From the dispatching order to the local experts' index lists.

    Assignment id a = t*k + j.  The queue of expert e is every assignment that chose e, in ascending
    a.  With a capacity only the first ``cap`` of a queue are kept.  The local experts' kept queues
    are laid end to end in ascending expert order:

      counts[i]   kept queue length of expert local_begin + i
      offsets     exclusive prefix sum of counts, length local_count + 1
      perm[r]     the assignment id held by packed row r
      inv_perm[t, j]  the packed row of assignment (t, j), or -1 if it is dropped or not local
    """
    expert_idx = np.asarray(expert_idx)
    T, k = expert_idx.shape
    assert 0 <= local_begin and local_begin + local_count <= E
    flat = expert_idx.reshape(-1)
    counts = np.zeros(local_count, dtype=np.int32)
    offsets = np.zeros(local_count + 1, dtype=np.int32)
    perm_parts = []
    inv_perm = np.full(T * k, -1, dtype=np.int32)
    for i in range(local_count):
        queue = np.flatnonzero(flat == local_begin + i)      # ascending assignment id
        if cap is not None:
            queue = queue[:cap]
        counts[i] = queue.size
        offsets[i + 1] = offsets[i] + queue.size
        inv_perm[queue] = offsets[i] + np.arange(queue.size)
        perm_parts.append(queue)
    perm = (np.concatenate(perm_parts) if perm_parts else np.zeros(0)).astype(np.int32)
    return counts, offsets, perm, inv_perm.reshape(T, k)


def slice_rows(x, perm, k):
    """The index selection that replaces the first all-to-all: x_sliced[r] = x[token of perm[r]]."""
    x = np.asarray(x)
    return x[np.asarray(perm, dtype=np.int64) // k]


# ----------------------------------------------------------------------------------------------
# Local experts (Section 3.3.2: N experts per device computed serially; FFN = GeLU(X A) B)
# ----------------------------------------------------------------------------------------------

def gelu_tanh(u):
    u = np.asarray(u, dtype=F64)
    return 0.5 * u * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (u + 0.044715 * u ** 3)))


def expert_ffn(x_sliced, offsets, W1, W2):
    """For each local expert i in turn: H_i = GeLU(X_i A_i), Y_i = H_i B_i.

    W1[i] is A_i with shape [d, F]; W2[i] is B_i with shape [F, d] (the paper's X A, H B form).
    Returns (H[A, F], y_sliced[A, d]) in float64, packed like x_sliced."""
    x_sliced = np.asarray(x_sliced, dtype=F64)
    n_local = len(offsets) - 1
    A = int(offsets[-1])
    F = W1[0].shape[1]
    d = W2[0].shape[1]
    H = np.zeros((A, F), dtype=F64)
    y = np.zeros((A, d), dtype=F64)
    for i in range(n_local):
        lo, hi = int(offsets[i]), int(offsets[i + 1])
        if hi == lo:
            continue
        H[lo:hi] = gelu_tanh(x_sliced[lo:hi] @ np.asarray(W1[i], dtype=F64))
        y[lo:hi] = H[lo:hi] @ np.asarray(W2[i], dtype=F64)
    return H, y


# ----------------------------------------------------------------------------------------------
# Combine (Algorithm 1: zeros_like(hidden_states), then the expert outputs go back to their rows)
# ----------------------------------------------------------------------------------------------

def combine(y_sliced, inv_perm, gate_w, d=None):
    """out[t] = sum over picks j (ascending) with inv_perm[t, j] >= 0 of gate_w[t, j] * y[row].
    Tokens with no kept local pick stay exactly zero."""
    y_sliced = np.asarray(y_sliced, dtype=F64)
    inv_perm = np.asarray(inv_perm)
    T, k = inv_perm.shape
    if d is None:
        d = y_sliced.shape[1]
    out = np.zeros((T, d), dtype=F64)
    for j in range(k):
        rows = inv_perm[:, j]
        kept = np.flatnonzero(rows >= 0)
        out[kept] += np.asarray(gate_w, dtype=F64)[kept, j][:, None] * y_sliced[rows[kept]]
    return out


# ----------------------------------------------------------------------------------------------
# Whole layer (Algorithm 1 without the closing all-reduce)
# ----------------------------------------------------------------------------------------------

def layer_forward(x, Wg, bias, W1, W2, *, E, k, local_begin, local_count, capacity_factor=0.0,
                  renorm=False, logits_in=None, logits_dtype=np.float32):
    """Returns a dict with every intermediate of the path and ``out``, the partial [T, d] output."""
    x = np.asarray(x)
    T, d = x.shape
    logits, expert_idx, gate_w = gate(x, Wg, bias, k, renorm, logits_in, logits_dtype)
    cap = capacity(capacity_factor, k, T, E)
    counts, offsets, perm, inv_perm = dispatch(expert_idx, E, local_begin, local_count, cap)
    x_sliced = slice_rows(x, perm, k)
    H, y_sliced = expert_ffn(x_sliced, offsets, W1, W2)
    out = combine(y_sliced, inv_perm, gate_w, d)
    return dict(logits=logits, expert_idx=expert_idx, gate_w=gate_w, capacity=cap, counts=counts,
                offsets=offsets, perm=perm, inv_perm=inv_perm, x_sliced=x_sliced, H=H,
                y_sliced=y_sliced, out=out)


def layer_forward_rows(token_rows, x, Wg, bias, W1, W2, *, E, k, local_begin, local_count,
                       capacity_factor=0.0, renorm=False, logits_in=None,
                       logits_dtype=np.float32):
    """The same layer, but the expert FFNs and the combine are evaluated only for the output rows
    listed in ``token_rows`` (gating and the dispatching order are still computed for every token,
    because a capacity drop depends on all earlier tokens).  Used where the full layer is too much
    float64 work: each sampled output row is computed one by one from the definition
    out[t] = sum_j [pick j local and kept] * gate_w[t, j] * FFN_{e_j}(x[t]).

    Returns (out_rows[len(token_rows), d], gating dict as in layer_forward)."""
    x = np.asarray(x)
    T, d = x.shape
    logits, expert_idx, gate_w = gate(x, Wg, bias, k, renorm, logits_in, logits_dtype)
    cap = capacity(capacity_factor, k, T, E)
    counts, offsets, perm, inv_perm = dispatch(expert_idx, E, local_begin, local_count, cap)
    token_rows = np.asarray(token_rows, dtype=np.int64)
    out_rows = np.zeros((token_rows.size, d), dtype=F64)
    for i in range(local_count):
        e = local_begin + i
        W1_e = W2_e = None
        for j in range(k):
            sel = np.flatnonzero((expert_idx[token_rows, j] == e) & (inv_perm[token_rows, j] >= 0))
            if sel.size == 0:
                continue
            if W1_e is None:
                W1_e = np.asarray(W1[i], dtype=F64)
                W2_e = np.asarray(W2[i], dtype=F64)
            t = token_rows[sel]
            h = gelu_tanh(np.asarray(x[t], dtype=F64) @ W1_e)
            out_rows[sel] += gate_w[t, j][:, None] * (h @ W2_e)
    info = dict(logits=logits, expert_idx=expert_idx, gate_w=gate_w, capacity=cap, counts=counts,
                offsets=offsets, perm=perm, inv_perm=inv_perm)
    return out_rows, info


def ffn_flops(n_assignments, d, F):
    """Multiply-add count x2 of the two expert GEMMs for ``n_assignments`` kept rows; with F = 4d and
    one pick per token this is the 16*b*s*h^2 of Section 3.2."""
    return 4 * int(n_assignments) * int(d) * int(F)


# ----------------------------------------------------------------------------------------------
# Backward of the layer (Section 3.2, footnote to Eq. 1: the backward pass costs about twice the
# forward; Section 3.3.4: it moves the same tensors between devices as the forward).  The paper
# prints no backward algorithm: it trains through the automatic differentiation of its framework, so
# what is written out here is the derivative of the forward above, term by term, by the chain rule.
# The picks (top-k, capacity drops) are piecewise constant in the inputs and carry no gradient.
# Everything is this device's partial sum, like the forward output: summed over the devices of a
# tensor-parallel group it is the gradient of the whole layer.
# ----------------------------------------------------------------------------------------------

def gelu_tanh_grad(u):
    """d/du of gelu_tanh.  With z = sqrt(2/pi) (u + 0.044715 u^3):
    0.5 (1 + tanh z) + 0.5 u (1 - tanh^2 z) sqrt(2/pi) (1 + 3 * 0.044715 u^2)."""
    u = np.asarray(u, dtype=F64)
    c = math.sqrt(2.0 / math.pi)
    th = np.tanh(c * (u + 0.044715 * u ** 3))
    return 0.5 * (1.0 + th) + 0.5 * u * (1.0 - th * th) * c * (1.0 + 3.0 * 0.044715 * u * u)


def expert_ffn_backward(x_sliced, offsets, W1, W2, dY):
    """Backward of expert_ffn for each local expert i in turn, given dY = dLoss/dY (packed rows):

        U_i = X_i A_i,  H_i = GeLU(U_i),  Y_i = H_i B_i
        dH_i = dY_i B_i^T,  dU_i = dH_i * GeLU'(U_i),  dX_i = dU_i A_i^T,
        dA_i = X_i^T dU_i,  dB_i = H_i^T dY_i.

    W1[i] = A_i [d, F], W2[i] = B_i [F, d].  Returns dict(dX[A, d], dW1[N, d, F], dW2[N, F, d], U, H,
    dH, dU), float64."""
    x_sliced = np.asarray(x_sliced, dtype=F64)
    dY = np.asarray(dY, dtype=F64)
    n_local = len(offsets) - 1
    A = int(offsets[-1])
    d, F = W1[0].shape
    U = np.zeros((A, F), dtype=F64)
    H = np.zeros((A, F), dtype=F64)
    dH = np.zeros((A, F), dtype=F64)
    dU = np.zeros((A, F), dtype=F64)
    dX = np.zeros((A, d), dtype=F64)
    dW1 = np.zeros((n_local, d, F), dtype=F64)
    dW2 = np.zeros((n_local, F, d), dtype=F64)
    for i in range(n_local):
        lo, hi = int(offsets[i]), int(offsets[i + 1])
        if hi == lo:
            continue
        A_i = np.asarray(W1[i], dtype=F64)
        B_i = np.asarray(W2[i], dtype=F64)
        U[lo:hi] = x_sliced[lo:hi] @ A_i
        H[lo:hi] = gelu_tanh(U[lo:hi])
        dH[lo:hi] = dY[lo:hi] @ B_i.T
        dU[lo:hi] = dH[lo:hi] * gelu_tanh_grad(U[lo:hi])
        dX[lo:hi] = dU[lo:hi] @ A_i.T
        dW1[i] = x_sliced[lo:hi].T @ dU[lo:hi]
        dW2[i] = H[lo:hi].T @ dY[lo:hi]
    return dict(dX=dX, dW1=dW1, dW2=dW2, U=U, H=H, dH=dH, dU=dU)


def gate_backward(logits, expert_idx, renorm, d_gate_w):
    """Gradient of the gate weights with respect to the logits, picks held fixed.

    p = softmax(logits);  w_j = p[e_j], or p[e_j] / S with S = sum_j p[e_j] when renorm.
    Without renorm  dp[e_j] = dw_j;  with renorm  dp[e_j] = (dw_j - sum_i dw_i w_i) / S.
    Softmax:  dlogits[e] = p[e] (dp[e] - sum_e' dp[e'] p[e']).   Returns dlogits [T, E], float64."""
    logits = np.asarray(logits, dtype=F64)
    T, E = logits.shape
    p = softmax_rows(logits)
    idx = np.asarray(expert_idx).astype(np.int64)
    dgw = np.asarray(d_gate_w, dtype=F64)
    picked = np.take_along_axis(p, idx, axis=1)
    if renorm:
        S = picked.sum(axis=1, keepdims=True)
        w = picked / S
        dpick = (dgw - (dgw * w).sum(axis=1, keepdims=True)) / S
    else:
        dpick = dgw
    dp = np.zeros((T, E), dtype=F64)
    np.put_along_axis(dp, idx, dpick, axis=1)        # a token picks an expert at most once
    return p * (dp - (dp * p).sum(axis=1, keepdims=True))


def layer_backward(x, Wg, bias, W1, W2, d_out, *, E, k, local_begin, local_count,
                   capacity_factor=0.0, renorm=False, logits_in=None, logits_dtype=np.float32):
    """Backward of layer_forward given d_out = dLoss/d(out) [T, d]; the forward is re-evaluated first.

        dY[r]       = gate_w[t, j] * d_out[t]                 for the kept local assignment (t, j) in row r
        d_gate_w[t, j] = <d_out[t], Y[r]>                       (0 for dropped / non-local picks)
        expert FFN backward                                     -> dX_sliced, dW1, dW2
        dx[t]       = sum over kept local (t, j) of dX_sliced[r]  +  dlogits[t] Wg^T
        dWg         = x^T dlogits,   dbias = column sums of dlogits

    Returns a dict with every intermediate, float64."""
    fwd = layer_forward(x, Wg, bias, W1, W2, E=E, k=k, local_begin=local_begin,
                        local_count=local_count, capacity_factor=capacity_factor, renorm=renorm,
                        logits_in=logits_in, logits_dtype=logits_dtype)
    x64 = np.asarray(x, dtype=F64)
    d_out = np.asarray(d_out, dtype=F64)
    T, d = x64.shape
    perm, inv_perm, gate_w = fwd["perm"], fwd["inv_perm"], fwd["gate_w"]
    tok = perm.astype(np.int64) // k
    pick = perm.astype(np.int64) % k
    dY = gate_w[tok, pick][:, None] * d_out[tok]
    d_gate_w = np.zeros((T, k), dtype=F64)
    d_gate_w[tok, pick] = np.einsum("rc,rc->r", d_out[tok], fwd["y_sliced"])
    ffn = expert_ffn_backward(fwd["x_sliced"], fwd["offsets"], W1, W2, dY)
    dx = np.zeros((T, d), dtype=F64)
    for j in range(k):
        rows = inv_perm[:, j]
        kept = np.flatnonzero(rows >= 0)
        dx[kept] += ffn["dX"][rows[kept]]
    dlogits = gate_backward(fwd["logits"], fwd["expert_idx"], renorm, d_gate_w)
    Wg64 = np.asarray(Wg, dtype=F64)
    dx_gate = dlogits @ Wg64.T
    return dict(fwd=fwd, dY=dY, d_gate_w=d_gate_w, dX_sliced=ffn["dX"], dW1=ffn["dW1"], dW2=ffn["dW2"],
                dU=ffn["dU"], dH=ffn["dH"], U=ffn["U"], dlogits=dlogits, dx_experts=dx, dx_gate=dx_gate,
                dx=dx + dx_gate, dWg=x64.T @ dlogits, dbias=dlogits.sum(axis=0))
