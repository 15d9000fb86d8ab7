"""Pins for the CPU oracle: what the paper prints, closed forms, invariants, textbook routines and
pure-Python brute force on tiny inputs.  No GPU, no HIP library.

Every brute-force helper here is written independently of oracle/ (scalar Python loops over the
per-token definition), so a dropped term, a wrong index, a transposed weight or a missing gate weight
in the oracle shows up as a mismatch."""

import math

import numpy as np
import pytest
import scipy.special

from oracle import ppmoe_oracle as O
from tests.conftest import read_golden

RNG = np.random.default_rng(20230411)


# ------------------------------------------------------------------ worked example, Section 3.3.3

def test_worked_example_index_lists():
    g = read_golden("worked_example_dispatch.txt")
    order = np.array(g["order"], dtype=np.int32).reshape(-1, 1)
    counts, offsets, perm, inv_perm = O.dispatch(order, E=4, local_begin=0, local_count=4)
    for e in range(4):
        assert perm[offsets[e]:offsets[e + 1]].tolist() == g[f"expert{e}"]
    assert counts.tolist() == [len(g[f"expert{e}"]) for e in range(4)]
    # index selection reproduces X_i = X[indices_i]
    X = RNG.standard_normal((8, 5))
    xs = O.slice_rows(X, perm, 1)
    for e in range(4):
        np.testing.assert_array_equal(xs[offsets[e]:offsets[e + 1]], X[g[f"expert{e}"]])


def test_worked_example_two_tensor_parallel_slices():
    """2 slices in the tensor-parallel group: device 0 holds experts {0,1}, device 1 holds {2,3};
    each slices only its own experts' tokens from the identical dispatching order."""
    g = read_golden("worked_example_dispatch.txt")
    order = np.array(g["order"], dtype=np.int32).reshape(-1, 1)
    _, off0, perm0, inv0 = O.dispatch(order, 4, 0, 2)
    _, off1, perm1, inv1 = O.dispatch(order, 4, 2, 2)
    assert perm0.tolist() == g["expert0"] + g["expert1"]
    assert perm1.tolist() == g["expert2"] + g["expert3"]
    # a token is local to exactly one of the two devices
    assert np.all((inv0 >= 0) ^ (inv1 >= 0))


# ------------------------------------------------------------------ gating

def brute_topk(logit_row, k):
    order = sorted(range(len(logit_row)), key=lambda e: (-float(logit_row[e]), e))
    return order[:k]


@pytest.mark.parametrize("E,k", [(1, 1), (4, 1), (8, 2), (16, 2), (5, 5), (64, 3)])
def test_topk_matches_full_sort_with_ties(E, k):
    T = 200
    logits = RNG.standard_normal((T, E)).astype(np.float32)
    # exact ties: duplicated values, an all-equal row, an all-zero row
    if E > 1:
        logits[::7, E - 1] = logits[::7, 0]
        logits[::11, :] = logits[::11, :1]
        logits[13, :] = 0.0
    got = O.top_k_picks(logits, k)
    for t in range(T):
        assert got[t].tolist() == brute_topk(logits[t], k)
        assert len(set(got[t].tolist())) == k


def test_tie_goes_to_lower_expert_index():
    logits = np.array([[1.0, 3.0, 3.0, 3.0], [0.0, 0.0, 0.0, 0.0], [2.0, 1.0, 2.0, 1.0]], np.float32)
    assert O.top_k_picks(logits, 2).tolist() == [[1, 2], [0, 1], [0, 2]]


def test_topk_shift_invariance_and_softmax_library():
    T, E = 64, 8
    logits = RNG.standard_normal((T, E)).astype(np.float32)
    shift = (RNG.integers(-8, 8, size=(T, 1))).astype(np.float32)      # exactly representable shifts
    a = O.top_k_picks(logits, 2)
    b = O.top_k_picks((logits.astype(np.float64) + shift), 2)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_allclose(O.softmax_rows(logits), scipy.special.softmax(logits.astype(np.float64), axis=1),
                               rtol=1e-14, atol=0)


def test_gate_weight_conventions():
    T, d, E = 50, 16, 6
    x = RNG.standard_normal((T, d))
    Wg = RNG.standard_normal((d, E)) * 0.3
    bias = RNG.standard_normal(E)
    # k = E without renormalisation: the weights are the whole softmax and sum to one
    logits, idx, w = O.gate(x, Wg, bias, E, renorm=False)
    np.testing.assert_allclose(w.sum(1), 1.0, rtol=1e-13)
    p = scipy.special.softmax(logits.astype(np.float64), axis=1)
    np.testing.assert_allclose(w, np.take_along_axis(p, idx.astype(np.int64), 1), rtol=1e-13)
    # picks come out in descending-logit order
    picked = np.take_along_axis(logits, idx.astype(np.int64), 1)
    assert np.all(np.diff(picked, axis=1) <= 0)
    # top-2 renormalised: sums to one, ratio equals the ratio of the probabilities
    _, idx2, w2 = O.gate(x, Wg, bias, 2, renorm=True)
    np.testing.assert_allclose(w2.sum(1), 1.0, rtol=1e-13)
    p2 = np.take_along_axis(p, idx2.astype(np.int64), 1)
    np.testing.assert_allclose(w2[:, 0] / w2[:, 1], p2[:, 0] / p2[:, 1], rtol=1e-12)
    # top-1: renormalised weight is exactly one, raw weight is the max probability
    _, idx1, w1 = O.gate(x, Wg, bias, 1, renorm=True)
    assert np.all(w1 == 1.0)
    _, idx1b, w1b = O.gate(x, Wg, bias, 1, renorm=False)
    np.testing.assert_array_equal(idx1, idx1b)
    np.testing.assert_allclose(w1b[:, 0], p.max(1), rtol=1e-13)
    # a single expert always gets weight one
    _, idxe1, we1 = O.gate(x, Wg[:, :1], None, 1, renorm=False)
    assert np.all(idxe1 == 0) and np.all(we1 == 1.0)


def test_router_logits_against_scalar_loops():
    T, d, E = 7, 9, 5
    x = RNG.standard_normal((T, d))
    Wg = RNG.standard_normal((d, E))
    bias = RNG.standard_normal(E)
    got = O.router_logits(x, Wg, bias)
    for t in range(T):
        for e in range(E):
            ref = math.fsum(x[t, i] * Wg[i, e] for i in range(d)) + bias[e]
            assert abs(got[t, e] - ref) < 1e-13
    # logits handed in are used verbatim
    lg = RNG.standard_normal((T, E)).astype(np.float32)
    out_lg, idx, _ = O.gate(None, None, None, 1, False, logits_in=lg)
    assert out_lg is lg or np.array_equal(out_lg, lg)
    np.testing.assert_array_equal(idx[:, 0], [brute_topk(r, 1)[0] for r in lg])


# ------------------------------------------------------------------ dispatching order / capacity

def brute_dispatch(expert_idx, E, e0, n, cap):
    """O((Tk)^2) predecessor counting, straight from the definition."""
    T, k = expert_idx.shape
    flat = [int(v) for v in expert_idx.reshape(-1)]
    pos = [sum(1 for b in range(a) if flat[b] == flat[a]) for a in range(len(flat))]
    kept = [(cap is None or pos[a] < cap) and e0 <= flat[a] < e0 + n for a in range(len(flat))]
    counts = [sum(1 for a in range(len(flat)) if kept[a] and flat[a] == e0 + i) for i in range(n)]
    offsets = [0]
    for c in counts:
        offsets.append(offsets[-1] + c)
    perm = [None] * offsets[-1]
    inv = [-1] * len(flat)
    for a in range(len(flat)):
        if kept[a]:
            r = offsets[flat[a] - e0] + pos[a]
            perm[r] = a
            inv[a] = r
    return counts, offsets, perm, np.array(inv).reshape(T, k)


@pytest.mark.parametrize("T,E,k,e0,n,cap", [
    (40, 4, 1, 0, 4, None), (40, 4, 2, 0, 4, None), (33, 8, 2, 2, 3, None), (64, 8, 2, 0, 8, 7),
    (64, 8, 1, 4, 4, 3), (50, 6, 3, 0, 6, 20), (17, 3, 3, 1, 2, None), (30, 5, 2, 0, 5, 1),
])
def test_dispatch_matches_predecessor_counting(T, E, k, e0, n, cap):
    logits = RNG.standard_normal((T, E)).astype(np.float32)
    logits[:, 0] += 1.0                                   # skew so queues overflow
    idx = O.top_k_picks(logits, k)
    counts, offsets, perm, inv = O.dispatch(idx, E, e0, n, cap)
    bc, bo, bp, bi = brute_dispatch(idx, E, e0, n, cap)
    assert counts.tolist() == bc and offsets.tolist() == bo and perm.tolist() == bp
    np.testing.assert_array_equal(inv, bi)


def test_dispatch_invariants():
    T, E, k = 500, 8, 2
    logits = RNG.standard_normal((T, E)).astype(np.float32)
    idx = O.top_k_picks(logits, k)
    counts, offsets, perm, inv = O.dispatch(idx, E, 0, E)
    # all local, no capacity: every assignment appears exactly once
    assert counts.sum() == T * k and sorted(perm.tolist()) == list(range(T * k))
    assert np.all(counts <= T)                            # at most b*s tokens per expert (Section 4.1)
    flat_inv = inv.reshape(-1)
    np.testing.assert_array_equal(flat_inv[perm], np.arange(perm.size))
    for e in range(E):
        seg = perm[offsets[e]:offsets[e + 1]]
        assert np.all(np.diff(seg) > 0)                   # ascending token order inside an expert
        assert np.all(idx.reshape(-1)[seg] == e)
    # capacity: counts clamp, and whatever is dropped comes after everything kept in that queue
    cap = 100
    c2, o2, p2, i2 = O.dispatch(idx, E, 0, E, cap)
    hist = np.bincount(idx.reshape(-1), minlength=E)
    np.testing.assert_array_equal(c2, np.minimum(hist, cap))
    for e in range(E):
        kept = p2[o2[e]:o2[e + 1]]
        dropped = np.flatnonzero((idx.reshape(-1) == e) & (i2.reshape(-1) < 0))
        if dropped.size and kept.size:
            assert dropped.min() > kept.max()


def test_capacity_formula():
    assert O.capacity(1.25, 2, 16384, 16) == 2560
    assert O.capacity(1.0, 1, 10, 4) == 3                 # ceil(2.5)
    assert O.capacity(0.0, 1, 10, 4) is None and O.capacity(-1.0, 2, 10, 4) is None
    # The factor is a float32 number.  float32(1.2) = 0x3F99999A = 1.2000000476837158203125 exactly,
    # times 20 / 4 = 6.0000002384185791015625: one more than the 6 a double-precision 1.2 would give.
    assert O.capacity(1.2, 1, 20, 4) == 7
    assert O.capacity(np.float32(1.2), 1, 20, 4) == 7
    assert O.capacity(1.5, 1, 20, 4) == 8                 # 1.5 is exact in float32: 7.5 -> 8
    # float32(0.7) = 0x3F333333 = 0.699999988079071044921875 < 0.7: 0.7 * 30 / 3 stays at 7
    assert O.capacity(0.7, 1, 30, 3) == 7


def test_all_tokens_to_one_expert_and_empty_experts():
    T = 37
    idx = np.full((T, 1), 2, dtype=np.int32)
    counts, offsets, perm, inv = O.dispatch(idx, 4, 0, 4)
    assert counts.tolist() == [0, 0, T, 0] and offsets.tolist() == [0, 0, 0, T, T]
    assert perm.tolist() == list(range(T)) and inv[:, 0].tolist() == list(range(T))
    # local range sees no traffic
    c, o, p, i = O.dispatch(idx, 4, 0, 2)
    assert c.tolist() == [0, 0] and p.size == 0 and np.all(i == -1)


# ------------------------------------------------------------------ expert FFN

def test_gelu_tanh_properties():
    u = np.linspace(-6, 6, 2001)
    g = O.gelu_tanh(u)
    assert O.gelu_tanh(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(g - O.gelu_tanh(-u), u, atol=1e-15)          # g(u) - g(-u) = u
    exact = 0.5 * u * (1.0 + scipy.special.erf(u / math.sqrt(2.0)))        # erf GeLU
    assert np.max(np.abs(g - exact)) < 5e-4                                  # known gap of the tanh form
    assert np.max(np.abs(g - exact)) > 1e-4                                  # ...and it IS the tanh form
    np.testing.assert_allclose(O.gelu_tanh(np.array([10.0, -10.0])), [10.0, 0.0], atol=1e-12)
    # one scalar value by hand: inner = sqrt(2/pi) * (1 + 0.044715)
    inner = 0.7978845608028654 * 1.044715
    assert abs(O.gelu_tanh(np.array([1.0]))[0] - 0.5 * (1.0 + math.tanh(inner))) < 1e-15


def scalar_ffn(v, A, B):
    """GeLU(v A) B for one token with scalar loops; A is [d, F], B is [F, d_out]."""
    d, F = A.shape
    h = []
    for f in range(F):
        u = math.fsum(v[i] * A[i, f] for i in range(d))
        h.append(0.5 * u * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (u + 0.044715 * u * u * u))))
    return [math.fsum(h[f] * B[f, o] for f in range(F)) for o in range(B.shape[1])]


def test_single_expert_reduces_to_dense_ffn():
    """E = 1, top-1: the layer is the dense FFN GeLU(X A) B (an MoE layer is a drop-in for an FFN)."""
    T, d, F = 12, 6, 10
    x = RNG.standard_normal((T, d))
    A = RNG.standard_normal((d, F)) * 0.5
    B = RNG.standard_normal((F, d)) * 0.5
    Wg = RNG.standard_normal((d, 1))
    res = O.layer_forward(x, Wg, None, [A], [B], E=1, k=1, local_begin=0, local_count=1)
    dense = 0.5 * (x @ A) * (1 + np.tanh(math.sqrt(2 / math.pi) * ((x @ A) + 0.044715 * (x @ A) ** 3))) @ B
    np.testing.assert_allclose(res["out"], dense, rtol=1e-12, atol=1e-13)
    for t in (0, 5, 11):
        np.testing.assert_allclose(res["out"][t], scalar_ffn(x[t], A, B), rtol=1e-12, atol=1e-13)
    # non-square weights catch a transposed operand: F != d on purpose
    assert res["H"].shape == (T, F)


def test_ffn_flop_closed_form():
    b, s, h = 4, 2048, 2048
    assert O.ffn_flops(b * s, h, 4 * h) == 16 * b * s * h * h


# ------------------------------------------------------------------ whole layer vs per-token brute force

def brute_layer(x, Wg, bias, W1, W2, E, k, e0, n, cap, renorm):
    """Per-token definition with scalar loops and float32-rounded logits for the pick."""
    T, d = x.shape
    logits = np.zeros((T, E), dtype=np.float32)
    for t in range(T):
        for e in range(E):
            logits[t, e] = np.float32(math.fsum(x[t, i] * Wg[i, e] for i in range(d)) + (0.0 if bias is None else bias[e]))
    picks, weights = [], []
    for t in range(T):
        row = [float(v) for v in logits[t]]
        m = max(row)
        ex = [math.exp(v - m) for v in row]
        z = math.fsum(ex)
        pk = brute_topk(row, k)
        w = [ex[e] / z for e in pk]
        if renorm:
            sw = math.fsum(w)
            w = [v / sw for v in w]
        picks.append(pk)
        weights.append(w)
    seen = [0] * E
    out = np.zeros((T, d))
    for t in range(T):
        for j in range(k):
            e = picks[t][j]
            pos = seen[e]
            seen[e] += 1
            if not (e0 <= e < e0 + n):
                continue
            if cap is not None and pos >= cap:
                continue
            y = scalar_ffn(x[t], W1[e - e0], W2[e - e0])
            for o in range(d):
                out[t, o] += weights[t][j] * y[o]
    return out, picks


@pytest.mark.parametrize("T,d,F,E,k,e0,n,cf,renorm", [
    (24, 8, 12, 4, 1, 0, 4, 0.0, False),
    (24, 8, 12, 4, 2, 0, 4, 0.0, True),
    (24, 8, 12, 4, 2, 1, 2, 0.0, True),
    (32, 6, 10, 8, 2, 0, 8, 1.0, True),
    (32, 6, 10, 8, 2, 2, 4, 0.5, False),
    (20, 8, 12, 3, 3, 0, 3, 0.0, False),
])
def test_layer_matches_per_token_brute_force(T, d, F, E, k, e0, n, cf, renorm):
    x = RNG.standard_normal((T, d))
    Wg = RNG.standard_normal((d, E)) * 0.5
    bias = RNG.standard_normal(E) * 0.5
    W1 = [RNG.standard_normal((d, F)) * 0.4 for _ in range(n)]
    W2 = [RNG.standard_normal((F, d)) * 0.4 for _ in range(n)]
    res = O.layer_forward(x, Wg, bias, W1, W2, E=E, k=k, local_begin=e0, local_count=n,
                          capacity_factor=cf, renorm=renorm)
    cap = O.capacity(cf, k, T, E)
    ref, picks = brute_layer(x, Wg, bias, W1, W2, E, k, e0, n, cap, renorm)
    assert res["expert_idx"].tolist() == picks
    np.testing.assert_allclose(res["out"], ref, rtol=1e-11, atol=1e-12)
    # sampled-row evaluation agrees with the full layer
    rows = np.array([0, T // 2, T - 1, 3])
    sub, _ = O.layer_forward_rows(rows, x, Wg, bias, W1, W2, E=E, k=k, local_begin=e0,
                                  local_count=n, capacity_factor=cf, renorm=renorm)
    np.testing.assert_allclose(sub, res["out"][rows], rtol=1e-12, atol=1e-13)


def test_partition_sum_equals_all_local_and_zero_rows():
    """Summing the partial outputs of the devices of a tensor-parallel group (what the all-reduce
    does) gives the all-local output; rows whose expert lives elsewhere are exactly zero."""
    T, d, F, E = 48, 8, 16, 8
    x = RNG.standard_normal((T, d))
    Wg = RNG.standard_normal((d, E))
    W1 = [RNG.standard_normal((d, F)) * 0.3 for _ in range(E)]
    W2 = [RNG.standard_normal((F, d)) * 0.3 for _ in range(E)]
    full = O.layer_forward(x, Wg, None, W1, W2, E=E, k=1, local_begin=0, local_count=E)
    total = np.zeros_like(full["out"])
    for e0 in range(0, E, 2):
        part = O.layer_forward(x, Wg, None, W1[e0:e0 + 2], W2[e0:e0 + 2], E=E, k=1, local_begin=e0,
                               local_count=2)
        not_local = ~((full["expert_idx"][:, 0] >= e0) & (full["expert_idx"][:, 0] < e0 + 2))
        assert np.all(part["out"][not_local] == 0.0)
        np.testing.assert_array_equal(part["expert_idx"], full["expert_idx"])   # identical order on every rank
        total += part["out"]
    np.testing.assert_array_equal(total, full["out"])      # top-1: one non-zero contributor per row
    # top-2 partition sum (two contributors per row: equal up to rounding)
    full2 = O.layer_forward(x, Wg, None, W1, W2, E=E, k=2, local_begin=0, local_count=E, renorm=True)
    tot2 = sum(O.layer_forward(x, Wg, None, W1[e0:e0 + 4], W2[e0:e0 + 4], E=E, k=2, local_begin=e0,
                               local_count=4, renorm=True)["out"] for e0 in (0, 4))
    np.testing.assert_allclose(tot2, full2["out"], rtol=1e-13, atol=1e-14)


def test_token_permutation_equivariance_without_capacity():
    T, d, F, E = 40, 8, 12, 4
    x = RNG.standard_normal((T, d))
    Wg = RNG.standard_normal((d, E))
    W1 = [RNG.standard_normal((d, F)) * 0.3 for _ in range(E)]
    W2 = [RNG.standard_normal((F, d)) * 0.3 for _ in range(E)]
    p = RNG.permutation(T)
    a = O.layer_forward(x, Wg, None, W1, W2, E=E, k=2, local_begin=0, local_count=E, renorm=True)
    b = O.layer_forward(x[p], Wg, None, W1, W2, E=E, k=2, local_begin=0, local_count=E, renorm=True)
    np.testing.assert_allclose(b["out"], a["out"][p], rtol=1e-12, atol=1e-13)


def test_gate_weight_scales_the_expert_output():
    """Doubling every logit gap changes the weights but not the picks: out must scale row by row with
    the gate weight (fails if the weight is not applied at all)."""
    T, d, F, E = 16, 6, 8, 4
    x = RNG.standard_normal((T, d))
    Wg = RNG.standard_normal((d, E))
    W1 = [RNG.standard_normal((d, F)) for _ in range(E)]
    W2 = [RNG.standard_normal((F, d)) for _ in range(E)]
    a = O.layer_forward(x, Wg, None, W1, W2, E=E, k=1, local_begin=0, local_count=E)
    b = O.layer_forward(x, 2 * Wg, None, W1, W2, E=E, k=1, local_begin=0, local_count=E)
    np.testing.assert_array_equal(a["expert_idx"], b["expert_idx"])
    np.testing.assert_allclose(b["out"] * a["gate_w"], a["out"] * b["gate_w"], rtol=1e-12, atol=1e-13)
    assert not np.allclose(a["gate_w"], b["gate_w"])


# ---- auxiliary balance loss (GShard form; the paper prints no formula: pinned by closed forms) ----

def test_aux_loss_closed_forms():
    E, T = 8, 64
    # all logits equal: probabilities 1/E, every token's first pick is expert 0 (ties -> lowest)
    lg = np.zeros((T, E), dtype=np.float32)
    idx = O.top_k_picks(lg, 1)
    r = O.aux_loss(lg, idx)
    assert r["first_counts"].tolist() == [T] + [0] * (E - 1)
    np.testing.assert_allclose(r["mean_prob"], 1.0 / E, rtol=1e-15)
    assert abs(r["l_aux"] - 1.0) < 1e-14            # E * (1/E * 1)
    # perfectly balanced routing, token t prefers expert t mod E by a margin L: by symmetry the
    # mean probability is exactly 1/E per expert and so is the first-pick share: l_aux = 1
    L = 3.0
    lg = np.zeros((T, E))
    lg[np.arange(T), np.arange(T) % E] = L
    r = O.aux_loss(lg, O.top_k_picks(lg, 1))
    assert r["first_counts"].tolist() == [T // E] * E
    np.testing.assert_allclose(r["mean_prob"], 1.0 / E, rtol=1e-14)
    assert abs(r["l_aux"] - 1.0) < 1e-13
    # every token prefers expert 2 with softmax probability q = e^a / (e^a + E - 1): l_aux = E q
    a = 1.7
    lg = np.zeros((T, E))
    lg[:, 2] = a
    q = math.exp(a) / (math.exp(a) + E - 1)
    r = O.aux_loss(lg, O.top_k_picks(lg, 1))
    assert abs(r["l_aux"] - E * q) < 1e-13
    assert abs(r["mean_prob"][2] - q) < 1e-15 and abs(r["mean_prob"][0] - (1 - q) / (E - 1)) < 1e-15


def test_aux_loss_against_scalar_loops_and_invariances():
    rng = np.random.default_rng(11)
    T, E = 37, 5
    lg = rng.normal(size=(T, E)).astype(np.float32)
    idx2 = O.top_k_picks(lg, 2)
    r = O.aux_loss(lg, idx2)
    # restated with scalar loops
    mean_prob = [0.0] * E
    counts = [0] * E
    for t in range(T):
        m = max(float(v) for v in lg[t])
        ex = [math.exp(float(v) - m) for v in lg[t]]
        z = sum(ex)
        for e in range(E):
            mean_prob[e] += ex[e] / z / T
        best = 0
        for e in range(1, E):
            if float(lg[t, e]) > float(lg[t, best]):
                best = e
        counts[best] += 1
    want = E * sum(mean_prob[e] * counts[e] / T for e in range(E))
    assert r["first_counts"].tolist() == counts
    np.testing.assert_allclose(r["mean_prob"], mean_prob, rtol=1e-13)
    assert abs(r["l_aux"] - want) < 1e-13
    # only the first pick counts: top-1 and top-2 gating of the same logits give the same loss
    assert O.aux_loss(lg, O.top_k_picks(lg, 1))["l_aux"] == r["l_aux"]
    # the order of the tokens does not matter (up to summation order)
    p = rng.permutation(T)
    assert abs(O.aux_loss(lg[p], idx2[p])["l_aux"] - r["l_aux"]) < 1e-13
    # probabilities sum to one, shares sum to one; Cauchy-Schwarz-free bounds: 0 < l_aux <= E
    assert abs(r["mean_prob"].sum() - 1.0) < 1e-14 and r["first_counts"].sum() == T
    assert 0.0 < r["l_aux"] <= E


# ------------------------------------------------------------------ backward (chain rule of the forward)

def _fd_layer(theta, name, base, R, kw, eps=1e-6):
    """Central finite difference of L = sum(out * R) with respect to every entry of one input."""
    g = np.zeros_like(theta)
    it = np.nditer(theta, flags=["multi_index"])
    for _ in it:
        idx = it.multi_index
        vals = []
        for sgn in (+1.0, -1.0):
            args = {k: (v.copy() if isinstance(v, np.ndarray) else [m.copy() for m in v] if isinstance(v, list) else v)
                    for k, v in base.items()}
            if isinstance(args[name], list):
                args[name][idx[0]][idx[1:]] += sgn * eps
            else:
                args[name][idx] += sgn * eps
            out = O.layer_forward(args["x"], args["Wg"], args["bias"], args["W1"], args["W2"], logits_dtype=None,
                                  **kw)["out"]
            vals.append(np.sum(out * R))
        g[idx] = (vals[0] - vals[1]) / (2 * eps)
    return g


@pytest.mark.parametrize("k,renorm,cf,local", [(1, False, 0.0, (0, 4)), (2, True, 0.0, (0, 4)), (2, False, 0.75, (0, 4)),
                                               (2, True, 0.0, (1, 2)), (3, True, 1.0, (0, 4))])
def test_layer_backward_against_finite_differences(k, renorm, cf, local):
    """Every gradient layer_backward returns (tokens, router matrix and bias, both expert matrices)
    against central differences of layer_forward, entry by entry, on a layer small enough for that;
    gate weights and picks of top-1 / top-2 / top-3, renormalised or not, capacity drops, a subset of
    the experts.  The picks stay fixed under the perturbation (the seed leaves margins)."""
    rng = np.random.default_rng(100 + k)
    T, d, F, E = 9, 5, 7, 4
    base = dict(x=rng.standard_normal((T, d)), Wg=rng.standard_normal((d, E)), bias=0.3 * rng.standard_normal(E),
                W1=[0.7 * rng.standard_normal((d, F)) for _ in range(E)],
                W2=[0.7 * rng.standard_normal((F, d)) for _ in range(E)])
    e0, n = local
    kw = dict(E=E, k=k, local_begin=e0, local_count=n, capacity_factor=cf, renorm=renorm)
    loc = dict(base, W1=base["W1"][e0:e0 + n], W2=base["W2"][e0:e0 + n])
    R = rng.standard_normal((T, d))
    logits = O.router_logits(base["x"], base["Wg"], base["bias"])
    srt = -np.sort(-logits, axis=1)
    assert (srt[:, :-1] - srt[:, 1:]).min() > 1e-3          # no pick flips under a 1e-6 perturbation
    bw = O.layer_backward(loc["x"], loc["Wg"], loc["bias"], loc["W1"], loc["W2"], R, logits_dtype=None, **kw)
    assert (bw["fwd"]["inv_perm"] >= 0).any()
    tol = dict(rtol=2e-6, atol=2e-8)
    np.testing.assert_allclose(bw["dx"], _fd_layer(loc["x"], "x", loc, R, kw), **tol)
    np.testing.assert_allclose(bw["dWg"], _fd_layer(loc["Wg"], "Wg", loc, R, kw), **tol)
    np.testing.assert_allclose(bw["dbias"], _fd_layer(loc["bias"], "bias", loc, R, kw), **tol)
    fd_w1 = _fd_layer(np.stack(loc["W1"]), "W1", loc, R, kw)
    fd_w2 = _fd_layer(np.stack(loc["W2"]), "W2", loc, R, kw)
    np.testing.assert_allclose(bw["dW1"], fd_w1, **tol)
    np.testing.assert_allclose(bw["dW2"], fd_w2, **tol)
    if cf > 0:
        assert (bw["fwd"]["inv_perm"] < 0).any()              # the capacity did drop something


def test_gelu_grad_against_finite_differences_and_limits():
    u = np.linspace(-6, 6, 1201)
    eps = 1e-6
    fd = (O.gelu_tanh(u + eps) - O.gelu_tanh(u - eps)) / (2 * eps)
    np.testing.assert_allclose(O.gelu_tanh_grad(u), fd, rtol=0, atol=1e-8)
    assert O.gelu_tanh_grad(np.array([0.0]))[0] == 0.5
    np.testing.assert_allclose(O.gelu_tanh_grad(np.array([9.0, -9.0])), [1.0, 0.0], atol=1e-12)
    # The erf form has GeLU'' = phi(u) (2 - u^2), so its derivative is smallest at u = -sqrt(2), where it
    # is Phi(-sqrt 2) - sqrt(2) phi(sqrt 2) = -0.12890; the tanh form stays within 1e-3 of that.  (With
    # the factor 3 of the cubic term's derivative dropped the minimum is -0.0998 at u = -1.38.)
    g = O.gelu_tanh_grad(u)
    exact_min = 0.5 * (1 + math.erf(-1.0)) - math.sqrt(2) * math.exp(-1.0) / math.sqrt(2 * math.pi)
    assert abs(exact_min - (-0.12890)) < 1e-5
    assert abs(g.min() - exact_min) < 1e-3 and abs(u[np.argmin(g)] + math.sqrt(2)) < 0.03


def test_expert_ffn_backward_reduces_to_the_dense_ffn_gradients():
    """One expert holding every row: the textbook gradients of Y = GeLU(X A) B, written out with
    numpy, and the finite difference of <Y, R> in a few entries of A and B."""
    rng = np.random.default_rng(5)
    n, d, F = 6, 4, 5
    X, A, Bm, R = (rng.standard_normal(s) for s in ((n, d), (d, F), (F, d), (n, d)))
    bw = O.expert_ffn_backward(X, np.array([0, n]), [A], [Bm], R)
    U = X @ A
    dU = (R @ Bm.T) * O.gelu_tanh_grad(U)
    np.testing.assert_allclose(bw["dX"], dU @ A.T, rtol=1e-13)
    np.testing.assert_allclose(bw["dW1"][0], X.T @ dU, rtol=1e-13)
    np.testing.assert_allclose(bw["dW2"][0], O.gelu_tanh(U).T @ R, rtol=1e-13)
    eps = 1e-6
    for (i, j) in ((0, 0), (3, 4), (2, 1)):
        Ap, Am = A.copy(), A.copy()
        Ap[i, j] += eps
        Am[i, j] -= eps
        fd = (np.sum(O.gelu_tanh(X @ Ap) @ Bm * R) - np.sum(O.gelu_tanh(X @ Am) @ Bm * R)) / (2 * eps)
        assert abs(bw["dW1"][0][i, j] - fd) < 1e-7


def test_gate_backward_rows_sum_to_zero_and_renormalised_weights_have_no_common_mode():
    """Softmax gradients sum to zero over the experts; with renormalised weights (which sum to one)
    a d_gate_w that is constant over the picks gives no gradient at all."""
    rng = np.random.default_rng(6)
    logits = rng.standard_normal((11, 6))
    idx = O.top_k_picks(logits, 3)
    dgw = rng.standard_normal((11, 3))
    for renorm in (False, True):
        g = O.gate_backward(logits, idx, renorm, dgw)
        np.testing.assert_allclose(g.sum(axis=1), 0.0, atol=1e-14)
    g = O.gate_backward(logits, idx, True, np.full((11, 3), 2.5))
    np.testing.assert_allclose(g, 0.0, atol=1e-14)
