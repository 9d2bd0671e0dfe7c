"""Pins for the oracle's router/top-k, expert FFN and whole layer (Sections 1, 2.1, 3.2).

Checked against closed forms, numpy library routines on cases where quantization is lossless,
brute force on tiny shapes, and invariants of the definition; never against the oracle itself.
"""
import numpy as np
import pytest

import oracle


def qmax(b):
    return (1 << (b - 1)) - 1


def lossless_matrix(rng, rows, cols, b, g, s0):
    """Integers in [-qmax, qmax] times a power-of-two step, every group holding a +-qmax:
    the quantizer reproduces it exactly, so a quantized FFN equals the float FFN on it."""
    ints = rng.integers(-qmax(b), qmax(b) + 1, size=(rows, cols))
    ints[:, ::g] = qmax(b) * rng.choice([-1, 1], size=(rows, cols // g))
    return (ints * s0).astype(np.float32)


def make_expert(rng, d, f, b, g, swiglu, lossless=False, std=0.02):
    if lossless:
        w_in = lossless_matrix(rng, f, d, b, g, 2.0 ** -6)
        w_out = lossless_matrix(rng, d, f, b, g, 2.0 ** -8)
        w_gate = lossless_matrix(rng, f, d, b, g, 2.0 ** -5) if swiglu else None
    else:
        w_in = (rng.standard_normal((f, d)) * std).astype(np.float32)
        w_out = (rng.standard_normal((d, f)) * std).astype(np.float32)
        w_gate = (rng.standard_normal((f, d)) * std).astype(np.float32) if swiglu else None
    qi, si = oracle.quantize_pack(w_in, b, g)
    qo, so = oracle.quantize_pack(w_out, b, g)
    qg, sg = oracle.quantize_pack(w_gate, b, g) if swiglu else (None, None)
    return oracle.Expert(b, qi, si, qo, so, qg, sg), (w_in, w_gate, w_out)


def dense_ffn(w_in, w_gate, w_out, x):
    """Textbook FFN in float64 with numpy matmul."""
    a = x.astype(np.float64) @ w_in.astype(np.float64).T
    if w_gate is None:
        h = np.maximum(a, 0.0)
    else:
        h = a / (1.0 + np.exp(-a)) * (x.astype(np.float64) @ w_gate.astype(np.float64).T)
    return h @ w_out.astype(np.float64).T, h


# ------------------------------------------------------------------ router / top-k
def test_softmax_sums_to_one_and_topk_matches_sorting():
    rng = np.random.default_rng(0)
    T, d, E = 64, 96, 16
    x = rng.standard_normal((T, d)).astype(np.float32)
    Wr = (rng.standard_normal((E, d)) * 0.2).astype(np.float32)
    bias = rng.standard_normal(E).astype(np.float32)
    for k in (1, 2, 3):
        idx, gate, probs, logits = oracle.router_topk(x, Wr, bias, k, False, want_logits=True)
        ref_logits = x.astype(np.float64) @ Wr.astype(np.float64).T + bias
        assert np.allclose(logits, ref_logits, rtol=0, atol=1e-12)
        assert np.allclose(probs.sum(1), 1.0, atol=1e-6)
        order = np.argsort(-ref_logits, axis=1, kind="stable")[:, :k]
        assert np.array_equal(idx, order.astype(np.int32))
        p_ref = np.exp(ref_logits - ref_logits.max(1, keepdims=True))
        p_ref /= p_ref.sum(1, keepdims=True)
        assert np.allclose(gate, np.take_along_axis(p_ref, order, 1), rtol=1e-6)
        assert np.all(np.diff(gate, axis=1) <= 0), "gates come out in descending order"


def test_renormalised_gates_equal_softmax_over_the_selected_logits():
    rng = np.random.default_rng(1)
    T, d, E, k = 32, 64, 8, 2
    x = rng.standard_normal((T, d)).astype(np.float32)
    Wr = (rng.standard_normal((E, d)) * 0.3).astype(np.float32)
    idx, gate, probs, logits = oracle.router_topk(x, Wr, None, k, True, want_logits=True)
    sel = np.take_along_axis(logits, idx.astype(np.int64), 1)
    ref = np.exp(sel - sel.max(1, keepdims=True))
    ref /= ref.sum(1, keepdims=True)
    assert np.allclose(gate, ref, rtol=1e-6)
    assert np.allclose(gate.sum(1), 1.0, atol=1e-6)
    # k = 1 with renormalisation: the single gate is exactly one
    _, g1, _ = oracle.router_topk(x, Wr, None, 1, True)
    assert np.all(g1 == 1.0)


def test_topk_ties_go_to_the_lowest_index():
    d, E = 8, 6
    x = np.ones((1, d), np.float32)
    Wr = np.zeros((E, d), np.float32)
    Wr[[1, 3, 4]] = 0.25          # three experts with exactly equal, largest logits
    idx, gate, probs = oracle.router_topk(x, Wr, None, 2, False)
    assert list(idx[0]) == [1, 3]
    assert gate[0, 0] == gate[0, 1]
    idx, _, _ = oracle.router_topk(x, np.zeros((E, d), np.float32), None, 3, False)
    assert list(idx[0]) == [0, 1, 2]


def test_softmax_is_stable_for_logits_far_outside_the_range_of_exp():
    """Logits of +-1e3 .. 1e4 (exp of them overflows a double): the probabilities still sum to one, are finite,
    the order follows the logits, and the gates equal the closed form computed on shifted logits."""
    E, d = 6, 4
    x = np.array([[1.0, 0.0, 0.0, 0.0], [0.0, 1.0, 0.0, 0.0], [0.0, 0.0, 1.0, 0.0]], np.float32)
    Wr = np.zeros((E, d), np.float32)
    Wr[:, 0] = [1000.0, 9999.0, -5000.0, 9998.0, 10000.0, 0.0]          # token 0: huge positive logits
    Wr[:, 1] = [-10000.0, -9000.0, -9001.0, -1e4, -9500.0, -9000.5]     # token 1: huge negative logits
    # token 2: every probability but the largest underflows to zero; the second choice is still the second
    # largest SCORE (the router's order, Section 2.1), not the lowest index among the zeros
    Wr[:, 2] = [-3000.0, 0.0, -2000.0, -1000.0, -4000.0, -1500.0]
    for renorm in (False, True):
        idx, gate, probs, logits = oracle.router_topk(x, Wr, None, 2, renorm, want_logits=True)
        assert np.all(np.isfinite(probs)) and np.all(np.isfinite(gate))
        assert np.allclose(probs.sum(1), 1.0, atol=1e-6)
        assert [list(r) for r in idx] == [[4, 1], [1, 5], [1, 3]]
        assert list(gate[2]) == [1.0, 0.0]
        for t in range(3):
            z = logits[t] - logits[t].max()
            p = np.exp(z) / np.exp(z).sum()
            want = p[idx[t]] / (p[idx[t]].sum() if renorm else 1.0)
            assert np.allclose(gate[t], want, rtol=1e-6)
            assert np.allclose(probs[t], p, rtol=1e-6, atol=1e-30)


def test_non_finite_logits_still_give_valid_expert_indices():
    """A NaN or +Inf hidden state makes the softmax undefined. The routing must stay total all the same (the
    indices are used as addresses): every index lies in [0, E), the k indices of a token are distinct, a token
    whose softmax is undefined takes the experts 0 .. k-1 with NaN gates, and the other tokens are untouched."""
    rng = np.random.default_rng(11)
    T, d, E, k = 5, 16, 7, 3
    x = rng.standard_normal((T, d)).astype(np.float32)
    Wr = rng.standard_normal((E, d)).astype(np.float32)
    clean = oracle.router_topk(x, Wr, None, k, True)
    xb = x.copy()
    xb[1, 3] = np.nan
    xb[3, 0] = np.inf
    idx, gate, probs = oracle.router_topk(xb, Wr, None, k, True)
    assert idx.min() >= 0 and idx.max() < E
    assert all(len(set(r)) == k for r in idx.tolist())
    for t in (1, 3):
        assert list(idx[t]) == [0, 1, 2] and np.all(np.isnan(gate[t]))
    for t in (0, 2, 4):
        assert np.array_equal(idx[t], clean[0][t]) and np.array_equal(gate[t], clean[1][t])
    # logits of -inf only remove experts from the choice; when fewer than k finite ones remain the rest are
    # taken in index order with probability zero
    Wb = np.zeros((4, 2), np.float32)
    Wb[:, 0] = [-np.inf, 2.0, -np.inf, -np.inf]
    idx, gate, probs = oracle.router_topk(np.array([[1.0, 0.0]], np.float32), Wb, None, 3, False)
    assert list(idx[0]) == [1, 0, 2] and list(gate[0]) == [1.0, 0.0, 0.0]


def test_router_bias_is_added_to_the_logits():
    d, E = 4, 5
    x = np.zeros((1, d), np.float32)
    bias = np.array([0, 0, 3, 0, 1], np.float32)
    idx, gate, probs = oracle.router_topk(x, np.zeros((E, d), np.float32), bias, 2, False)
    assert list(idx[0]) == [2, 4]
    p = np.exp(bias - 3.0); p /= p.sum()
    assert np.allclose(probs[0], p, rtol=1e-6)


# ------------------------------------------------------------------ expert FFN
@pytest.mark.parametrize("b", (2, 4, 8))
@pytest.mark.parametrize("swiglu", (False, True))
def test_ffn_on_lossless_weights_equals_numpy_dense_ffn(b, swiglu):
    """Asymmetric shapes (d != f, T > 1) so a transposed operand or a swapped matrix cannot pass."""
    rng = np.random.default_rng(20 + b)
    d, f, g, T = 64, 160, 32, 3
    ex, (w_in, w_gate, w_out) = make_expert(rng, d, f, b, g, swiglu, lossless=True)
    x = rng.standard_normal((T, d)).astype(np.float32)
    y, h = oracle.expert_ffn(ex, d, f, g, int(swiglu), x, want_h=True)
    y_ref, h_ref = dense_ffn(w_in, w_gate, w_out, x)
    assert np.allclose(h, h_ref, rtol=2e-7, atol=1e-30)
    assert np.allclose(y, y_ref, rtol=1e-6, atol=1e-6 * np.abs(y_ref).max())


def test_ffn_integer_exact_case():
    """Integer weights (scale 1 = power of two) and integer x: the ReLU FFN is integer arithmetic."""
    rng = np.random.default_rng(5)
    d, f, g, b = 32, 64, 32, 4
    w_in = lossless_matrix(rng, f, d, b, g, 1.0)
    w_out = lossless_matrix(rng, d, f, b, g, 1.0)
    ex = oracle.Expert(b, *oracle.quantize_pack(w_in, b, g), *oracle.quantize_pack(w_out, b, g))
    x = rng.integers(-3, 4, size=(2, d)).astype(np.float32)
    y = oracle.expert_ffn(ex, d, f, g, 0, x)
    h = np.maximum(x.astype(np.int64) @ w_in.astype(np.int64).T, 0)
    assert np.array_equal(y.astype(np.int64), h @ w_out.astype(np.int64).T)


@pytest.mark.parametrize("swiglu", (False, True))
def test_ffn_brute_force_tiny(swiglu):
    """d=8, f=16, g=4: python loops over an independently unpacked copy of the codes."""
    rng = np.random.default_rng(11)
    d, f, g, b = 8, 16, 4, 4
    ex, _ = make_expert(rng, d, f, b, g, swiglu, std=0.5)
    x = rng.standard_normal((1, d)).astype(np.float32)

    def deq(packed, scales, rows, cols):
        W = np.zeros((rows, cols))
        for o in range(rows):
            word = int.from_bytes(packed[o].tobytes(), "little")
            for i in range(cols):
                u = (word >> (i * b)) & 15
                W[o, i] = float(scales[o, i // g].view(np.float16)) * (u - 8)
        return W

    Wi, Wo = deq(ex.q_in, ex.s_in, f, d), deq(ex.q_out, ex.s_out, d, f)
    Wg = deq(ex.q_gate, ex.s_gate, f, d) if swiglu else None
    h = []
    for o in range(f):
        a = sum(Wi[o, i] * float(x[0, i]) for i in range(d))
        if swiglu:
            bb = sum(Wg[o, i] * float(x[0, i]) for i in range(d))
            h.append(a / (1 + np.exp(-a)) * bb)
        else:
            h.append(max(a, 0.0))
    y_ref = [sum(Wo[o, i] * h[i] for i in range(f)) for o in range(d)]
    y = oracle.expert_ffn(ex, d, f, g, int(swiglu), x)
    assert np.allclose(y[0], y_ref, rtol=1e-6, atol=1e-7)


def test_ffn_zero_input_negative_preactivations_and_homogeneity():
    rng = np.random.default_rng(12)
    d, f, g, b = 64, 128, 32, 4
    ex, (w_in, _, w_out) = make_expert(rng, d, f, b, g, False)
    x = rng.standard_normal((2, d)).astype(np.float32)
    assert np.all(oracle.expert_ffn(ex, d, f, g, 0, np.zeros((1, d), np.float32)) == 0)
    y1 = oracle.expert_ffn(ex, d, f, g, 0, x)
    y2 = oracle.expert_ffn(ex, d, f, g, 0, 2 * x)
    assert np.array_equal(y2, 2 * y1), "ReLU FFN is positively homogeneous; doubling is exact in binary"
    # all pre-activations negative -> zero output: non-negative x against strictly negative wi
    w_neg = -np.abs(w_in) - 1e-3
    exn = oracle.Expert(b, *oracle.quantize_pack(w_neg, b, g), ex.q_out, ex.s_out)
    assert np.all(oracle.expert_ffn(exn, d, f, g, 0, np.abs(x) + 0.1) == 0)


@pytest.mark.parametrize("swiglu", (False, True))
def test_int8_expert_close_to_float_dense_ffn(swiglu):
    """An 8-bit expert reproduces the unquantized fp32 FFN to about 1e-2 relative.

    The level is set by the quantizer, not by the FFN code: with groups of 32 Gaussian weights
    the step is about 2.07 sigma / 127, i.e. a relative weight noise of 2.07 / 127 / sqrt(12) = 0.47 %,
    and an FFN of m matrices carries about sqrt(m) times that: 0.67 % (ReLU, m=2), 0.81 % (SwiGLU, m=3).
    So the bound is 1e-2 for ReLU and 1.25e-2 for SwiGLU, in the 2-norm per token; the measured
    weight noise is checked against the same prediction so the two claims hang together."""
    rng = np.random.default_rng(13)
    d, f, g = 768, 1536, 32
    ex, (w_in, w_gate, w_out) = make_expert(rng, d, f, 8, g, swiglu)
    x = rng.standard_normal((4, d)).astype(np.float32)
    y = oracle.expert_ffn(ex, d, f, g, int(swiglu), x)
    y_ref, _ = dense_ffn(w_in, w_gate, w_out, x)
    rel = np.linalg.norm(y - y_ref, axis=1) / np.linalg.norm(y_ref, axis=1)
    assert np.all(rel < (1.25e-2 if swiglu else 1e-2))
    w_hat = oracle.dequant(ex.q_in, ex.s_in, d, 8, g)
    noise = np.linalg.norm(w_hat - w_in) / np.linalg.norm(w_in)
    assert 0.0040 < noise < 0.0054
    m = 3 if swiglu else 2
    assert np.all(rel > 0.6 * np.sqrt(m) * noise) and np.all(rel < 1.6 * np.sqrt(m) * noise)
    # a 4-bit copy of the same weights is about 127/7 = 18x worse
    ex4, _ = make_expert(np.random.default_rng(13), d, f, 4, g, swiglu)
    y4 = oracle.expert_ffn(ex4, d, f, g, int(swiglu), x)
    rel4 = np.linalg.norm(y4 - y_ref, axis=1) / np.linalg.norm(y_ref, axis=1)
    assert np.all(rel4 > 10 * rel) and np.all(rel4 < 30 * rel)


def test_ffn_tokens_are_independent():
    rng = np.random.default_rng(14)
    d, f, g = 64, 96, 32
    ex, _ = make_expert(rng, d, f, 4, g, True)
    x = rng.standard_normal((5, d)).astype(np.float32)
    y = oracle.expert_ffn(ex, d, f, g, 1, x)
    for t in range(5):
        assert np.array_equal(oracle.expert_ffn(ex, d, f, g, 1, x[t:t + 1])[0], y[t])


# ------------------------------------------------------------------ whole layer
def build_layer(rng, d, f, E, g, swiglu, bits=None, lossless=False):
    bits = bits or [(2, 4, 8)[e % 3] for e in range(E)]
    experts, dense = [], []
    for e in range(E):
        ex, ws = make_expert(rng, d, f, bits[e], g, swiglu, lossless=lossless)
        experts.append(ex)
        dense.append(ws)
    Wr = (rng.standard_normal((E, d)) * 0.2).astype(np.float32)
    return experts, dense, Wr


@pytest.mark.parametrize("swiglu,k,renorm", [(False, 1, False), (True, 2, True), (True, 2, False)])
def test_layer_equals_gate_weighted_sum_of_dense_ffns_on_lossless_weights(swiglu, k, renorm):
    rng = np.random.default_rng(30)
    d, f, E, g, T = 64, 96, 6, 32, 7
    experts, dense, Wr = build_layer(rng, d, f, E, g, swiglu, lossless=True)
    x = rng.standard_normal((T, d)).astype(np.float32)
    y, idx, gate = oracle.layer_forward(experts, d, f, g, int(swiglu), k, renorm, Wr, None, x)
    logits = x.astype(np.float64) @ Wr.astype(np.float64).T
    p = np.exp(logits - logits.max(1, keepdims=True)); p /= p.sum(1, keepdims=True)
    for t in range(T):
        order = np.argsort(-logits[t], kind="stable")[:k]
        assert list(idx[t]) == list(order)
        gts = p[t, order] / (p[t, order].sum() if renorm else 1.0)
        ref = sum(gts[j] * dense_ffn(*dense[order[j]], x[t:t + 1])[0][0] for j in range(k))
        assert np.allclose(y[t], ref, rtol=1e-5, atol=1e-6 * np.abs(ref).max())


def test_one_hot_routing_equals_a_single_dense_ffn():
    rng = np.random.default_rng(31)
    d, f, E, g, T = 64, 96, 5, 32, 4
    experts, dense, Wr = build_layer(rng, d, f, E, g, False, lossless=True)
    x = rng.standard_normal((T, d)).astype(np.float32)
    bias = np.zeros(E, np.float32); bias[3] = 50.0
    y, idx, gate = oracle.layer_forward(experts, d, f, g, 0, 1, False, Wr, bias, x)
    assert np.all(idx == 3) and np.allclose(gate, 1.0, atol=1e-6)
    ref, _ = dense_ffn(*dense[3], x)
    assert np.allclose(y, ref, rtol=1e-5, atol=1e-6 * np.abs(ref).max())


def test_permuting_experts_with_router_rows_leaves_output_unchanged_and_layer_is_pure():
    rng = np.random.default_rng(32)
    d, f, E, g, T = 64, 96, 6, 32, 5
    experts, _, Wr = build_layer(rng, d, f, E, g, True)
    x = rng.standard_normal((T, d)).astype(np.float32)
    y, idx, gate = oracle.layer_forward(experts, d, f, g, 1, 2, True, Wr, None, x)
    y_again, idx_again, _ = oracle.layer_forward(experts, d, f, g, 1, 2, True, Wr, None, x)
    assert np.array_equal(y, y_again) and np.array_equal(idx, idx_again)   # Section 4.2: results never depend on history
    perm = rng.permutation(E)
    yp, idxp, gatep = oracle.layer_forward([experts[i] for i in perm], d, f, g, 1, 2, True, Wr[perm], None, x)
    assert np.array_equal(perm[idxp], idx)
    assert np.array_equal(gatep, gate) and np.array_equal(yp, y)


def test_layer_handles_zero_tokens():
    rng = np.random.default_rng(33)
    experts, _, Wr = build_layer(rng, 32, 64, 3, 32, False)
    y, idx, gate = oracle.layer_forward(experts, 32, 64, 32, 0, 1, False, Wr, None, np.zeros((0, 32), np.float32))
    assert y.shape == (0, 32) and idx.shape == (0, 1)


# ------------------------------------------------------------------ routing given by the caller
@pytest.mark.parametrize("swiglu", (False, True))
def test_given_routing_equals_gate_weighted_sum_of_dense_ffns_on_lossless_weights(swiglu):
    """Section 3.1 ("Applicability"), static routing: the experts of a token are given. On losslessly
    quantizable weights the result is the plain gate-weighted sum of textbook dense FFNs; an index outside
    [0, E) contributes nothing, an expert named twice counts twice."""
    rng = np.random.default_rng(40)
    d, f, E, g, T, k = 64, 96, 6, 32, 6, 2
    experts, dense, _ = build_layer(rng, d, f, E, g, swiglu, lossless=True)
    x = rng.standard_normal((T, d)).astype(np.float32)
    idx = np.array([[0, 5], [3, 3], [2, -1], [E, 1], [4, 0], [7, -3]], np.int32)
    gate = rng.uniform(0.1, 1.5, size=(T, k)).astype(np.float32)
    y = oracle.layer_forward_routed(experts, d, f, g, int(swiglu), k, x, idx, gate)
    for t in range(T):
        ref = np.zeros(d)
        for j in range(k):
            if 0 <= idx[t, j] < E:
                ref += np.float64(gate[t, j]) * dense_ffn(*dense[idx[t, j]], x[t:t + 1])[0][0]
        assert np.allclose(y[t], ref, rtol=1e-5, atol=1e-6 * max(np.abs(ref).max(), 1e-3))
    assert np.all(y[5] == 0.0)


def test_given_routing_with_the_routers_own_decision_reproduces_the_layer():
    rng = np.random.default_rng(41)
    d, f, E, g, T, k = 64, 96, 5, 32, 5, 2
    experts, _, Wr = build_layer(rng, d, f, E, g, True, lossless=False)
    x = rng.standard_normal((T, d)).astype(np.float32)
    y, idx, gate = oracle.layer_forward(experts, d, f, g, 1, k, True, Wr, None, x)
    y2 = oracle.layer_forward_routed(experts, d, f, g, 1, k, x, idx, gate)
    assert np.array_equal(y, y2)
