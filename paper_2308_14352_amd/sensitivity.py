"""Bitwidth-sensitivity harness on synthetic data (Section 3.2, "Profiling expert importance" and "Selecting
expert-wise bitwidths").

The paper ranks the experts of a model by the accuracy the model loses on validation sets when one expert
alone is run at INT2, then lowers the bitwidth of the least important experts one by one while the loss stays
within a tolerated bound. Accuracy needs the trained models and their datasets; this harness keeps the
procedure and replaces the measure by one that needs neither: the relative error of the layer's (or one
expert's) output against the same computation on the unquantized weights, over a batch of tokens. Everything
quantized runs through the library's own kernels (`moe_quantize_pack`, `moe_expert_ffn_q`,
`moe_layer_forward`); the unquantized reference is plain float64 torch arithmetic on the same device.
"""
import numpy as np
import torch

from . import binding as B


def dense_ffn(w, x, swiglu):
    """Unquantized expert FFN in float64: w = {"w_in", "w_out"[, "w_gate"]} fp32 tensors, x [T][d]."""
    xd = x.double()
    a = xd @ w["w_in"].double().t()
    if swiglu:
        h = a * torch.sigmoid(a) * (xd @ w["w_gate"].double().t())
    else:
        h = torch.relu(a)
    return h @ w["w_out"].double().t()


def pack_expert(w, bits, group):
    q_in, s_in = B.moe_quantize_pack(w["w_in"], bits, group)
    q_out, s_out = B.moe_quantize_pack(w["w_out"], bits, group)
    q_g = s_g = None
    if "w_gate" in w:
        q_g, s_g = B.moe_quantize_pack(w["w_gate"], bits, group)
    return B.PackedExpert(bits, q_in, s_in, q_out, s_out, q_g, s_g)


def _layer(experts, weights, top_k, group, swiglu, renorm, router_w, router_bias):
    d_ff, d_model = weights[0]["w_in"].shape
    return B.Layer(d_model, d_ff, top_k, group, B.MOEQ_ACT_SWIGLU if swiglu else B.MOEQ_ACT_RELU, renorm, B.MOEQ_F32,
                   router_w, router_bias, experts, B.MOEQ_OUT_CANONICAL)


def _rel(y, ref):
    return float(torch.linalg.norm(y.double() - ref) / torch.linalg.norm(ref))


def expert_errors(weights, x, group, swiglu, bits_list=(2, 4, 8)):
    """errors[e][i] = ||FFN_q(x) - FFN(x)|| / ||FFN(x)|| of expert e quantized to bits_list[i], over the tokens x
    (fp32 [T][d] on the GPU). Every expert sees every token: the measure is a property of the expert."""
    E = len(weights)
    router_w = torch.zeros((E, x.shape[1]), dtype=torch.float32, device=x.device)
    out = np.zeros((E, len(bits_list)))
    refs = [dense_ffn(w, x, swiglu) for w in weights]
    for i, b in enumerate(bits_list):
        experts = [pack_expert(w, b, group) for w in weights]
        layer = _layer(experts, weights, 1, group, swiglu, False, router_w, None)
        for e in range(E):
            out[e, i] = _rel(B.moe_expert_ffn_q(layer, e, x), refs[e])
        del layer, experts
    return out


def importance_order(errors_low):
    """Experts from the least to the most important: ascending error at the lowest bitwidth (ties: lower index)."""
    return [int(e) for e in np.argsort(np.asarray(errors_low), kind="stable")]


def layer_loss(weights, bits_table, x, top_k, group, swiglu, renorm, router_w, router_bias, packed=None):
    """Relative error of the layer's output with the experts at bits_table against unquantized experts under
    the same routing (the routing does not depend on the experts' bitwidths). packed: optional cache
    {(expert, bits): PackedExpert}."""
    packed = {} if packed is None else packed
    experts = []
    for e, b in enumerate(bits_table):
        if (e, b) not in packed:
            packed[(e, b)] = pack_expert(weights[e], b, group)
        experts.append(packed[(e, b)])
    layer = _layer(experts, weights, top_k, group, swiglu, renorm, router_w, router_bias)
    y, idx, gate = B.moe_layer_forward(layer, x, want_routing=True)
    ref = torch.zeros_like(y, dtype=torch.float64)
    for e in range(len(weights)):
        hit = (idx == e)
        rows = hit.any(dim=1).nonzero().flatten()
        if rows.numel() == 0:
            continue
        g = (gate.double() * hit).sum(dim=1)[rows]
        ref[rows] += g[:, None] * dense_ffn(weights[e], x[rows], swiglu)
    return _rel(y, ref)


def select_bitwidths(weights, x, top_k, group, swiglu, renorm, router_w, router_bias, tolerable_loss,
                     lo_bits=2, hi_bits=4, order=None):
    """The paper's second step with the output error as the loss: all experts start at hi_bits; following the
    importance list, the K least important ones go to lo_bits, K growing while the layer's loss stays within
    tolerable_loss. Returns (bits_table, K, loss at K, losses tried)."""
    E = len(weights)
    if order is None:
        order = importance_order(expert_errors(weights, x, group, swiglu, (lo_bits,))[:, 0])
    packed = {}
    table = [hi_bits] * E
    args = (x, top_k, group, swiglu, renorm, router_w, router_bias, packed)
    tried = [layer_loss(weights, table, *args)]
    K = 0
    while K < E:
        cand = list(table)
        cand[order[K]] = lo_bits
        loss = layer_loss(weights, cand, *args)
        if loss > tolerable_loss:
            break
        tried.append(loss)
        table = cand
        K += 1
    return table, K, tried[-1], tried
