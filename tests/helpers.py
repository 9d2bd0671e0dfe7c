"""Shared by the GPU parity tests and the smoke check: builds the SAME synthetic layer twice, once as
device tensors packed by the library's own quantizer and once as host arrays packed by the oracle's.
The two sides share only the fp32 weight bits they start from."""
import numpy as np
import torch

import gen
import oracle
import paper_2308_14352_amd as moeq


def pack_expert_gpu(w, bits, group, group_out=None):
    """fp32 device weights dict -> moeq.PackedExpert via the library's device quantizer."""
    q_in, s_in = moeq.moe_quantize_pack(w["w_in"], bits, group)
    q_out, s_out = moeq.moe_quantize_pack(w["w_out"], bits, group_out or group)
    q_g = s_g = None
    if "w_gate" in w:
        q_g, s_g = moeq.moe_quantize_pack(w["w_gate"], bits, group)
    return moeq.PackedExpert(bits, q_in, s_in, q_out, s_out, q_g, s_g)


def pack_expert_oracle(w, bits, group, group_out=None):
    """fp32 weights dict (any device) -> oracle.Expert via the oracle's quantizer, on the host."""
    host = {k: v.detach().cpu().numpy() for k, v in w.items()}
    q_in, s_in = oracle.quantize_pack(host["w_in"], bits, group)
    q_out, s_out = oracle.quantize_pack(host["w_out"], bits, group_out or group)
    q_g = s_g = None
    if "w_gate" in host:
        q_g, s_g = oracle.quantize_pack(host["w_gate"], bits, group)
    return oracle.Expert(bits, q_in, s_in, q_out, s_out, q_g, s_g)


def build_layer_pair(cfg, layer_id, device, bits_table=None, want_oracle=True, columns=False, stream=False):
    """Returns (moeq.Layer on `device`, [oracle.Expert] or None, Wr, bias). columns: the layer holds W_out in
    the dword-column-major layout (the one-kernel decode path); stream: W_in / W_gate in the row-block stream
    layout as well (the integer-dot streaming kernel); layer.canonical keeps the canonical experts."""
    bits_table = bits_table or gen.bitwidth_table(cfg, layer_id)
    gpu_experts, orc_experts = [], []
    for e in range(cfg.n_experts):
        w = gen.expert_weights(cfg, layer_id, e, device)
        gpu_experts.append(pack_expert_gpu(w, bits_table[e], cfg.group))
        if want_oracle:
            orc_experts.append(pack_expert_oracle(w, bits_table[e], cfg.group))
        del w
    Wr, bias = gen.router_weights(cfg, layer_id, device)
    canonical = gpu_experts
    if stream:
        gpu_experts = [e.with_stream_layout(cfg.d_model, cfg.d_ff, cfg.group) for e in canonical]
    elif columns:
        gpu_experts = [e.with_out_columns(cfg.d_ff, cfg.group) for e in canonical]
    layer = moeq.Layer(cfg.d_model, cfg.d_ff, cfg.top_k, cfg.group,
                       moeq.MOEQ_ACT_SWIGLU if cfg.swiglu else moeq.MOEQ_ACT_RELU, cfg.renorm,
                       moeq.MOEQ_BF16 if cfg.x_dtype == "bf16" else moeq.MOEQ_F32, Wr, bias, gpu_experts,
                       moeq.MOEQ_OUT_COLUMNS if (columns or stream) else moeq.MOEQ_OUT_CANONICAL,
                       moeq.MOEQ_IN_STREAM if stream else moeq.MOEQ_IN_CANONICAL)
    layer.canonical = canonical
    return layer, (orc_experts if want_oracle else None), Wr, bias


def oracle_layer(cfg, orc_experts, Wr, bias, x):
    return oracle.layer_forward(orc_experts, cfg.d_model, cfg.d_ff, cfg.group, int(cfg.swiglu), cfg.top_k,
                                cfg.renorm, Wr.detach().cpu().numpy(),
                                None if bias is None else bias.detach().cpu().numpy(),
                                x.detach().float().cpu().numpy())


def rel_err(y, y_ref):
    """Per-token max-norm relative error: ||y - y_ref||_inf / ||y_ref||_inf."""
    y = np.asarray(y, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    den = np.abs(y_ref).max(axis=-1)
    den = np.where(den == 0, 1.0, den)
    return np.abs(y - y_ref).max(axis=-1) / den


def near_tie_tokens(cfg, Wr, bias, x, gap=1e-5):
    """Tokens whose k-th and (k+1)-th (or two selected) router logits are closer than `gap`
    (computed by the oracle in double); their top-k order is not required to be bit-exact."""
    _, _, _, logits = oracle.router_topk(x.detach().float().cpu().numpy(), Wr.detach().cpu().numpy(),
                                         None if bias is None else bias.detach().cpu().numpy(),
                                         cfg.top_k, cfg.renorm, want_logits=True)
    srt = -np.sort(-logits, axis=1)
    k = cfg.top_k
    gaps = srt[:, :k] - srt[:, 1:k + 1] if srt.shape[1] > k else srt[:, :k - 1] - srt[:, 1:k]
    return np.where(gaps.min(axis=1) < gap)[0] if gaps.size else np.array([], dtype=np.int64)
