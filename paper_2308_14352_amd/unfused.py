"""The paper's own execution flow for one expert, kept as a comparison: decompress, then compute in FP32.

Section 3.2 ("Expert-wise bitwidth adaptation") stores an expert compressed, decompresses it to FP32 when it
is activated and then runs the ordinary dense FFN on the FP32 copy. The library's kernels never form that
copy (decompression is fused into the GEMV/GEMM); this module runs the unfused flow on the same packed expert
so the two can be compared on the same inputs: the decompression is the library's `moe_dequantize` kernel,
the dense FFN is plain fp32 torch arithmetic (rocBLAS). It is a yardstick for benchmarks and tests, not a
path the product takes.
"""
import torch

from . import binding as B


def dequantize_expert(ex, d_model, d_ff, group, out=None):
    """FP32 copies {"w_in", "w_out"[, "w_gate"]} of a PackedExpert whose W_out is in the canonical layout.
    `out` may hold tensors of the right shapes to be overwritten (the decompression buffer of the paper)."""
    def deq(q, s, cols, name):
        if out is not None and name in out:
            rows = q.shape[0]
            B._check(B.lib().moe_dequantize(B._ptr(q), B._ptr(s), rows, cols, ex.bits, group, B._ptr(out[name]),
                                            B._stream(None)), "moe_dequantize")
            return out[name]
        return B.moe_dequantize(q, s, cols, ex.bits, group)
    w = {"w_in": deq(ex.q_in, ex.s_in, d_model, "w_in"), "w_out": deq(ex.q_out, ex.s_out, d_ff, "w_out")}
    if ex.q_gate is not None:
        w["w_gate"] = deq(ex.q_gate, ex.s_gate, d_model, "w_gate")
    return w


def dense_ffn_fp32(w, x):
    """y [T][d_model] fp32 of the dense FFN on FP32 weights; x [T][d_model] in fp32 or bf16."""
    xf = x.float()
    a = xf @ w["w_in"].t()
    if "w_gate" in w:
        h = a * torch.sigmoid(a) * (xf @ w["w_gate"].t())
    else:
        h = torch.relu(a)
    return h @ w["w_out"].t()


def expert_ffn_unfused(ex, d_model, d_ff, group, x, out=None):
    """Decompress the expert, then the dense FFN (what `moe_expert_ffn_q` computes without the FP32 copy)."""
    return dense_ffn_fp32(dequantize_expert(ex, d_model, d_ff, group, out), x)
