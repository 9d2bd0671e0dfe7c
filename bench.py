#!/usr/bin/env python3
"""Benchmark of the mixed-bitwidth MoE layer forward on one MI355X.

A step is one decode step of the whole stack: every MoE layer of the workload runs router ->
top-k -> dequantize-fused expert FFNs -> gate-weighted combine on that step's hidden states, the
layers strictly in order on one stream. Inputs (packed experts, router weights, all hidden states)
are resident in HBM before the timed region. Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4|c1|c2|c2b8|c3|c3b8] [--no-extras]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes per launch of k_moe_stream on the c4 stack from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per
# dispatch, each scaled by what the counter reads for a plain pass over 1 GiB: factors 2.000 and 1.000), mean
# over the dispatches of `bench.py --no-extras --no-cpu-baseline --no-graph --layers 4 --steps 6 --warmup 2`,
# whose algorithmic bytes per launch are 130.4 MB. A stored figure, not measured in this run: counters need the
# profiler. The summary with the commands is profiles/k_moe_stream_c4_pmc.md.
PMC_TRAFFIC_C4_STREAM = {"fetch_bytes": 132.0e6, "write_bytes": 3.67e6, "algorithmic_bytes_same_slice": 130.4e6,
                         "source": "profiles/k_moe_stream_c4_pmc.md (rocprofv3 --pmc, stored; not re-measured here)"}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="c4", choices=["c1", "c2", "c2b8", "c3", "c3b8", "c4"])
    ap.add_argument("--no-extras", action="store_true", help="skip the short runs of the other decode workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="launch every layer from Python instead of a HIP graph")
    ap.add_argument("--layers", type=int, default=None, help="debug: truncate the stack")
    ap.add_argument("--pmc-calibrate", action="store_true",
                    help="run only a plain elementwise pass over 1 GiB (reads 1 GiB, writes 1 GiB) and exit: the "
                         "known-size kernel that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--shared-expert-probe", action="store_true",
                    help="run only calls of 8 tokens on a c3-shaped layer whose routing is given: all tokens on one "
                         "expert, 4 experts with 2 tokens each (neighbouring tokens / tokens 4 apart), 8 different "
                         "experts; 4 calls of each pattern in this order, every call on experts no earlier call touched "
                         "(the run rocprofv3's FETCH_SIZE per dispatch is read from)")
    ap.add_argument("--prefill-only", action="store_true",
                    help="run only the c5 prefill layer call (the run its rocprofv3 summaries are made from), "
                         "print its figures as one JSON line and exit")
    ap.add_argument("--layout", default="auto", choices=["auto", "stream", "columns", "canonical"],
                    help="weight layout: stream = W_in/W_gate in the row-block stream layout + W_out in columns (the "
                         "integer-dot streaming kernel; d_model 4096, groups of 128), columns = W_out in columns (one "
                         "streaming kernel per layer call), canonical = the two-kernel path on the boundary format, "
                         "auto = stream where the shape allows it, else columns for single-token steps and "
                         "for the Mixtral-sized experts, canonical for small layers with several tokens")
    return ap.parse_args()


class Stack:
    """All layers of one workload, packed in HBM, plus the hidden states of every (step, layer)."""

    def __init__(self, cfg, batch, steps, dev, n_layers=None, columns=True, stream=False, group_in=None,
                 group_out=None):
        import torch
        import gen
        import paper_2308_14352_amd as moeq
        self.cfg, self.batch, self.steps, self.columns, self.stream = cfg, batch, steps, columns or stream, stream
        self.L = n_layers or cfg.n_layers
        g_in, g_out = group_in or cfg.group, group_out or cfg.group
        self.layers, self.bits = [], []
        act = moeq.MOEQ_ACT_SWIGLU if cfg.swiglu else moeq.MOEQ_ACT_RELU
        xdt = moeq.MOEQ_BF16 if cfg.x_dtype == "bf16" else moeq.MOEQ_F32
        for l in range(self.L):
            bits = gen.bitwidth_table(cfg, l)
            experts = []
            for e in range(cfg.n_experts):
                w = gen.expert_weights(cfg, l, e, dev)
                q_in, s_in = moeq.moe_quantize_pack(w["w_in"], bits[e], g_in)
                q_out, s_out = moeq.moe_quantize_pack(w["w_out"], bits[e], g_out)
                q_g = s_g = None
                if cfg.swiglu:
                    q_g, s_g = moeq.moe_quantize_pack(w["w_gate"], bits[e], g_in)
                ex = moeq.PackedExpert(bits[e], q_in, s_in, q_out, s_out, q_g, s_g)
                if stream:
                    experts.append(ex.with_stream_layout(cfg.d_model, cfg.d_ff, cfg.group))
                    del q_in, s_in, q_g, s_g
                else:
                    experts.append(ex.with_out_columns(cfg.d_ff, g_out) if columns else ex)
                del w, ex, q_out, s_out
            Wr, bias = gen.router_weights(cfg, l, dev)
            self.layers.append(moeq.Layer(cfg.d_model, cfg.d_ff, cfg.top_k, cfg.group, act, cfg.renorm, xdt, Wr,
                                          bias, experts,
                                          moeq.MOEQ_OUT_COLUMNS if (columns or stream) else moeq.MOEQ_OUT_CANONICAL,
                                          moeq.MOEQ_IN_STREAM if stream else moeq.MOEQ_IN_CANONICAL,
                                          group_in=g_in, group_out=g_out))
            self.bits.append(bits)
        torch.cuda.synchronize()
        # hidden states of every (step, layer): [steps][L][batch][d]
        self.x_all = torch.stack([torch.stack([gen.hidden(cfg, l, s, batch, dev) for l in range(self.L)])
                                  for s in range(steps)])
        self.xs = torch.empty_like(self.x_all[0])               # staging: the current step's inputs
        self.y = torch.empty((self.L, batch, cfg.d_model), dtype=torch.float32, device=dev)
        self.ws = torch.empty(max(l.workspace_bytes(batch) for l in self.layers), dtype=torch.uint8, device=dev)
        self.packed_bytes = sum(e.nbytes() for l in self.layers for e in l.experts)

    def routing(self):
        """Top-k indices of every (step, layer, token), computed up front (untimed) for byte accounting."""
        import torch
        import paper_2308_14352_amd as moeq
        out = []
        for s in range(self.steps):
            out.append(torch.stack([moeq.moe_router_topk(self.layers[l], self.x_all[s, l])[0]
                                    for l in range(self.L)]))
        torch.cuda.synchronize()
        return torch.stack(out).cpu().numpy()                   # [steps][L][batch][k]

    def algorithmic_bytes(self, idx):
        """Bytes the path must move per (step, layer): packed codes+scales of the DISTINCT activated
        experts, the router weights (+bias), the hidden states in and the outputs out."""
        import numpy as np
        cfg = self.cfg
        xb = 2 if cfg.x_dtype == "bf16" else 4
        per = np.zeros((self.steps, self.L))
        for l, layer in enumerate(self.layers):
            eb = np.array([e.nbytes() for e in layer.experts], dtype=np.float64)
            fixed = layer.router_w.numel() * 4 + (0 if layer.router_bias is None else cfg.n_experts * 4) \
                + self.batch * cfg.d_model * (xb + 4)
            for s in range(self.steps):
                per[s, l] = eb[np.unique(idx[s, l])].sum() + fixed
        return per

    def run_step_eager(self, s):
        import paper_2308_14352_amd as moeq
        self.xs.copy_(self.x_all[s])
        for l in range(self.L):
            moeq.moe_layer_forward(self.layers[l], self.xs[l], y=self.y[l], ws=self.ws)

    def capture(self):
        import torch
        import paper_2308_14352_amd as moeq
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for l in range(self.L):
                moeq.moe_layer_forward(self.layers[l], self.xs[l], y=self.y[l], ws=self.ws)
        return g

    def run_step_graph(self, g, s):
        self.xs.copy_(self.x_all[s])
        g.replay()


def time_steps(stack, steps, warmup, use_graph, passes=5):
    """W warm-up steps, then the K steps timed `passes` times over (each pass: exactly K steps between two
    synchronisations). Returns (seconds of the median pass, seconds of every pass, graph)."""
    import torch
    g = None
    if use_graph:
        g = stack.capture()                       # a fresh layer's first call may be captured
    run = (lambda s: stack.run_step_graph(g, s)) if use_graph else stack.run_step_eager
    for s in range(warmup):
        run(s % stack.steps)
    times = []
    for _ in range(passes):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(steps):
            run(s % stack.steps)
        torch.cuda.synchronize()
        times.append(time.perf_counter() - t0)
    return sorted(times)[len(times) // 2], times, g


class HipEvents:
    """Raw HIP events through ctypes on the HIP runtime torch already loaded (plumbing only)."""

    def __init__(self):
        import ctypes as C
        self.C = C
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventSynchronize.argtypes = [C.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]
        self.pool = []

    def new(self):
        ev = self.C.c_void_p()
        assert self.hip.hipEventCreate(self.C.byref(ev)) == 0
        self.pool.append(ev)
        return ev

    def ms(self, a, b):
        out = self.C.c_float(0)
        assert self.hip.hipEventSynchronize(b) == 0
        assert self.hip.hipEventElapsedTime(self.C.byref(out), a, b) == 0
        return out.value

    def close(self):
        for ev in self.pool:
            self.hip.hipEventDestroy(ev)
        self.pool = []


def dominant_kernel_events(stack, steps, idx):
    """Eager pass over `steps` steps with a HIP event pair the library attaches to the dominant kernel
    of every layer call (begin and end of the kernel's execution on its stream): k_moe_decode (the whole layer
    but the final sum of partial vectors) with W_out in columns, else k_ffn_in (phase 1, about two thirds
    of the bytes). Returns (mean duration in ms, mean algorithmic bytes of that kernel, and for single-token
    calls the same two figures grouped by the bitwidths of the chosen experts)."""
    import numpy as np
    import torch
    import paper_2308_14352_amd as moeq
    from paper_2308_14352_amd import binding
    cfg = stack.cfg
    evs = HipEvents()
    pairs, nbytes, mixes = [], [], []
    xb = 2 if cfg.x_dtype == "bf16" else 4
    for s in range(steps):
        sd = s % stack.steps
        stack.xs.copy_(stack.x_all[sd])
        for l in range(stack.L):
            a, b = evs.new(), evs.new()
            binding.moe_layer_profile_kernel(stack.layers[l], binding.MOEQ_KERNEL_FUSED if stack.columns
                                             else binding.MOEQ_KERNEL_FFN_IN, a.value, b.value)
            moeq.moe_layer_forward(stack.layers[l], stack.xs[l], y=stack.y[l], ws=stack.ws)
            binding.moe_layer_profile_kernel(stack.layers[l], 0)
            pairs.append((a, b))
            layer = stack.layers[l]
            if stack.columns:       # router weights (+bias), x, every (token, choice) slot's whole expert
                tot = stack.batch * cfg.d_model * xb + layer.router_w.numel() * 4 \
                    + (0 if layer.router_bias is None else cfg.n_experts * 4)
            else:                   # x, logits, the h vectors out
                tot = stack.batch * cfg.d_model * xb + stack.batch * cfg.top_k * cfg.d_ff * 4 \
                    + stack.batch * cfg.n_experts * 4
            for t in range(stack.batch):                 # the kernel streams every (token, choice) slot
                for e in idx[sd, l, t]:
                    ex = layer.experts[int(e)]
                    tensors = (ex.q_in, ex.s_in, ex.q_gate, ex.s_gate) + ((ex.q_out, ex.s_out) if stack.columns else ())
                    for tns in tensors:
                        if tns is not None:
                            tot += tns.numel() * tns.element_size()
            nbytes.append(tot)
            mixes.append("+".join(str(b) for b in sorted(layer.experts[int(e)].bits for e in idx[sd, l, 0])))
    torch.cuda.synchronize()
    ms = [evs.ms(a, b) for a, b in pairs]
    evs.close()
    by_mix = {}
    if stack.batch == 1:
        for m in sorted(set(mixes)):
            sel = [i for i, mm in enumerate(mixes) if mm == m]
            t, nb = float(np.mean([ms[i] for i in sel])), float(np.mean([nbytes[i] for i in sel]))
            by_mix[m] = {"launches": len(sel), "avg_launch_ms": t, "bytes_per_launch": nb, "GBps": nb / t / 1e6}
    return float(np.mean(ms)), float(np.mean(nbytes)), by_mix


def cpu_baseline(stack, dev, budget_layers):
    """The CPU oracle on a bounded sample: `budget_layers` (step 0, layer l) pairs, each the full
    paper-order path (decompress the activated experts to fp32, FFN, combine). The oracle quantizes its
    own copy of the weights from the same fp32 bits; only its forward pass is timed."""
    import numpy as np
    import gen
    import oracle
    cfg = stack.cfg
    total, n, one_core = 0.0, 0, 0.0
    all_cores = oracle.num_threads()
    for l in range(min(budget_layers, stack.L)):
        Wr, bias = gen.router_weights(cfg, l, dev)
        x = stack.x_all[0, l].float().cpu().numpy()
        Wr_h = Wr.cpu().numpy()
        b_h = None if bias is None else bias.cpu().numpy()
        idx, _, _ = oracle.router_topk(x, Wr_h, b_h, cfg.top_k, cfg.renorm)
        dummy = oracle.Expert(4, np.zeros(1, np.uint8), np.zeros(1, np.uint16), np.zeros(1, np.uint8),
                              np.zeros(1, np.uint16), np.zeros(1, np.uint8), np.zeros(1, np.uint16))
        experts = [dummy] * cfg.n_experts
        for e in sorted(set(idx.flatten().tolist())):
            w = {k: v.cpu().numpy() for k, v in gen.expert_weights(cfg, l, e, dev).items()}
            b = stack.bits[l][e]
            qi, si = oracle.quantize_pack(w["w_in"], b, cfg.group)
            qo, so = oracle.quantize_pack(w["w_out"], b, cfg.group)
            qg, sg = oracle.quantize_pack(w["w_gate"], b, cfg.group) if cfg.swiglu else (None, None)
            experts[e] = oracle.Expert(b, qi, si, qo, so, qg, sg)
            del w
        t0 = time.perf_counter()
        oracle.layer_forward(experts, cfg.d_model, cfg.d_ff, cfg.group, int(cfg.swiglu), cfg.top_k, cfg.renorm,
                             Wr_h, b_h, x)
        total += time.perf_counter() - t0
        n += 1
        if l == 0:                                  # the same token-layer once more on a single core
            oracle.set_num_threads(1)
            t0 = time.perf_counter()
            oracle.layer_forward(experts, cfg.d_model, cfg.d_ff, cfg.group, int(cfg.swiglu), cfg.top_k, cfg.renorm,
                                 Wr_h, b_h, x)
            one_core = time.perf_counter() - t0
            oracle.set_num_threads(all_cores)
    per_layer = total / n
    return {"value": stack.batch / (per_layer * stack.L), "unit": "tokens/s", "cores": all_cores,
            "kind": "oracle",
            "one_core": {"value": stack.batch / (one_core * stack.L), "unit": "tokens/s",
                         "sample": f"step 0 of layer 0 (1 token-layer), {one_core * 1e3:.1f} ms"},
            "build": oracle.BUILD_FLAGS,
            "sample": f"step 0 of layers 0..{n - 1} ({n} token-layers, batch {stack.batch}); "
                      f"{per_layer * 1e3:.1f} ms per token-layer, scaled to the {stack.L}-layer stack"}


def run_prefill(dev, reps=5, columns=False, stream=False):
    """c5: one Mixtral-8x7B-shaped layer, 2048 tokens in one call (grouped GEMMs on the matrix cores).
    columns: W_out in the dword-column-major layout the decode kernels want (GEMM 2 then gathers its words);
    stream: W_in / W_gate in the stream layout of the decode kernel as well (the layer a decode stack holds)."""
    import torch
    import gen
    import paper_2308_14352_amd as moeq
    cfg = gen.CONFIGS["c5"]
    T = cfg.prefill_tokens
    st = Stack(cfg, T, 1, dev, 1, columns=columns, stream=stream)
    layer, x = st.layers[0], st.x_all[0, 0]
    y = torch.empty((T, cfg.d_model), dtype=torch.float32, device=dev)
    ws = torch.empty(layer.workspace_bytes(T), dtype=torch.uint8, device=dev)
    for _ in range(2):
        moeq.moe_layer_forward(layer, x, y=y, ws=ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        moeq.moe_layer_forward(layer, x, y=y, ws=ws)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / reps
    flops = 2.0 * 3 * cfg.d_model * cfg.d_ff * T * cfg.top_k
    return {"tokens_per_s": T / dt, "ms_per_call": dt * 1e3, "tokens": T, "achieved_TFLOPs": flops / dt / 1e12,
            "mfma_f16_peak_TFLOPs": 2500.0, "frac_of_mfma_peak": flops / dt / 2.5e15,
            "packed_GB": st.packed_bytes / 1e9, "bitwidths": st.bits[0],
            "layout": "stream" if stream else ("columns" if columns else "canonical")}


def run_unfused_comparison(dev, reps=10):
    """One Mixtral-shaped 4-bit expert at batch 1: the fused kernels against the paper's own flow (Section 3.2:
    decompress the activated expert to FP32, then a dense FP32 FFN), the decompression by the library's
    kernel into a preallocated buffer, the dense FFN by fp32 matrix products (rocBLAS through torch)."""
    import torch
    import gen
    import paper_2308_14352_amd as moeq
    from paper_2308_14352_amd import unfused
    cfg = gen.CONFIGS["c4"]
    w = gen.expert_weights(cfg, 0, 0, dev)
    q_in, s_in = moeq.moe_quantize_pack(w["w_in"], 4, cfg.group)
    q_out, s_out = moeq.moe_quantize_pack(w["w_out"], 4, cfg.group)
    q_g, s_g = moeq.moe_quantize_pack(w["w_gate"], 4, cfg.group)
    del w
    ex = moeq.PackedExpert(4, q_in, s_in, q_out, s_out, q_g, s_g)
    Wr, bias = gen.router_weights(cfg, 0, dev)
    layer = moeq.Layer(cfg.d_model, cfg.d_ff, 1, cfg.group, moeq.MOEQ_ACT_SWIGLU, cfg.renorm, moeq.MOEQ_BF16,
                       Wr[:1].contiguous(), None, [ex.with_out_columns(cfg.d_ff, cfg.group)], moeq.MOEQ_OUT_COLUMNS)
    x = gen.hidden(cfg, 0, 0, 1, dev)
    buf = {"w_in": torch.empty((cfg.d_ff, cfg.d_model), dtype=torch.float32, device=dev),
           "w_gate": torch.empty((cfg.d_ff, cfg.d_model), dtype=torch.float32, device=dev),
           "w_out": torch.empty((cfg.d_model, cfg.d_ff), dtype=torch.float32, device=dev)}
    y = torch.empty((1, cfg.d_model), dtype=torch.float32, device=dev)
    ws = layer.workspace(1)

    def timed(fn):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps * 1e3

    fused_ms = timed(lambda: moeq.moe_expert_ffn_q(layer, 0, x, y=y, ws=ws))
    deq_ms = timed(lambda: unfused.dequantize_expert(ex, cfg.d_model, cfg.d_ff, cfg.group, buf))
    dense_ms = timed(lambda: unfused.dense_ffn_fp32(buf, x))
    y_f = moeq.moe_expert_ffn_q(layer, 0, x)
    y_u = unfused.expert_ffn_unfused(ex, cfg.d_model, cfg.d_ff, cfg.group, x, buf)
    torch.cuda.synchronize()
    diff = float((y_f - y_u).abs().max() / y_u.abs().max())
    return {"expert": "c4 shape, 4 bits, one token", "fused_ms": fused_ms, "decompress_ms": deq_ms,
            "dense_fp32_ffn_ms": dense_ms, "unfused_over_fused": (deq_ms + dense_ms) / fused_ms,
            "max_rel_diff": diff, "fp32_copy_GB": 3 * cfg.d_model * cfg.d_ff * 4 / 1e9}


def run_shared_expert_probe(dev, layout):
    """Calls of 8 tokens with caller-given routing (moe_layer_forward_routed) on one c3-shaped layer whose 128
    experts are all 4-bit: how many bytes a call fetches when its tokens share experts is read from rocprofv3's
    FETCH_SIZE of the dispatches, in the order stated in `order`."""
    import torch
    import gen
    import paper_2308_14352_amd as moeq
    cfg = gen.CONFIGS["c3"]
    columns = layout == "columns"
    experts = []
    for e in range(cfg.n_experts):
        w = gen.expert_weights(cfg, 0, e, dev)
        q = [moeq.moe_quantize_pack(m, 4, cfg.group) for m in (w["w_in"], w["w_out"])]
        ex = moeq.PackedExpert(4, q[0][0], q[0][1], q[1][0], q[1][1], None, None)
        experts.append(ex.with_out_columns(cfg.d_ff, cfg.group) if columns else ex)
    Wr, bias = gen.router_weights(cfg, 0, dev)
    layer = moeq.Layer(cfg.d_model, cfg.d_ff, 1, cfg.group, moeq.MOEQ_ACT_RELU, 0, moeq.MOEQ_F32, Wr, bias, experts,
                       moeq.MOEQ_OUT_COLUMNS if columns else moeq.MOEQ_OUT_CANONICAL)
    T = 8
    x = gen.hidden(cfg, 0, 0, T, dev)
    gate = torch.ones((T, 1), dtype=torch.float32, device=dev)
    patterns = {"one_expert": [0] * 8, "four_experts_neighbours": [0, 0, 1, 1, 2, 2, 3, 3],
                "four_experts_apart": [0, 1, 2, 3, 0, 1, 2, 3], "eight_experts": list(range(8))}
    base, order = 0, []
    for name, pat in patterns.items():
        for _ in range(4):
            idx = torch.tensor([[base + v] for v in pat], dtype=torch.int32, device=dev)
            moeq.moe_layer_forward_routed(layer, x, idx, gate)
            torch.cuda.synchronize()
            base += max(pat) + 1
            order.append(name)
    assert base <= cfg.n_experts
    return {"layout": layout if layout != "auto" else "canonical", "tokens_per_call": T, "order": order,
            "expert_bytes": experts[0].nbytes(),
            "distinct_experts": {k: len(set(v)) for k, v in patterns.items()}}


WORKLOADS = {"c1": ("c1", 1), "c2": ("c2", 1), "c2b8": ("c2", 8), "c3": ("c3", 1), "c3b8": ("c3", 8), "c4": ("c4", 1)}
DEFAULT_STEPS = {"c1": 64, "c2": 512, "c2b8": 256, "c3": 256, "c3b8": 256, "c4": 128}


def run_workload(name, steps, warmup, use_graph, dev, n_layers=None, want_events=True, layout="columns",
                 per_channel=False):
    import gen
    cfg_id, batch = WORKLOADS[name]
    cfg = gen.CONFIGS[cfg_id]
    n_distinct = min(steps, cfg.steps)
    # per_channel: one float16 scale per channel of each matrix (Section 3.2) instead of the configuration's groups
    stack = Stack(cfg, batch, n_distinct, dev, n_layers, columns=layout != "canonical", stream=layout == "stream",
                  group_in=cfg.d_model if per_channel else None, group_out=cfg.d_ff if per_channel else None)
    idx = stack.routing()
    bytes_sl = stack.algorithmic_bytes(idx)
    elapsed, pass_times, _ = time_steps(stack, steps, warmup, use_graph)
    # bytes over the timed steps (steps may wrap around the distinct inputs)
    order = [s % n_distinct for s in range(steps)]
    total_bytes = float(bytes_sl[order].sum())
    res = {
        "tokens_per_s": steps * batch / elapsed,
        "layer_tokens_per_s": steps * batch * stack.L / elapsed,
        "ms_per_step": elapsed / steps * 1e3,
        "algorithmic_GBps": total_bytes / elapsed / 1e9,
        "bytes_per_layer_call": total_bytes / (steps * stack.L),
        "layers": stack.L, "batch": batch, "steps": steps,
        "packed_GB": stack.packed_bytes / 1e9,
        "ms_per_step_passes": [t / steps * 1e3 for t in pass_times],
    }
    if want_events:
        ms, kb, by_mix = dominant_kernel_events(stack, min(steps, 32), idx)
        res["kernel_ms"] = ms
        res["kernel_bytes"] = kb
        res["kernel_by_mix"] = by_mix
    if batch > 1:
        import numpy as np
        distinct = np.mean([len(np.unique(idx[s % n_distinct, l])) for s in range(steps) for l in range(stack.L)])
        res["distinct_experts_per_layer_call"] = float(distinct)
        res["pairs_per_layer_call"] = batch * cfg.top_k
    if cfg.bias_rule == "hotset":
        import numpy as np
        hot_share = []
        for l in range(stack.L):
            hot = (stack.layers[l].router_bias > 0).cpu().numpy()
            hot_share.append(hot[idx[:, l].reshape(-1)].mean())
        res["hot_expert_share"] = float(np.mean(hot_share))
    return stack, res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); multi-GPU runs are not part of it",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import gen
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.pmc_calibrate:
        a = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        for _ in range(3):
            torch.add(a, 1.0, out=b)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "torch.add over 2^28 fp32", "read_bytes": a.numel() * 4,
                          "write_bytes": b.numel() * 4}))
        return
    if args.shared_expert_probe:
        print(json.dumps({"shared_expert_probe": run_shared_expert_probe(dev, args.layout)}))
        return
    if args.prefill_only:
        print(json.dumps({"c5_prefill": run_prefill(dev, reps=args.steps or 5, columns=args.layout == "columns",
                                                    stream=args.layout == "stream")}))
        return
    name = args.workload
    steps = args.steps or DEFAULT_STEPS[name]
    use_graph = not args.no_graph
    def pick_layout(workload):
        c = gen.CONFIGS[WORKLOADS[workload][0]]
        batch = WORKLOADS[workload][1]
        if args.layout != "auto":
            return args.layout
        # auto: the stream layout where the integer-dot kernel takes the shape; else the one-kernel path for
        # single-token steps (measured faster on every configuration) and for the large layers; small layers
        # with several tokens per step run faster on the two-kernel path
        if c.d_model == 4096 and c.group == 128:
            return "stream"
        return "columns" if (batch == 1 or c.d_model * c.d_ff >= (1 << 24)) else "canonical"
    layout = pick_layout(name)
    columns = layout != "canonical"
    stack, res = run_workload(name, steps, args.warmup, use_graph, dev, args.layers, layout=layout)
    cfg = stack.cfg
    achieved = res["kernel_bytes"] / (res["kernel_ms"] * 1e-3) / 1e9
    out = {
        "metric": "decode MoE-layer tokens/s + achieved HBM GB/s on packed experts (% peak)",
        "value": res["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "passes": len(res["ms_per_step_passes"]),
        "ms_per_step_passes": res["ms_per_step_passes"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "i32" if layout == "stream" else "f32", "data": "synthetic",
        "dtype_note": ("hidden states enter as block-floating-point integers (one power of two per 128 columns, "
                       "15 bits), codes as stored; every group's dot product is an exact int32 sum of 4- or 8-bit "
                       "digit products; group scales, offsets, the activation and the gate-weighted sum are fp32"
                       if layout == "stream" else
                       "codes and activations enter the multipliers as binary16 (codes exactly; hidden states after "
                       "a per-token power-of-two scaling), every product and sum is fp32; scales and offsets are "
                       "applied in fp32"),
        "config": {"workload": f"{name}: {cfg.name}", "layers": stack.L, "d_model": cfg.d_model, "d_ff": cfg.d_ff,
                   "experts": cfg.n_experts, "top_k": cfg.top_k, "act": cfg.act, "group": cfg.group,
                   "batch": stack.batch, "x_dtype": cfg.x_dtype, "bitwidths": cfg.bit_rule,
                   "packed_GB": round(res["packed_GB"], 3), "launch": "hip-graph" if use_graph else "eager",
                   "layout": layout},
        "layer_tokens_per_s": res["layer_tokens_per_s"],
        "algorithmic_GBps": res["algorithmic_GBps"],
        "pct_hbm_peak": 100.0 * res["algorithmic_GBps"] / HBM_PEAK_GBS,
        "roofline": {"bound": "hbm",
                     "kernel": ("k_moe_stream (router + top-k + dequantize-fused FFN of every d_ff slice, integer dot "
                                "products)" if layout == "stream" else
                                "k_moe_decode (router + top-k + dequantize-fused FFN of every d_ff slice)" if columns
                                else "k_ffn_in (phase 1: top-k + dequantize-fused W_in/W_gate GEMVs)"),
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "bytes_per_launch": res["kernel_bytes"], "avg_launch_ms": res["kernel_ms"],
                     "traffic": None},
    }
    if res["kernel_by_mix"]:
        # the same kernel figures grouped by the bitwidths of the experts the token chose
        out["roofline"]["by_expert_bitwidths"] = res["kernel_by_mix"]
    if name == "c4" and layout == "stream":
        t = PMC_TRAFFIC_C4_STREAM
        out["roofline"]["traffic"] = t["fetch_bytes"] + t["write_bytes"]
        out["roofline"]["traffic_detail"] = t
    if stack.batch > 1:
        # FETCH_SIZE of the layer call's kernels is compared against these: bytes of the DISTINCT activated experts
        out["distinct_experts_per_layer_call"] = res["distinct_experts_per_layer_call"]
        out["distinct_expert_bytes_per_layer_call"] = res["bytes_per_layer_call"]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(stack, dev, 4 if name == "c4" else 12)
    del stack
    torch.cuda.empty_cache()
    if not args.no_extras:
        extras = {}
        for other, k in (("c1", 64), ("c2", 256), ("c2b8", 128), ("c3", 128), ("c3b8", 128)):
            if other == name:
                continue
            st, r = run_workload(other, k, args.warmup, use_graph, dev, want_events=False,
                                 layout=pick_layout(other))
            extras[other] = {"layout": pick_layout(other)}
            extras[other].update({kk: r[kk] for kk in ("tokens_per_s", "layer_tokens_per_s", "ms_per_step",
                                                  "algorithmic_GBps", "bytes_per_layer_call", "layers", "batch", "steps",
                                                  "packed_GB", "distinct_experts_per_layer_call", "pairs_per_layer_call")
                             if kk in r})
            if "hot_expert_share" in r:
                extras[other]["hot_expert_share"] = r["hot_expert_share"]
            del st
            torch.cuda.empty_cache()
        st, r = run_workload("c1", 64, args.warmup, use_graph, dev, want_events=False, layout="columns", per_channel=True)
        extras["c1_per_channel_scales"] = {"layout": "columns", "group_in": 768, "group_out": 3072}
        extras["c1_per_channel_scales"].update({kk: r[kk] for kk in ("tokens_per_s", "ms_per_step", "algorithmic_GBps",
                                                                      "layers", "batch", "steps", "packed_GB")})
        del st
        torch.cuda.empty_cache()
        extras["c5_prefill"] = run_prefill(dev)
        extras["c5_prefill_stream_layout"] = run_prefill(dev, stream=True)
        extras["c4_expert_fused_vs_unfused"] = run_unfused_comparison(dev)
        out["other_workloads"] = extras
    print(json.dumps(out))


if __name__ == "__main__":
    main()
