"""Seeded tensors and bitwidth tables for the five benchmark configurations.

Every tensor is a pure function of (MASTER_SEED, configuration, layer, expert, tensor
name, step) and of the device it is drawn on (torch's CPU and GPU generators produce
different streams). A test that compares the GPU library with the CPU oracle draws a
tensor ONCE and hands the same bits to both sides (a host copy for the oracle).
"""
from dataclasses import dataclass, field, replace

import torch

MASTER_SEED = 230814352
_MASK = (1 << 64) - 1


def _splitmix64(z):
    z = (z + 0x9E3779B97F4A7C15) & _MASK
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK
    return z ^ (z >> 31)


def seed_for(*parts):
    """63-bit seed from the master seed and a tuple of small integers / short strings."""
    z = MASTER_SEED
    for p in parts:
        if isinstance(p, str):
            p = int.from_bytes(p.encode()[:8].ljust(8, b"\0"), "little")
        z = _splitmix64(z ^ (int(p) & _MASK))
    return z >> 1


def _generator(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def normal(shape, std, seed, device="cpu"):
    """fp32 N(0, std^2) tensor, seeded."""
    g = _generator(seed, device)
    t = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    if std != 1.0:
        t.mul_(std)
    return t


@dataclass(frozen=True)
class Config:
    name: str
    cid: int                 # index in the benchmark's configuration list
    d_model: int
    d_ff: int
    n_experts: int
    top_k: int
    act: str                 # "relu" (wi, wo) or "swiglu" (w1, w3, w2)
    group: int               # quantization group size along the input dimension
    n_layers: int
    renorm: bool             # gates divided by the sum of the selected probabilities
    x_dtype: str             # "f32" or "bf16": storage type of the hidden states
    bit_rule: str            # how the per-expert bitwidth table is drawn
    weight_std: float = 0.02
    router_std: float = 0.02
    bias_rule: str = "none"  # "none" | "hotset" | "normal"
    bias_param: float = 0.0
    steps: int = 1           # decode steps (tokens per sequence) the benchmark runs
    batches: tuple = (1,)    # tokens per call
    prefill_tokens: int = 0

    @property
    def swiglu(self):
        return self.act == "swiglu"


# Hot-set bias of the Switch-base-64 stack: 13 of 64 experts per layer get this much added
# to their router logit. The value was chosen offline (bisection on tokens drawn from this
# module) so that about 60 % of the tokens pick a hot expert; the benchmark reports the
# share it actually observes.
_C2_HOT_BIAS = 0.445

CONFIGS = {
    "c1": Config("switch-1layer-8e", 0, 768, 3072, 8, 1, "relu", 32, 1, False, "f32",
                 "uniform248", steps=64),
    "c2": Config("switch-base-64-stack", 1, 768, 3072, 64, 1, "relu", 32, 6, False, "f32",
                 "mix_30_50_20", bias_rule="hotset", bias_param=_C2_HOT_BIAS, steps=512),
    "c3": Config("switch-large-128-stack", 2, 1024, 4096, 128, 1, "relu", 64, 12, False, "f32",
                 "int4_25pct2_10pct8", steps=256, batches=(1, 8)),
    "c4": Config("mixtral-8x7b-decode-stack", 3, 4096, 14336, 8, 2, "swiglu", 128, 32, True, "bf16",
                 "bernoulli24", steps=128),
    "c5": Config("mixtral-8x7b-prefill-layer", 4, 4096, 14336, 8, 2, "swiglu", 128, 1, True, "bf16",
                 "uniform48", router_std=1.0 / 64.0, bias_rule="normal", bias_param=0.5,
                 steps=1, batches=(2048,), prefill_tokens=2048),
}


def tiny_config(base, d_model, d_ff, n_experts=None, n_layers=None, group=None):
    """A shrunken copy of a configuration (same rules, smaller shapes) for quick parity cases."""
    c = CONFIGS[base]
    return replace(c, name=c.name + "-tiny", d_model=d_model, d_ff=d_ff,
                   n_experts=n_experts or c.n_experts, n_layers=n_layers or c.n_layers,
                   group=group or c.group)


def _randperm(n, seed):
    return torch.randperm(n, generator=_generator(seed, "cpu")).tolist()


def _randint(n, high, seed):
    return torch.randint(0, high, (n,), generator=_generator(seed, "cpu")).tolist()


def bitwidth_table(cfg, layer):
    """Per-expert bitwidths of one layer (list of ints in {2,4,8}); host-side, seeded."""
    E = cfg.n_experts
    seed = seed_for(cfg.cid, layer, "bits")
    rule = cfg.bit_rule
    if rule in ("uniform248", "uniform48"):
        choices = [2, 4, 8] if rule == "uniform248" else [4, 8]
        draw = [choices[i] for i in _randint(E, len(choices), seed)]
        # every choice appears at least once when there is room for it
        pos = _randperm(E, seed + 1)
        for j, b in enumerate(choices):
            if b not in draw and j < E:
                draw[pos[j]] = b
        return draw
    if rule == "mix_30_50_20":
        n2, n8 = int(0.30 * E), int(round(0.20 * E))
        table = [2] * n2 + [8] * n8 + [4] * (E - n2 - n8)
    elif rule == "int4_25pct2_10pct8":
        n2, n8 = int(0.25 * E), int(round(0.10 * E))
        table = [2] * n2 + [8] * n8 + [4] * (E - n2 - n8)
    elif rule == "bernoulli24":
        return [(2, 4)[i] for i in _randint(E, 2, seed)]
    else:
        raise ValueError(rule)
    perm = _randperm(E, seed)
    return [table[perm[i]] for i in range(E)]


def expert_weights(cfg, layer, expert, device="cpu"):
    """fp32 weights of one expert: {"w_in": [f][d], "w_out": [d][f]} plus "w_gate": [f][d] for SwiGLU.

    w_in is wi (ReLU) or w1 (SwiGLU); w_gate is w3; w_out is wo or w2. Output-major layout
    (row = output channel) so that quantization groups run along the input dimension.
    """
    d, f = cfg.d_model, cfg.d_ff
    out = {"w_in": normal((f, d), cfg.weight_std, seed_for(cfg.cid, layer, expert, "w_in"), device),
           "w_out": normal((d, f), cfg.weight_std, seed_for(cfg.cid, layer, expert, "w_out"), device)}
    if cfg.swiglu:
        out["w_gate"] = normal((f, d), cfg.weight_std, seed_for(cfg.cid, layer, expert, "w_gate"), device)
    return out


def router_weights(cfg, layer, device="cpu"):
    """(Wr [E][d] fp32, bias [E] fp32 or None)."""
    E, d = cfg.n_experts, cfg.d_model
    Wr = normal((E, d), cfg.router_std, seed_for(cfg.cid, layer, "router"), device)
    bias = None
    if cfg.bias_rule == "hotset":
        n_hot = max(1, round(0.2 * E))
        hot = _randperm(E, seed_for(cfg.cid, layer, "hotset"))[:n_hot]
        b = torch.zeros(E, dtype=torch.float32)
        b[hot] = cfg.bias_param
        bias = b.to(device)
    elif cfg.bias_rule == "normal":
        bias = normal((E,), cfg.bias_param, seed_for(cfg.cid, layer, "rbias"), "cpu").to(device)
    return Wr, bias


def hidden(cfg, layer, step, n_tokens, device="cpu"):
    """Hidden states [n_tokens][d] ~ N(0,1) of one (step, layer): fp32, or bf16 when the
    configuration stores them so. Each (step, layer) has its own seed: the attention blocks
    that would connect the layers of a real model are not part of this workload."""
    x = normal((n_tokens, cfg.d_model), 1.0, seed_for(cfg.cid, layer, step, "x"), device)
    return x.to(torch.bfloat16) if cfg.x_dtype == "bf16" else x
