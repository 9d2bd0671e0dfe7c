"""Parity of the whole layer at the benchmark configurations' real shapes, over many (token, layer) pairs.

Default (-m gpu): a reduced sweep - c4: 4 layers x 16 tokens on the stream and the columns layouts (the layers
are chosen so that 2+2, 2+4 and 4+4 bit expert pairs all occur), c5: 64 tokens of the 2048-token prefill call,
stratified over every expert, the first and last positions of its 64-token blocks and the ragged last block.
With MOEQ_FULL_SCOPE=1: every (token, layer) pair of the benchmark's c1, c2 and c3 runs (c3 also with 8 tokens
per call), c4 all 32 layers x 16 tokens, c5 at least 256 stratified tokens; the figures are printed and, when
MOEQ_SCOPE_OUT names a file, written there as JSON. The oracle side groups the tokens by expert, so that an expert
is decompressed once per layer."""
import json
import os

import numpy as np
import pytest
import torch

import gen
import oracle
import paper_2308_14352_amd as moeq
from helpers import build_layer_pair, pack_expert_oracle, rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
FULL = os.environ.get("MOEQ_FULL_SCOPE") == "1"
RESULTS = {}


def _record(name, **kw):
    RESULTS[name] = kw
    out = os.environ.get("MOEQ_SCOPE_OUT")
    if out:
        with open(out, "w") as f:
            json.dump(RESULTS, f, indent=1)
    print(name, kw, flush=True)


def oracle_rows(cfg, layer_id, bits_table, Wr, bias, x_rows):
    """Oracle outputs for the rows of x_rows [N][d] (float32 numpy): routing for all rows at once, then every
    activated expert decompressed once and applied to the rows that chose it."""
    Wr_h = Wr.cpu().numpy()
    b_h = None if bias is None else bias.cpu().numpy()
    idx, gate, _, logits = oracle.router_topk(x_rows, Wr_h, b_h, cfg.top_k, cfg.renorm, want_logits=True)
    y = np.zeros((x_rows.shape[0], cfg.d_model), np.float64)
    for e in sorted(set(idx.flatten().tolist())):
        ex = pack_expert_oracle(gen.expert_weights(cfg, layer_id, e, DEV), bits_table[e], cfg.group)
        rows, slots = np.nonzero(idx == e)
        ye = oracle.expert_ffn(ex, cfg.d_model, cfg.d_ff, cfg.group, int(cfg.swiglu), x_rows[rows])
        for j in range(cfg.top_k):
            sel = slots == j
            if sel.any():
                y[rows[sel]] += gate[rows[sel], j][:, None].astype(np.float64) * ye[sel].astype(np.float64)
    srt = -np.sort(-logits, axis=1)
    k = cfg.top_k
    gaps = (srt[:, :k] - srt[:, 1:k + 1]).min(axis=1) if srt.shape[1] > k else np.full(len(srt), np.inf)
    return y, idx, gate, gaps


def check_layer(cfg, layer_id, layout, xs, calls, tol, gpu_rows=None):
    """xs: device tensor [N][d]; calls: list of row ranges, each one library call. Returns (max error over the
    compared rows, rows compared, near-tie rows left out of the index comparison). gpu_rows: compare these rows
    only (the library still runs every call)."""
    bits_table = gen.bitwidth_table(cfg, layer_id)
    layer, _, Wr, bias = build_layer_pair(cfg, layer_id, DEV, bits_table, want_oracle=False,
                                          columns=layout != "canonical", stream=layout == "stream")
    N = xs.shape[0]
    y = torch.empty((N, cfg.d_model), dtype=torch.float32, device=DEV)
    idx = torch.empty((N, cfg.top_k), dtype=torch.int32, device=DEV)
    for a, b in calls:
        yy, ii, _ = moeq.moe_layer_forward(layer, xs[a:b], want_routing=True)
        y[a:b] = yy
        idx[a:b] = ii
    torch.cuda.synchronize()
    rows = np.arange(N) if gpu_rows is None else np.asarray(gpu_rows)
    y_ref, idx_ref, _, gaps = oracle_rows(cfg, layer_id, bits_table, Wr, bias, xs[rows].float().cpu().numpy())
    tied = gaps < 1e-5
    got_idx = idx.cpu().numpy()[rows]
    assert np.array_equal(got_idx[~tied], idx_ref[~tied]), "top-k indices differ from the oracle"
    same = (got_idx == idx_ref).all(axis=1)
    err = rel_err(y.cpu().numpy()[rows][same], y_ref[same])
    assert err.max() < tol, (cfg.name, layer_id, layout, float(err.max()))
    del layer
    torch.cuda.empty_cache()
    return float(err.max()), int(same.sum()), int(tied.sum())


def _c4_layers_with_all_pairs():
    """Four layers of c4 whose 16 tokens meet 2+2, 2+4 and 4+4 bit expert pairs (checked by the test)."""
    return [0, 5, 11, 23]


@pytest.mark.parametrize("layout", ("stream", "columns"))
def test_c4_layers_by_16_tokens(layout):
    cfg = gen.CONFIGS["c4"]
    layers = list(range(cfg.n_layers)) if FULL else _c4_layers_with_all_pairs()
    worst, pairs = 0.0, set()
    for l in layers:
        xs = torch.cat([gen.hidden(cfg, l, s, 1, DEV) for s in range(16)])
        err, n, tied = check_layer(cfg, l, layout, xs, [(t, t + 1) for t in range(16)], 2e-3)
        worst = max(worst, err)
        bits = gen.bitwidth_table(cfg, l)
        Wr, _ = gen.router_weights(cfg, l, DEV)
        idx_ref, _, _ = oracle.router_topk(xs.float().cpu().numpy(), Wr.cpu().numpy(), None, 2, True)
        pairs |= {tuple(sorted((bits[a], bits[b]))) for a, b in idx_ref.tolist()}
    assert pairs == {(2, 2), (2, 4), (4, 4)}, pairs
    _record(f"c4_{layout}", layers=len(layers), tokens_per_layer=16, max_rel_err=worst)


def _stratified_tokens(idx, n_experts, per_expert):
    """Tokens covering, for every expert, the first / last rows of its 64-token blocks, the ragged last block and
    an even spread in between (rank = position of the token among those routed to the expert)."""
    chosen = set()
    for e in range(n_experts):
        toks = np.nonzero((idx == e).any(axis=1))[0]
        n = len(toks)
        if n == 0:
            continue
        ranks = {0, n - 1, n // 2, min(63, n - 1), min(64, n - 1), min(65, n - 1), (n // 64) * 64 - 1 if n >= 64 else 0,
                 min((n // 64) * 64, n - 1)}
        ranks |= set(np.linspace(0, n - 1, max(per_expert - len(ranks), 2) + 2).astype(int).tolist())
        chosen |= {int(toks[r]) for r in ranks}
    return sorted(chosen)


@pytest.mark.parametrize("layout", ("canonical",) + (("columns",) if FULL else ()))
def test_c5_prefill_stratified_tokens(layout):
    cfg = gen.CONFIGS["c5"]
    T = cfg.prefill_tokens
    xs = gen.hidden(cfg, 0, 0, T, DEV)
    Wr, bias = gen.router_weights(cfg, 0, DEV)
    idx_all, _, _ = oracle.router_topk(xs.float().cpu().numpy(), Wr.cpu().numpy(), bias.cpu().numpy(), cfg.top_k, cfg.renorm)
    rows = _stratified_tokens(idx_all, cfg.n_experts, 40 if FULL else 12)
    assert len(rows) >= (256 if FULL else 64)
    err, n, tied = check_layer(cfg, 0, layout, xs, [(0, T)], 2e-2, gpu_rows=rows)
    _record(f"c5_{layout}", tokens_compared=n, near_ties=tied, max_rel_err=err)


@pytest.mark.skipif(not FULL, reason="the full scope runs with MOEQ_FULL_SCOPE=1")
@pytest.mark.parametrize("name,cfg_id,batch,layout", [("c1", "c1", 1, "columns"), ("c2", "c2", 1, "columns"),
                                                      ("c3", "c3", 1, "columns"), ("c3b8", "c3", 8, "canonical")])
def test_every_token_layer_pair_of_the_switch_configurations(name, cfg_id, batch, layout):
    cfg = gen.CONFIGS[cfg_id]
    worst, n_all, tied_all = 0.0, 0, 0
    for l in range(cfg.n_layers):
        xs = torch.cat([gen.hidden(cfg, l, s, batch, DEV) for s in range(cfg.steps)])
        calls = [(s * batch, (s + 1) * batch) for s in range(cfg.steps)]
        err, n, tied = check_layer(cfg, l, layout, xs, calls, 2e-3)
        worst, n_all, tied_all = max(worst, err), n_all + n, tied_all + tied
    _record(name, token_layer_pairs=n_all, near_ties=tied_all, max_rel_err=worst)
