"""moe_layer_forward_static (no workspace argument, no allocation: the scratch is a fixed array in the library's
device code) against moe_layer_forward, through the C ABI: same kernels, so the outputs must be bit-identical,
on two calls in a row, the second with a smaller input; and the size limit is reported as an error."""
import numpy as np
import pytest
import torch

import gen
import paper_2308_14352_amd as moeq
from paper_2308_14352_amd import binding
from helpers import build_layer_pair, oracle_layer, rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("base,d,f,E,columns,T1,T2", [
    ("c4", 512, 1792, 8, True, 5, 2),       # one-kernel path
    ("c3", 512, 1024, 32, False, 8, 3),     # two-kernel path
    ("c5", 512, 1024, 8, False, 70, 40),    # grouped GEMMs, then fewer tokens through the same scratch
    ("c5", 512, 1024, 8, True, 40, 1),      # grouped GEMMs, then one token through the one-kernel path
    ("c4", 4096, 256, 8, "stream", 2, 1),   # the streaming kernel on integer dot products (stream layout)
])
def test_static_entry_matches_the_workspace_entry_on_two_calls_in_a_row(base, d, f, E, columns, T1, T2):
    cfg = gen.tiny_config(base, d, f, n_experts=E, n_layers=1)
    layer, orc_experts, Wr, bias = build_layer_pair(cfg, 0, DEV, columns=columns is True, stream=columns == "stream")
    assert layer.workspace_bytes(T1) <= binding.moe_static_scratch_bytes()
    x1 = gen.hidden(cfg, 0, 0, T1, DEV)
    x2 = gen.hidden(cfg, 0, 1, T2, DEV)
    want1 = moeq.moe_layer_forward(layer, x1, want_routing=True)
    want2 = moeq.moe_layer_forward(layer, x2, want_routing=True)
    torch.cuda.synchronize()
    got1 = binding.moe_layer_forward_static(layer, x1, want_routing=True)
    got2 = binding.moe_layer_forward_static(layer, x2, want_routing=True)     # smaller input, stale scratch behind it
    torch.cuda.synchronize()
    for got, want in ((got1, want1), (got2, want2)):
        assert torch.equal(got[0], want[0]) and torch.equal(got[1], want[1]) and torch.equal(got[2], want[2])
    # and against the oracle, to the decode / prefill bars
    y_ref, idx_ref, _ = oracle_layer(cfg, orc_experts, Wr, bias, x2)
    assert np.array_equal(got2[1].cpu().numpy(), idx_ref)
    assert rel_err(got2[0].cpu().numpy(), y_ref).max() < (2e-2 if T2 >= 32 else 2e-3)


def test_static_entry_rejects_what_does_not_fit_its_scratch():
    cfg = gen.tiny_config("c5", 1024, 4096, n_experts=4, n_layers=1)
    layer, _, _, _ = build_layer_pair(cfg, 0, DEV, want_oracle=False)
    T = 512                                         # the grouped path's staging alone is 512 x 2 x 4096 x 4 bytes
    assert layer.workspace_bytes(T) > binding.moe_static_scratch_bytes()
    x = gen.hidden(cfg, 0, 0, T, DEV)
    with pytest.raises(moeq.MoeqError) as ei:
        binding.moe_layer_forward_static(layer, x)
    assert ei.value.status == binding.MOEQ_EWORKSPACE
    y = binding.moe_layer_forward_static(layer, x[:0])        # zero tokens: a no-op
    assert y.shape[0] == 0
