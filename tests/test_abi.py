"""CPU-only checks of the boundary: the library loads, exports every declared symbol, and rejects bad
arguments before touching the device. No compute call is made here."""
import ctypes as C
import os
import re

import pytest

from conftest import ROOT, golden_path
from paper_2308_14352_amd import binding as B


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "moeq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    names = declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in moeq.h but not exported"
    assert sorted(B.EXPORTS) == names


def test_status_strings():
    assert B.status_str(B.MOEQ_OK) == "ok"
    assert "workspace" in B.status_str(B.MOEQ_EWORKSPACE)


def test_packed_bytes_matches_the_papers_expert_sizes():
    """Section 4.2 / 4.3 print sizes that fix the expert shape d=768, d_ff=3072 with no biases."""
    vals = {}
    for line in open(golden_path("paper_sizes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, v, unit, _ = [s.strip() for s in line.split("|")]
        vals[k] = float(v)
    fp32_expert = 2 * 768 * 3072 * 4
    assert abs(10 * fp32_expert / 1e6 - vals["expert_buffer_10_experts_st_base"]) / 180 < 0.06
    assert abs(0.2e9 / fp32_expert - vals["experts_per_0.2GB_st_base_8"]) < 1.0
    # all experts at INT4 with one fp16 scale per channel (the paper's granularity, group = cols)
    q1, s1 = B.moe_packed_bytes(3072, 768, 4, 768)
    q2, s2 = B.moe_packed_bytes(768, 3072, 4, 3072)
    int4_expert = q1 + s1 + q2 + s2
    assert q1 == 3072 * 768 // 2 and s1 == 3072 * 2
    n_exp = int(vals["st_base_8_total_experts"])
    non_expert = vals["storage_st_base_8_fp32"] * 1e9 - n_exp * fp32_expert
    est = (non_expert + n_exp * int4_expert) / 1e9
    assert abs(est - vals["storage_st_base_8_int4_experts"]) / 0.85 < 0.05


@pytest.mark.parametrize("rows,cols,bits,group,expect", [
    (3072, 768, 2, 32, (3072 * 768 // 4, 3072 * 24 * 2)),
    (3072, 768, 4, 32, (3072 * 768 // 2, 3072 * 24 * 2)),
    (3072, 768, 8, 32, (3072 * 768, 3072 * 24 * 2)),
    (14336, 4096, 4, 128, (14336 * 2048, 14336 * 32 * 2)),
    (8, 64, 3, 32, (0, 0)), (8, 60, 4, 32, (0, 0)), (0, 64, 4, 32, (0, 0)),
])
def test_packed_bytes(rows, cols, bits, group, expect):
    assert B.moe_packed_bytes(rows, cols, bits, group) == expect


def _desc(**kw):
    ex = (B.moeq_expert * 2)(B.moeq_expert(4, 16, 16, None, None, 16, 16), B.moeq_expert(4, 16, 16, None, None, 16, 16))
    d = dict(d_model=64, d_ff=128, n_experts=2, top_k=1, group=32, act=0, renorm=0, x_dtype=0,
             router_w=16, router_bias=None, experts=ex, out_layout=0)
    d.update(kw)
    return B.moeq_layer_desc(**d), ex


@pytest.mark.parametrize("kw,status", [
    (dict(d_model=0), B.MOEQ_EINVAL),
    (dict(top_k=3), B.MOEQ_EINVAL),
    (dict(group=48), B.MOEQ_EINVAL),          # 64 % 48 != 0
    (dict(act=7), B.MOEQ_EINVAL),
    (dict(x_dtype=5), B.MOEQ_EINVAL),
    (dict(router_w=None), B.MOEQ_EINVAL),
    (dict(out_layout=2), B.MOEQ_EINVAL),
    (dict(out_layout=1, d_model=64, d_ff=136, group=8), B.MOEQ_EUNSUPPORTED),   # d_ff is not a multiple of 16
    (dict(out_layout=1, d_model=16384, d_ff=16384, group=32), B.MOEQ_EUNSUPPORTED),  # beyond the one-kernel path
    (dict(group=16, d_model=64, d_ff=128), B.MOEQ_EUNSUPPORTED),
])
def test_layer_create_rejects_bad_descriptions_before_any_device_call(kw, status):
    desc, _keep = _desc(**kw)
    h = C.c_void_p()
    st = B.lib().moe_layer_create(C.byref(desc), C.c_void_p(256), 4096, C.byref(h))
    assert st == status and not h.value


def test_layer_create_rejects_bad_experts():
    for bad in (B.moeq_expert(3, 16, 16, None, None, 16, 16), B.moeq_expert(4, None, 16, None, None, 16, 16),
                B.moeq_expert(4, 8, 16, None, None, 16, 16)):
        ex = (B.moeq_expert * 2)(B.moeq_expert(4, 16, 16, None, None, 16, 16), bad)
        desc, _ = _desc(experts=ex)
        h = C.c_void_p()
        assert B.lib().moe_layer_create(C.byref(desc), C.c_void_p(256), 4096, C.byref(h)) == B.MOEQ_EINVAL
    # SwiGLU needs the gate matrix
    desc, _ = _desc(act=1)
    h = C.c_void_p()
    assert B.lib().moe_layer_create(C.byref(desc), C.c_void_p(256), 4096, C.byref(h)) == B.MOEQ_EINVAL
    # table buffer too small / misaligned
    desc, _ = _desc()
    assert B.lib().moe_layer_create(C.byref(desc), C.c_void_p(256), 64, C.byref(h)) == B.MOEQ_EINVAL
    assert B.lib().moe_layer_create(C.byref(desc), C.c_void_p(260), 4096, C.byref(h)) == B.MOEQ_EINVAL


def test_compute_entry_points_reject_null_handles_and_shapes():
    L = B.lib()
    assert L.moe_router_topk(None, None, 1, None, None, None, None, 0, None) == B.MOEQ_EINVAL
    assert L.moe_layer_forward(None, None, 1, None, None, None, None, 0, None) == B.MOEQ_EINVAL
    assert L.moe_layer_forward_routed(None, None, 1, C.c_void_p(256), C.c_void_p(256), None, None, 0, None) == B.MOEQ_EINVAL
    assert L.moe_layer_forward_routed(None, None, 1, None, None, None, None, 0, None) == B.MOEQ_EINVAL
    assert L.moe_expert_ffn_q(None, 0, None, 1, None, 0, None, None, 0, None) == B.MOEQ_EINVAL
    assert L.moe_quantize_pack(None, 1, 64, 4, 32, None, None, None) == B.MOEQ_EINVAL
    assert L.moe_quantize_pack(C.c_void_p(256), 1, 64, 5, 32, C.c_void_p(256), C.c_void_p(256), None) == B.MOEQ_EINVAL
    assert L.moe_quantize_pack(C.c_void_p(256), 1, 60, 4, 30, C.c_void_p(256), C.c_void_p(256), None) == B.MOEQ_EINVAL
    assert L.moe_unpack_codes(C.c_void_p(256), 1, 64, 3, C.c_void_p(256), None) == B.MOEQ_EINVAL
    assert L.moe_dequantize(C.c_void_p(256), C.c_void_p(256), 1, 64, 4, 48, C.c_void_p(256), None) == B.MOEQ_EINVAL
    assert L.moe_workspace_bytes(None, 4) == 0
    assert L.moe_layer_path(None, 4) == -1
    assert B.moe_layer_table_bytes(8) == 8 * 64 and B.moe_layer_table_bytes(0) == 0
    p = C.c_void_p(256)
    q = C.c_void_p(4096)
    assert L.moe_prepare_out(None, p, 4, 64, 4, 32, q, q, None) == B.MOEQ_EINVAL
    assert L.moe_prepare_out(p, p, 6, 64, 4, 32, q, q, None) == B.MOEQ_EINVAL        # rows not a multiple of 4
    assert L.moe_prepare_out(p, p, 4, 64, 4, 32, p, q, None) == B.MOEQ_EINVAL        # in place
    assert L.moe_unprepare_out(p, p, 4, 64, 3, 32, q, q, None) == B.MOEQ_EINVAL
