"""ctypes front end of the CPU oracle (oracle/moe_oracle.cc).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's cpu_baseline
leg may import this module; the product package never does. Arrays are numpy,
host memory; every function is a thin marshalling layer over the C entry points.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.cc")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")


def build(force=True):
    """Compile the oracle with g++ (strict IEEE: no fast-math, no contraction)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["g++", "-std=c++17", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-shared", "-fPIC", _SRC, "-o", _LIB]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


class _Expert(C.Structure):
    _fields_ = [("bits", C.c_int32),
                ("q_in", C.c_void_p), ("s_in", C.c_void_p),
                ("q_gate", C.c_void_p), ("s_gate", C.c_void_p),
                ("q_out", C.c_void_p), ("s_out", C.c_void_p)]


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        _lib = C.CDLL(_LIB)
        _lib.orc_f32_to_f16.restype = C.c_uint16
        _lib.orc_f32_to_f16.argtypes = [C.c_float]
        _lib.orc_f16_to_f32.restype = C.c_float
        _lib.orc_f16_to_f32.argtypes = [C.c_uint16]
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _chk(rc, what):
    if rc != 0:
        raise ValueError(f"oracle: {what} rejected its arguments")


def f32_to_f16_bits(v):
    return int(lib().orc_f32_to_f16(float(np.float32(v))))


def f16_bits_to_f32(h):
    return float(lib().orc_f16_to_f32(int(h)))


def num_threads():
    return int(lib().orc_num_threads())


def set_num_threads(n):
    """OpenMP threads of the following calls (a timing knob of the benchmark's baseline leg)."""
    lib().orc_set_num_threads(C.c_int(int(n)))


BUILD_FLAGS = "g++ -std=c++17 -O2 -fopenmp -ffp-contract=off -fno-fast-math"


def quantize(w, bits, group):
    """w [rows][cols] fp32 -> (q int8 [rows][cols], scales uint16(fp16 bits) [rows][cols/group])."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    rows, cols = w.shape
    q = np.empty((rows, cols), np.int8)
    s = np.empty((rows, cols // max(group, 1)), np.uint16)
    _chk(lib().orc_quantize(_p(w), C.c_int64(rows), C.c_int64(cols), C.c_int(bits), C.c_int(group),
                            _p(q), _p(s)), "quantize")
    return q, s


def pack(q, bits):
    q = np.ascontiguousarray(q, dtype=np.int8)
    rows, cols = q.shape
    out = np.empty((rows, cols * bits // 8), np.uint8)
    _chk(lib().orc_pack(_p(q), C.c_int64(rows), C.c_int64(cols), C.c_int(bits), _p(out)), "pack")
    return out


def unpack(packed, cols, bits):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    rows = packed.shape[0]
    q = np.empty((rows, cols), np.int8)
    _chk(lib().orc_unpack(_p(packed), C.c_int64(rows), C.c_int64(cols), C.c_int(bits), _p(q)), "unpack")
    return q


def dequant(packed, scales, cols, bits, group):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint16)
    rows = packed.shape[0]
    w = np.empty((rows, cols), np.float32)
    _chk(lib().orc_dequant(_p(packed), _p(scales), C.c_int64(rows), C.c_int64(cols), C.c_int(bits),
                           C.c_int(group), _p(w)), "dequant")
    return w


def quantize_pack(w, bits, group):
    """Convenience: quantize then pack. Returns (packed uint8 [rows][cols*bits/8], scales uint16)."""
    q, s = quantize(w, bits, group)
    return pack(q, bits), s


def router_topk(x, Wr, bias, k, renorm, want_logits=False):
    """x [T][d] fp32, Wr [E][d] fp32 -> idx int32 [T][k], gate fp32 [T][k], probs fp32 [T][E]."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    Wr = np.ascontiguousarray(Wr, dtype=np.float32)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    T, d = x.shape
    E = Wr.shape[0]
    assert Wr.shape[1] == d
    idx = np.empty((T, k), np.int32)
    gate = np.empty((T, k), np.float32)
    probs = np.empty((T, E), np.float32)
    logits = np.empty((T, E), np.float64) if want_logits else None
    _chk(lib().orc_router_topk(_p(x), C.c_int32(T), C.c_int32(d), _p(Wr), _p(b), C.c_int32(E),
                               C.c_int32(k), C.c_int32(int(renorm)), _p(idx), _p(gate), _p(probs),
                               _p(logits)), "router_topk")
    if want_logits:
        return idx, gate, probs, logits
    return idx, gate, probs


class Expert:
    """Packed weights of one expert, host side. Keeps the numpy arrays alive."""

    def __init__(self, bits, q_in, s_in, q_out, s_out, q_gate=None, s_gate=None):
        self.bits = int(bits)
        self.q_in = np.ascontiguousarray(q_in, np.uint8)
        self.s_in = np.ascontiguousarray(s_in, np.uint16)
        self.q_out = np.ascontiguousarray(q_out, np.uint8)
        self.s_out = np.ascontiguousarray(s_out, np.uint16)
        self.q_gate = None if q_gate is None else np.ascontiguousarray(q_gate, np.uint8)
        self.s_gate = None if s_gate is None else np.ascontiguousarray(s_gate, np.uint16)

    def c_struct(self):
        return _Expert(self.bits, _p(self.q_in), _p(self.s_in), _p(self.q_gate), _p(self.s_gate),
                       _p(self.q_out), _p(self.s_out))


def expert_ffn(ex, d, f, g, act, x, want_h=False):
    """y_e [T][d] = W_out^ act(W_in^ x). act: 0 ReLU, 1 SwiGLU."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    T = x.shape[0]
    assert x.shape[1] == d
    y = np.empty((T, d), np.float32)
    h = np.empty((T, f), np.float32) if want_h else None
    st = ex.c_struct()
    _chk(lib().orc_expert_ffn(C.byref(st), C.c_int32(d), C.c_int32(f), C.c_int32(g), C.c_int32(act),
                              _p(x), C.c_int32(T), _p(y), _p(h)), "expert_ffn")
    return (y, h) if want_h else y


def layer_forward(experts, d, f, g, act, k, renorm, Wr, bias, x):
    """Whole MoE layer. Returns (y [T][d] fp32, idx [T][k] int32, gate [T][k] fp32)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    Wr = np.ascontiguousarray(Wr, dtype=np.float32)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    T = x.shape[0]
    E = len(experts)
    arr = (_Expert * E)(*[e.c_struct() for e in experts])
    y = np.empty((T, d), np.float32)
    idx = np.empty((T, k), np.int32)
    gate = np.empty((T, k), np.float32)
    _chk(lib().orc_layer_forward(arr, C.c_int32(E), C.c_int32(d), C.c_int32(f), C.c_int32(g),
                                 C.c_int32(act), C.c_int32(k), C.c_int32(int(renorm)), _p(Wr), _p(b),
                                 _p(x), C.c_int32(T), _p(y), _p(idx), _p(gate)), "layer_forward")
    return y, idx, gate


def layer_forward_routed(experts, d, f, g, act, k, x, idx, gate):
    """The layer for a routing that is already decided: idx [T][k] int32, gate [T][k] fp32. Returns y [T][d]."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    gate = np.ascontiguousarray(gate, dtype=np.float32)
    T = x.shape[0]
    E = len(experts)
    arr = (_Expert * E)(*[e.c_struct() for e in experts])
    y = np.empty((T, d), np.float32)
    _chk(lib().orc_layer_forward_routed(arr, C.c_int32(E), C.c_int32(d), C.c_int32(f), C.c_int32(g),
                                        C.c_int32(act), C.c_int32(k), _p(x), C.c_int32(T), _p(idx), _p(gate),
                                        _p(y)), "layer_forward_routed")
    return y
