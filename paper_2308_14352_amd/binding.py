"""Thin ctypes binding of libmoeq.so: same names as include/moeq.h, argument marshalling only.

torch is used for device memory and streams; every step of the path runs in the library's HIP
kernels. There is no fallback: if the library is missing the import of a compute call raises.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# MOEQ_LIB lets a developer point the binding at another build of the same library.
LIB_PATH = os.environ.get("MOEQ_LIB") or os.path.join(_HERE, "libmoeq.so")

MOEQ_OK, MOEQ_EINVAL, MOEQ_EUNSUPPORTED, MOEQ_EWORKSPACE, MOEQ_EDEVICE = range(5)
MOEQ_ACT_RELU, MOEQ_ACT_SWIGLU = 0, 1
MOEQ_F32, MOEQ_BF16 = 0, 1
MOEQ_OUT_CANONICAL, MOEQ_OUT_COLUMNS = 0, 1
MOEQ_IN_CANONICAL, MOEQ_IN_STREAM = 0, 1


class MoeqError(RuntimeError):
    def __init__(self, status, what):
        self.status = int(status)
        super().__init__(f"{what}: {status_str(status)} (status {int(status)})")


class moeq_expert(C.Structure):
    _fields_ = [("bits", C.c_int32),
                ("q_in", C.c_void_p), ("s_in", C.c_void_p),
                ("q_gate", C.c_void_p), ("s_gate", C.c_void_p),
                ("q_out", C.c_void_p), ("s_out", C.c_void_p)]


class moeq_layer_desc(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("d_ff", C.c_int32), ("n_experts", C.c_int32),
                ("top_k", C.c_int32), ("group", C.c_int32), ("act", C.c_int32),
                ("renorm", C.c_int32), ("x_dtype", C.c_int32),
                ("router_w", C.c_void_p), ("router_bias", C.c_void_p),
                ("experts", C.POINTER(moeq_expert)), ("out_layout", C.c_int32), ("in_layout", C.c_int32),
                ("group_in", C.c_int32), ("group_out", C.c_int32)]


_lib = None


def lib():
    """Loads libmoeq.so (building it first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    L.moe_status_str.restype = C.c_char_p
    L.moe_status_str.argtypes = [C.c_int]
    L.moe_layer_table_bytes.restype = sz
    L.moe_layer_table_bytes.argtypes = [i32]
    L.moe_packed_bytes.restype = sz
    L.moe_packed_bytes.argtypes = [i64, i64, i32, i32, C.POINTER(sz)]
    L.moe_layer_create.restype = C.c_int
    L.moe_layer_create.argtypes = [C.POINTER(moeq_layer_desc), vp, sz, C.POINTER(vp)]
    L.moe_layer_destroy.restype = None
    L.moe_layer_destroy.argtypes = [vp]
    L.moe_layer_profile_kernel.restype = C.c_int
    L.moe_layer_profile_kernel.argtypes = [vp, i32, vp, vp]
    L.moe_workspace_bytes.restype = sz
    L.moe_workspace_bytes.argtypes = [vp, i32]
    L.moe_layer_path.restype = i32
    L.moe_layer_path.argtypes = [vp, i32]
    L.moe_router_topk.restype = C.c_int
    L.moe_router_topk.argtypes = [vp, vp, i32, vp, vp, vp, vp, sz, vp]
    L.moe_expert_ffn_q.restype = C.c_int
    L.moe_expert_ffn_q.argtypes = [vp, i32, vp, i32, vp, i32, vp, vp, sz, vp]
    L.moe_layer_forward.restype = C.c_int
    L.moe_layer_forward.argtypes = [vp, vp, i32, vp, vp, vp, vp, sz, vp]
    L.moe_static_scratch_bytes.restype = sz
    L.moe_static_scratch_bytes.argtypes = []
    L.moe_layer_forward_static.restype = C.c_int
    L.moe_layer_forward_static.argtypes = [vp, vp, i32, vp, vp, vp, vp]
    L.moe_layer_forward_routed.restype = C.c_int
    L.moe_layer_forward_routed.argtypes = [vp, vp, i32, vp, vp, vp, vp, sz, vp]
    L.moe_quantize_pack.restype = C.c_int
    L.moe_quantize_pack.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp]
    L.moe_unpack_codes.restype = C.c_int
    L.moe_unpack_codes.argtypes = [vp, i64, i64, i32, vp, vp]
    L.moe_dequantize.restype = C.c_int
    L.moe_dequantize.argtypes = [vp, vp, i64, i64, i32, i32, vp, vp]
    L.moe_stream_bytes.restype = sz
    L.moe_stream_bytes.argtypes = [i64, i64, i32, i32]
    L.moe_prepare_in.restype = C.c_int
    L.moe_prepare_in.argtypes = [vp, vp, i64, i64, i32, i32, vp, vp]
    L.moe_unprepare_in.restype = C.c_int
    L.moe_unprepare_in.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp]
    for fn in (L.moe_prepare_out, L.moe_unprepare_out):
        fn.restype = C.c_int
        fn.argtypes = [vp, vp, i64, i64, i32, i32, vp, vp, vp]
    _lib = L
    return L


EXPORTS = ["moe_status_str", "moe_layer_profile_kernel", "moe_layer_table_bytes", "moe_packed_bytes", "moe_layer_create",
           "moe_layer_destroy", "moe_workspace_bytes", "moe_layer_path", "moe_router_topk", "moe_expert_ffn_q",
           "moe_layer_forward", "moe_layer_forward_routed", "moe_layer_forward_static", "moe_static_scratch_bytes", "moe_quantize_pack", "moe_unpack_codes", "moe_dequantize", "moe_prepare_out",
           "moe_unprepare_out", "moe_prepare_in", "moe_unprepare_in", "moe_stream_bytes"]


def status_str(st):
    return lib().moe_status_str(int(st)).decode()


def _check(st, what):
    if st != MOEQ_OK:
        raise MoeqError(st, what)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


MOEQ_KERNEL_FFN_IN, MOEQ_KERNEL_FFN_OUT, MOEQ_KERNEL_FUSED = 1, 2, 3
MOEQ_PATH_TWO_KERNELS, MOEQ_PATH_ONE_KERNEL, MOEQ_PATH_ONE_KERNEL_MX, MOEQ_PATH_GROUPED_GEMM, MOEQ_PATH_STREAM = 0, 1, 2, 3, 4


def moe_layer_profile_kernel(layer, which, start_event=None, stop_event=None):
    """which: 0 (off) or one of the MOEQ_KERNEL_* ids; events are raw hipEvent_t handles (ints)."""
    _check(lib().moe_layer_profile_kernel(layer.handle, int(which), C.c_void_p(start_event), C.c_void_p(stop_event)),
           "moe_layer_profile_kernel")


def moe_packed_bytes(rows, cols, bits, group):
    """(code bytes, scale bytes) of a packed [rows][cols] matrix; (0, 0) for an invalid shape."""
    sb = C.c_size_t(0)
    qb = lib().moe_packed_bytes(rows, cols, bits, group, C.byref(sb))
    return int(qb), int(sb.value)


def moe_layer_table_bytes(n_experts):
    return int(lib().moe_layer_table_bytes(n_experts))


def moe_quantize_pack(w, bits, group, stream=None):
    """w: device fp32 [rows][cols] -> (codes uint8 [rows][cols*bits/8], scales int16-typed fp16 bits [rows][cols/group])."""
    assert w.is_cuda and w.dtype == torch.float32 and w.is_contiguous() and w.dim() == 2
    rows, cols = w.shape
    qb, sb = moe_packed_bytes(rows, cols, bits, group)
    if qb == 0:
        raise MoeqError(MOEQ_EINVAL, "moe_quantize_pack")
    q = torch.empty((rows, cols * bits // 8), dtype=torch.uint8, device=w.device)
    s = torch.empty((rows, cols // group), dtype=torch.float16, device=w.device)
    _check(lib().moe_quantize_pack(_ptr(w), rows, cols, bits, group, _ptr(q), _ptr(s), _stream(stream)),
           "moe_quantize_pack")
    return q, s


def moe_unpack_codes(q, cols, bits, stream=None):
    rows = q.shape[0]
    out = torch.empty((rows, cols), dtype=torch.int8, device=q.device)
    _check(lib().moe_unpack_codes(_ptr(q), rows, cols, bits, _ptr(out), _stream(stream)), "moe_unpack_codes")
    return out


def moe_dequantize(q, s, cols, bits, group, stream=None):
    rows = q.shape[0]
    out = torch.empty((rows, cols), dtype=torch.float32, device=q.device)
    _check(lib().moe_dequantize(_ptr(q), _ptr(s), rows, cols, bits, group, _ptr(out), _stream(stream)),
           "moe_dequantize")
    return out


def moe_prepare_out(q, s, cols, bits, group, stream=None):
    """Canonical W_out (codes [rows][cols*bits/8], scales [rows][cols/group]) -> dword-column-major copies
    (codes uint8 [cols*bits/32][rows*4], scales [cols/group][rows])."""
    rows = q.shape[0]
    qc = torch.empty((cols * bits // 32, rows * 4), dtype=torch.uint8, device=q.device)
    sc = torch.empty((cols // group, rows), dtype=torch.float16, device=q.device)
    _check(lib().moe_prepare_out(_ptr(q), _ptr(s), rows, cols, bits, group, _ptr(qc), _ptr(sc), _stream(stream)),
           "moe_prepare_out")
    return qc, sc


def moe_unprepare_out(qc, sc, cols, bits, group, stream=None):
    """Inverse of moe_prepare_out."""
    rows = sc.shape[1]
    q = torch.empty((rows, cols * bits // 8), dtype=torch.uint8, device=qc.device)
    s = torch.empty((rows, cols // group), dtype=torch.float16, device=qc.device)
    _check(lib().moe_unprepare_out(_ptr(qc), _ptr(sc), rows, cols, bits, group, _ptr(q), _ptr(s), _stream(stream)),
           "moe_unprepare_out")
    return q, s


def moe_stream_bytes(rows, cols, bits, group):
    return int(lib().moe_stream_bytes(rows, cols, bits, group))


def moe_prepare_in(q, s, cols, bits, group, stream=None):
    """Canonical W_in / W_gate (codes [rows][cols*bits/8], scales [rows][cols/group]) -> one stream buffer (uint8)."""
    rows = q.shape[0]
    n = moe_stream_bytes(rows, cols, bits, group)
    if n == 0:
        raise MoeqError(MOEQ_EUNSUPPORTED, "moe_prepare_in")
    buf = torch.empty(n, dtype=torch.uint8, device=q.device)
    _check(lib().moe_prepare_in(_ptr(q), _ptr(s), rows, cols, bits, group, _ptr(buf), _stream(stream)), "moe_prepare_in")
    return buf


def moe_unprepare_in(buf, rows, cols, bits, group, stream=None):
    """Inverse of moe_prepare_in: (codes, scales) in the canonical format."""
    q = torch.empty((rows, cols * bits // 8), dtype=torch.uint8, device=buf.device)
    s = torch.empty((rows, cols // group), dtype=torch.float16, device=buf.device)
    _check(lib().moe_unprepare_in(_ptr(buf), rows, cols, bits, group, _ptr(q), _ptr(s), _stream(stream)),
           "moe_unprepare_in")
    return q, s


class PackedExpert:
    """Device tensors of one expert in the boundary format (keeps them alive). q_out/s_out are in the
    layout the owning Layer is created with."""

    def __init__(self, bits, q_in, s_in, q_out, s_out, q_gate=None, s_gate=None):
        self.bits = int(bits)
        self.q_in, self.s_in, self.q_out, self.s_out = q_in, s_in, q_out, s_out
        self.q_gate, self.s_gate = q_gate, s_gate

    def with_out_columns(self, d_ff, group):
        """A copy of this expert (canonical W_out) whose W_out is in the dword-column-major layout."""
        qc, sc = moe_prepare_out(self.q_out, self.s_out, d_ff, self.bits, group)
        return PackedExpert(self.bits, self.q_in, self.s_in, qc, sc, self.q_gate, self.s_gate)

    def with_stream_layout(self, d_model, d_ff, group):
        """A copy of this expert (canonical) for a MOEQ_IN_STREAM layer: W_in / W_gate as stream buffers (their
        scales inside), W_out in the dword-column-major layout."""
        qc, sc = moe_prepare_out(self.q_out, self.s_out, d_ff, self.bits, group)
        b_in = moe_prepare_in(self.q_in, self.s_in, d_model, self.bits, group)
        b_gate = None if self.q_gate is None else moe_prepare_in(self.q_gate, self.s_gate, d_model, self.bits, group)
        return PackedExpert(self.bits, b_in, None, qc, sc, b_gate, None)

    def nbytes(self):
        ts = [self.q_in, self.s_in, self.q_out, self.s_out, self.q_gate, self.s_gate]
        return sum(t.numel() * t.element_size() for t in ts if t is not None)

    def c_struct(self):
        return moeq_expert(self.bits, _ptr(self.q_in), _ptr(self.s_in), _ptr(self.q_gate), _ptr(self.s_gate),
                           _ptr(self.q_out), _ptr(self.s_out))


class Layer:
    """Owner of a moeq_layer handle and of the device tensors it borrows."""

    def __init__(self, d_model, d_ff, top_k, group, act, renorm, x_dtype, router_w, router_bias, experts,
                 out_layout=MOEQ_OUT_CANONICAL, in_layout=MOEQ_IN_CANONICAL, group_in=0, group_out=0):
        self.out_layout = out_layout
        self.in_layout = in_layout
        self.group_in, self.group_out = group_in or group, group_out or group
        self.d_model, self.d_ff, self.top_k, self.group = d_model, d_ff, top_k, group
        self.n_experts = len(experts)
        self.experts = list(experts)
        self.router_w, self.router_bias = router_w, router_bias
        self.x_dtype = x_dtype
        dev = router_w.device
        self._table = torch.empty(max(moe_layer_table_bytes(self.n_experts), 16), dtype=torch.uint8, device=dev)
        arr = (moeq_expert * self.n_experts)(*[e.c_struct() for e in self.experts])
        desc = moeq_layer_desc(d_model, d_ff, self.n_experts, top_k, group, act, int(bool(renorm)), x_dtype,
                               _ptr(router_w), _ptr(router_bias), arr, out_layout, in_layout, group_in, group_out)
        h = C.c_void_p()
        _check(lib().moe_layer_create(C.byref(desc), _ptr(self._table), self._table.numel(), C.byref(h)),
               "moe_layer_create")
        self._h = h
        self._ws = None

    def __del__(self):
        h = getattr(self, "_h", None)
        if h and callable(lib):          # at interpreter shutdown the module's names may already be gone
            lib().moe_layer_destroy(h)
            self._h = None

    @property
    def handle(self):
        return self._h

    def workspace_bytes(self, max_tokens):
        return int(lib().moe_workspace_bytes(self._h, max_tokens))

    def path(self, n_tokens):
        """MOEQ_PATH_* constant: the kernels a layer call with n_tokens tokens runs."""
        return int(lib().moe_layer_path(self._h, n_tokens))

    def workspace(self, n_tokens):
        need = self.workspace_bytes(n_tokens)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.router_w.device)
        return self._ws


def moe_router_topk(layer, x, want_probs=False, ws=None, stream=None):
    T = x.shape[0]
    dev = x.device
    if ws is None:
        ws = layer.workspace(T)
    idx = torch.empty((T, layer.top_k), dtype=torch.int32, device=dev)
    gate = torch.empty((T, layer.top_k), dtype=torch.float32, device=dev)
    probs = torch.empty((T, layer.n_experts), dtype=torch.float32, device=dev) if want_probs else None
    _check(lib().moe_router_topk(layer.handle, _ptr(x), T, _ptr(idx), _ptr(gate), _ptr(probs), _ptr(ws), ws.numel(),
                                 _stream(stream)), "moe_router_topk")
    return (idx, gate, probs) if want_probs else (idx, gate)


def moe_expert_ffn_q(layer, expert, x, gate=None, y=None, accumulate=False, ws=None, stream=None):
    T = x.shape[0]
    if y is None:
        y = torch.empty((T, layer.d_model), dtype=torch.float32, device=x.device)
    if ws is None:
        ws = layer.workspace(T)
    _check(lib().moe_expert_ffn_q(layer.handle, expert, _ptr(x), T, _ptr(gate), int(bool(accumulate)), _ptr(y),
                                  _ptr(ws), ws.numel(), _stream(stream)), "moe_expert_ffn_q")
    return y


def moe_layer_forward(layer, x, y=None, want_routing=False, ws=None, stream=None):
    T = x.shape[0]
    dev = x.device
    if y is None:
        y = torch.empty((T, layer.d_model), dtype=torch.float32, device=dev)
    idx = gate = None
    if want_routing:
        idx = torch.empty((T, layer.top_k), dtype=torch.int32, device=dev)
        gate = torch.empty((T, layer.top_k), dtype=torch.float32, device=dev)
    if ws is None:
        ws = layer.workspace(T)
    _check(lib().moe_layer_forward(layer.handle, _ptr(x), T, _ptr(y), _ptr(idx), _ptr(gate), _ptr(ws), ws.numel(),
                                   _stream(stream)), "moe_layer_forward")
    return (y, idx, gate) if want_routing else y


def moe_static_scratch_bytes():
    return int(lib().moe_static_scratch_bytes())


def moe_layer_forward_static(layer, x, y=None, want_routing=False, stream=None):
    """moe_layer_forward without a workspace argument (the library's fixed scratch array is used)."""
    T = x.shape[0]
    dev = x.device
    if y is None:
        y = torch.empty((T, layer.d_model), dtype=torch.float32, device=dev)
    idx = gate = None
    if want_routing:
        idx = torch.empty((T, layer.top_k), dtype=torch.int32, device=dev)
        gate = torch.empty((T, layer.top_k), dtype=torch.float32, device=dev)
    _check(lib().moe_layer_forward_static(layer.handle, _ptr(x), T, _ptr(y), _ptr(idx), _ptr(gate), _stream(stream)),
           "moe_layer_forward_static")
    return (y, idx, gate) if want_routing else y


def moe_layer_forward_routed(layer, x, idx, gate, y=None, ws=None, stream=None):
    """The layer with the routing given by the caller: idx [T][top_k] int32, gate [T][top_k] fp32 (device)."""
    T = x.shape[0]
    if y is None:
        y = torch.empty((T, layer.d_model), dtype=torch.float32, device=x.device)
    if ws is None:
        ws = layer.workspace(T)
    _check(lib().moe_layer_forward_routed(layer.handle, _ptr(x), T, _ptr(idx), _ptr(gate), _ptr(y), _ptr(ws),
                                          ws.numel(), _stream(stream)), "moe_layer_forward_routed")
    return y
