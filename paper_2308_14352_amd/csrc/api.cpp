// Host side of the C ABI: argument validation, workspace carving, kernel dispatch.
// Every check runs before the first HIP call, so the error paths work on a host without a GPU.
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "moeq_internal.h"

using namespace moeq;

struct moeq_layer {
  LayerDims dims;
  const float* router_w;
  const float* router_bias;
  const DevExpert* table;          // device
  std::vector<int32_t> bits;       // host copy of the bitwidth table
  int32_t bits_mask;               // or of the bitwidths in the table (2 | 4 | 8)
  int32_t out_layout;              // layout of W_out (MOEQ_OUT_CANONICAL or MOEQ_OUT_COLUMNS)
  int32_t in_layout;               // layout of W_in / W_gate (MOEQ_IN_CANONICAL or MOEQ_IN_STREAM)
  FusedPlan plan;                  // split of the one-kernel path (out_layout == MOEQ_OUT_COLUMNS)
  // measurement aid (moe_layer_profile_kernel): events to record around one kernel of this layer's calls
  int32_t prof_which = 0;
  hipEvent_t prof_start = nullptr, prof_stop = nullptr;
};

namespace {

inline bool bits_ok(int32_t b) { return b == 2 || b == 4 || b == 8; }

inline bool group_ok(int32_t g, int32_t bits) {
  if (g <= 0 || g % 32) return false;
  if (bits == 2 && !(g == 32 || g % 64 == 0)) return false;
  return true;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Workspace carving. Both paths keep idx, gate and logits; the two-kernel path adds the chosen experts'
// records and h (fp32), the one-kernel path the partial output vectors.
struct WsLayout {
  size_t idx_off, gate_off, logits_off, sel_off, h_off, part_off, prefill_off, total;
};

// Calls with at least this many tokens run as grouped GEMMs on the matrix cores (when the shape allows);
// fewer tokens run the streaming decode kernels, token by token.
constexpr int64_t kPrefillMinTokens = 32;
// The one-kernel path takes the tokens of a call in launches of at most this many, so that the buffer of
// partial output vectors (tokens x slices x d_model floats) does not grow with the call.
constexpr int32_t kDecodeChunk = 32;
bool use_prefill(const moeq_layer* layer, int64_t T);

WsLayout ws_layout(const moeq_layer* layer, int64_t T) {
  const LayerDims& L = layer->dims;
  WsLayout w{};
  const size_t slots = (size_t)T * L.top_k;
  w.idx_off = 0;
  w.gate_off = align_up(slots * sizeof(int32_t), 256);
  w.logits_off = w.gate_off + align_up(slots * sizeof(float), 256);
  const size_t tail = w.logits_off + align_up((size_t)T * (size_t)L.n_experts * sizeof(float), 256);
  if (layer->out_layout == MOEQ_OUT_COLUMNS) {
    const size_t chunk = (size_t)(T < kDecodeChunk ? T : kDecodeChunk);
    const size_t part = align_up(chunk * (size_t)layer->plan.n_slices * (size_t)L.d_model * sizeof(float), 256);
    w.part_off = tail;
    w.prefill_off = tail;           // a call uses one of the two
    const size_t grouped = use_prefill(layer, T) ? prefill_ws(L, T).total : 0;
    w.total = tail + (part > grouped ? part : grouped);
  } else {
    w.sel_off = tail;
    w.h_off = w.sel_off + align_up(slots * sizeof(DevExpert), 256);
    w.total = w.h_off + align_up(slots * (size_t)L.d_ff * sizeof(float), 256);
    if (use_prefill(layer, T)) {      // moe_layer_forward takes the grouped path; the single-expert call keeps h
      w.prefill_off = w.total;
      w.total = w.prefill_off + prefill_ws(L, T).total;
    }
  }
  return w;
}

bool use_prefill(const moeq_layer* layer, int64_t T) {
  static const bool off = [] { const char* v = std::getenv("MOEQ_NO_PREFILL"); return v && v[0] == '1'; }();
  // (the grouped GEMMs read W_in / W_gate in the canonical and in the stream layout, W_out in both of its layouts)
  return !off && T >= kPrefillMinTokens && prefill_supported(layer->dims);
}

// Routers with at most this many experts are evaluated inside the one-kernel path by every workgroup;
// larger ones by the router kernel first (MOEQ_INLINE_ROUTER overrides, for experiments).
int inline_router_max() {
  static const int v = [] {
    const char* e = std::getenv("MOEQ_INLINE_ROUTER");
    const int want = e ? std::atoi(e) : 16, cap = fused_inline_router_max();
    return want < cap ? want : cap;
  }();
  return v;
}

inline moeq_status dev(hipError_t e) { return e == hipSuccess ? MOEQ_OK : MOEQ_EDEVICE; }

// Scratch of moe_layer_forward_static: device memory that belongs to the library's code object, so that the
// entry point needs neither a workspace from its caller nor an allocation. Every GPU the library runs on
// holds its own copy of the array at its own address; the name below is only a host-side handle, the
// address on the current device comes from hipGetSymbolAddress (once per device) and is what the kernels
// and every other use get.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
void* g_scratch_ptr[kMaxDevices] = {};

// Address of `scratch` on the current device (nullptr when HIP refuses), looked up on first use per device.
void* static_scratch() {
  int devid = -1;
  if (hipGetDevice(&devid) != hipSuccess || devid < 0 || devid >= kMaxDevices) return nullptr;
  void* p = __atomic_load_n(&g_scratch_ptr[devid], __ATOMIC_ACQUIRE);
  if (p) return p;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
    (void)hipGetLastError();
    return nullptr;
  }
  __atomic_store_n(&g_scratch_ptr[devid], p, __ATOMIC_RELEASE);   // racing threads store the same value
  return p;
}

// Measurement aid (moe_layer_profile_kernel): records the layer's two events around one kernel launch.
struct ScopedEvents {
  const moeq_layer* l; bool on; hipStream_t st;
  ScopedEvents(const moeq_layer* layer, int32_t which, hipStream_t s)
      : l(layer), on(layer->prof_which == which && layer->prof_start && layer->prof_stop), st(s) {
    if (on) (void)hipEventRecord(l->prof_start, st);
  }
  ~ScopedEvents() { if (on) (void)hipEventRecord(l->prof_stop, st); }
};

}  // namespace

extern "C" {

const char* moe_status_str(moeq_status st) {
  switch (st) {
    case MOEQ_OK: return "ok";
    case MOEQ_EINVAL: return "invalid argument";
    case MOEQ_EUNSUPPORTED: return "unsupported configuration";
    case MOEQ_EWORKSPACE: return "workspace missing or too small";
    case MOEQ_EDEVICE: return "HIP call failed";
  }
  return "unknown status";
}

size_t moe_layer_table_bytes(int32_t n_experts) {
  return n_experts > 0 ? (size_t)n_experts * sizeof(DevExpert) : 0;
}

size_t moe_packed_bytes(int64_t rows, int64_t cols, int32_t bits, int32_t group, size_t* scale_bytes_opt) {
  if (scale_bytes_opt) *scale_bytes_opt = 0;
  if (rows <= 0 || cols <= 0 || !bits_ok(bits) || group <= 0 || cols % group || (cols * bits) % 8) return 0;
  if (scale_bytes_opt) *scale_bytes_opt = (size_t)rows * (size_t)(cols / group) * 2;
  return (size_t)rows * (size_t)(cols * bits / 8);
}

moeq_status moe_layer_create(const moeq_layer_desc* desc, void* table_dev, size_t table_bytes,
                             moeq_layer** out) {
  if (out) *out = nullptr;
  if (!desc || !out || !table_dev || !desc->experts || !desc->router_w) return MOEQ_EINVAL;
  const int32_t d = desc->d_model, f = desc->d_ff, E = desc->n_experts, k = desc->top_k;
  // group_in / group_out, each falling back to the shorthand `group`
  const int32_t g = desc->group_in > 0 ? desc->group_in : desc->group;
  const int32_t go = desc->group_out > 0 ? desc->group_out : desc->group;
  if (desc->group_in < 0 || desc->group_out < 0) return MOEQ_EINVAL;
  if (d <= 0 || f <= 0 || E <= 0 || k <= 0 || g <= 0 || go <= 0) return MOEQ_EINVAL;
  if (k > E) return MOEQ_EINVAL;
  if (desc->act != MOEQ_ACT_RELU && desc->act != MOEQ_ACT_SWIGLU) return MOEQ_EINVAL;
  if (desc->x_dtype != MOEQ_F32 && desc->x_dtype != MOEQ_BF16) return MOEQ_EINVAL;
  if (desc->out_layout != MOEQ_OUT_CANONICAL && desc->out_layout != MOEQ_OUT_COLUMNS) return MOEQ_EINVAL;
  if (desc->in_layout != MOEQ_IN_CANONICAL && desc->in_layout != MOEQ_IN_STREAM) return MOEQ_EINVAL;
  const bool stream = desc->in_layout == MOEQ_IN_STREAM;
  if (stream && desc->out_layout != MOEQ_OUT_COLUMNS) return MOEQ_EINVAL;
  if (d % g || f % go) return MOEQ_EINVAL;
  if (((uintptr_t)table_dev & 15u) || table_bytes < moe_layer_table_bytes(E)) return MOEQ_EINVAL;
  if (k > 8 || E > 1024 || d > 32768 || f > 32768 || d % 8 || f % 8) return MOEQ_EUNSUPPORTED;
  const LayerDims dims{d, f, E, k, g, desc->act, desc->renorm ? 1 : 0, desc->x_dtype == MOEQ_BF16 ? 1 : 0, go};
  FusedPlan plan{0, 0, 0, 0};
  if (stream) {
    if (!stream_supported(dims)) return MOEQ_EUNSUPPORTED;
    plan = FusedPlan{64, stream_slices(dims), 512, 0};
  } else if (desc->out_layout == MOEQ_OUT_COLUMNS) {
    plan = plan_fused(dims);
    if (!plan.SW) return MOEQ_EUNSUPPORTED;
  }
  std::vector<DevExpert> tab((size_t)E);
  std::memset(tab.data(), 0, tab.size() * sizeof(DevExpert));
  std::vector<int32_t> bits((size_t)E);
  for (int32_t e = 0; e < E; ++e) {
    const moeq_expert& x = desc->experts[e];
    if (!bits_ok(x.bits)) return MOEQ_EINVAL;
    if (!x.q_in || (!stream && !x.s_in) || !x.q_out || !x.s_out) return MOEQ_EINVAL;
    if (desc->act == MOEQ_ACT_SWIGLU && (!x.q_gate || (!stream && !x.s_gate))) return MOEQ_EINVAL;
    if (((int64_t)d * x.bits) % 128 || ((int64_t)f * x.bits) % 128) return MOEQ_EINVAL;
    if (!group_ok(g, x.bits) || !group_ok(go, x.bits)) return MOEQ_EUNSUPPORTED;
    const uintptr_t align_or = (uintptr_t)x.q_in | (uintptr_t)x.q_out | (uintptr_t)x.q_gate;
    if (align_or & 15u) return MOEQ_EINVAL;  // 16-byte loads on the code rows
    if (((uintptr_t)x.s_in | (uintptr_t)x.s_out | (uintptr_t)x.s_gate) & 1u) return MOEQ_EINVAL;
    DevExpert& t = tab[(size_t)e];
    std::memset(&t, 0, sizeof(t));
    t.q_in = (const uint8_t*)x.q_in;     t.s_in = (const uint16_t*)x.s_in;
    t.q_gate = (const uint8_t*)x.q_gate; t.s_gate = (const uint16_t*)x.s_gate;
    t.q_out = (const uint8_t*)x.q_out;   t.s_out = (const uint16_t*)x.s_out;
    t.bits = x.bits;
    bits[(size_t)e] = x.bits;
  }
  moeq_layer* L = new (std::nothrow) moeq_layer();
  if (!L) return MOEQ_EDEVICE;
  L->dims = dims;
  L->router_w = desc->router_w;
  L->router_bias = desc->router_bias;
  L->table = (const DevExpert*)table_dev;
  L->bits_mask = 0;
  for (int32_t b : bits) L->bits_mask |= b;
  L->bits = std::move(bits);
  L->out_layout = desc->out_layout;
  L->in_layout = desc->in_layout;
  L->plan = plan;
  if (hipMemcpy(table_dev, tab.data(), tab.size() * sizeof(DevExpert), hipMemcpyHostToDevice) != hipSuccess ||
      init_attrs_decode_fused() != hipSuccess || init_attrs_ffn_decode() != hipSuccess ||
      init_attrs_prefill() != hipSuccess) {
    (void)hipGetLastError();
    delete L;
    return MOEQ_EDEVICE;
  }
  (void)static_scratch();   // set-up time is the place for the symbol lookup; the entry point repeats it if needed
  *out = L;
  return MOEQ_OK;
}

void moe_layer_destroy(moeq_layer* layer) { delete layer; }

size_t moe_workspace_bytes(const moeq_layer* layer, int32_t max_tokens) {
  if (!layer || max_tokens <= 0) return 0;
  return ws_layout(layer, max_tokens).total;
}

moeq_status moe_router_topk(const moeq_layer* layer, const void* x, int32_t n_tokens, int32_t* topk_idx,
                            float* topk_gate, float* probs_opt, void* ws, size_t ws_bytes, void* stream) {
  if (!layer || n_tokens < 0) return MOEQ_EINVAL;
  if (n_tokens == 0) return MOEQ_OK;
  if (!x || !topk_idx || !topk_gate || ((uintptr_t)x & 15u)) return MOEQ_EINVAL;
  if (n_tokens > 65535) return MOEQ_EUNSUPPORTED;
  const WsLayout w = ws_layout(layer, n_tokens);
  if (!ws || ws_bytes < w.total) return MOEQ_EWORKSPACE;
  if ((uintptr_t)ws & 255u) return MOEQ_EINVAL;
  float* logits = (float*)((char*)ws + w.logits_off);
  hipStream_t st = (hipStream_t)stream;
  if (launch_router_logits(layer->dims, layer->router_w, layer->router_bias, x, n_tokens, logits, st) != hipSuccess)
    return MOEQ_EDEVICE;
  return dev(launch_topk(layer->dims, logits, n_tokens, topk_idx, topk_gate, probs_opt, st));
}

moeq_status moe_expert_ffn_q(const moeq_layer* layer, int32_t expert, const void* x, int32_t n_tokens,
                             const float* gate_opt, int32_t accumulate, float* y, void* ws, size_t ws_bytes,
                             void* stream) {
  if (!layer || n_tokens < 0) return MOEQ_EINVAL;
  if (expert < 0 || expert >= layer->dims.n_experts) return MOEQ_EINVAL;
  if (n_tokens == 0) return MOEQ_OK;
  if (!x || !y || ((uintptr_t)x & 15u) || ((uintptr_t)y & 3u)) return MOEQ_EINVAL;
  if (n_tokens > 65535) return MOEQ_EUNSUPPORTED;
  const WsLayout w = ws_layout(layer, n_tokens);
  if (!ws || ws_bytes < w.total) return MOEQ_EWORKSPACE;
  if ((uintptr_t)ws & 255u) return MOEQ_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  if (layer->out_layout == MOEQ_OUT_COLUMNS) {
    float* part = (float*)((char*)ws + w.part_off);
    const size_t x_row = (size_t)layer->dims.d_model * (layer->dims.x_bf16 ? 2 : 4);
    for (int32_t t0 = 0; t0 < n_tokens; t0 += kDecodeChunk) {
      const int32_t n = n_tokens - t0 < kDecodeChunk ? n_tokens - t0 : kDecodeChunk;
      const hipError_t le = layer->in_layout == MOEQ_IN_STREAM
          ? launch_moe_stream(layer->dims, layer->table, nullptr, nullptr, nullptr, expert,
                              gate_opt ? gate_opt + t0 : nullptr, nullptr, nullptr, layer->bits_mask,
                              (const char*)x + (size_t)t0 * x_row, n, part, nullptr, nullptr, st)
          : launch_moe_decode(layer->dims, layer->plan, layer->table, nullptr, nullptr, nullptr, expert,
                              gate_opt ? gate_opt + t0 : nullptr, nullptr, nullptr, layer->bits[(size_t)expert],
                              (const char*)x + (size_t)t0 * x_row, n, part, nullptr, nullptr, st);
      if (le != hipSuccess) return MOEQ_EDEVICE;
      if (launch_reduce_partials(part, layer->plan.n_slices, layer->dims.d_model, n, accumulate ? 1 : 0,
                                 y + (size_t)t0 * layer->dims.d_model, st) != hipSuccess)
        return MOEQ_EDEVICE;
    }
    return MOEQ_OK;
  }
  float* h = (float*)((char*)ws + w.h_off);
  hipError_t e = launch_ffn_in(layer->dims, layer->table, nullptr, nullptr, nullptr, nullptr, expert, x, n_tokens, h,
                               st);
  if (e != hipSuccess) return MOEQ_EDEVICE;
  return dev(launch_ffn_out(layer->dims, layer->table, nullptr, gate_opt, expert, accumulate ? 1 : 0, h, n_tokens, y,
                            st));
}

// The layer with the routing computed here (given_idx == nullptr) or supplied by the caller.
static moeq_status layer_forward_impl(const moeq_layer* layer, const void* x, int32_t n_tokens, float* y,
                                      int32_t* topk_idx_opt, float* topk_gate_opt, const int32_t* given_idx,
                                      const float* given_gate, void* ws, size_t ws_bytes, void* stream) {
  if (!layer || n_tokens < 0) return MOEQ_EINVAL;
  if (n_tokens == 0) return MOEQ_OK;
  if (!x || !y || ((uintptr_t)x & 15u) || ((uintptr_t)y & 3u)) return MOEQ_EINVAL;
  if ((int64_t)n_tokens * layer->dims.top_k > 65535) return MOEQ_EUNSUPPORTED;
  const LayerDims& L = layer->dims;
  const WsLayout w = ws_layout(layer, n_tokens);
  if (!ws || ws_bytes < w.total) return MOEQ_EWORKSPACE;
  if ((uintptr_t)ws & 255u) return MOEQ_EINVAL;
  const bool given = given_idx != nullptr;
  int32_t* idx = topk_idx_opt ? topk_idx_opt : (int32_t*)((char*)ws + w.idx_off);
  float* gate = topk_gate_opt ? topk_gate_opt : (float*)((char*)ws + w.gate_off);
  hipStream_t st = (hipStream_t)stream;
  float* logits = (float*)((char*)ws + w.logits_off);
  if (given && launch_take_routing(given_idx, given_gate, n_tokens * L.top_k, L.n_experts, idx, gate, st) != hipSuccess)
    return MOEQ_EDEVICE;
  if (use_prefill(layer, n_tokens)) {
    // batched path: router kernels, then the pairs grouped by expert through two quantized GEMMs
    if (!given) {
      if (launch_router_logits(L, layer->router_w, layer->router_bias, x, n_tokens, logits, st) != hipSuccess)
        return MOEQ_EDEVICE;
      if (launch_topk(L, logits, n_tokens, idx, gate, nullptr, st) != hipSuccess) return MOEQ_EDEVICE;
    }
    const PrefillWs pw = prefill_ws(L, n_tokens);
    return dev(launch_prefill(L, layer->table, x, n_tokens, idx, gate, (char*)ws + w.prefill_off, pw, y,
                              layer->out_layout == MOEQ_OUT_COLUMNS, layer->in_layout == MOEQ_IN_STREAM, st));
  }
  if (layer->out_layout == MOEQ_OUT_COLUMNS) {
    // one streaming kernel for the whole layer, then the ordered sum of its partial output vectors
    const bool stream = layer->in_layout == MOEQ_IN_STREAM;
    const float* lg = nullptr;
    if (!given && L.n_experts > (stream ? (inline_router_max() < stream_inline_router_max() ? inline_router_max()
                                                                                             : stream_inline_router_max())
                                        : inline_router_max())) {
      if (launch_router_logits(L, layer->router_w, layer->router_bias, x, n_tokens, logits, st) != hipSuccess)
        return MOEQ_EDEVICE;
      lg = logits;
    }
    float* part = (float*)((char*)ws + w.part_off);
    const size_t x_row = (size_t)L.d_model * (L.x_bf16 ? 2 : 4);
    for (int32_t t0 = 0; t0 < n_tokens; t0 += kDecodeChunk) {
      const int32_t n = n_tokens - t0 < kDecodeChunk ? n_tokens - t0 : kDecodeChunk;
      const size_t s0 = (size_t)t0 * (size_t)L.top_k;
      // the profiling events, when asked for, bracket the kernel's own execution (not its dispatch)
      const bool prof = t0 == 0 && layer->prof_which == MOEQ_KERNEL_FUSED && layer->prof_start && layer->prof_stop;
      const hipError_t le = stream
          ? launch_moe_stream(L, layer->table, layer->router_w, layer->router_bias,
                              lg ? lg + (size_t)t0 * L.n_experts : nullptr, -1, nullptr, given ? idx + s0 : nullptr,
                              given ? gate + s0 : nullptr, layer->bits_mask, (const char*)x + (size_t)t0 * x_row, n,
                              part, given ? nullptr : idx + s0, given ? nullptr : gate + s0, st,
                              prof ? layer->prof_start : nullptr, prof ? layer->prof_stop : nullptr)
          : launch_moe_decode(L, layer->plan, layer->table, layer->router_w, layer->router_bias,
                              lg ? lg + (size_t)t0 * L.n_experts : nullptr, -1, nullptr, given ? idx + s0 : nullptr,
                              given ? gate + s0 : nullptr, layer->bits_mask, (const char*)x + (size_t)t0 * x_row, n,
                              part, given ? nullptr : idx + s0, given ? nullptr : gate + s0, st,
                              prof ? layer->prof_start : nullptr, prof ? layer->prof_stop : nullptr);
      if (le != hipSuccess) return MOEQ_EDEVICE;
      if (launch_reduce_partials(part, layer->plan.n_slices, L.d_model, n, 0, y + (size_t)t0 * L.d_model, st) !=
          hipSuccess)
        return MOEQ_EDEVICE;
    }
    return MOEQ_OK;
  }
  float* h = (float*)((char*)ws + w.h_off);
  DevExpert* sel_tab = (DevExpert*)((char*)ws + w.sel_off);
  if (!given && launch_router_logits(L, layer->router_w, layer->router_bias, x, n_tokens, logits, st) != hipSuccess)
    return MOEQ_EDEVICE;
  {
    ScopedEvents ev(layer, MOEQ_KERNEL_FFN_IN, st);
    if (launch_ffn_in(L, layer->table, given ? nullptr : logits, idx, gate, sel_tab, -1, x, n_tokens, h, st) !=
        hipSuccess)
      return MOEQ_EDEVICE;
  }
  ScopedEvents ev(layer, MOEQ_KERNEL_FFN_OUT, st);
  return dev(launch_ffn_out(L, layer->table, sel_tab, gate, -1, 0, h, n_tokens, y, st));
}

moeq_status moe_layer_forward(const moeq_layer* layer, const void* x, int32_t n_tokens, float* y,
                              int32_t* topk_idx_opt, float* topk_gate_opt, void* ws, size_t ws_bytes,
                              void* stream) {
  return layer_forward_impl(layer, x, n_tokens, y, topk_idx_opt, topk_gate_opt, nullptr, nullptr, ws, ws_bytes,
                            stream);
}

moeq_status moe_layer_forward_routed(const moeq_layer* layer, const void* x, int32_t n_tokens,
                                     const int32_t* topk_idx, const float* topk_gate, float* y, void* ws,
                                     size_t ws_bytes, void* stream) {
  if (n_tokens > 0 && (!topk_idx || !topk_gate)) return MOEQ_EINVAL;
  if (((uintptr_t)topk_idx | (uintptr_t)topk_gate) & 3u) return MOEQ_EINVAL;
  return layer_forward_impl(layer, x, n_tokens, y, nullptr, nullptr, topk_idx, topk_gate, ws, ws_bytes, stream);
}

size_t moe_static_scratch_bytes(void) { return kStaticScratchBytes; }

moeq_status moe_layer_forward_static(const moeq_layer* layer, const void* x, int32_t n_tokens, float* y,
                                     int32_t* topk_idx_opt, float* topk_gate_opt, void* stream) {
  if (!layer || n_tokens < 0) return MOEQ_EINVAL;
  if (n_tokens == 0) return MOEQ_OK;
  if (ws_layout(layer, n_tokens).total > kStaticScratchBytes) return MOEQ_EWORKSPACE;   // beyond the fixed scratch
  void* ws = static_scratch();
  if (!ws) return MOEQ_EDEVICE;
  return layer_forward_impl(layer, x, n_tokens, y, topk_idx_opt, topk_gate_opt, nullptr, nullptr, ws,
                            kStaticScratchBytes, stream);
}

int32_t moe_layer_path(const moeq_layer* layer, int32_t n_tokens) {
  if (!layer || n_tokens < 1) return -1;
  if (use_prefill(layer, n_tokens)) return MOEQ_PATH_GROUPED_GEMM;
  if (layer->in_layout == MOEQ_IN_STREAM) return MOEQ_PATH_STREAM;
  if (layer->out_layout == MOEQ_OUT_COLUMNS) return layer->plan.mx ? MOEQ_PATH_ONE_KERNEL_MX : MOEQ_PATH_ONE_KERNEL;
  return MOEQ_PATH_TWO_KERNELS;
}

moeq_status moe_layer_profile_kernel(moeq_layer* layer, int32_t which, void* start_event, void* stop_event) {
  if (!layer || which < 0 || which > MOEQ_KERNEL_FUSED) return MOEQ_EINVAL;
  if (which != 0 && (!start_event || !stop_event)) return MOEQ_EINVAL;
  layer->prof_which = which;
  layer->prof_start = which ? (hipEvent_t)start_event : nullptr;
  layer->prof_stop = which ? (hipEvent_t)stop_event : nullptr;
  return MOEQ_OK;
}

moeq_status moe_quantize_pack(const float* w, int64_t rows, int64_t cols, int32_t bits, int32_t group,
                              void* q_out, void* s_out, void* stream) {
  if (!w || !q_out || !s_out || rows < 0 || cols <= 0) return MOEQ_EINVAL;
  if (!bits_ok(bits) || group <= 0 || cols % group || group % 4 || (cols * bits) % 128) return MOEQ_EINVAL;
  if (((uintptr_t)w & 15u) || ((uintptr_t)q_out & 3u) || ((uintptr_t)s_out & 1u)) return MOEQ_EINVAL;
  if (rows == 0) return MOEQ_OK;
  if (rows * (cols / group) > (int64_t)1 << 40) return MOEQ_EUNSUPPORTED;
  return dev(launch_quantize_pack(w, rows, cols, bits, group, (uint8_t*)q_out, (uint16_t*)s_out,
                                  (hipStream_t)stream));
}

// Canonical <-> dword-column-major: a transposition of the 32-bit words of the code rows and of the scales.
static moeq_status relayout_out(const void* q_src, const void* s_src, int64_t rows, int64_t cols, int32_t bits,
                                int32_t group, void* q_dst, void* s_dst, bool to_columns, void* stream) {
  if (!q_src || !s_src || !q_dst || !s_dst || rows <= 0 || cols <= 0) return MOEQ_EINVAL;
  if (!bits_ok(bits) || group <= 0 || cols % group || (cols * bits) % 32 || rows % 4) return MOEQ_EINVAL;
  if (q_src == q_dst || s_src == s_dst) return MOEQ_EINVAL;
  if (((uintptr_t)q_src | (uintptr_t)q_dst) & 15u) return MOEQ_EINVAL;
  if (((uintptr_t)s_src | (uintptr_t)s_dst) & 1u) return MOEQ_EINVAL;
  const int64_t words = cols * bits / 32, groups = cols / group;
  hipStream_t st = (hipStream_t)stream;
  hipError_t e = to_columns ? launch_transpose(q_src, rows, words, 4, q_dst, st)
                            : launch_transpose(q_src, words, rows, 4, q_dst, st);
  if (e != hipSuccess) return MOEQ_EDEVICE;
  e = to_columns ? launch_transpose(s_src, rows, groups, 2, s_dst, st)
                 : launch_transpose(s_src, groups, rows, 2, s_dst, st);
  return dev(e);
}

moeq_status moe_prepare_out(const void* q, const void* s, int64_t rows, int64_t cols, int32_t bits, int32_t group,
                            void* q_cols, void* s_cols, void* stream) {
  return relayout_out(q, s, rows, cols, bits, group, q_cols, s_cols, true, stream);
}

moeq_status moe_unprepare_out(const void* q_cols, const void* s_cols, int64_t rows, int64_t cols, int32_t bits,
                              int32_t group, void* q, void* s, void* stream) {
  return relayout_out(q_cols, s_cols, rows, cols, bits, group, q, s, false, stream);
}

size_t moe_stream_bytes(int64_t rows, int64_t cols, int32_t bits, int32_t group) {
  if (rows <= 0 || !bits_ok(bits) || cols != 4096 || group != 128 || rows % 8) return 0;
  return (size_t)rows * ((size_t)cols * (size_t)bits / 8 + (size_t)(cols / group) * 2);
}

static moeq_status relayout_in(const void* q, const void* s, int64_t rows, int64_t cols, int32_t bits, int32_t group,
                               const void* stream_buf, bool to_stream, void* stream) {
  if (!q || !s || !stream_buf || rows <= 0 || cols <= 0 || !bits_ok(bits) || group <= 0) return MOEQ_EINVAL;
  if (!moe_stream_bytes(rows, cols, bits, group)) return MOEQ_EUNSUPPORTED;
  if (((uintptr_t)q | (uintptr_t)stream_buf) & 15u) return MOEQ_EINVAL;
  if ((uintptr_t)s & 1u) return MOEQ_EINVAL;
  if (q == stream_buf || s == stream_buf) return MOEQ_EINVAL;
  return dev(launch_relayout_in(q, s, rows, bits, (void*)stream_buf, to_stream, (hipStream_t)stream));
}

moeq_status moe_prepare_in(const void* q, const void* s, int64_t rows, int64_t cols, int32_t bits, int32_t group,
                           void* stream_buf, void* stream) {
  return relayout_in(q, s, rows, cols, bits, group, stream_buf, true, stream);
}

moeq_status moe_unprepare_in(const void* stream_buf, int64_t rows, int64_t cols, int32_t bits, int32_t group, void* q,
                             void* s, void* stream) {
  return relayout_in(q, s, rows, cols, bits, group, stream_buf, false, stream);
}

moeq_status moe_unpack_codes(const void* q, int64_t rows, int64_t cols, int32_t bits, int8_t* codes_out,
                             void* stream) {
  if (!q || !codes_out || rows < 0 || cols <= 0) return MOEQ_EINVAL;
  if (!bits_ok(bits) || (cols * bits) % 8) return MOEQ_EINVAL;
  if (rows == 0) return MOEQ_OK;
  return dev(launch_unpack_codes((const uint8_t*)q, rows, cols, bits, codes_out, (hipStream_t)stream));
}

moeq_status moe_dequantize(const void* q, const void* s, int64_t rows, int64_t cols, int32_t bits,
                           int32_t group, float* w_out, void* stream) {
  if (!q || !s || !w_out || rows < 0 || cols <= 0) return MOEQ_EINVAL;
  if (!bits_ok(bits) || group <= 0 || cols % group || (cols * bits) % 8) return MOEQ_EINVAL;
  if (rows == 0) return MOEQ_OK;
  return dev(launch_dequantize((const uint8_t*)q, (const uint16_t*)s, rows, cols, bits, group, w_out,
                               (hipStream_t)stream));
}

}  // extern "C"
