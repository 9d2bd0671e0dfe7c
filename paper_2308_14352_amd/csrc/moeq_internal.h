// Internal declarations shared by the host API and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moeq.h"

namespace moeq {

// Device-resident view of one expert (the expert table is an array of these).
struct alignas(64) DevExpert {
  const uint8_t* q_in;
  const uint16_t* s_in;
  const uint8_t* q_gate;
  const uint16_t* s_gate;
  const uint8_t* q_out;
  const uint16_t* s_out;
  int32_t bits;
  int32_t pad_[3];
};
static_assert(sizeof(DevExpert) == 64, "expert table entry is 64 bytes");

// group: scale group of W_in / W_gate (along d_model); group_out: of W_out (along d_ff).
struct LayerDims {
  int32_t d_model, d_ff, n_experts, top_k, group, act, renorm, x_bf16, group_out;
};

// Launchers (defined in the .hip files). All enqueue on `st` and return the launch status.

// logits[t][e] = router_w[e] . x[t] (+ bias[e])
hipError_t launch_router_logits(const LayerDims& L, const float* router_w, const float* router_bias,
                                const void* x, int32_t T, float* logits, hipStream_t st);
// softmax + top-k of every token from its logits
hipError_t launch_topk(const LayerDims& L, const float* logits, int32_t T, int32_t* idx, float* gate,
                       float* probs, hipStream_t st);

// idx[i], gate[i] = the caller's routing of pair i, or (0, 0.0f) when its expert index is not in [0, E).
hipError_t launch_take_routing(const int32_t* idx_in, const float* gate_in, int32_t n, int32_t E, int32_t* idx,
                               float* gate, hipStream_t st);

// Phase 1 of the expert FFN: h[slot][f] = act(W_in x [, W_gate x]), stored as fp32.
// fixed_expert >= 0: every token uses that expert (slot == token). Otherwise each workgroup derives
// the token's top-k from `logits`, the routing is written to idx_out/gate_out, the chosen experts'
// table records to sel_tab[slot], and slot = token * top_k + j; with logits == nullptr the routing is
// READ from idx_out/gate_out instead (caller-supplied routing, already validated).
hipError_t launch_ffn_in(const LayerDims& L, const DevExpert* table, const float* logits,
                         int32_t* idx_out, float* gate_out, DevExpert* sel_tab, int32_t fixed_expert,
                         const void* x, int32_t T, float* h, hipStream_t st);

// Phase 2 + combine: y[t] (+)= sum_j gate * W_out h[slot].
hipError_t launch_ffn_out(const LayerDims& L, const DevExpert* table, const DevExpert* sel_tab,
                          const float* gate, int32_t fixed_expert, int32_t accumulate,
                          const float* h, int32_t T, float* y, hipStream_t st);

// ---- one-kernel decode path (W_out in the dword-column-major layout) -------------------------------
// Split of a layer for the fused kernel: slices of SW columns of d_ff, one workgroup of `threads` per
// (slice, token). SW == 0: the shape does not fit the scheme. mx != 0: the matrix-core variant of the kernel
// runs.
struct FusedPlan { int32_t SW, n_slices, threads, mx; };
FusedPlan plan_fused(const LayerDims& L);

// Router (inline when logits == nullptr: at most fused_inline_router_max() experts) + top-k + both FFN
// phases of every (slice, token); writes the partial outputs part[T][n_slices][d]. fixed_expert >= 0: that
// expert for every token, gate_in[T] or 1. route_idx / route_gate non-null: the routing is given ([T][k],
// validated), no router runs. bits_mask: bitwidths the call can meet (2 | 4 | 8 or-ed). ev_start / ev_stop
// (both or none): events that receive the begin and end of the kernel's own execution.
int fused_inline_router_max();
hipError_t launch_moe_decode(const LayerDims& L, const FusedPlan& plan, const DevExpert* table,
                             const float* router_w, const float* router_bias, const float* logits,
                             int32_t fixed_expert, const float* gate_in, const int32_t* route_idx,
                             const float* route_gate, int32_t bits_mask, const void* x, int32_t T, float* part,
                             int32_t* idx_out, float* gate_out, hipStream_t st, hipEvent_t ev_start = nullptr,
                             hipEvent_t ev_stop = nullptr);
// y[t] (+)= sum_s part[t][s], fixed order.
hipError_t launch_reduce_partials(const float* part, int n_slices, int d, int32_t T, int accumulate,
                                  float* y, hipStream_t st);
// out[c][r] = in[r][c], elements of 2 or 4 bytes.
hipError_t launch_transpose(const void* in, int64_t rows, int64_t cols, int elem_bytes, void* out,
                            hipStream_t st);

// Per-kernel attributes (the dynamic LDS ceiling) for the current device, set at layer creation so that no
// compute call has to: a fresh layer's first call can then be recorded into a graph like any other.
hipError_t init_attrs_decode_fused();
hipError_t init_attrs_ffn_decode();
hipError_t init_attrs_prefill();

// ---- one-kernel decode path on integer dot products (W_in / W_gate in the row-block stream layout, W_out in
// the dword-column-major layout; d_model 4096, scale groups of 128 columns). Arguments as launch_moe_decode;
// the partial outputs are part[T][stream_slices(L)][d].
bool stream_supported(const LayerDims& L);
int stream_inline_router_max();
int stream_slices(const LayerDims& L);
hipError_t launch_moe_stream(const LayerDims& L, const DevExpert* table, const float* router_w,
                             const float* router_bias, const float* logits, int32_t fixed_expert,
                             const float* gate_in, const int32_t* route_idx, const float* route_gate,
                             int32_t bits_mask, const void* x, int32_t T, float* part, int32_t* idx_out,
                             float* gate_out, hipStream_t st, hipEvent_t ev_start = nullptr,
                             hipEvent_t ev_stop = nullptr);
// canonical (q, s) <-> stream buffer of a [rows][4096] matrix, groups of 128 columns
hipError_t launch_relayout_in(const void* q, const void* s, int64_t rows, int bits, void* stream_buf, bool to_stream,
                              hipStream_t st);

// ---- batched (prefill) path: pairs grouped by expert, two quantized GEMMs on the matrix cores ----------
// Byte offsets of the pieces of the prefill workspace (all 256-byte aligned).
struct PrefillWs {
  size_t poff, boff, nblk, blocks, gpair, ginv, gexp, xa, ha, hf, ypair, total;
  size_t max_blocks;
};
bool prefill_supported(const LayerDims& L);
PrefillWs prefill_ws(const LayerDims& L, int64_t T);
// idx / gate: the routing of the T tokens ([T][k], already computed). out_columns / in_stream: the layouts of W_out and
// of W_in / W_gate.
hipError_t launch_prefill(const LayerDims& L, const DevExpert* table, const void* x, int32_t T,
                          const int32_t* idx, const float* gate, char* ws, const PrefillWs& w, float* y,
                          bool out_columns, bool in_stream, hipStream_t st);

hipError_t launch_quantize_pack(const float* w, int64_t rows, int64_t cols, int bits, int group,
                                uint8_t* q, uint16_t* s, hipStream_t st);
hipError_t launch_unpack_codes(const uint8_t* q, int64_t rows, int64_t cols, int bits, int8_t* codes,
                               hipStream_t st);
hipError_t launch_dequantize(const uint8_t* q, const uint16_t* s, int64_t rows, int64_t cols, int bits,
                             int group, float* w, hipStream_t st);

}  // namespace moeq
