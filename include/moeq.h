/* moeq.h - C ABI of the MI355X (gfx950) mixed-bitwidth MoE layer forward.
 *
 * The path (EdgeMoE, arxiv 2308.14352): a router sends every token to its top-K experts
 * (Section 1, Section 2.1); each expert is an independent FFN whose weights are stored at a
 * per-expert bitwidth (INT2/INT4/INT8) by linear, scale-only quantization with float16
 * scales and are decompressed by the mirror map before use (Section 3.2); the K expert
 * outputs are combined with the router's gate weights. Here the decompression is fused into
 * the FFN kernels: packed codes are streamed from HBM once and never materialised as floats.
 *
 * Conventions
 *   - "dev" pointers are device (HBM) pointers owned by the caller; "host" pointers are host
 *     memory. The library borrows them for the duration of a call (for moe_layer_create: for
 *     the lifetime of the layer handle) and never frees them.
 *   - The library allocates no device memory. Scratch comes in through `ws` (size from
 *     moe_workspace_bytes); the per-layer expert table lives in a caller-provided device
 *     buffer (size from moe_layer_table_bytes).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream). Compute entry
 *     points only enqueue work and return; they never synchronise. Results are valid once
 *     the stream reaches the end of the enqueued work. The top-k indices stay on the device
 *     between the router and the expert kernels.
 *   - Every entry point validates its arguments before the first HIP call and reports
 *     problems as a status code; nothing throws, nothing aborts.
 *   - Calls that share a workspace, and all compute calls on one layer handle, must be ordered on
 *     one stream (or otherwise serialised).
 *   - Range of the hidden states (Section 4.1, "Baselines": the decompressed weights are used in FP32
 *     arithmetic, so the path's range is fp32's). The kernels multiply in binary16 x integer code and
 *     accumulate in fp32; before that, every token's hidden state - and every intermediate vector h -
 *     is multiplied by a power of two of its own that brings its largest magnitude to about 2^14, and
 *     the result is scaled back in fp32. Accuracy therefore does not depend on the scale of a token as
 *     long as its largest magnitude lies in [2^-96, 2^124] and the exact results fit fp32; elements more
 *     than 2^29 times smaller than the token's largest one lose relative precision. A token that holds
 *     a NaN or an infinity gets the experts 0 .. top_k-1, NaN gates and a non-finite output; other tokens
 *     of the call are not affected and no invalid address is formed.
 *   - Token limits: moe_router_topk and moe_expert_ffn_q take at most 65535 tokens per call,
 *     moe_layer_forward(_routed) at most 65535 / top_k (else MOEQ_EUNSUPPORTED).
 *
 * Packed weight format (the boundary format; "canonical")
 *   A matrix W[rows][cols] (row = output channel, cols = input dimension) at b bits with group
 *   size g (g consecutive input indices of one row share a scale; g = cols is the paper's
 *   per-channel case):
 *     codes : rows * cols*b/8 bytes, row-major. Element i of a row is the unsigned field
 *             u = q + 2^(b-1) (q in [-(2^(b-1)-1), 2^(b-1)-1]) at bits [i*b mod 8, +b) of byte
 *             floor(i*b/8). cols*b must be a multiple of 128 (16-byte rows).
 *     scales: rows * cols/g IEEE binary16 values, row-major. W^[o][i] = scale[o][i/g] * q[o][i].
 *             Every entry point uses a scale as the binary16 value it is, sign bit included
 *             (moe_quantize_pack writes none below zero).
 *
 * Dword-column-major layout of W_out (optional, made from the canonical one by moe_prepare_out)
 *   The same bits, transposed in units of 32-bit words: codes[w][r] = word w (little-endian) of canonical
 *   row r, for w < cols*b/32; scales[g][r] = canonical scale[r][g]. rows must be a multiple of 4. With
 *   W_out in this layout a layer's decode calls run as one streaming kernel per call (each workgroup
 *   takes a slice of d_ff through both FFN matrices) plus a small ordered reduction.
 *
 * Row-block stream layout of W_in / W_gate (optional, made by moe_prepare_in; cols = 4096, g = 128)
 *   Codes and scales of a matrix in ONE buffer of rows * (cols*b/8 + cols/g*2) bytes, cut into blocks of
 *   RB = 16/b rows (8, 4, 2 rows at 2, 4, 8 bits). A block is 8 tiles of 1 KB followed by 64 * RB bytes of
 *   scales. Tile t holds part t % (b/2) of row t / (b/2) of the block: its 16-byte piece l (l = 0..63) is the
 *   canonical bytes [16 * ((b/2) * l + part), +16) of that row, so that piece l of every tile of a row lies in
 *   the columns [64 l, 64 l + 64). The scale bytes of piece l are the RB/2 binary16 values
 *   scale[row0 + (l & 1) * RB/2 + i][l >> 1], i < RB/2. A pure permutation of the canonical bytes: a wavefront
 *   of the decode kernel reads a block front to back, its lanes always own the same columns, and the scales
 *   arrive in the same memory pages as the codes they belong to. With W_in / W_gate in this layout and W_out
 *   in the dword-column-major one a decode call runs as one streaming kernel on integer dot products.
 */
#ifndef MOEQ_H
#define MOEQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MOEQ_OK = 0,
  MOEQ_EINVAL = 1,       /* malformed argument (null pointer, bad shape, bad bitwidth ...)   */
  MOEQ_EUNSUPPORTED = 2, /* well-formed but outside what the kernels cover                    */
  MOEQ_EWORKSPACE = 3,   /* ws is NULL or smaller than moe_workspace_bytes() for this call    */
  MOEQ_EDEVICE = 4       /* a HIP call failed (no device, launch error); see hipGetLastError  */
} moeq_status;

typedef enum { MOEQ_ACT_RELU = 0, MOEQ_ACT_SWIGLU = 1 } moeq_act;
typedef enum { MOEQ_F32 = 0, MOEQ_BF16 = 1 } moeq_dtype;
typedef enum { MOEQ_OUT_CANONICAL = 0, MOEQ_OUT_COLUMNS = 1 } moeq_out_layout;
typedef enum { MOEQ_IN_CANONICAL = 0, MOEQ_IN_STREAM = 1 } moeq_in_layout;

/* One expert's packed weights: dev pointers, read-only, in the canonical format.
 * ReLU   (Switch-style): h = relu(W_in x),            y = W_out h;   q_gate/s_gate = NULL
 * SwiGLU (Mixtral-style): h = silu(W_in x) * (W_gate x), y = W_out h
 * W_in, W_gate: [d_ff][d_model]; W_out: [d_model][d_ff] (q_out/s_out in the layout the layer's
 * out_layout names). `bits` is this expert's entry of the per-expert bitwidth table (Section 3.2,
 * "Selecting expert-wise bitwidths").                                                        */
typedef struct moeq_expert {
  int32_t bits; /* 2, 4 or 8 */
  const void *q_in, *s_in;
  const void *q_gate, *s_gate;
  const void *q_out, *s_out;
} moeq_expert;

/* Description of one MoE layer (host struct). */
typedef struct moeq_layer_desc {
  int32_t d_model, d_ff, n_experts, top_k, group;
  int32_t act;              /* moeq_act                                                        */
  int32_t renorm;           /* 0: gate = softmax probability of the chosen expert;
                               1: gates divided by the sum of the K chosen probabilities      */
  int32_t x_dtype;          /* moeq_dtype of the hidden states; outputs are always fp32        */
  const float *router_w;    /* dev [n_experts][d_model] fp32                                   */
  const float *router_bias; /* dev [n_experts] fp32 or NULL                                    */
  const moeq_expert *experts; /* host array [n_experts] of dev pointers                        */
  int32_t out_layout;       /* moeq_out_layout of every expert's q_out / s_out                 */
  int32_t in_layout;        /* moeq_in_layout of every expert's W_in / W_gate. MOEQ_IN_STREAM: q_in and
                               q_gate point to stream buffers (moe_prepare_in), s_in / s_gate are not
                               read (may be NULL); needs out_layout = MOEQ_OUT_COLUMNS                */
  int32_t group_in;         /* scale group of W_in / W_gate along d_model; 0: `group`                  */
  int32_t group_out;        /* scale group of W_out along d_ff; 0: `group`. group_in = d_model with
                               group_out = d_ff is Section 3.2's scheme: one float16 scale per channel
                               of each matrix                                                          */
} moeq_layer_desc;

typedef struct moeq_layer moeq_layer; /* opaque, host-side handle */

/* ---- set-up (not on the hot path) -------------------------------------------------------- */

/* Bytes of device memory the expert table of a layer with n_experts experts needs (one record per expert:
 * its bitwidth - the per-expert bitwidth table of Section 3.2 - and the addresses of its packed matrices). */
size_t moe_layer_table_bytes(int32_t n_experts);

/* Validates `desc`, copies the expert table into `table_dev` (synchronous copy) and returns a
 * handle. `table_dev` (dev, >= moe_layer_table_bytes(n_experts), 16-byte aligned) and every
 * pointer in `desc` must stay valid until moe_layer_destroy. All per-device set-up happens here (the kernels'
 * shared-memory ceilings, the scratch lookup of moe_layer_forward_static), with the device current on which
 * the layer will run: every compute call on the layer, the first one included, only enqueues kernels and may
 * be recorded into a HIP graph. Limits: d_model a multiple of the scale group of W_in / W_gate, d_ff of the
 * scale group of W_out (`group` for both unless group_in / group_out say otherwise); each group a multiple of
 * 32 (a multiple of 64 or exactly 32 for 2-bit experts);
 * d_model*bits and d_ff*bits multiples of 128 for every expert; 1 <= top_k <= min(8, n_experts);
 * n_experts <= 1024; d_model, d_ff <= 32768. With out_layout = MOEQ_OUT_COLUMNS also: group and d_ff
 * multiples of 16, d_model <= 8192 (else MOEQ_EUNSUPPORTED). With in_layout = MOEQ_IN_STREAM also: out_layout =
 * MOEQ_OUT_COLUMNS, d_model = 4096, group = 128, d_ff a multiple of 64 (else MOEQ_EUNSUPPORTED); calls on such a
 * layer run the streaming kernel below 32 tokens and the grouped GEMMs from 32 tokens on where their shape rules
 * hold (d_ff a multiple of 256 with d_ff / 128 a multiple of 4; else the streaming kernel, 32 tokens per launch):
 * one copy of the weights serves decode and prefill.
 * Errors: MOEQ_EINVAL, MOEQ_EUNSUPPORTED, MOEQ_EDEVICE (copy failed). */
moeq_status moe_layer_create(const moeq_layer_desc *desc, void *table_dev, size_t table_bytes,
                             moeq_layer **out);
void moe_layer_destroy(moeq_layer *layer);

/* Workspace bytes needed by any compute call on `layer` with up to max_tokens tokens (the routing, the router
 * logits, and what the path of Section 2.1 needs between its kernels: h, or the partial output vectors, or
 * the grouped path's staging). Host-only arithmetic. */
size_t moe_workspace_bytes(const moeq_layer *layer, int32_t max_tokens);

/* Which kernels moe_layer_forward / moe_layer_forward_routed run for a call with n_tokens tokens on
 * `layer` (the choice depends on the layer's shape and W_out layout and on the token count only, so a
 * caller or a test can know it beforehand). The three paths compute the same layer (Section 3.1, the
 * MoE layer: router, top-k experts, gate-weighted sum). Returns -1 for a null layer or n_tokens < 1.
 * Host-only. */
#define MOEQ_PATH_TWO_KERNELS 0    /* canonical layout: router, phase-1 and phase-2 GEMV kernels          */
#define MOEQ_PATH_ONE_KERNEL 1     /* columns layout: one streaming kernel per 32 tokens, vector instr.   */
#define MOEQ_PATH_ONE_KERNEL_MX 2  /* columns layout: the same with matrix-core instructions              */
#define MOEQ_PATH_GROUPED_GEMM 3   /* 32 tokens or more, either layout: pairs grouped by expert, GEMMs   */
#define MOEQ_PATH_STREAM 4         /* stream + columns layouts: one streaming kernel on integer dot products */
int32_t moe_layer_path(const moeq_layer *layer, int32_t n_tokens);

/* Codes bytes of a packed [rows][cols] matrix; *scale_bytes_opt receives the bytes of its scales.
 * Returns 0 when the arguments are not a valid packed shape. Host-only arithmetic. */
size_t moe_packed_bytes(int64_t rows, int64_t cols, int32_t bits, int32_t group,
                        size_t *scale_bytes_opt);

/* ---- the path ---------------------------------------------------------------------------- */

/* Router: logits = router_w x (+ bias), p = softmax(logits), the top_k largest (ties to the lowest
 * expert index, results in descending gate order), gates per `renorm` (Section 1; Section 2.1).
 * x: dev [n_tokens][d_model] in the layer's x_dtype. topk_idx: dev [n_tokens][top_k] int32.
 * topk_gate: dev [n_tokens][top_k] fp32. probs_opt: dev [n_tokens][n_experts] fp32 or NULL.
 * ws holds the logits between the two kernels. n_tokens == 0 is a no-op. */
moeq_status moe_router_topk(const moeq_layer *layer, const void *x, int32_t n_tokens,
                            int32_t *topk_idx, float *topk_gate, float *probs_opt, void *ws,
                            size_t ws_bytes, void *stream);

/* One expert's dequantize-fused FFN on n_tokens tokens (Section 3.2: decompress, then use):
 * y[t] (+)= gate[t] * W_out^ act(W_in^ x[t]). gate_opt: dev [n_tokens] fp32 or NULL (= 1).
 * accumulate != 0 adds into y, else overwrites. y: dev [n_tokens][d_model] fp32. */
moeq_status moe_expert_ffn_q(const moeq_layer *layer, int32_t expert, const void *x,
                             int32_t n_tokens, const float *gate_opt, int32_t accumulate,
                             float *y, void *ws, size_t ws_bytes, void *stream);

/* The whole layer (Section 1; Section 2.1, the sparse MoE layer; Section 3.2 for the experts' weights): router,
 * top-k, the chosen experts' FFNs on their decompressed weights, gate-weighted combine:
 * y[t] = sum_j gate[t][j] * FFN_{idx[t][j]}(x[t]). topk_idx_opt / topk_gate_opt (dev, may be NULL)
 * receive the routing decision. */
moeq_status moe_layer_forward(const moeq_layer *layer, const void *x, int32_t n_tokens, float *y,
                              int32_t *topk_idx_opt, float *topk_gate_opt, void *ws,
                              size_t ws_bytes, void *stream);

/* moe_layer_forward for callers that cannot allocate and have no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc. Same computation, same kernels, same
 * results; the scratch that `ws` brings in elsewhere is a fixed array inside the library's device code
 * (moe_static_scratch_bytes() bytes, 8 MiB, held on every GPU the library runs on until the process ends).
 * The call allocates nothing and frees nothing. Returns MOEQ_EWORKSPACE when
 * moe_workspace_bytes(layer, n_tokens) exceeds that size (e.g. more than 2 tokens per call on a
 * Mixtral-sized layer in the columns layout: split the call), MOEQ_EDEVICE when the array's address cannot be
 * obtained. All calls on one GPU share the one array, which keeps the previous call's contents (nothing in
 * it needs clearing: every piece is written before it is read): calls that overlap on one GPU - two streams,
 * two threads - race; order them on one stream. x, y, topk_*_opt, stream as for moe_layer_forward. */
size_t moe_static_scratch_bytes(void);
moeq_status moe_layer_forward_static(const moeq_layer *layer, const void *x, int32_t n_tokens, float *y,
                                     int32_t *topk_idx_opt, float *topk_gate_opt, void *stream);

/* The layer with the routing GIVEN by the caller instead of computed by the router: static-routing
 * layers (Section 3.1, "Applicability": hash layers, expert-choice layers - the experts of a token
 * follow from the input tokens, not from its hidden state):
 * y[t] = sum_j topk_gate[t][j] * FFN_{topk_idx[t][j]}(x[t]).
 * topk_idx: dev [n_tokens][top_k] int32; topk_gate: dev [n_tokens][top_k] fp32; both read-only and
 * 4-byte aligned. The layer's router weights are not read. A pair whose expert index is outside
 * [0, n_experts) contributes nothing (the arrays live on the device, so no error can be raised for
 * it); the same expert may appear more than once for a token. Workspace, limits, alignment and
 * errors as for moe_layer_forward. */
moeq_status moe_layer_forward_routed(const moeq_layer *layer, const void *x, int32_t n_tokens,
                                     const int32_t *topk_idx, const float *topk_gate, float *y,
                                     void *ws, size_t ws_bytes, void *stream);

/* ---- compression primitives (offline side of the path, Section 3.2) ---------------------- */

/* Quantize and pack on the device: w dev [rows][cols] fp32 -> codes (q_out) and fp16 scales (s_out)
 * in the canonical format. scale = fp16(absmax/qmax) (nearest even, moved one fp16 step up if the
 * largest element would otherwise clamp), q = rint(w/scale) with fp32 division. */
moeq_status moe_quantize_pack(const float *w, int64_t rows, int64_t cols, int32_t bits,
                              int32_t group, void *q_out, void *s_out, void *stream);

/* Packed codes -> signed codes, one int8 per weight (dev [rows][cols]); for bit-exact checks. */
moeq_status moe_unpack_codes(const void *q, int64_t rows, int64_t cols, int32_t bits,
                             int8_t *codes_out, void *stream);

/* Stand-alone decompression (the paper's own step): packed -> fp32 dev [rows][cols]. */
moeq_status moe_dequantize(const void *q, const void *s, int64_t rows, int64_t cols, int32_t bits,
                           int32_t group, float *w_out, void *stream);

/* W_out of one expert, canonical -> dword-column-major (see the top of this file) and back: device to
 * device, out of place (source and destination must not overlap). rows = d_model (a multiple of 4), cols =
 * d_ff; q buffers are rows*cols*bits/8 bytes (16-byte aligned), s buffers rows*cols/group binary16 values.
 * Both are pure permutations: moe_unprepare_out(moe_prepare_out(q, s)) returns q and s bit for bit. */
moeq_status moe_prepare_out(const void *q, const void *s, int64_t rows, int64_t cols, int32_t bits,
                            int32_t group, void *q_cols, void *s_cols, void *stream);
moeq_status moe_unprepare_out(const void *q_cols, const void *s_cols, int64_t rows, int64_t cols,
                              int32_t bits, int32_t group, void *q, void *s, void *stream);

/* W_in or W_gate of one expert, canonical -> row-block stream layout (see the top of this file) and back:
 * device to device, out of place. rows = d_ff (a multiple of 8), cols = d_model = 4096, group = 128 (else
 * MOEQ_EUNSUPPORTED); `stream_buf` holds moe_stream_bytes(rows, cols, bits, group) bytes, 16-byte aligned.
 * Both are pure permutations: moe_unprepare_in(moe_prepare_in(q, s)) returns q and s bit for bit.
 * moe_stream_bytes returns 0 for a shape the layout does not cover. */
size_t moe_stream_bytes(int64_t rows, int64_t cols, int32_t bits, int32_t group);
moeq_status moe_prepare_in(const void *q, const void *s, int64_t rows, int64_t cols, int32_t bits,
                           int32_t group, void *stream_buf, void *stream);
moeq_status moe_unprepare_in(const void *stream_buf, int64_t rows, int64_t cols, int32_t bits,
                             int32_t group, void *q, void *s, void *stream);

/* Measurement aid, per layer. While `which` names a kernel, every moe_layer_forward call on THIS
 * layer records start_event just before and stop_event just after that kernel on the call's stream
 * (hipEvent_t handles created by the caller with timing enabled, which must outlive the setting),
 * so a benchmark can time the dominant kernel alone. For MOEQ_KERNEL_FUSED the two events are
 * attached to the kernel launch itself and receive the begin and end of the kernel's execution
 * (what a kernel trace reports), without the dispatch before it. which = 0 turns it off (the
 * default). The setting is part of the layer handle: change it only while no other thread is
 * inside a call on the same layer, and turn it off before a call is captured into a graph. */
#define MOEQ_KERNEL_FFN_IN 1  /* phase 1: top-k + W_in / W_gate GEMVs (Section 3.2, dequantize-fused) */
#define MOEQ_KERNEL_FFN_OUT 2 /* phase 2: W_out GEMVs + gate-weighted combine                          */
#define MOEQ_KERNEL_FUSED 3   /* the one-kernel paths: router, top-k and both phases of every d_ff slice */
moeq_status moe_layer_profile_kernel(moeq_layer *layer, int32_t which, void *start_event, void *stop_event);

const char *moe_status_str(moeq_status st);

#ifdef __cplusplus
}
#endif
#endif /* MOEQ_H */
