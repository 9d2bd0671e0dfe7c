// Dequantize-fused expert FFN for decode (one to a few tokens): bandwidth-bound GEMVs that stream the
// packed INT2/INT4/INT8 rows of the activated experts with 128-bit loads, unpack the codes in
// registers and accumulate in fp32 (Section 3.2: the weights are decompressed by the mirror of the
// linear quantization before use; here that mirror map is applied on the fly and the fp32 copy of
// the expert is never written).
//
// The streaming core lives in decode_core.h.
#include "decode_core.h"

namespace moeq {
namespace {

__global__ __launch_bounds__(64) void k_topk(LayerDims L, const float* __restrict__ logits, int32_t* __restrict__ idx,
                                             float* __restrict__ gate, float* __restrict__ probs) {
  const int t = blockIdx.x;
  topk_from_logits(logits + (size_t)t * L.n_experts, L.n_experts, L.top_k, L.renorm, threadIdx.x,
                   idx + (size_t)t * L.top_k, gate + (size_t)t * L.top_k,
                   probs ? probs + (size_t)t * L.n_experts : nullptr);
}

// Caller-supplied routing (static-routing layers, Section 3.1 "Applicability": the experts of a token are
// known from the input, no router runs): copies idx / gate of the n = T * k pairs to the workspace; a pair
// whose expert index is outside [0, E) becomes expert 0 with gate 0, i.e. contributes nothing, so that the
// kernels behind can trust what they read.
__global__ __launch_bounds__(256) void k_take_routing(const int32_t* __restrict__ idx_in, const float* __restrict__ gate_in,
                                                      int32_t n, int32_t E, int32_t* __restrict__ idx, float* __restrict__ gate) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int32_t e = idx_in[i];
  const bool ok = e >= 0 && e < E;
  idx[i] = ok ? e : 0;
  gate[i] = ok ? gate_in[i] : 0.f;
}

// ---------------------------------------------------------------------------------------------
template <int BITS, bool SWIGLU, typename Stage>
__device__ __forceinline__ void ffn_in_tasks(const DevExpert& ex, int tid, int nwaves, int d, int f, int group,
                                             int row_begin, int row_end, float up, float* __restrict__ h_out,
                                             const uint32_t* XP, const float* XK, Stage stage) {
  constexpr int NM = SWIGLU ? 2 : 1;
  const int C = d / Fmt<BITS>::WPC;
  const int P = lanes_per_row(C), RW = 64 / P;
  const int lane = tid & 63, wave = tid >> 6;
  const int nrm = pick_nrm(row_end - row_begin, RW, nwaves, P, kBlock / NM);
  const bool two = (BITS == 2) && (group == 32);
  const uint8_t* q_in = uniform_ptr(ex.q_in);
  const uint16_t* s_in = uniform_ptr(ex.s_in);
  const uint8_t* q_gate = SWIGLU ? uniform_ptr(ex.q_gate) : nullptr;
  const uint16_t* s_gate = SWIGLU ? uniform_ptr(ex.s_gate) : nullptr;
  // `up` undoes the normalisation of the staged activations; h stays fp32 (phase 2 normalises it for itself)
  auto epi = [&](int row, const float (&r)[NM], int) {
    const float a = r[0] * up;
    float v;
    if constexpr (SWIGLU) v = a / (1.0f + __expf(-a)) * (r[NM - 1] * up);
    else v = fmaxf(a, 0.f);
    h_out[row] = v;
  };
  auto run = [&](auto nrm_tag, auto two_tag) {
    constexpr int NRM = decltype(nrm_tag)::value;
    constexpr bool TWO = decltype(two_tag)::value;
    if constexpr (SWIGLU) {
      const uint8_t* const qq[2] = {q_in, q_gate};
      const uint16_t* const ss[2] = {s_in, s_gate};
      gemv_stream<BITS, NRM, 2, TWO>(qq, ss, d, group, f, row_begin, row_end, lane, wave, nwaves, 1, XP, XK, epi, stage);
    } else {
      const uint8_t* const qq[1] = {q_in};
      const uint16_t* const ss[1] = {s_in};
      gemv_stream<BITS, NRM, 1, TWO>(qq, ss, d, group, f, row_begin, row_end, lane, wave, nwaves, 1, XP, XK, epi, stage);
    }
  };
  using T_ = std::true_type;
  using F_ = std::false_type;
  if constexpr (BITS == 2) {
    if (two) {
      if (!SWIGLU && nrm == 4) run(std::integral_constant<int, SWIGLU ? 2 : 4>{}, T_{});
      else if (nrm >= 2) run(std::integral_constant<int, 2>{}, T_{});
      else run(std::integral_constant<int, 1>{}, T_{});
      return;
    }
  }
  if (!SWIGLU && nrm == 4) run(std::integral_constant<int, SWIGLU ? 2 : 4>{}, F_{});
  else if (nrm >= 2) run(std::integral_constant<int, 2>{}, F_{});
  else run(std::integral_constant<int, 1>{}, F_{});
}

// Copies the table records of the k chosen experts into LDS (sel_x), so that nothing later in the
// kernel waits on a chain of dependent global loads. src_idx == nullptr: the single expert `fixed`.
__device__ __forceinline__ void load_selected(DevExpert* sel_x, const DevExpert* __restrict__ table,
                                              const int* src_idx, int fixed, int k, int E) {
  const int t = threadIdx.x;
  if (t < k * 4) {
    const int j = t >> 2, part = t & 3;
    const int e = min(max(src_idx ? src_idx[j] : fixed, 0), E - 1);   // an address: kept inside the table
    ((uint4*)&sel_x[j])[part] = ((const uint4*)&table[e])[part];
  }
}

// Phase 1 of one token for the rows [row_begin, row_end) of d_ff: for each chosen expert
// h[slot][r] = act(W_in[r] . x [, W_gate[r] . x]), written as fp32. The activations are already in RAW
// (LDS, linear binary16, normalised: `up` is the factor that undoes it) and the chosen experts' records in
// sel_x (LDS). The k
// experts are handled in passes of `spp`: the activation layouts a pass needs (one per distinct
// bitwidth) are staged together, then every wavefront streams its tasks of all the pass's experts
// without a barrier. Called by every thread of the workgroup; the first barrier inside also orders
// RAW and sel_x.
__device__ __forceinline__ void phase1_body(const LayerDims& L, const DevExpert* sel_x, int k, size_t slot0, float up,
                                            float* __restrict__ h, int row_begin, int row_end, int spp,
                                            const uint16_t* RAW, uint32_t* LAY, int nwaves) {
  const int d = L.d_model, f = L.d_ff;
  const int lay_words = d / 2 + d / 16;         // one layout: d/2 pair words + d/16 offset terms
  const bool sw = L.act == MOEQ_ACT_SWIGLU;
  __syncthreads();  // RAW and sel_x are complete
  for (int j0 = 0; j0 < k; j0 += spp) {
    const int j1 = min(k, j0 + spp);
    if (j0 > 0) __syncthreads();  // every wavefront is done with the previous pass's layouts
    for (int j = j0; j < j1; ++j) {
      const DevExpert ex = sel_x[j];
      int li = j;
      for (int i = j - 1; i >= j0; --i)
        if (sel_x[i].bits == ex.bits) li = i;
      const uint32_t* XP = LAY + (li - j0) * lay_words;
      const float* XK = (const float*)(XP + d / 2);
      float* h_out = h + (slot0 + j) * f;
      // Opaque copy of the thread index: keeps the per-variant lane arithmetic inside this iteration
      // instead of being hoisted (and spilled) ahead of the loop for every bitwidth at once.
      int tid = threadIdx.x;
      asm volatile("" : "+v"(tid));
      // The first expert of a pass stages, behind its first weight loads, one activation layout per
      // distinct bitwidth of the pass (layout index = first slot of the pass with that bitwidth).
      const bool do_stage = (j == j0);
      auto stage = [&]() {
        if (!do_stage) return;
        for (int jj = j0; jj < j1; ++jj) {
          const int bits = sel_x[jj].bits;
          bool first = true;
          for (int i = j0; i < jj; ++i) first = first && (sel_x[i].bits != bits);
          if (!first) continue;
          uint32_t* XPs = LAY + (jj - j0) * lay_words;
          float* XKs = (float*)(XPs + d / 2);
          if (bits == 2) permute_x<2>(RAW, d, L.group, tid, blockDim.x, XPs, XKs);
          else if (bits == 4) permute_x<4>(RAW, d, L.group, tid, blockDim.x, XPs, XKs);
          else permute_x<8>(RAW, d, L.group, tid, blockDim.x, XPs, XKs);
        }
        __syncthreads();
      };
      auto run = [&](auto bits_tag) {
        constexpr int BITS = decltype(bits_tag)::value;
        if (sw) ffn_in_tasks<BITS, true>(ex, tid, nwaves, d, f, L.group, row_begin, row_end, up, h_out, XP, XK, stage);
        else ffn_in_tasks<BITS, false>(ex, tid, nwaves, d, f, L.group, row_begin, row_end, up, h_out, XP, XK, stage);
      };
      switch (ex.bits) {
        case 2: run(std::integral_constant<int, 2>{}); break;
        case 4: run(std::integral_constant<int, 4>{}); break;
        default: run(std::integral_constant<int, 8>{}); break;
      }
    }
  }
}

// Stand-alone phase 1: (optionally) top-k from the router logits, then phase1_body. Workgroup 0 of a
// token also publishes the routing (idx, gate) and the chosen experts' records (sel_tab) for phase 2.
__global__ __launch_bounds__(1024) void k_ffn_in(LayerDims L, const DevExpert* __restrict__ table,
                                                 const float* __restrict__ logits, int32_t* __restrict__ idx_out,
                                                 float* __restrict__ gate_out, DevExpert* __restrict__ sel_tab,
                                                 int32_t fixed_expert, const void* __restrict__ x,
                                                 float* __restrict__ h, int32_t rows_per_wg,
                                                 int32_t slots_per_pass) {
  extern __shared__ uint32_t smem[];
  __shared__ int sel_e[8];
  __shared__ float sel_g[8];
  __shared__ DevExpert sel_x[8];
  __shared__ float red[16];
  const int d = L.d_model, f = L.d_ff;
  const int token = blockIdx.y;
  uint16_t* RAW = (uint16_t*)smem;              // d halfs, then the layouts
  uint32_t* LAY = smem + d / 2;
  const int k = fixed_expert >= 0 ? 1 : L.top_k;
  const size_t xbytes = L.x_bf16 ? 2 : 4;
  const float up = stage_normalised((const char*)x + (size_t)token * d * xbytes, L.x_bf16 ? X_BF16 : X_F32, d,
                                    threadIdx.x, blockDim.x, RAW, red);
  if (fixed_expert < 0) {
    if (logits) {
      if (threadIdx.x < 64) topk_from_logits(logits + (size_t)token * L.n_experts, L.n_experts, k, L.renorm,
                                             threadIdx.x, sel_e, sel_g, nullptr);
    } else if (threadIdx.x < k) {   // the routing is given: idx_out / gate_out already hold it
      sel_e[threadIdx.x] = idx_out[(size_t)token * k + threadIdx.x];
      sel_g[threadIdx.x] = gate_out[(size_t)token * k + threadIdx.x];
    }
    __syncthreads();
    load_selected(sel_x, table, sel_e, -1, k, L.n_experts);
    if (logits && blockIdx.x == 0 && threadIdx.x < k) {
      idx_out[(size_t)token * k + threadIdx.x] = sel_e[threadIdx.x];
      gate_out[(size_t)token * k + threadIdx.x] = sel_g[threadIdx.x];
    }
    if (blockIdx.x == 0) {
      __syncthreads();
      if (threadIdx.x < k * 4)
        ((uint4*)&sel_tab[(size_t)token * k])[threadIdx.x] = ((const uint4*)sel_x)[threadIdx.x];
    }
  } else {
    load_selected(sel_x, table, nullptr, fixed_expert, 1, L.n_experts);
  }
  const int row_begin = blockIdx.x * rows_per_wg;
  const int row_end = min(f, row_begin + rows_per_wg);
  phase1_body(L, sel_x, k, fixed_expert >= 0 ? (size_t)token : (size_t)token * k, up, h, row_begin, row_end,
              slots_per_pass, RAW, LAY, (int)(blockDim.x >> 6));
}

// ---------------------------------------------------------------------------------------------
// Number of wavefront teams that split every row of a phase-2 GEMV along its length: the rows a
// workgroup owns are few and long, so without the split most wavefronts would have no task.
__host__ __device__ inline int pick_ks(int rows_in_wg, int RW, int nwaves, int Jfull) {
  const int tasks1 = (rows_in_wg + RW - 1) / RW;   // tasks at one row per lane group
  int ks = 1;
  while (ks < kMaxKs && tasks1 * ks * 2 <= nwaves && ks * 2 <= Jfull && nwaves % (ks * 2) == 0) ks *= 2;
  return ks;
}

template <int BITS, typename Stage>
__device__ __forceinline__ void ffn_out_tasks(const DevExpert& ex, int tid, int nwaves, int d, int f, int group,
                                              float g, const float* up, int row_begin, int row_end, int rows_per_wg,
                                              float* ybuf, const uint32_t* XP, const float* XK, Stage stage) {
  const int C = f / Fmt<BITS>::WPC;
  const int P = lanes_per_row(C), RW = 64 / P;
  const int lane = tid & 63, wave = tid >> 6;
  const int ks = pick_ks(row_end - row_begin, RW, nwaves, C / P);
  const int nrm = pick_nrm(row_end - row_begin, RW, nwaves / ks, P, kBlock);
  const bool two = (BITS == 2) && (group == 32);
  const uint8_t* const qq[1] = {uniform_ptr(ex.q_out)};
  const uint16_t* const ss[1] = {uniform_ptr(ex.s_out)};
  // ybuf: [kMaxKs][rows_per_wg] partial sums of this expert; teams beyond ks are zeroed by the caller
  // *up (LDS, written by stage()) undoes the normalisation of this expert's h
  auto epi = [&](int row, const float (&r)[1], int part) {
    ybuf[part * rows_per_wg + (row - row_begin)] = g * (r[0] * *up);
  };
  auto run = [&](auto nrm_tag, auto two_tag) {
    constexpr int NRM = decltype(nrm_tag)::value;
    constexpr bool TWO = decltype(two_tag)::value;
    gemv_stream<BITS, NRM, 1, TWO>(qq, ss, f, group, d, row_begin, row_end, lane, wave, nwaves, ks, XP, XK, epi, stage);
  };
  using T_ = std::true_type;
  using F_ = std::false_type;
  if constexpr (BITS == 2) {
    if (two) {
      if (nrm == 4) run(std::integral_constant<int, 4>{}, T_{});
      else if (nrm == 2) run(std::integral_constant<int, 2>{}, T_{});
      else run(std::integral_constant<int, 1>{}, T_{});
      return;
    }
  }
  if (nrm == 4) run(std::integral_constant<int, 4>{}, F_{});
  else if (nrm == 2) run(std::integral_constant<int, 2>{}, F_{});
  else run(std::integral_constant<int, 1>{}, F_{});
}

// Phase 2 + combine of one token for the rows [row_begin, row_end) of d_model:
// y[t][r] (+)= sum_j gate_j * W_out_j[r] . h[slot_j]. Experts are handled in passes of `spp`: their
// activation vectors (fp32 in h) are normalised, converted to binary16 and staged in the pair order of
// their expert's bitwidth, every wavefront streams its tasks of all of them without a barrier,
// each expert's contribution lands in its own LDS row buffer, and the buffers are summed in top-k order
// at the end: ordered, no atomics, every output written once.
// sel_x: the k chosen experts' records (LDS); gate_tok: their gates (LDS or global), may be null (= 1).
__device__ __forceinline__ void phase2_body(const LayerDims& L, const DevExpert* sel_x, const float* gate_tok, int k,
                                            int accumulate, size_t slot0, const float* __restrict__ h,
                                            float* __restrict__ y_out, int row_begin, int row_end, int rows_per_wg,
                                            int spp, uint32_t* smem, float* red, float* s_up, int nwaves) {
  const int d = L.d_model, f = L.d_ff;
  const int lay_words = f / 2 + f / 16;          // pair words + offset terms of one activation vector
  float* ybuf = (float*)smem;                    // [k][kMaxKs][rows_per_wg]
  uint32_t* LAY = smem + k * kMaxKs * rows_per_wg;   // [spp][lay_words]
  uint16_t* RAW = (uint16_t*)(LAY + spp * lay_words);   // [f] one normalised h vector, linear binary16
  for (int i = threadIdx.x; i < k * kMaxKs * rows_per_wg; i += blockDim.x) ybuf[i] = 0.f;
  __syncthreads();  // sel_x / gates are complete
  for (int j0 = 0; j0 < k; j0 += spp) {
    const int j1 = min(k, j0 + spp);
    if (j0 > 0) __syncthreads();  // every wavefront is done with the previous pass's activations
    for (int j = j0; j < j1; ++j) {
      const float g = gate_tok ? gate_tok[j] : 1.0f;
      const DevExpert ex = sel_x[j];
      const uint32_t* XP = LAY + (j - j0) * lay_words;
      const float* XK = (const float*)(XP + f / 2);
      int tid = threadIdx.x;       // opaque copy: keeps per-variant lane arithmetic out of the prologue
      asm volatile("" : "+v"(tid));
      // The first expert of a pass stages, behind its first weight loads, the activation vectors of all the
      // pass's experts: each is normalised into RAW, then put in the pair order of its expert's bitwidth with
      // its offset terms.
      const bool do_stage = (j == j0);
      auto stage = [&]() {
        if (!do_stage) return;
        for (int jj = j0; jj < j1; ++jj) {
          const float u = stage_normalised(h + (slot0 + jj) * f, X_F32, f, tid, blockDim.x, RAW, red);
          if (tid == 0) s_up[jj] = u;
          __syncthreads();   // RAW is complete
          uint32_t* XPs = LAY + (jj - j0) * lay_words;
          float* XKs = (float*)(XPs + f / 2);
          const int bits = sel_x[jj].bits;
          if (bits == 2) permute_x<2>(RAW, f, L.group_out, tid, blockDim.x, XPs, XKs);
          else if (bits == 4) permute_x<4>(RAW, f, L.group_out, tid, blockDim.x, XPs, XKs);
          else permute_x<8>(RAW, f, L.group_out, tid, blockDim.x, XPs, XKs);
          __syncthreads();   // the layout and s_up are complete; RAW may be overwritten
        }
      };
      auto run = [&](auto bits_tag) {
        constexpr int BITS = decltype(bits_tag)::value;
        ffn_out_tasks<BITS>(ex, tid, nwaves, d, f, L.group_out, g, s_up + j, row_begin, row_end, rows_per_wg,
                            ybuf + j * kMaxKs * rows_per_wg, XP, XK, stage);
      };
      switch (ex.bits) {
        case 2: run(std::integral_constant<int, 2>{}); break;
        case 4: run(std::integral_constant<int, 4>{}); break;
        default: run(std::integral_constant<int, 8>{}); break;
      }
    }
  }
  __syncthreads();
  for (int i = row_begin + (int)threadIdx.x; i < row_end; i += blockDim.x) {
    float acc = accumulate ? y_out[i] : 0.f;
    for (int j = 0; j < k; ++j) {      // experts in top-k order, teams in order: a fixed summation order
      float e_sum = 0.f;
      for (int pt = 0; pt < kMaxKs; ++pt) e_sum += ybuf[(j * kMaxKs + pt) * rows_per_wg + (i - row_begin)];
      acc += e_sum;
    }
    y_out[i] = acc;
  }
}

// Stand-alone phase 2. sel_tab: the chosen experts' records written by phase 1 (fixed_expert < 0).
__global__ __launch_bounds__(1024) void k_ffn_out(LayerDims L, const DevExpert* __restrict__ table,
                                                  const DevExpert* __restrict__ sel_tab, const float* __restrict__ gate,
                                                  int32_t fixed_expert, int32_t accumulate,
                                                  const float* __restrict__ h, float* __restrict__ y,
                                                  int32_t rows_per_wg, int32_t slots_per_pass) {
  extern __shared__ uint32_t smem[];
  __shared__ DevExpert sel_x[8];
  __shared__ float sel_g[8];
  __shared__ float red[16];
  __shared__ float s_up[8];
  const int d = L.d_model;
  const int token = blockIdx.y;
  const int k = fixed_expert >= 0 ? 1 : L.top_k;
  const size_t slot0 = fixed_expert >= 0 ? (size_t)token : (size_t)token * k;
  if (fixed_expert >= 0) {
    load_selected(sel_x, table, nullptr, fixed_expert, 1, L.n_experts);
  } else if (threadIdx.x < k * 4) {
    ((uint4*)sel_x)[threadIdx.x] = ((const uint4*)&sel_tab[slot0])[threadIdx.x];
  }
  if (threadIdx.x < k) sel_g[threadIdx.x] = gate ? gate[slot0 + threadIdx.x] : 1.0f;
  const int row_begin = blockIdx.x * rows_per_wg;
  const int row_end = min(d, row_begin + rows_per_wg);
  phase2_body(L, sel_x, sel_g, k, accumulate, slot0, h, y + (size_t)token * d, row_begin, row_end, rows_per_wg,
              slots_per_pass, smem, red, s_up, (int)(blockDim.x >> 6));
}

int num_cus() {
  static int cus = 0;
  if (!cus) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
      cus = prop.multiProcessorCount;
    if (cus <= 0) cus = 256;
  }
  return cus;
}

constexpr size_t kLdsBudget = 150 * 1024;  // of the 160 KB per compute unit; the rest covers static LDS

// Rows per workgroup and wavefronts per workgroup for a GEMV over `rows` output rows split over
// `target` workgroups. Row ranges are multiples of the rows a wavefront covers per step at the widest
// bitwidth (64/min_P) so that tasks never straddle workgroups.
struct Split { int rows_per_wg, gx, threads; };
Split plan_rows(int rows, int min_P, int target, int nrm_max) {
  const int RWmax = 64 / min_P;
  if (target < 1) target = 1;
  int rpw = (rows + target - 1) / target;
  rpw = (rpw + RWmax - 1) / RWmax * RWmax;
  if (rpw < RWmax) rpw = RWmax;
  Split s;
  s.rows_per_wg = rpw;
  s.gx = (rows + rpw - 1) / rpw;
  // wavefronts per workgroup: the count in [4, 16] that leaves the fewest idle task slots, more on ties
  int best_w = 4;
  double best_eff = -1.0;
  for (int w = 16; w >= 4; --w) {
    const int nrm = pick_nrm(rpw, RWmax, w, min_P, nrm_max);
    const int tasks = (rpw + RWmax * nrm - 1) / (RWmax * nrm);
    const int rounds = (tasks + w - 1) / w;
    const double eff = (double)tasks / ((double)rounds * w);
    if (eff > best_eff + 1e-9) { best_eff = eff; best_w = w; }
  }
  s.threads = best_w * 64;
  return s;
}

// Phase 2 rows are few and long: wavefronts beyond one per task team up along the row (pick_ks), so the
// workgroup is widened to the largest power-of-two multiple of the planned size that still fits.
int phase2_threads(int threads) {
  int w = threads / 64;
  while (w * 2 <= 16) w *= 2;
  return w * 64;
}

int wgs_per_token(int T) {
  const int cus = num_cus();
  int target = cus / (T < 1 ? 1 : (T > cus ? cus : T));
  return target < 1 ? 1 : target;
}

int min_lanes_per_row(int cols) {
  int P = 64;
  for (int b = 2; b <= 8; b *= 2) {
    if ((cols * b) % 128) continue;
    const int p = lanes_per_row(cols * b / 128);
    if (p < P) P = p;
  }
  return P;
}

// LDS bytes and slots per pass of the two phases.
struct PhaseLds { size_t bytes; int spp; };
PhaseLds phase1_lds(const LayerDims& L, int k) {
  const size_t raw = (size_t)L.d_model * 2;
  const size_t lay = ((size_t)L.d_model / 2 + (size_t)L.d_model / 16) * 4;
  int spp = (int)((kLdsBudget - raw) / lay);   // layouts that fit: at most one per slot of a pass, 3 distinct
  if (spp > k) spp = k;
  if (spp > 3) spp = 3;
  if (spp < 1) spp = 1;
  return {raw + (size_t)spp * lay, spp};
}
PhaseLds phase2_lds(const LayerDims& L, int k, int rows_per_wg) {
  const size_t ybuf = (size_t)k * kMaxKs * rows_per_wg * 4;
  const size_t raw = (size_t)L.d_ff * 2;         // one normalised h vector on its way into the pair order
  const size_t per_slot = ((size_t)L.d_ff / 2 + (size_t)L.d_ff / 16) * 4;
  int spp = (int)((kLdsBudget - ybuf - raw) / per_slot);
  if (spp > k) spp = k;
  if (spp < 1) spp = 1;
  return {ybuf + raw + (size_t)spp * per_slot, spp};
}


}  // namespace

hipError_t init_attrs_ffn_decode() {
  (void)num_cus();
  if (hipError_t e = hipFuncSetAttribute((const void*)k_ffn_in, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBudget);
      e != hipSuccess)
    return e;
  return hipFuncSetAttribute((const void*)k_ffn_out, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBudget);
}

hipError_t launch_topk(const LayerDims& L, const float* logits, int32_t T, int32_t* idx, float* gate, float* probs,
                       hipStream_t st) {
  hipLaunchKernelGGL(k_topk, dim3(T), dim3(64), 0, st, L, logits, idx, gate, probs);
  return hipGetLastError();
}

hipError_t launch_take_routing(const int32_t* idx_in, const float* gate_in, int32_t n, int32_t E, int32_t* idx,
                               float* gate, hipStream_t st) {
  hipLaunchKernelGGL(k_take_routing, dim3((n + 255) / 256), dim3(256), 0, st, idx_in, gate_in, n, E, idx, gate);
  return hipGetLastError();
}

hipError_t launch_ffn_in(const LayerDims& L, const DevExpert* table, const float* logits, int32_t* idx_out,
                         float* gate_out, DevExpert* sel_tab, int32_t fixed_expert, const void* x, int32_t T,
                         float* h, hipStream_t st) {
  const Split sp = plan_rows(L.d_ff, min_lanes_per_row(L.d_model), wgs_per_token(T),
                             L.act == MOEQ_ACT_SWIGLU ? kBlock / 2 : kBlock);
  const PhaseLds pl = phase1_lds(L, fixed_expert >= 0 ? 1 : L.top_k);
  if (pl.bytes > kLdsBudget) return hipErrorInvalidValue;   // the ceiling init_attrs_ffn_decode() asked for
  hipLaunchKernelGGL(k_ffn_in, dim3(sp.gx, T), dim3(sp.threads), pl.bytes, st, L, table, logits, idx_out, gate_out,
                     sel_tab, fixed_expert, x, h, sp.rows_per_wg, pl.spp);
  return hipGetLastError();
}

hipError_t launch_ffn_out(const LayerDims& L, const DevExpert* table, const DevExpert* sel_tab, const float* gate,
                          int32_t fixed_expert, int32_t accumulate, const float* h, int32_t T, float* y,
                          hipStream_t st) {
  Split sp = plan_rows(L.d_model, min_lanes_per_row(L.d_ff), wgs_per_token(T), kBlock);
  sp.threads = phase2_threads(sp.threads);
  const PhaseLds pl = phase2_lds(L, fixed_expert >= 0 ? 1 : L.top_k, sp.rows_per_wg);
  if (pl.bytes > kLdsBudget) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_ffn_out, dim3(sp.gx, T), dim3(sp.threads), pl.bytes, st, L, table, sel_tab, gate, fixed_expert,
                     accumulate, h, y, sp.rows_per_wg, pl.spp);
  return hipGetLastError();
}

}  // namespace moeq
