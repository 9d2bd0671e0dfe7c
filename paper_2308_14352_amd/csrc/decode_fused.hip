// The whole MoE layer of a decode call in ONE streaming kernel plus a small reduction
// (Section 1, Section 2.1: router, top-k, the chosen experts' FFNs, gate-weighted combine; Section 3.2:
// the experts' weights are decompressed by the mirror of the linear quantization before use - here
// on the fly, in registers).
//
// Work split. The hidden dimension d_ff is cut into slices of SW columns; workgroup (slice, token)
// computes, for every chosen expert, the SW entries h[slice] = act(W_in[slice rows] x [, W_gate ...])
// and at once multiplies them into the matching SW columns of W_out for ALL d_model output rows,
// which gives a partial output vector. No workgroup ever waits for another one: the only exchange is
// the final sum of the partial vectors, done by a second, tiny kernel in a fixed order (no atomics, the
// result is bit-reproducible). The router (or, for many experts, the top-k on logits computed by the
// router kernel) is evaluated redundantly by every workgroup, with identical arithmetic, so all
// workgroups of a token agree on the routing without talking to each other.
//
// W_out is read in the "dword-column-major" layout (moe_prepare_out): the 32-bit words of the canonical
// packed rows transposed, qT[w][r] = word w of row r, scales sT[g][r]. A lane then owns four consecutive
// output rows, a 128-bit load brings one word (32/b codes along d_ff) of each of them, consecutive
// lanes read consecutive addresses, and the partial dot products need no cross-lane reduction at all.
#include <cstdlib>

#include "decode_core.h"

namespace moeq {
namespace {

constexpr int kRbMax = 2;          // output row blocks (of 4 rows) per thread in phase 2
constexpr int kP2Unroll = 8;       // 128-bit loads in flight per thread in phase 2
constexpr int kInlineMaxE = 1024;  // size of the in-kernel logits buffer

// Position (in binary16 units) of column `col` of a slice in the pair layout phase 2 reads, and the
// power of two its activation is pre-divided by. Word w of a row holds CPD = 32/b codes; its PPD = CPD/2
// pair registers sit at words [w*PPD, (w+1)*PPD) in the order dword_dot<b> consumes them.
template <int BITS>
__device__ __forceinline__ int slice_pair_index(int col, float& prescale) {
  constexpr int CPD = 32 / BITS, PPD = CPD / 2;
  const int w = col / CPD, pos = col % CPD;
  int pi, half;
  if (BITS == 8) {
    pi = pos & 1; half = pos >> 1; prescale = 1.0f;
  } else if (BITS == 4) {
    pi = pos & 3; half = pos >> 2; prescale = (pi & 1) ? 0.0625f : 1.0f;
  } else {
    pi = pos & 7; half = pos >> 3;
    const int e = pi < 5 ? pi : pi - 5;
    prescale = 1.0f / (float)(1 << (2 * e));
  }
  return (w * PPD + pi) * 2 + half;
}

struct FusedParams {
  LayerDims L;
  const DevExpert* table;
  const float* Wr;
  const float* bias;
  const float* logits;    // non-null: router logits [T][E] computed beforehand; null: computed here
  int32_t fixed_expert;   // >= 0: every token uses this expert (no routing)
  const float* gate_in;   // fixed-expert mode: [T] or null (= 1)
  const void* x;          // [T][d] in the layer's dtype
  float* part;            // [T][n_slices][d] partial outputs
  int32_t* idx_out;       // [T][k] or null
  float* gate_out;        // [T][k] or null
  int32_t SW;             // slice width (columns of d_ff): a multiple of 16 that divides the group size
};

// Phase 1 of one expert on the rows [row_begin, row_end) of W_in (and W_gate): h values go to LDS as
// binary16, once linear (HL) and once in the pair layout of this expert's bitwidth (HP).
template <int BITS, bool SWIGLU>
__device__ __forceinline__ void fused_in_tasks(const DevExpert& ex, int tid, int nwaves, int d, int f, int group,
                                               int row_begin, int row_end, uint16_t* HL, uint16_t* HP,
                                               const uint32_t* XP, const float* XK) {
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
  auto epi = [&](int row, const float (&r)[NM], int) {
    float v;
    if constexpr (SWIGLU) v = r[0] / (1.0f + __expf(-r[0])) * r[1];
    else v = fmaxf(r[0], 0.f);
    const uint32_t hb = f32_to_f16_bits(v);
    const int c = row - row_begin;
    HL[c] = (uint16_t)hb;
    float ps;
    const int si = slice_pair_index<BITS>(c, ps);
    HP[si] = (uint16_t)f32_to_f16_bits(f16_bits_to_f32(hb) * ps);
  };
  auto no_stage = []() {};
  auto run = [&](auto nrm_tag, auto two_tag) {
    constexpr int NRM = decltype(nrm_tag)::value;
    constexpr bool TWO = decltype(two_tag)::value;
    if constexpr (SWIGLU) {
      const uint8_t* const qq[2] = {q_in, q_gate};
      const uint16_t* const ss[2] = {s_in, s_gate};
      gemv_stream<BITS, NRM, 2, TWO>(qq, ss, d, group, f, row_begin, row_end, lane, wave, nwaves, 1, XP, XK, epi, no_stage);
    } else {
      const uint8_t* const qq[1] = {q_in};
      const uint16_t* const ss[1] = {s_in};
      gemv_stream<BITS, NRM, 1, TWO>(qq, ss, d, group, f, row_begin, row_end, lane, wave, nwaves, 1, XP, XK, epi, no_stage);
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

// Phase 2 of one expert: yacc[i][r] += gate * s[row][grp] * sum_{col in slice} (u - 2^(b-1)) * h[col] for the
// thread's row blocks. qT/sT are the dword-column-major codes and scales of W_out.
template <int BITS>
__device__ __forceinline__ void fused_out(const DevExpert& ex, int tid, int nthreads, int d, int group, int slice,
                                          int SW, float gate, const uint16_t* HL, const uint16_t* HP,
                                          float (&yacc)[kRbMax][4]) {
  constexpr int CPD = 32 / BITS, PPD = CPD / 2;
  const int lane = tid & 63;
  const int DW = SW / CPD;
  const int w0 = slice * DW;
  const int grp = (slice * SW) / group;
  // offset term: 2^(b-1) * 2^-24 * (sum of the slice's activations), the same in every wavefront
  float hs = 0.f;
  for (int c = lane; c < SW; c += 64) hs += f16_bits_to_f32(HL[c]);
  hs = wave_sum(hs);
  const float K = hs * (Fmt<BITS>::OFF * 5.9604644775390625e-08f);
  const uint8_t* qT = uniform_ptr(ex.q_out);
  const uint8_t* sT = (const uint8_t*)uniform_ptr(ex.s_out);
  const uint32_t* HPw = (const uint32_t*)HP;
  const int nrb = d / 4;
#pragma unroll
  for (int i = 0; i < kRbMax; ++i) {
    const int rb = tid + i * nthreads;
    if (rb < nrb) {
      const uint2 sraw = *(const uint2*)(sT + ((size_t)grp * d + 4 * (size_t)rb) * 2);
      float acc[4] = {0.f, 0.f, 0.f, 0.f};
      for (int wb = 0; wb < DW; wb += kP2Unroll) {
        uint4 t[kP2Unroll];
#pragma unroll
        for (int u = 0; u < kP2Unroll; ++u)
          if (wb + u < DW) t[u] = load_stream16(qT + ((size_t)(w0 + wb + u) * d + 4 * (size_t)rb) * 4);
#pragma unroll
        for (int u = 0; u < kP2Unroll; ++u)
          if (wb + u < DW) {
            uint32_t xr[PPD];
#pragma unroll
            for (int p = 0; p < PPD; ++p) xr[p] = HPw[(wb + u) * PPD + p];
            acc[0] = dword_dot<BITS>(t[u].x, xr, acc[0]);
            acc[1] = dword_dot<BITS>(t[u].y, xr, acc[1]);
            acc[2] = dword_dot<BITS>(t[u].z, xr, acc[2]);
            acc[3] = dword_dot<BITS>(t[u].w, xr, acc[3]);
          }
      }
      const float g24 = gate * 16777216.0f;
      yacc[i][0] = fmaf(f16_bits_to_f32(sraw.x & 0xffffu) * g24, acc[0] - K, yacc[i][0]);
      yacc[i][1] = fmaf(f16_bits_to_f32(sraw.x >> 16) * g24, acc[1] - K, yacc[i][1]);
      yacc[i][2] = fmaf(f16_bits_to_f32(sraw.y & 0xffffu) * g24, acc[2] - K, yacc[i][2]);
      yacc[i][3] = fmaf(f16_bits_to_f32(sraw.y >> 16) * g24, acc[3] - K, yacc[i][3]);
    }
  }
}

template <bool BF16>
__global__ __launch_bounds__(1024) void k_moe_decode(FusedParams P) {
  extern __shared__ uint32_t smem[];
  __shared__ int sel_e[8];
  __shared__ float sel_g[8];
  __shared__ DevExpert sel_x[8];
  __shared__ float lg[kInlineMaxE];
  const LayerDims& L = P.L;
  const int d = L.d_model, f = L.d_ff, E = L.n_experts, SW = P.SW;
  const int slice = blockIdx.x, token = blockIdx.y;
  const int nthreads = blockDim.x, nwaves = nthreads >> 6;
  const int k = P.fixed_expert >= 0 ? 1 : L.top_k;
  const int lay_words = d / 2 + d / 16;
  uint16_t* RAW = (uint16_t*)smem;                 // [d] activations, linear binary16
  uint16_t* HLs = RAW + d;                         // [k][SW] h of every chosen expert, linear binary16
  uint16_t* HPs = HLs + k * SW;                    // [k][SW] the same in the pair layout of the expert's bitwidth
  uint32_t* LAY = (uint32_t*)(HPs + k * SW);       // [<= 3][lay_words] staged activations, one per distinct bitwidth
  const size_t xbytes = BF16 ? 2 : 4;
  const char* xt = (const char*)P.x + (size_t)token * d * xbytes;

  copy_x_to_lds(xt, BF16 ? X_BF16 : X_F32, d, threadIdx.x, nthreads, RAW);
  if (P.fixed_expert < 0) {
    const float* lgp;
    if (P.logits) {
      lgp = P.logits + (size_t)token * E;
    } else {
      // router: wavefront w scores the experts w, w + nwaves, ... in fp32 on the unrounded activations
      const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
      for (int e = wave; e < E; e += nwaves) {
        const float* wr = P.Wr + (size_t)e * d;
        float acc = 0.f;
        for (int i = lane * 4; i < d; i += 256) {
          const float4 w = *(const float4*)(wr + i);
          float4 v;
          if (BF16) {
            const uint2 b = *(const uint2*)((const uint16_t*)xt + i);
            v = make_float4(bf16_bits_to_f32(b.x & 0xffffu), bf16_bits_to_f32(b.x >> 16),
                            bf16_bits_to_f32(b.y & 0xffffu), bf16_bits_to_f32(b.y >> 16));
          } else {
            v = *(const float4*)((const float*)xt + i);
          }
          acc = fmaf(w.x, v.x, acc); acc = fmaf(w.y, v.y, acc); acc = fmaf(w.z, v.z, acc); acc = fmaf(w.w, v.w, acc);
        }
        acc = wave_sum(acc);
        if (lane == 0) lg[e] = acc + (P.bias ? P.bias[e] : 0.f);
      }
      __syncthreads();
      lgp = lg;
    }
    if (threadIdx.x < 64) topk_from_logits(lgp, E, k, L.renorm, threadIdx.x, sel_e, sel_g, nullptr);
    __syncthreads();
    if (threadIdx.x < k * 4) {
      const int j = threadIdx.x >> 2, part = threadIdx.x & 3;
      ((uint4*)&sel_x[j])[part] = ((const uint4*)&P.table[sel_e[j]])[part];
    }
    if (slice == 0 && threadIdx.x < k) {
      if (P.idx_out) P.idx_out[(size_t)token * k + threadIdx.x] = sel_e[threadIdx.x];
      if (P.gate_out) P.gate_out[(size_t)token * k + threadIdx.x] = sel_g[threadIdx.x];
    }
  } else {
    if (threadIdx.x < 4) ((uint4*)&sel_x[0])[threadIdx.x] = ((const uint4*)&P.table[P.fixed_expert])[threadIdx.x];
    if (threadIdx.x == 0) sel_g[0] = P.gate_in ? P.gate_in[token] : 1.0f;
  }
  __syncthreads();  // RAW, sel_x, sel_g are complete

  // one staged activation layout per distinct bitwidth among the chosen experts, in first-use order
  uint32_t lay_of = 0;  // 2 bits per slot: the layout its expert reads
  {
    int n_lay = 0;
    for (int j = 0; j < k; ++j) {
      const int bits = sel_x[j].bits;
      int li = -1;
      for (int i = 0; i < j; ++i)
        if (li < 0 && sel_x[i].bits == bits) li = (int)((lay_of >> (2 * i)) & 3u);
      if (li < 0) {
        li = n_lay++;
        uint32_t* XPs = LAY + li * lay_words;
        float* XKs = (float*)(XPs + d / 2);
        if (bits == 2) permute_x<2>(RAW, d, L.group, threadIdx.x, nthreads, XPs, XKs);
        else if (bits == 4) permute_x<4>(RAW, d, L.group, threadIdx.x, nthreads, XPs, XKs);
        else permute_x<8>(RAW, d, L.group, threadIdx.x, nthreads, XPs, XKs);
      }
      lay_of |= (uint32_t)li << (2 * j);
    }
  }
  __syncthreads();

  const int row_begin = slice * SW, row_end = row_begin + SW;
  const bool sw = L.act == MOEQ_ACT_SWIGLU;
  float yacc[kRbMax][4];
#pragma unroll
  for (int i = 0; i < kRbMax; ++i)
#pragma unroll
    for (int r = 0; r < 4; ++r) yacc[i][r] = 0.f;

  for (int j = 0; j < k; ++j) {
    const DevExpert ex = sel_x[j];
    const uint32_t* XP = LAY + (int)((lay_of >> (2 * j)) & 3u) * lay_words;
    const float* XK = (const float*)(XP + d / 2);
    uint16_t* HL = HLs + j * SW;
    uint16_t* HP = HPs + j * SW;
    const float gate = sel_g[j];
    int tid = threadIdx.x;  // opaque copy: keeps the per-bitwidth lane arithmetic inside this iteration
    asm volatile("" : "+v"(tid));
    auto run = [&](auto bits_tag) {
      constexpr int BITS = decltype(bits_tag)::value;
      if (sw) fused_in_tasks<BITS, true>(ex, tid, nwaves, d, f, L.group, row_begin, row_end, HL, HP, XP, XK);
      else fused_in_tasks<BITS, false>(ex, tid, nwaves, d, f, L.group, row_begin, row_end, HL, HP, XP, XK);
      __syncthreads();  // this expert's h slice is complete in LDS
      fused_out<BITS>(ex, tid, nthreads, d, L.group, slice, SW, gate, HL, HP, yacc);
    };
    switch (ex.bits) {
      case 2: run(std::integral_constant<int, 2>{}); break;
      case 4: run(std::integral_constant<int, 4>{}); break;
      default: run(std::integral_constant<int, 8>{}); break;
    }
  }

  float* out = P.part + ((size_t)token * gridDim.x + slice) * d;
#pragma unroll
  for (int i = 0; i < kRbMax; ++i) {
    const int rb = (int)threadIdx.x + i * nthreads;
    if (rb < d / 4) ((float4*)out)[rb] = make_float4(yacc[i][0], yacc[i][1], yacc[i][2], yacc[i][3]);
  }
}

// y[t][r] (+)= sum over the slices of part[t][s][r], in a fixed order. Workgroup = 64 outputs x 16 slice
// teams: team g sums the slices g, g+16, ... for its 4 outputs, then the 16 team sums are added in order.
__global__ __launch_bounds__(256) void k_reduce_partials(const float* __restrict__ part, int n_slices, int d,
                                                         int accumulate, float* __restrict__ y) {
  __shared__ float4 red[16][16];
  const int token = blockIdx.y;
  const int rq = threadIdx.x & 15, sg = threadIdx.x >> 4;
  const int r0 = blockIdx.x * 64 + rq * 4;
  float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
  if (r0 < d) {
    const float* p = part + (size_t)token * n_slices * d + r0;
    for (int s = sg; s < n_slices; s += 16) {
      const float4 v = *(const float4*)(p + (size_t)s * d);
      a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
    }
  }
  red[sg][rq] = a;
  __syncthreads();
  if (threadIdx.x < 16 && r0 < d) {
    float4 t = red[0][rq];
#pragma unroll
    for (int g = 1; g < 16; ++g) {
      const float4 v = red[g][rq];
      t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w;
    }
    float4* o = (float4*)(y + (size_t)token * d + r0);
    if (accumulate) {
      const float4 v = *o;
      t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w;
    }
    *o = t;
  }
}

// out[c][r] = in[r][c] for a [rows][cols] matrix of T-sized elements (32 x 32 tiles through LDS).
template <typename T>
__global__ __launch_bounds__(256) void k_transpose(const T* __restrict__ in, int64_t rows, int64_t cols,
                                                   T* __restrict__ out) {
  __shared__ T tile[32][33];
  const int64_t c0 = (int64_t)blockIdx.x * 32, r0 = (int64_t)blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int i = ty; i < 32; i += 8)
    if (r0 + i < rows && c0 + tx < cols) tile[i][tx] = in[(r0 + i) * cols + c0 + tx];
  __syncthreads();
  for (int i = ty; i < 32; i += 8)
    if (c0 + i < cols && r0 + tx < rows) out[(c0 + i) * rows + r0 + tx] = tile[tx][i];
}

int cu_count() {
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

constexpr size_t kFusedLdsBudget = 150 * 1024;

size_t fused_lds_bytes(const LayerDims& L, int k, int SW) {
  const int nl = k < 3 ? k : 3;
  return (size_t)L.d_model * 2 + (size_t)k * SW * 4 + (size_t)nl * ((size_t)L.d_model / 2 + (size_t)L.d_model / 16) * 4;
}

}  // namespace

// Slice width: a multiple of 16 columns (one 32-bit word of 2-bit codes) that divides the group size, so that
// a slice has one scale per output row; the widest one that still gives at least 3/4 of a workgroup per
// compute unit, else the narrowest.
FusedPlan plan_fused(const LayerDims& L) {
  FusedPlan p{0, 0, 0};
  if (L.d_model % 8 || L.d_ff % 16 || L.group % 16) return p;
  static const int forced = [] { const char* v = std::getenv("MOEQ_SLICE"); return v ? std::atoi(v) : 0; }();
  const int want = cu_count() * 3 / 4;
  int best = 0;
  for (int sw = 16; sw <= 256; sw *= 2) {
    if (L.group % sw || L.d_ff % sw) break;
    if (best == 0 || L.d_ff / sw >= want) best = sw;
    if (forced == sw) { best = sw; break; }
  }
  if (!best) return p;
  int nt = (L.d_model / 4 + 63) / 64 * 64;
  if (nt < 256) nt = 256;
  if (nt > 1024) nt = 1024;
  static const int forced_nt = [] { const char* v = std::getenv("MOEQ_THREADS"); return v ? std::atoi(v) : 0; }();
  if (forced_nt >= 64 && forced_nt <= 1024 && forced_nt % 64 == 0) nt = forced_nt;
  if ((int64_t)nt * kRbMax * 4 < L.d_model) return p;   // every output row needs an owner
  if (fused_lds_bytes(L, L.top_k, best) > kFusedLdsBudget) return p;
  p.SW = best;
  p.n_slices = L.d_ff / best;
  p.threads = nt;
  return p;
}

hipError_t launch_moe_decode(const LayerDims& L, const FusedPlan& plan, const DevExpert* table, const float* router_w,
                             const float* router_bias, const float* logits, int32_t fixed_expert,
                             const float* gate_in, const void* x, int32_t T, float* part, int32_t* idx_out,
                             float* gate_out, hipStream_t st) {
  if (!plan.SW || T < 1 || T > 65535) return hipErrorInvalidValue;
  if (!logits && fixed_expert < 0 && L.n_experts > kInlineMaxE) return hipErrorInvalidValue;
  const int k = fixed_expert >= 0 ? 1 : L.top_k;
  const size_t lds = fused_lds_bytes(L, k, plan.SW);
  FusedParams P{L, table, router_w, router_bias, logits, fixed_expert, gate_in, x, part, idx_out, gate_out, plan.SW};
  static size_t granted[2] = {0, 0};
  const int v = L.x_bf16 ? 1 : 0;
  auto kernel = L.x_bf16 ? k_moe_decode<true> : k_moe_decode<false>;
  if (lds > 48 * 1024 && lds > granted[v]) {
    hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    granted[v] = lds;
  }
  hipLaunchKernelGGL(kernel, dim3(plan.n_slices, T), dim3(plan.threads), lds, st, P);
  return hipGetLastError();
}

hipError_t launch_reduce_partials(const float* part, int n_slices, int d, int32_t T, int accumulate, float* y,
                                  hipStream_t st) {
  hipLaunchKernelGGL(k_reduce_partials, dim3((d + 63) / 64, T), dim3(256), 0, st, part, n_slices, d, accumulate, y);
  return hipGetLastError();
}

hipError_t launch_transpose(const void* in, int64_t rows, int64_t cols, int elem_bytes, void* out, hipStream_t st) {
  const int64_t gx = (cols + 31) / 32, gy = (rows + 31) / 32;
  if (gx > 0x7fffffff || gy > 65535) return hipErrorInvalidValue;
  const dim3 grid((unsigned)gx, (unsigned)gy), block(256);
  if (elem_bytes == 4)
    hipLaunchKernelGGL(k_transpose<uint32_t>, grid, block, 0, st, (const uint32_t*)in, rows, cols, (uint32_t*)out);
  else if (elem_bytes == 2)
    hipLaunchKernelGGL(k_transpose<uint16_t>, grid, block, 0, st, (const uint16_t*)in, rows, cols, (uint16_t*)out);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace moeq
