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

#include <hip/hip_ext.h>

#include "decode_core.h"

namespace moeq {
namespace {

constexpr int kRbMax = 4;          // output row blocks (of 4 rows) per thread in phase 2
constexpr int kBurst = 8;          // 128-bit loads a thread issues back to back before it consumes them
constexpr int kInlineMaxE = 64;    // the router is evaluated in the kernel for at most this many experts
constexpr int kMaxSegs = 8;        // router work units per expert: d_model <= 2048 * kMaxSegs on the one-kernel path
constexpr int kTabLds = 64;        // expert records kept in LDS when the layer has at most this many experts

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
  const int32_t* route_idx;   // non-null: the routing is given, [T][k] expert indices (validated) ...
  const float* route_gate;    // ... and gates; no router runs
  const void* x;          // [T][d] in the layer's dtype
  float* part;            // [T][n_slices][d] partial outputs
  int32_t* idx_out;       // [T][k] or null
  float* gate_out;        // [T][k] or null
  int32_t SW;             // slice width (columns of d_ff): a multiple of 16 that divides the group size
  int32_t bits_mask;      // bitwidths present among the experts this call can pick (bit 1: INT2, 2: INT4, 3: INT8)
};

// Layout slot of a bitwidth: its rank among the bitwidths present in the layer.
__device__ __forceinline__ int layout_slot(int bits_mask, int bits) {
  const int bit = bits == 2 ? 1 : bits == 4 ? 2 : 3;
  return __popc((unsigned)bits_mask & ((1u << bit) - 1u));
}

// ---------------------------------------------------------------------------------------------
// Phase 1 of one expert: the rows [row_begin, row_begin + n_rows) of W_in (and W_gate) against the
// staged activations. P lanes share a row (RW = 64/P rows per wavefront load), J = chunks per lane
// and row. The tiles (one 128-bit load per lane, plus its scale) of a wavefront are grouped in bursts
// of RGB row groups x JC chunk steps x NM matrices (four tiles); a wavefront walks the bursts of its
// row-group sets (J/JC bursts per set) with two register sets: the loads of
// burst b+1 are issued before the arithmetic of burst b, so 4 to 8 loads per lane are always in flight.
template <int BITS, int NM, int JC, int RGB>
struct P1Burst {
  uint4 t[RGB][JC][NM];
  uint32_t sc[RGB][JC][NM];
};

template <int BITS, int NM, int JC, int RGB, typename Epilogue>
__device__ __forceinline__ void p1_stream(const uint8_t* const (&q)[NM], const uint8_t* const (&s)[NM], int d,
                                          int group, int row_begin, int n_rows, int P, int J, int lane, int wave,
                                          int nwaves, const uint32_t* XP, const float* XK, Epilogue epilogue) {
  constexpr int WPC = Fmt<BITS>::WPC, PPC = Fmt<BITS>::PPC;
  using Burst = P1Burst<BITS, NM, JC, RGB>;
  const int C = d / WPC;
  const int RW = 64 / P;
  const int n_rg = (n_rows + RW - 1) / RW;
  const int n_sets = (n_rg + RGB - 1) / RGB;
  const int JB = J / JC;                                                     // bursts per row-group set
  // Wavefront w owns the contiguous run of sets [w*spw, (w+1)*spw) and starts at a position that depends
  // on the workgroup: at any moment the loads of a workgroup are spread over its whole block of rows, and
  // those of different workgroups over different parts of theirs, which keeps all memory channels busy
  // (workgroups walking their blocks in lockstep would otherwise hit the same few channels together).
  const int spw = (n_sets + nwaves - 1) / nwaves;
  const int set_begin = wave * spw;
  const int my_sets = max(0, min(spw, n_sets - set_begin));
  const int rot = my_sets > 0 ? (int)blockIdx.x % my_sets : 0;
  const int nb = my_sets * JB;
  const int p = lane & (P - 1), rsub = lane / P;
  const uint32_t row_bytes = (uint32_t)C * 16u;
  const uint32_t ng2 = (uint32_t)(d / group) * 2u;
  const int gsh = group_shift(group);
  const bool two = (BITS == 2) && (group == 32);
  const uint4* XP4 = (const uint4*)XP;

  auto issue = [&](Burst& B, int b) __attribute__((always_inline)) {
    const int si = b / JB, j0 = (b - si * JB) * JC;
    const int sr = si + rot < my_sets ? si + rot : si + rot - my_sets;
    const int rg0 = (set_begin + sr) * RGB;
#pragma unroll
    for (int i = 0; i < RGB; ++i) {
      // rows past the slice are clamped: computed and dropped
      const uint32_t row = (uint32_t)(row_begin + min((rg0 + i) * RW + rsub, n_rows - 1));
      const uint32_t qoff = row * row_bytes + (uint32_t)p * 16u;
      const uint32_t soff = row * ng2;
#pragma unroll
      for (int jj = 0; jj < JC; ++jj) {
        const uint32_t c = (uint32_t)(p + (j0 + jj) * P);
        const uint32_t g0 = div_group(c * (uint32_t)WPC, group, gsh) * 2u;
#pragma unroll
        for (int m = 0; m < NM; ++m) {
          B.t[i][jj][m] = load_stream16(q[m] + (qoff + (uint32_t)(j0 + jj) * (uint32_t)P * 16u));
          if (two) B.sc[i][jj][m] = gload_u32(s[m] + (soff + g0));
          else B.sc[i][jj][m] = gload_u16(s[m] + (soff + g0));
        }
      }
    }
  };

  float tot[NM * RGB];
  auto compute = [&](const Burst& B, int b) __attribute__((always_inline)) {
    const int si = b / JB, j0 = (b - si * JB) * JC;
    const int sr = si + rot < my_sets ? si + rot : si + rot - my_sets;
    const int rg0 = (set_begin + sr) * RGB;
    if (j0 == 0) {
#pragma unroll
      for (int v = 0; v < NM * RGB; ++v) tot[v] = 0.f;
    }
    // Per chunk step, the two halves of the chunk one after the other, so that only half of the chunk's
    // activation pairs are in registers at a time. The offset term enters as the start value of the
    // dot-product chain; the factor 2^24 of the subnormal trick is applied once per row.
#pragma unroll
    for (int jj = 0; jj < JC; ++jj) {
      const int c = p + (j0 + jj) * P;
      float k0, k1 = 0.f;
      if (two) { k0 = XK[2 * c]; k1 = XK[2 * c + 1]; }
      else k0 = XK[c];
      float a[RGB][NM];
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        uint32_t xr[PPC / 2];
#pragma unroll
        for (int qq = 0; qq < PPC / 8; ++qq) {
          const uint4 t4 = XP4[(h * (PPC / 8) + qq) * C + c];
          xr[4 * qq] = t4.x; xr[4 * qq + 1] = t4.y; xr[4 * qq + 2] = t4.z; xr[4 * qq + 3] = t4.w;
        }
#pragma unroll
        for (int i = 0; i < RGB; ++i)
#pragma unroll
          for (int m = 0; m < NM; ++m) {
            const uint4 w = B.t[i][jj][m];
            const float start = h == 0 ? -k0 : (two ? -k1 : a[i][m]);
            float v = dword_dot<BITS>(h ? w.z : w.x, &xr[0], start);
            v = dword_dot<BITS>(h ? w.w : w.y, &xr[PPC / 4], v);
            a[i][m] = v;
            if (two) {
              const uint32_t sraw = B.sc[i][jj][m];
              tot[m * RGB + i] = fmaf(f16_bits_to_f32(h ? (sraw >> 16) : (sraw & 0xffffu)), v, tot[m * RGB + i]);
            }
          }
      }
      if (!two) {
#pragma unroll
        for (int i = 0; i < RGB; ++i)
#pragma unroll
          for (int m = 0; m < NM; ++m)
            tot[m * RGB + i] = fmaf(f16_bits_to_f32(B.sc[i][jj][m]), a[i][m], tot[m * RGB + i]);
      }
    }
    if (j0 + JC == J) {
      fold_rows<RGB, NM>(tot, P, lane);
      if (p < RGB && (rg0 + p) * RW + rsub < n_rows) {
        float r[NM];
#pragma unroll
        for (int m = 0; m < NM; ++m) r[m] = tot[m * RGB] * 16777216.0f;
        epilogue(row_begin + (rg0 + p) * RW + rsub, r);
      }
    }
  };

  Burst A, Bb;
  if (nb > 0) issue(A, 0);
  for (int b = 0; b < nb; b += 2) {
    if (b + 1 < nb) issue(Bb, b + 1);
    compute(A, b);
    if (b + 2 < nb) issue(A, b + 2);
    if (b + 1 < nb) compute(Bb, b + 1);
  }
}

// Phase 1 of one expert on the SW rows of its slice: the h values go to LDS as fp32 (HF); `up` undoes the
// normalisation of the staged activations.
template <int BITS, bool SWIGLU>
__device__ __forceinline__ void fused_in(const DevExpert* ex, int tid, int nwaves, int d, int group, int row_begin,
                                         int SW, float up, float* HF, const uint32_t* XP, const float* XK) {
  constexpr int NM = SWIGLU ? 2 : 1;
  const int C = d / Fmt<BITS>::WPC;
  const int P = lanes_per_row(C), J = C / P;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  auto epi = [&](int row, const float (&r)[NM]) __attribute__((always_inline)) {
    const float a = r[0] * up;
    float v;
    if constexpr (SWIGLU) v = a / (1.0f + __expf(-a)) * (r[NM - 1] * up);
    else v = fmaxf(a, 0.f);
    HF[row - row_begin] = v;
  };
  const uint8_t* q0 = uniform_ptr(ex->q_in);
  const uint8_t* s0 = (const uint8_t*)uniform_ptr(ex->s_in);
  const uint8_t* q1 = SWIGLU ? uniform_ptr(ex->q_gate) : nullptr;
  const uint8_t* s1 = SWIGLU ? (const uint8_t*)uniform_ptr(ex->s_gate) : nullptr;
  auto run = [&](auto jc_tag, auto rgb_tag) __attribute__((always_inline)) {
    constexpr int JC = decltype(jc_tag)::value, RGB = decltype(rgb_tag)::value;
    if constexpr (SWIGLU) {
      const uint8_t* const qq[2] = {q0, q1};
      const uint8_t* const ss[2] = {s0, s1};
      p1_stream<BITS, 2, JC, RGB>(qq, ss, d, group, row_begin, SW, P, J, lane, wave, nwaves, XP, XK, epi);
    } else {
      const uint8_t* const qq[1] = {q0};
      const uint8_t* const ss[1] = {s0};
      p1_stream<BITS, 1, JC, RGB>(qq, ss, d, group, row_begin, SW, P, J, lane, wave, nwaves, XP, XK, epi);
    }
  };
  // A burst is four tiles: two chunk steps when a row has an even number of them, and as many row groups
  // as that leaves room for - one only when the fold could not take more (it needs RGB <= P).
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  using I4 = std::integral_constant<int, 4>;
  constexpr int RGB1 = 4 / NM, RGB2 = 2 / NM;   // row groups per burst at JC = 1 and JC = 2
  if (J % 2 == 0) {
    if constexpr (RGB2 > 1) { if (P >= RGB2) { run(I2{}, std::integral_constant<int, RGB2>{}); return; } }
    run(I2{}, I1{});
  } else {
    if (P >= RGB1) { run(I1{}, std::integral_constant<int, RGB1>{}); return; }
    run(I1{}, I1{});
  }
}

// ---------------------------------------------------------------------------------------------
// Between the phases (all threads, between two barriers): the h slice of every chosen expert (fp32 in HF) is
// normalised by its own power of two (stage_normalised's rule, over the SW values of the slice), converted to
// binary16 and stored linear (HL) and in the pair layout of the expert's bitwidth (HP); uph[j] receives the
// factor that undoes the normalisation. One wavefront per expert, SW <= 256.
__device__ __forceinline__ void stage_h_slices(const float* HF, int k, int SW, const DevExpert* tabp, const int* sel_e,
                                               uint16_t* HLs, uint16_t* HPs, float* uph, int lane, int wave,
                                               int nwaves) {
  for (int j = wave; j < k; j += nwaves) {
    const int bits = __builtin_amdgcn_readfirstlane(tabp[sel_e[j]].bits);
    float v[4];
    float m = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = lane + 64 * i;
      v[i] = c < SW ? HF[j * SW + c] : 0.f;
      m = fmaxf(m, fabsf(v[i]));
    }
    const int e = norm_exponent(wave_max(m));
    const float dn = pow2f(-e);
    uint16_t* HL = HLs + j * SW;
    uint16_t* HP = HPs + j * SW;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = lane + 64 * i;
      if (c < SW) {
        const uint32_t hb = f32_to_f16_bits(v[i] * dn);
        HL[c] = (uint16_t)hb;
        float ps;
        const int si = bits == 2 ? slice_pair_index<2>(c, ps) : bits == 4 ? slice_pair_index<4>(c, ps)
                                                                          : slice_pair_index<8>(c, ps);
        HP[si] = (uint16_t)f32_to_f16_bits(f16_bits_to_f32(hb) * ps);
      }
    }
    if (lane == 0) uph[j] = pow2f(e);
  }
}

// ---------------------------------------------------------------------------------------------
// Phase 2 of one expert: Y[row] (+)= gate * s[row][grp] * sum_{col in slice} (u - 2^(b-1)) * h[col] for the
// thread's row blocks rb = tid + i*nthreads (4 rows each). qT/sT are the dword-column-major codes and
// scales of W_out; Y is the workgroup's partial output vector in LDS (every row block has one owner, so
// no synchronisation is needed on it). A burst is RBC row blocks x DWC words; the first burst's loads
// are issued by p2_issue before the barrier that completes h, the rest inside fused_out.
template <int BITS, int DWC>
struct P2Burst {
  static constexpr int RBC = (kBurst / DWC) < kRbMax ? (kBurst / DWC) : kRbMax;
  uint4 t[RBC][DWC];
  uint2 sc[RBC];
};

// qT_w: the codes at word column w_first (uniform); a tile is at qT_w + w * d*4 + rb*16.
template <int BITS, int DWC>
__device__ __forceinline__ void p2_issue(P2Burst<BITS, DWC>& b, const uint8_t* qT_w, const uint8_t* sT_g, int d,
                                         int nrb, int tid, int nthreads, int i0, bool want_scales) {
  constexpr int RBC = P2Burst<BITS, DWC>::RBC;
#pragma unroll
  for (int i = 0; i < RBC; ++i) {
    const int rb = tid + (i0 + i) * nthreads;
    if (rb < nrb) {
      if (want_scales) b.sc[i] = gload_u32x2(sT_g + (uint32_t)rb * 8u);
#pragma unroll
      for (int w = 0; w < DWC; ++w)
        b.t[i][w] = load_stream16(qT_w + (size_t)w * ((size_t)d * 4) + (uint32_t)rb * 16u);
    }
  }
}

template <int BITS, int DWC>
__device__ __forceinline__ void fused_out(P2Burst<BITS, DWC>& first, const uint8_t* qT_s, const uint8_t* sT_g,
                                          int tid, int nthreads, int d, int SW, float gate, bool first_expert,
                                          const uint16_t* HL, const uint16_t* HP, float4* Y) {
  constexpr int CPD = 32 / BITS, PPD = CPD / 2;
  constexpr int RBC = P2Burst<BITS, DWC>::RBC;
  const int lane = tid & 63;
  const int DW = SW / CPD;              // a multiple of DWC
  // offset term: 2^(b-1) * 2^-24 * (sum of the slice's activations), the same in every wavefront
  float hs = 0.f;
  for (int c = lane; c < SW; c += 64) hs += f16_bits_to_f32(HL[c]);
  hs = wave_sum(hs);
  const float K = hs * (Fmt<BITS>::OFF * 5.9604644775390625e-08f);
  const uint32_t* HPw = (const uint32_t*)HP;
  const int nrb = d / 4;
  const int RB = (nrb + nthreads - 1) / nthreads;
  auto consume = [&](const P2Burst<BITS, DWC>& cur, int wb, float (&acc)[RBC][4]) __attribute__((always_inline)) {
#pragma unroll
    for (int w = 0; w < DWC; ++w) {
      __builtin_amdgcn_sched_barrier(0);   // one word column at a time: bounds the live pair registers
      uint32_t xr[PPD];
#pragma unroll
      for (int pp = 0; pp < PPD; ++pp) xr[pp] = HPw[(wb + w) * PPD + pp];
#pragma unroll
      for (int i = 0; i < RBC; ++i) {
        acc[i][0] = dword_dot<BITS>(cur.t[i][w].x, xr, acc[i][0]);
        acc[i][1] = dword_dot<BITS>(cur.t[i][w].y, xr, acc[i][1]);
        acc[i][2] = dword_dot<BITS>(cur.t[i][w].z, xr, acc[i][2]);
        acc[i][3] = dword_dot<BITS>(cur.t[i][w].w, xr, acc[i][3]);
      }
    }
  };
#pragma unroll
  for (int i0 = 0; i0 < kRbMax; i0 += RBC) {
    if (i0 < RB) {
      float acc[RBC][4];
#pragma unroll
      for (int i = 0; i < RBC; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[i][r] = 0.f;
      uint2 sc[RBC];
      // first burst of this row-block set: the one issued before the barrier, or a fresh one
      {
        P2Burst<BITS, DWC> cur;
        if (i0 != 0) p2_issue<BITS, DWC>(cur, qT_s, sT_g, d, nrb, tid, nthreads, i0, true);
        const P2Burst<BITS, DWC>& use = (i0 == 0) ? first : cur;
#pragma unroll
        for (int i = 0; i < RBC; ++i) sc[i] = use.sc[i];
        consume(use, 0, acc);
      }
      for (int wb = DWC; wb < DW; wb += DWC) {
        P2Burst<BITS, DWC> cur;
        p2_issue<BITS, DWC>(cur, qT_s + (size_t)wb * ((size_t)d * 4), sT_g, d, nrb, tid, nthreads, i0, false);
        consume(cur, wb, acc);
      }
#pragma unroll
      for (int i = 0; i < RBC; ++i) {
        const int rb = tid + (i0 + i) * nthreads;
        if (rb < nrb) {
          float4 y = first_expert ? make_float4(0.f, 0.f, 0.f, 0.f) : Y[rb];
          // (acc - K) * 2^24 is the sum in the normalised domain; the gate carries the factor that undoes the
          // normalisation of h
          y.x = fmaf(f16_bits_to_f32(sc[i].x & 0xffffu) * gate, (acc[i][0] - K) * 16777216.0f, y.x);
          y.y = fmaf(f16_bits_to_f32(sc[i].x >> 16) * gate, (acc[i][1] - K) * 16777216.0f, y.y);
          y.z = fmaf(f16_bits_to_f32(sc[i].y & 0xffffu) * gate, (acc[i][2] - K) * 16777216.0f, y.z);
          y.w = fmaf(f16_bits_to_f32(sc[i].y >> 16) * gate, (acc[i][3] - K) * 16777216.0f, y.w);
          Y[rb] = y;
        }
      }
    }
  }
}

// Phase 2 of one expert of one (slice, token). The first expert's call holds the barriers between the
// phases and, between them, the staging of h (`between`); its first burst does not depend on h and is in
// flight across them. gate: the expert's gate times the factor that undoes the normalisation of its h,
// read through a pointer because it is known only after the staging.
template <int BITS, int DWC, typename Between>
__device__ __forceinline__ void fused_expert_out(const DevExpert* ex, int tid, int nthreads, int d, int group,
                                                 int slice, int SW, float gate_j, const float* uph_j,
                                                 bool first_expert, const uint16_t* HL, const uint16_t* HP, float4* Y,
                                                 Between between) {
  // first_expert: the call that also waits for phase 1 (of every expert) to be complete
  constexpr int CPD = 32 / BITS;
  // this slice's first word column of the codes, and its scale group, as uniform pointers
  const uint8_t* qT_s = uniform_ptr(ex->q_out) + (size_t)(slice * (SW / CPD)) * ((size_t)d * 4);
  const uint8_t* sT_g = (const uint8_t*)uniform_ptr(ex->s_out) + (size_t)((slice * SW) / group) * ((size_t)d * 2);
  P2Burst<BITS, DWC> first;
  p2_issue<BITS, DWC>(first, qT_s, sT_g, d, d / 4, tid, nthreads, 0, true);
  if (first_expert) {
    __syncthreads();  // the h slices of all chosen experts are complete in LDS (fp32)
    between();        // normalised, converted, put in pair order
    __syncthreads();
  }
  fused_out<BITS, DWC>(first, qT_s, sT_g, tid, nthreads, d, SW, gate_j * *uph_j, first_expert, HL, HP, Y);
}

// ---------------------------------------------------------------------------------------------
// Matrix-core variant of the two phases. Unpacking costs half a vector instruction per weight, the
// multiply-accumulate another half; handing the second half to the matrix cores (which otherwise idle)
// about halves the vector work, which is what bounds this kernel at 2 and 4 bits. One
// v_mfma_f32_16x16x32_f16 computes D[token][row] += sum_k X[token][k] * W[row][k] for 16 rows and 32
// values of k: lane l supplies 8 consecutive k (block kb = l/16) of weight row n = l%16 as the B operand,
// the activations are the A operand (all 16 token rows carry the same single token here), and the
// result for weight row n arrives in lane n, element 0. The weights enter exactly as in the vector
// path: masked code fields read as binary16 subnormals (the matrix cores honour them) against
// activations pre-divided by the fields' powers of two, in the same staged pair order; the reduction
// over k happens inside the instruction, so no cross-lane folding is needed.
constexpr int kMxSlice = 64;   // slice width of the matrix-core variant

// Phase 1 on the matrix cores, with the same coalesced row reads as the vector path. A tile is a
// contiguous run of a row covering 16 lane columns x 4 k blocks: 1 KB (2048 columns at 4 bits, 1024 at 8
// bits) read as 16 bytes per lane, or 512 bytes (2048 columns at 2 bits) read as 8 bytes per lane. Lane
// (n, kb) takes the piece 4*n + kb of the run, so that the four lanes the instruction sums over (same n)
// hold four consecutive pieces: 128 columns (64 at 8 bits), inside one scale group. Since every lane
// column n then covers a different range of k, the activations go in with the A-operand row m holding the
// activations of column group m: D[m][n] is the dot product of weight group n with activation group m, and
// the useful results are the diagonal m == n (16 group dot products per instruction chain), found in lane
// n + 16*(n/4), element n%4. Each diagonal lane scales its group's dot product with its own group scale
// and accumulates; a wavefront sum per row finishes the dot product.
//
// The rows of the slice, for all chosen experts, form one list of tasks (expert, then row); a task is the
// row's bursts (a burst = two tiles of each matrix). Wavefront w takes the tasks w, w + nwaves, ... Two
// register sets alternate: both are requested ahead, the set that was just consumed is requested again
// at once, and since the list does not stop at the change of expert the loads never drain there. Past
// the end of the list a wavefront requests a few bytes of the activation vector instead (cached, ignored),
// so that the loop holds no condition around its loads: every path issues the same number, and the
// arithmetic of a set waits for that set alone.
// The hardware serves the oldest wavefront of a SIMD first, which lets the four wavefronts of a SIMD drift
// apart by a third of the phase; each wavefront therefore lowers its own priority as its list gets
// shorter, so that the ones that are behind are served first and all reach the barrier together.
// (Handing tasks out through a counter in LDS was tried: the LDS atomics alone cost more than the drift.)
struct MxSet1 { uint4 t[2][2]; uint32_t sc[2][2]; };   // [tile of the burst][matrix]

struct MxTag1 { int valid, t, j, r, jb, bits, JB; };   // what a requested set holds: task, expert slot, row, burst

struct MxWalk1 {          // the next burst to request, and what the bursts of that expert need
  int t, valid, j, r, jb; // task, task in range; expert slot, row of the slice, burst of the row
  int bits, JB;           // of the expert at slot j: its bitwidth and bursts per row
  // the same load instructions serve every bitwidth, the differences are in these values
  const uint8_t* q[2];
  const uint8_t* s[2];
  uint32_t row_bytes, tile_bytes, tile_groups2;   // bytes of a row, of a tile; 2 * scale groups of a tile
  uint32_t lane_off, lane_g2;                     // per lane: byte offset in a tile, 2 * group of its piece in a tile
};

template <bool SWIGLU>
__device__ __forceinline__ void mx1_enter(MxWalk1& w, const DevExpert* ex, int d, int gsh, int lane) {
  w.bits = __builtin_amdgcn_readfirstlane(ex->bits);
  w.JB = d / (w.bits == 8 ? 2048 : 4096);
  w.q[0] = uniform_ptr(ex->q_in);
  w.s[0] = (const uint8_t*)uniform_ptr(ex->s_in);
  if constexpr (SWIGLU) {
    w.q[1] = uniform_ptr(ex->q_gate);
    w.s[1] = (const uint8_t*)uniform_ptr(ex->s_gate);
  } else {
    w.q[1] = w.q[0];
    w.s[1] = w.s[0];
  }
  const int m = lane & 15, kb = lane >> 4;
  w.row_bytes = (uint32_t)d * (uint32_t)w.bits / 8u;
  w.tile_bytes = w.bits == 2 ? 512u : 1024u;
  w.tile_groups2 = ((w.bits == 8 ? 1024u : 2048u) >> gsh) * 2u;
  // 2-bit codes: the lane's piece is 8 bytes at 32*m + 8*kb; it reads the aligned 16 bytes that hold it
  w.lane_off = w.bits == 2 ? (uint32_t)(32 * m + 16 * (kb >> 1)) : (uint32_t)(4 * m + kb) * 16u;
  const uint32_t lane_col = w.bits == 2 ? (uint32_t)(128 * m) : (uint32_t)(4 * m + kb) * (128u / (uint32_t)w.bits);
  w.lane_g2 = (lane_col >> gsh) * 2u;
}

// Requests the burst at w (two tiles of each matrix and the scales of the lane's pieces) and notes in tag
// what the set will hold. row0 = first row of the slice, ng2 = bytes of a row of scales; idle = cached
// bytes (at least 2 KB + 1 KB) to read when the list is exhausted.
template <int NM>
__device__ __forceinline__ void mx1_issue(MxSet1& S, MxTag1& tag, const MxWalk1& w, uint32_t row0, uint32_t ng2,
                                          const uint8_t* idle, int lane) {
  tag.valid = w.valid; tag.t = w.t; tag.j = w.j; tag.r = w.r; tag.jb = w.jb; tag.bits = w.bits; tag.JB = w.JB;
  const uint32_t row = row0 + (uint32_t)w.r, t0 = (uint32_t)w.jb * 2u;
  const uint32_t qoff = w.valid ? row * w.row_bytes + t0 * w.tile_bytes + w.lane_off : (uint32_t)lane * 16u;
  const uint32_t soff = w.valid ? row * ng2 + t0 * w.tile_groups2 + w.lane_g2 : (uint32_t)lane * 2u;
#pragma unroll
  for (int jj = 0; jj < 2; ++jj)
#pragma unroll
    for (int mm = 0; mm < NM; ++mm) {
      const uint8_t* qb = w.valid ? w.q[mm] : idle;
      const uint8_t* sb = w.valid ? w.s[mm] : idle;
      S.t[jj][mm] = load_stream16(qb + (qoff + (jj ? w.tile_bytes : 0u)));
      S.sc[jj][mm] = gload_u16(sb + (soff + (jj ? w.tile_groups2 : 0u)));
    }
}

// The arithmetic of one burst: adds the lane's share of the row's dot products to acc. dm[i] is 1 in the
// lane that holds a diagonal result in element i, else 0. KS holds the negated offset terms of the lane
// column ranges: the accumulation of D[m][.] starts there, so the diagonal comes out with its offset
// already taken off (the other entries are never looked at).
template <int BITS, int NM>
__device__ __forceinline__ void mx1_burst(const MxSet1& S, int jb, int d, int lane, const float (&dm)[4],
                                          const uint4* XP4, const float* KS, float (&acc)[NM]) {
  constexpr int WPC = 128 / BITS;
  const int C = d / WPC;
  const int m = lane & 15, kb = lane >> 4;
#pragma unroll
  for (int jj = 0; jj < 2; ++jj) {
    const int j = jb * 2 + jj;
    const float4 k4 = *(const float4*)(KS + 16 * j + 4 * kb);
    const float4_t init = {k4.x, k4.y, k4.z, k4.w};
    float4_t D[NM];
#pragma unroll
    for (int mm = 0; mm < NM; ++mm) D[mm] = init;
    if constexpr (BITS == 2) {
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
          const half8_t A = as_half8(XP4[(2 * (2 * (kb & 1) + t) + hh) * C + 32 * j + 2 * m + (kb >> 1)]);
#pragma unroll
          for (int mm = 0; mm < NM; ++mm) {
            // the lane's 8 bytes are the upper half of the 16 loaded ones when kb is odd
            const uint4 wd = S.t[jj][mm];
            const uint32_t dw = t ? ((kb & 1) ? wd.w : wd.y) : ((kb & 1) ? wd.z : wd.x);
            D[mm] = mfma16(A, hh ? codes8<2, 1>(dw, 0u) : codes8<2, 0>(dw, 0u), D[mm]);
          }
        }
    } else {
      constexpr int NI = BITS == 4 ? 4 : 2;
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const half8_t A = as_half8(XP4[i * C + 64 * j + 4 * m + kb]);
#pragma unroll
        for (int mm = 0; mm < NM; ++mm) {
          const uint4 wd = S.t[jj][mm];
          if constexpr (BITS == 4) D[mm] = mfma16(A, codes8<4, 0>(i == 0 ? wd.x : i == 1 ? wd.y : i == 2 ? wd.z : wd.w, 0u), D[mm]);
          else D[mm] = mfma16(A, i == 0 ? codes8<8, 0>(wd.x, wd.y) : codes8<8, 0>(wd.z, wd.w), D[mm]);
        }
      }
    }
#pragma unroll
    for (int mm = 0; mm < NM; ++mm) {
      // exactly one of the four products is non-zero in a diagonal lane, none elsewhere
      const float dv = fmaf(D[mm][3], dm[3], fmaf(D[mm][2], dm[2], fmaf(D[mm][1], dm[1], D[mm][0] * dm[0])));
      acc[mm] = fmaf(f16_bits_to_f32(S.sc[jj][mm]), dv, acc[mm]);
    }
  }
}

// Activation of one row of the slice (r: its pre-activations, normalisation of x already undone).
template <bool SWIGLU, int NM>
__device__ __forceinline__ float mx1_activation(const float (&r)[NM]) {
  if constexpr (SWIGLU) return r[0] / (1.0f + __expf(-r[0])) * r[NM - 1];
  else return fmaxf(r[0], 0.f);
}

// One requested burst: the arithmetic, and, when it completes a row, the sum of the lanes' shares over the
// 16-lane rows of the wavefront; the lanes i, 16 + i, 32 + i, 48 + i keep these four partial sums of the
// wavefront's i-th finished row (rows_done counts them, at most 16), and the caller adds them and applies the
// activation to all rows at once (every 16 rows and when the list is through).
template <int BITS, bool SWIGLU>
__device__ __forceinline__ void mx1_compute(const MxSet1& S, const MxTag1& tag, int d, int lane, const float (&dm)[4],
                                            const uint32_t* XP, const float* KS, float (&acc)[SWIGLU ? 2 : 1],
                                            float (&keep)[SWIGLU ? 2 : 1], int& rows_done) {
  constexpr int NM = SWIGLU ? 2 : 1;
  if (tag.jb == 0) {
#pragma unroll
    for (int mm = 0; mm < NM; ++mm) acc[mm] = 0.f;
  }
  mx1_burst<BITS, NM>(S, tag.jb, d, lane, dm, (const uint4*)XP, KS, acc);
  if (tag.jb + 1 == tag.JB) {
#pragma unroll
    for (int mm = 0; mm < NM; ++mm) {
      // sums over the four 16-lane rows of the wavefront; the four of them are added when the rows are flushed
      float r = acc[mm];
      r += dpp<kDppXor1>(r);
      r += dpp<kDppXor2>(r);
      r += dpp<kDppRor4>(r);
      r += dpp<kDppRor8>(r);
      keep[mm] = (lane & 15) == rows_done ? r : keep[mm];
    }
    ++rows_done;
  }
}

// Phase 2 on the matrix cores: a wavefront takes groups of 64 output rows; lane (n, kb) loads the 16-byte
// tile with word column 4*step + kb (8-bit codes: the word columns 8*step + 2*kb and + 1) of the rows
// 64*g + 4*n .. + 3, and instruction i multiplies row 4*n + i of every lane (here all A-operand rows
// carry the same activations and the result for row n of the instruction arrives in lane n, element 0).
// A register set holds four tiles: the tiles of GPS row groups. As in phase 1 the wavefront walks one
// list of sets through all chosen experts with two register sets; the first set is requested before the
// barrier that completes h.
struct MxSet2 { uint4 t[4]; uint2 sc[4]; };

template <int BITS>
struct P2Mx {
  static constexpr int DW = kMxSlice * BITS / 32;                   // word columns of a slice: 4 / 8 / 16
  static constexpr int TPR = BITS == 2 ? 1 : (BITS == 4 ? 2 : 4);   // tiles per row group and lane
  static constexpr int GPS = 4 / TPR;                               // row groups per register set
};

struct MxWalk2 {
  int j, set, n_sets, bits;      // expert slot, set of the expert, its number of sets
  // for the loads only (one instruction sequence for every bitwidth):
  const uint8_t* qT_s;           // the slice's first word column of the expert's W_out
  const uint8_t* sT_g;           // the slice's scale row
  uint32_t slot_q[4], slot_s[4]; // byte offsets of the four tiles / scale vectors of a set
  uint32_t set_q, set_s;         // byte strides from set to set
  uint32_t lane_q, lane_s;       // per lane
};

__device__ __forceinline__ void mx2_enter(MxWalk2& w, const DevExpert* ex, int d, int slice, int gsh, int lane,
                                          int wave, int nwaves) {
  w.bits = __builtin_amdgcn_readfirstlane(ex->bits);
  const int dw = kMxSlice * w.bits / 32;
  const int tpr = w.bits == 2 ? 1 : (w.bits == 4 ? 2 : 4), gps = 4 / tpr;
  w.qT_s = uniform_ptr(ex->q_out) + (size_t)(slice * dw) * ((size_t)d * 4);
  w.sT_g = (const uint8_t*)uniform_ptr(ex->s_out) + (size_t)((slice * kMxSlice) >> gsh) * ((size_t)d * 2);
  w.n_sets = (d >> 6) / (gps * nwaves);
  w.set = 0;
  const int n = lane & 15, kb = lane >> 4;
  const uint32_t col_bytes = (uint32_t)d * 4u;           // bytes of a word column
#pragma unroll
  for (int sl = 0; sl < 4; ++sl) {
    const int i = sl / tpr, tt = sl - i * tpr;           // row group of the set, tile of the row group
    const int wc = w.bits == 8 ? 8 * (tt >> 1) + (tt & 1) : 4 * tt;
    w.slot_q[sl] = (uint32_t)wc * col_bytes + (uint32_t)(i * nwaves) * 256u;
    w.slot_s[sl] = (uint32_t)((sl % gps) * nwaves) * 128u;   // slots past the set's row groups repeat one
  }
  w.set_q = (uint32_t)(gps * nwaves) * 256u;
  w.set_s = (uint32_t)(gps * nwaves) * 128u;
  w.lane_q = (uint32_t)(w.bits == 8 ? 2 * kb : kb) * col_bytes + (uint32_t)(64 * wave + 4 * n) * 4u;
  w.lane_s = (uint32_t)(64 * wave + 4 * n) * 2u;
}

// Row groups of a set: wave + (set * GPS + i) * nwaves, all below d / 64 (the plan makes d / 64 a multiple
// of 4 * nwaves).
__device__ __forceinline__ void mx2_issue(MxSet2& S, const MxWalk2& w) {
  const uint32_t q0 = w.lane_q + (uint32_t)w.set * w.set_q;
  const uint32_t s0 = w.lane_s + (uint32_t)w.set * w.set_s;
#pragma unroll
  for (int sl = 0; sl < 4; ++sl) {
    S.t[sl] = load_stream16(w.qT_s + (q0 + w.slot_q[sl]));
    S.sc[sl] = gload_u32x2(w.sT_g + (s0 + w.slot_s[sl]));
  }
}

template <int BITS>
__device__ __forceinline__ void mx2_compute(const MxSet2& S, const MxWalk2& w, int d, int lane, int wave, int nwaves,
                                            const uint4* HP4, float K, float gu, float4* Y) {
  constexpr int TPR = P2Mx<BITS>::TPR, GPS = P2Mx<BITS>::GPS;
  const int n = lane & 15, kb = lane >> 4;
  const float4_t zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < GPS; ++i) {
    const int g = wave + (w.set * GPS + i) * nwaves;
    {
      float4_t D[4] = {zero, zero, zero, zero};
      if constexpr (BITS == 4) {
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          const half8_t A = as_half8(HP4[4 * tt + kb]);
          const uint4 t = S.t[i * TPR + tt];
          D[0] = mfma16(A, codes8<4, 0>(t.x, 0u), D[0]);
          D[1] = mfma16(A, codes8<4, 0>(t.y, 0u), D[1]);
          D[2] = mfma16(A, codes8<4, 0>(t.z, 0u), D[2]);
          D[3] = mfma16(A, codes8<4, 0>(t.w, 0u), D[3]);
        }
      } else if constexpr (BITS == 2) {
        const half8_t A0 = as_half8(HP4[2 * kb]), A1 = as_half8(HP4[2 * kb + 1]);
        const uint4 t = S.t[i];
        D[0] = mfma16(A0, codes8<2, 0>(t.x, 0u), D[0]); D[0] = mfma16(A1, codes8<2, 1>(t.x, 0u), D[0]);
        D[1] = mfma16(A0, codes8<2, 0>(t.y, 0u), D[1]); D[1] = mfma16(A1, codes8<2, 1>(t.y, 0u), D[1]);
        D[2] = mfma16(A0, codes8<2, 0>(t.z, 0u), D[2]); D[2] = mfma16(A1, codes8<2, 1>(t.z, 0u), D[2]);
        D[3] = mfma16(A0, codes8<2, 0>(t.w, 0u), D[3]); D[3] = mfma16(A1, codes8<2, 1>(t.w, 0u), D[3]);
      } else {
#pragma unroll
        for (int st = 0; st < 2; ++st) {
          const half8_t A = as_half8(HP4[4 * st + kb]);
          const uint4 t0 = S.t[2 * st], t1 = S.t[2 * st + 1];
          D[0] = mfma16(A, codes8<8, 0>(t0.x, t1.x), D[0]);
          D[1] = mfma16(A, codes8<8, 0>(t0.y, t1.y), D[1]);
          D[2] = mfma16(A, codes8<8, 0>(t0.z, t1.z), D[2]);
          D[3] = mfma16(A, codes8<8, 0>(t0.w, t1.w), D[3]);
        }
      }
      if (lane < 16) {
        float4 y = w.j == 0 ? make_float4(0.f, 0.f, 0.f, 0.f) : Y[16 * g + n];
        // (D - K) * 2^24 is the sum in the normalised domain; gu = gate * the factor that undoes h's normalisation
        y.x = fmaf(f16_bits_to_f32(S.sc[i].x & 0xffffu) * gu, (D[0][0] - K) * 16777216.0f, y.x);
        y.y = fmaf(f16_bits_to_f32(S.sc[i].x >> 16) * gu, (D[1][0] - K) * 16777216.0f, y.y);
        y.z = fmaf(f16_bits_to_f32(S.sc[i].y & 0xffffu) * gu, (D[2][0] - K) * 16777216.0f, y.z);
        y.w = fmaf(f16_bits_to_f32(S.sc[i].y >> 16) * gu, (D[3][0] - K) * 16777216.0f, y.w);
        Y[16 * g + n] = y;
      }
    }
  }
}

// MAXT: the largest workgroup the variant is launched with (small layers run 256 threads and then have four
// times the registers per thread).
template <bool SWIGLU, bool MX, int MAXT = 1024>
__global__ __launch_bounds__(MAXT) void k_moe_decode(FusedParams P) {
  extern __shared__ uint32_t smem[];
  __shared__ int sel_e[8];
  __shared__ float sel_g[8];
  __shared__ int sel_b[8];                                // bitwidths of the chosen experts
  __shared__ float rpart[kInlineMaxE * (kMaxSegs + 1)];   // router partial sums, unit u = e * n_seg + seg
  __shared__ DevExpert tab[kTabLds];
  __shared__ float red[16];                               // per-wavefront maxima of |x|
  __shared__ float uph[8];                                // per chosen expert: undoes the normalisation of its h slice
  const LayerDims& L = P.L;
  const int d = L.d_model, E = L.n_experts, SW = P.SW;
  const int token = blockIdx.y;
  // Workgroups are handed to the eight XCDs in turn (workgroup number modulo 8), each with its own L2. XCD x
  // gets the contiguous slices x * G/8 .. (x+1) * G/8 - 1: neighbouring slices share the scale vectors of a
  // W_out group and read adjacent rows of W_in, which then meet in one L2 (35.3 against 36.0 us per launch).
  const int slice = (gridDim.x & 7u) == 0 ? (int)((blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3))
                                          : (int)blockIdx.x;
  const int nthreads = blockDim.x, nwaves = nthreads >> 6;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int k = P.fixed_expert >= 0 ? 1 : L.top_k;
  const int lay_words = d / 2 + d / 16;
  const bool bf16 = L.x_bf16 != 0;
  uint16_t* RAW = (uint16_t*)smem;                 // [d] activations, linear binary16
  uint16_t* HLs = RAW + d;                         // [k][SW] h of every chosen expert, linear binary16
  uint16_t* HPs = HLs + k * SW;                    // [k][SW] the same in the pair layout of the expert's bitwidth
  float4* Y = (float4*)(HPs + k * SW);             // [d/4] this workgroup's partial output vector
  float* HF = (float*)(Y + d / 4);                 // [k][SW] h of every chosen expert as phase 1 leaves it (fp32)
  uint32_t* LAY = (uint32_t*)(HF + k * SW);        // [#bitwidths][lay_words] staged activations
  const char* xt = (const char*)P.x + (size_t)token * d * (bf16 ? 2 : 4);
  const bool routed = P.fixed_expert < 0;
  const bool given = routed && P.route_idx != nullptr;
  const bool inline_router = routed && !P.logits && !given;
  const bool tab_in_lds = routed && E <= kTabLds;

  // ---- everything that depends on nothing but the inputs is requested at once: the activations, the
  // expert records, the router rows
  // The activations: a thread's first 8 values stay in registers until the largest magnitude of the vector is
  // known (stage_normalised's scheme, spread over the prologue so that its loads share a memory round trip with
  // the router's).
  const int xkind = bf16 ? X_BF16 : X_F32;
  const int n_items = d / 8;
  XItem xit;
#pragma unroll
  for (int q = 0; q < 8; ++q) xit.v[q] = 0.f;
  bool staged = false;
  auto stage_inputs = [&]() __attribute__((always_inline)) {
    if ((int)threadIdx.x < n_items) xit = load_x_item(xt, xkind, threadIdx.x);
    if (tab_in_lds && (int)threadIdx.x < E * 4) ((uint4*)tab)[threadIdx.x] = ((const uint4*)P.table)[threadIdx.x];
    staged = true;
  };
  // router work unit = (expert, segment of seg_cols columns), one wavefront each; segments are sized so
  // that the units about fill the wavefronts, at most eight 128-bit loads of the router row per lane
  int n_seg = (d + 2047) / 2048;
  if (inline_router) {
    while (n_seg * 2 <= kMaxSegs && E * n_seg * 2 <= nwaves && d >= n_seg * 2 * 256) n_seg *= 2;
    const int seg_cols = ((d + n_seg - 1) / n_seg + 255) / 256 * 256;
    for (int u = wave; u < E * n_seg; u += nwaves) {
      const int e = u / n_seg, seg = u - e * n_seg;
      const float* wr = P.Wr + (size_t)e * d;
      const int c_end = min(d, (seg + 1) * seg_cols);
      float4 w[8], v[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int i = seg * seg_cols + q * 256 + lane * 4;
        w[q] = make_float4(0.f, 0.f, 0.f, 0.f);
        v[q] = w[q];
        if (i < c_end) {
          w[q] = *(const float4*)(wr + i);
          if (bf16) {
            const uint2 b = *(const uint2*)((const uint16_t*)xt + i);
            v[q] = make_float4(bf16_bits_to_f32(b.x & 0xffffu), bf16_bits_to_f32(b.x >> 16),
                               bf16_bits_to_f32(b.y & 0xffffu), bf16_bits_to_f32(b.y >> 16));
          } else {
            v[q] = *(const float4*)((const float*)xt + i);
          }
        }
      }
      if (!staged) stage_inputs();   // behind the router loads: one memory round trip for both
      float acc = 0.f;
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        acc = fmaf(w[q].x, v[q].x, acc); acc = fmaf(w[q].y, v[q].y, acc);
        acc = fmaf(w[q].z, v[q].z, acc); acc = fmaf(w[q].w, v[q].w, acc);
      }
      acc = wave_sum(acc);
      if (lane == 0) rpart[u] = acc;
    }
  }
  if (!staged) stage_inputs();
  {
    float m = item_absmax(xit);
    for (int i = threadIdx.x + nthreads; i < n_items; i += nthreads) m = fmaxf(m, item_absmax(load_x_item(xt, xkind, i)));
    m = wave_max(m);
    if (lane == 0) red[wave] = m;
  }
  __syncthreads();  // red, tab, rpart are complete
  float up;         // undoes the normalisation of the activations
  {
    float M = 0.f;
    for (int w = 0; w < nwaves; ++w) M = fmaxf(M, red[w]);
    const int e = norm_exponent(M);
    const float dn = pow2f(-e);
    up = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, pow2f(e))));   // uniform
    uint4* RAW4 = (uint4*)RAW;
    if ((int)threadIdx.x < n_items) RAW4[threadIdx.x] = item_to_f16(xit, dn);
    for (int i = threadIdx.x + nthreads; i < n_items; i += nthreads) RAW4[i] = item_to_f16(load_x_item(xt, xkind, i), dn);
  }
  __syncthreads();  // RAW is complete

  // ---- wavefront 0 turns the router sums into the top-k while the others stage the activations for
  // every bitwidth the layer holds (the staging does not depend on the routing)
  auto route = [&]() __attribute__((always_inline)) {
    if (given) {
      if (lane < k) {
        sel_e[lane] = P.route_idx[(size_t)token * k + lane];
        sel_g[lane] = P.route_gate[(size_t)token * k + lane];
      }
    } else if (routed) {
      if (inline_router) {
        float* lg = rpart + E * n_seg;            // the logits go behind the partial sums
        if (lane < E) {
          float t = 0.f;
          for (int sg = 0; sg < n_seg; ++sg) t += rpart[lane * n_seg + sg];
          lg[lane] = t + (P.bias ? P.bias[lane] : 0.f);
        }
        topk_from_logits(lg, E, k, L.renorm, lane, sel_e, sel_g, nullptr);   // same wavefront wrote lg
      } else {
        topk_from_logits(P.logits + (size_t)token * E, E, k, L.renorm, lane, sel_e, sel_g, nullptr);
      }
    } else if (lane == 0) {
      sel_e[0] = P.fixed_expert;
      sel_g[0] = P.gate_in ? P.gate_in[token] : 1.0f;
    }
    // the indices become addresses of expert records: whatever produced them, they stay inside the table
    if (lane < k) sel_e[lane] = min(max(sel_e[lane], 0), E - 1);
  };
  auto stage_layouts = [&](int st, int sn) __attribute__((always_inline)) {
    // behind the staged pairs of a bitwidth: its offset terms (matrix-core variant: negated, per range of
    // a lane column)
    if (P.bits_mask & 2) {
      uint32_t* XPs = LAY + layout_slot(P.bits_mask, 2) * lay_words;
      permute_x<2, MX>(RAW, d, L.group, st, sn, XPs, (float*)(XPs + d / 2));
    }
    if (P.bits_mask & 4) {
      uint32_t* XPs = LAY + layout_slot(P.bits_mask, 4) * lay_words;
      permute_x<4, MX>(RAW, d, L.group, st, sn, XPs, (float*)(XPs + d / 2));
    }
    if (P.bits_mask & 8) {
      uint32_t* XPs = LAY + layout_slot(P.bits_mask, 8) * lay_words;
      permute_x<8, MX>(RAW, d, L.group, st, sn, XPs, (float*)(XPs + d / 2));
    }
  };
  auto publish_routing = [&]() __attribute__((always_inline)) {
    if (routed && !given && slice == 0 && (int)threadIdx.x < k) {
      if (P.idx_out) P.idx_out[(size_t)token * k + threadIdx.x] = sel_e[threadIdx.x];
      if (P.gate_out) P.gate_out[(size_t)token * k + threadIdx.x] = sel_g[threadIdx.x];
    }
  };

  if constexpr (MX) {
    constexpr int NM = SWIGLU ? 2 : 1;
    if (wave == 0) {
      route();
      if (lane < k) sel_b[lane] = (tab_in_lds ? tab[sel_e[lane]] : P.table[sel_e[lane]]).bits;
    } else {
      stage_layouts(threadIdx.x - 64, nthreads - 64);
    }
    __syncthreads();  // layouts, sel_e, sel_g are complete
    publish_routing();
    const DevExpert* tabp = tab_in_lds ? tab : P.table;
    const int gsh = __builtin_ctz((unsigned)L.group);           // the plan admits powers of two only
    const int m16 = lane & 15, kb4 = lane >> 4;
    float dm[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) dm[i] = (kb4 == (m16 >> 2) && (m16 & 3) == i) ? 1.f : 0.f;
    // ---- phase 1: tasks (expert slot t / SW, row of the slice from t % SW); wavefront w takes w, w + nwaves, ...
    const uint32_t row0 = (uint32_t)(slice * SW);
    const uint32_t ng2 = (uint32_t)(d >> gsh) * 2u;
    const int n_tasks = k * SW;
    const int wsh = __builtin_ctz((unsigned)nwaves);           // the plan: nwaves divides 64
    MxWalk1 wi;
    wi.j = -1;
    auto take = [&](int t) __attribute__((always_inline)) {
      wi.t = t;
      wi.valid = t < n_tasks;
      wi.jb = 0;
      if (wi.valid) {
        // SW == 64. Consecutive tasks are rows 4 apart, rotated by the slice: what the workgroup reads at
        // any moment is spread over its whole block of rows, and differently in every workgroup
        const int j = t >> 6, u = t & 63;
        wi.r = ((u & 15) << 2) | (((u >> 4) + slice) & 3);
        if (j != wi.j) {
          wi.j = j;
          mx1_enter<SWIGLU>(wi, tabp + sel_e[j], d, gsh, lane);
        }
      }
    };
    auto issue = [&](MxSet1& S, MxTag1& tag) __attribute__((always_inline)) {
      mx1_issue<NM>(S, tag, wi, row0, ng2, (const uint8_t*)xt, lane);
      if (wi.valid && ++wi.jb == wi.JB) take(wi.t + nwaves);
    };
    float acc[NM], keep[NM];
#pragma unroll
    for (int mm = 0; mm < NM; ++mm) keep[mm] = 0.f;
    int rows_done = 0, rows_flushed = 0;
    // the activation of the wavefront's parked rows: lane i holds the task wave + (rows_flushed + i) * nwaves
    auto flush_rows = [&]() __attribute__((always_inline)) {
#pragma unroll
      for (int mm = 0; mm < NM; ++mm) {
        keep[mm] += __shfl_xor(keep[mm], 16);
        keep[mm] += __shfl_xor(keep[mm], 32);
      }
      if (lane < rows_done) {
        const int t = wave + (rows_flushed + lane) * nwaves, j = t >> 6, u = t & 63;
        const int c = ((u & 15) << 2) | (((u >> 4) + slice) & 3);
        float r[NM];
#pragma unroll
        for (int mm = 0; mm < NM; ++mm) r[mm] = keep[mm] * 16777216.0f * up;
        HF[j * SW + c] = mx1_activation<SWIGLU, NM>(r);
      }
      rows_flushed += rows_done;
      rows_done = 0;
#pragma unroll
      for (int mm = 0; mm < NM; ++mm) keep[mm] = 0.f;
    };
    auto compute = [&](const MxSet1& S, const MxTag1& tag) __attribute__((always_inline)) {
      const uint32_t* XP = LAY + layout_slot(P.bits_mask, tag.bits) * lay_words;
      const float* KS = (const float*)(XP + d / 2);
      switch (tag.bits) {
        case 2: mx1_compute<2, SWIGLU>(S, tag, d, lane, dm, XP, KS, acc, keep, rows_done); break;
        case 4: mx1_compute<4, SWIGLU>(S, tag, d, lane, dm, XP, KS, acc, keep, rows_done); break;
        default: mx1_compute<8, SWIGLU>(S, tag, d, lane, dm, XP, KS, acc, keep, rows_done); break;
      }
      if (rows_done == 16) flush_rows();
    };
    {
      MxSet1 A, B;
      MxTag1 ta, tb;
      take(wave);                     // n_tasks >= 64 > wave
      issue(A, ta);
      issue(B, tb);
      // priority by the tasks still ahead, finest near the end of the list where the drift would show
      auto prio = [&](int t) __attribute__((always_inline)) {
        const int left = (n_tasks - 1 - t) >> wsh;        // tasks after this one (nwaves is a power of two here)
        if (left >= 3) __builtin_amdgcn_s_setprio(3);
        else if (left == 2) __builtin_amdgcn_s_setprio(2);
        else if (left == 1) __builtin_amdgcn_s_setprio(1);
        else __builtin_amdgcn_s_setprio(0);
      };
      while (ta.valid) {
        prio(ta.t);
        compute(A, ta);
        issue(A, ta);
        if (tb.valid) {
          prio(tb.t);
          compute(B, tb);
        }
        issue(B, tb);
      }
      __builtin_amdgcn_s_setprio(0);
    }
    if (rows_done > 0) flush_rows();
    // ---- phase 2: one list of register sets through all chosen experts; the first set is requested ahead
    // of the barrier between the phases
    MxWalk2 vi, vc;
    vi.j = 0;
    mx2_enter(vi, tabp + sel_e[0], d, slice, gsh, lane, wave, nwaves);
    vc = vi;
    int ns = 0;
    for (int j = 0; j < k; ++j) {
      const int bits = __builtin_amdgcn_readfirstlane(tabp[sel_e[j]].bits);
      const int gps = bits == 2 ? 4 : (bits == 4 ? 2 : 1);
      ns += d / (64 * gps * nwaves);
    }
    auto advance2 = [&](MxWalk2& w) __attribute__((always_inline)) {
      if (++w.set == w.n_sets) {
        if (++w.j < k) mx2_enter(w, tabp + sel_e[w.j], d, slice, gsh, lane, wave, nwaves);
      }
    };
    auto issue2 = [&](MxSet2& S) __attribute__((always_inline)) {
      mx2_issue(S, vi);
      advance2(vi);
    };
    float K2 = 0.f, gu = 0.f;
    auto compute2 = [&](const MxSet2& S) __attribute__((always_inline)) {
      if (vc.set == 0) {
        // offset term of the expert: the sum of its h slice (one value per lane, kMxSlice == 64)
        const float hs = wave_sum(f16_bits_to_f32(HLs[vc.j * SW + lane]));
        K2 = hs * ((float)(1 << (vc.bits - 1)) * 5.9604644775390625e-08f);
        gu = sel_g[vc.j] * uph[vc.j];
      }
      const uint4* HP4 = (const uint4*)(HPs + vc.j * SW);
      switch (vc.bits) {
        case 2: mx2_compute<2>(S, vc, d, lane, wave, nwaves, HP4, K2, gu, Y); break;
        case 4: mx2_compute<4>(S, vc, d, lane, wave, nwaves, HP4, K2, gu, Y); break;
        default: mx2_compute<8>(S, vc, d, lane, wave, nwaves, HP4, K2, gu, Y); break;
      }
      advance2(vc);
    };
    {
      MxSet2 A, B;
      issue2(A);                      // ns >= 1
      __syncthreads();                // the h slices of all chosen experts are complete in LDS (fp32)
      stage_h_slices(HF, k, SW, tabp, sel_e, HLs, HPs, uph, lane, wave, nwaves);
      __syncthreads();                // ... and staged for phase 2
      // as in phase 1, a wavefront's priority falls with the sets it has left
      auto prio2 = [&](int left) __attribute__((always_inline)) {
        if (left >= 3) __builtin_amdgcn_s_setprio(3);
        else if (left == 2) __builtin_amdgcn_s_setprio(2);
        else if (left == 1) __builtin_amdgcn_s_setprio(1);
        else __builtin_amdgcn_s_setprio(0);
      };
      int b = 0;
      for (; b + 2 < ns; b += 2) {
        issue2(B);
        prio2(ns - 1 - b);
        compute2(A);
        issue2(A);
        prio2(ns - 2 - b);
        compute2(B);
      }
      if (b + 1 < ns) {
        issue2(B);
        prio2(1);
        compute2(A);
        prio2(0);
        compute2(B);
      } else {
        compute2(A);
      }
      __builtin_amdgcn_s_setprio(0);
    }
    __syncthreads();   // Y was written by the lanes that hold the instruction results, it is read by all
  } else {
  if (wave == 0) route();
  else stage_layouts(threadIdx.x - 64, nthreads - 64);
  __syncthreads();  // layouts, sel_e, sel_g are complete
  publish_routing();
  // ---- phase 1 of every chosen expert, back to back: no wavefront waits for another one here
  for (int j = 0; j < k; ++j) {
    const int e = sel_e[j];
    const DevExpert* ex = tab_in_lds ? &tab[e] : &P.table[e];
    const int bits = __builtin_amdgcn_readfirstlane(ex->bits);
    const uint32_t* XP = LAY + layout_slot(P.bits_mask, bits) * lay_words;
    const float* XK = (const float*)(XP + d / 2);
    int tid = threadIdx.x;  // opaque copy: keeps the per-bitwidth lane arithmetic inside this iteration
    asm volatile("" : "+v"(tid));
    switch (bits) {
      case 2: fused_in<2, SWIGLU>(ex, tid, nwaves, d, L.group, slice * SW, SW, up, HF + j * SW, XP, XK); break;
      case 4: fused_in<4, SWIGLU>(ex, tid, nwaves, d, L.group, slice * SW, SW, up, HF + j * SW, XP, XK); break;
      default: fused_in<8, SWIGLU>(ex, tid, nwaves, d, L.group, slice * SW, SW, up, HF + j * SW, XP, XK); break;
    }
  }
  // ---- phase 2 of every chosen expert (the first one's call holds the barriers between the phases and the
  // staging of h between them)
  const DevExpert* tabv = tab_in_lds ? tab : P.table;
  auto between = [&]() __attribute__((always_inline)) {
    stage_h_slices(HF, k, SW, tabv, sel_e, HLs, HPs, uph, lane, wave, nwaves);
  };
  for (int j = 0; j < k; ++j) {
    const int e = sel_e[j];
    const DevExpert* ex = tab_in_lds ? &tab[e] : &P.table[e];
    const int bits = __builtin_amdgcn_readfirstlane(ex->bits);
    const uint16_t* HL = HLs + j * SW;
    const uint16_t* HP = HPs + j * SW;
    const float gate = sel_g[j];
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    auto run = [&](auto bits_tag) __attribute__((always_inline)) {
      constexpr int BITS = decltype(bits_tag)::value;
      const int DW = SW * BITS / 32;
      if (DW >= 8) fused_expert_out<BITS, 8>(ex, tid, nthreads, d, L.group_out, slice, SW, gate, uph + j, j == 0, HL, HP, Y, between);
      else if (DW == 4) fused_expert_out<BITS, 4>(ex, tid, nthreads, d, L.group_out, slice, SW, gate, uph + j, j == 0, HL, HP, Y, between);
      else if (DW == 2) fused_expert_out<BITS, 2>(ex, tid, nthreads, d, L.group_out, slice, SW, gate, uph + j, j == 0, HL, HP, Y, between);
      else fused_expert_out<BITS, 1>(ex, tid, nthreads, d, L.group_out, slice, SW, gate, uph + j, j == 0, HL, HP, Y, between);
    };
    switch (bits) {
      case 2: run(std::integral_constant<int, 2>{}); break;
      case 4: run(std::integral_constant<int, 4>{}); break;
      default: run(std::integral_constant<int, 8>{}); break;
    }
  }

  }

  // (vector path: every row block was accumulated by the thread that now writes it out)
  float4* out = (float4*)(P.part + ((size_t)token * gridDim.x + slice) * d);
  for (int rb = threadIdx.x; rb < d / 4; rb += nthreads) out[rb] = Y[rb];
}

// y[t][r] (+)= sum over the slices of part[t][s][r], in a fixed order. Workgroup = 16 outputs x 64 slice
// teams: team g sums the slices g, g+64, ... for its 4 outputs, then the 64 team sums are added in a fixed
// tree (a butterfly over the lanes of a wavefront, then the wavefronts in order). Small workgroups on many
// compute units: the kernel is one memory round trip long.
__global__ __launch_bounds__(256) void k_reduce_partials(const float* __restrict__ part, int n_slices, int d,
                                                         int accumulate, float* __restrict__ y) {
  __shared__ float4 red[4][4];
  const int token = blockIdx.y;
  const int rq = threadIdx.x & 3, sg = threadIdx.x >> 2;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bool in_range = (int)blockIdx.x * 16 + rq * 4 < d;     // d is a multiple of 8, not always of 16
  const int r0 = min((int)blockIdx.x * 16 + rq * 4, d - 4);   // clamped columns are summed but not written
  float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
  const float* p = part + (size_t)token * n_slices * d + r0;
  // four slices per pass, requested together (one memory round trip per pass); slices past the end read the
  // last one and are weighted with zero, so that the loads need no condition
  for (int s0 = sg; s0 < n_slices; s0 += 256) {
    float4 v[4];
    float w[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int s = s0 + 64 * u;
      w[u] = s < n_slices ? 1.f : 0.f;
      v[u] = *(const float4*)(p + (size_t)min(s, n_slices - 1) * d);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      a.x = fmaf(v[u].x, w[u], a.x); a.y = fmaf(v[u].y, w[u], a.y);
      a.z = fmaf(v[u].z, w[u], a.z); a.w = fmaf(v[u].w, w[u], a.w);
    }
  }
  // the 16 teams of a wavefront (lanes 4 apart hold the same columns) in a fixed butterfly, then the four
  // wavefronts in order
#pragma unroll
  for (int off = 4; off < 64; off <<= 1) {
    a.x += __shfl_xor(a.x, off); a.y += __shfl_xor(a.y, off);
    a.z += __shfl_xor(a.z, off); a.w += __shfl_xor(a.w, off);
  }
  if (lane < 4) red[wave][lane] = a;
  __syncthreads();
  if (threadIdx.x < 4 && in_range) {
    float4 t = red[0][rq];
#pragma unroll
    for (int wv = 1; wv < 4; ++wv) {
      const float4 v = red[wv][rq];
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

size_t fused_lds_bytes(const LayerDims& L, int k, int SW, int n_layouts) {
  return (size_t)L.d_model * 2 + (size_t)k * SW * 8 + (size_t)L.d_model * 4 +
         (size_t)n_layouts * ((size_t)L.d_model / 2 + (size_t)L.d_model / 16) * 4;
}

}  // namespace

// Slice width: a multiple of 16 columns (one 32-bit word of 2-bit codes) that divides the group size, so that
// a slice has one scale per output row; the widest one that still gives at least 3/4 of a workgroup per
// compute unit, else the narrowest.
FusedPlan plan_fused(const LayerDims& L) {
  FusedPlan p{0, 0, 0, 0};
  if (L.d_model % 8 || L.d_ff % 16 || L.group_out % 16) return p;
  static const int forced = [] { const char* v = std::getenv("MOEQ_SLICE"); return v ? std::atoi(v) : 0; }();
  const int want = cu_count() * 3 / 4;
  int best = 0;
  for (int sw = 16; sw <= 256; sw *= 2) {
    if (L.group_out % sw || L.d_ff % sw) break;
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
  // Matrix-core variant: scale groups of 128, 256, 512 or 1024 columns, 64-column slices,
  // rows that are whole bursts (two tiles) at every bitwidth (4096 columns), and wavefronts that share the
  // rows of a slice and the 64-row groups of the output evenly.
  static const bool no_mx = [] { const char* v = std::getenv("MOEQ_NO_MFMA"); return v && v[0] == '1'; }();
  const int mx = (!no_mx && best == kMxSlice && L.group == L.group_out && L.group % 128 == 0 && (L.group & (L.group - 1)) == 0 && L.group <= 1024 &&
                  L.d_model % 4096 == 0 && kMxSlice % (nt / 64) == 0 && L.d_model % (4 * nt) == 0) ? 1 : 0;
  if (fused_lds_bytes(L, L.top_k, best, 3) > kFusedLdsBudget) return p;
  if (L.d_model > 2048 * kMaxSegs) return p;
  p.SW = best;
  p.n_slices = L.d_ff / best;
  p.threads = nt;
  p.mx = mx;
  return p;
}

int fused_inline_router_max() { return kInlineMaxE; }

hipError_t init_attrs_decode_fused() {
  (void)cu_count();
  const void* ks[6] = {(const void*)k_moe_decode<false, false>, (const void*)k_moe_decode<true, false>,
                       (const void*)k_moe_decode<false, true>, (const void*)k_moe_decode<true, true>,
                       (const void*)k_moe_decode<false, false, 256>, (const void*)k_moe_decode<true, false, 256>};
  for (const void* kf : ks)
    if (hipError_t e = hipFuncSetAttribute(kf, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFusedLdsBudget); e != hipSuccess)
      return e;
  return hipSuccess;
}

hipError_t launch_moe_decode(const LayerDims& L, const FusedPlan& plan, const DevExpert* table, const float* router_w,
                             const float* router_bias, const float* logits, int32_t fixed_expert,
                             const float* gate_in, const int32_t* route_idx, const float* route_gate,
                             int32_t bits_mask, const void* x, int32_t T, float* part, int32_t* idx_out,
                             float* gate_out, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
  if (!plan.SW || T < 1 || T > 65535 || !(bits_mask & 14)) return hipErrorInvalidValue;
  if (!logits && !route_idx && fixed_expert < 0 && L.n_experts > kInlineMaxE) return hipErrorInvalidValue;
  if ((route_idx != nullptr) != (route_gate != nullptr)) return hipErrorInvalidValue;
  const int k = fixed_expert >= 0 ? 1 : L.top_k;
  const int n_layouts = ((bits_mask >> 1) & 1) + ((bits_mask >> 2) & 1) + ((bits_mask >> 3) & 1);
  const size_t lds = fused_lds_bytes(L, k, plan.SW, n_layouts);
  FusedParams P{L, table, router_w, router_bias, logits, fixed_expert, gate_in, route_idx, route_gate, x, part,
                idx_out, gate_out, plan.SW, bits_mask};
  const bool sw = L.act == MOEQ_ACT_SWIGLU, mx = plan.mx != 0;
  const bool small = !mx && plan.threads <= 256;
  auto kernel = mx ? (sw ? k_moe_decode<true, true> : k_moe_decode<false, true>)
                   : small ? (sw ? k_moe_decode<true, false, 256> : k_moe_decode<false, false, 256>)
                           : (sw ? k_moe_decode<true, false> : k_moe_decode<false, false>);
  if (lds > kFusedLdsBudget) return hipErrorInvalidValue;   // the ceiling init_attrs_decode_fused() asked for
  if (ev_start && ev_stop)
    hipExtLaunchKernelGGL(kernel, dim3(plan.n_slices, T), dim3(plan.threads), lds, st, ev_start, ev_stop, 0, P);
  else
    hipLaunchKernelGGL(kernel, dim3(plan.n_slices, T), dim3(plan.threads), lds, st, P);
  return hipGetLastError();
}

hipError_t launch_reduce_partials(const float* part, int n_slices, int d, int32_t T, int accumulate, float* y,
                                  hipStream_t st) {
  hipLaunchKernelGGL(k_reduce_partials, dim3((d + 15) / 16, T), dim3(256), 0, st, part, n_slices, d, accumulate, y);
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
