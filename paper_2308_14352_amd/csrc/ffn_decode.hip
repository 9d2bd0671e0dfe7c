// Dequantize-fused expert FFN for decode (one to a few tokens): bandwidth-bound GEMVs that stream the
// packed INT2/INT4/INT8 rows of the activated experts with 128-bit loads, unpack the codes in
// registers and accumulate in fp32 (Section 3.2: the weights are decompressed by the mirror of the
// linear quantization before use; here that mirror map is applied on the fly and the fp32 copy of
// the expert is never written).
//
// Arithmetic. A 16-byte chunk of a packed row holds 128/b codes. A mask (and one shift per dword)
// isolates two codes at a time in the mantissa bits of the two halves of a register; read as a pair of
// binary16 subnormals these are exactly u * 4^j * 2^-24, and one v_dot2_f32_f16 multiplies the pair
// with the matching pair of activations (converted to binary16 once per workgroup and pre-divided by
// 4^j, an exact scaling) and adds into an fp32 accumulator. Per scale group the code offset and
// the scale are applied once: total += (s * 2^24) * (acc - 2^(b-1) * sum(x) * 2^-24). That is about
// 1.1 vector instructions per weight at every bitwidth.
//
// Work split. P lanes of a wavefront share a row (P = the largest power of two dividing the chunks
// per row, at most 64); a lane walks its chunks j = p, p+P, ... and, for each, NR rows that share the
// activation registers (for SwiGLU the rows of w1 and w3 are interleaved as "virtual rows"). Loads
// run D tiles ahead of the arithmetic through a register ring. Row totals are folded across the P
// lanes with a transposing butterfly (about one shuffle per row). A workgroup owns a fixed range of
// output rows for all k chosen experts of its token, so the gate-weighted sum over the experts is
// ordered and needs no atomics.
#include <hip/hip_fp16.h>

#include <type_traits>

#include "moeq_internal.h"

namespace moeq {
namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

template <int BITS>
struct Fmt {
  static constexpr int WPC = 128 / BITS;  // weights per 16-byte chunk
  static constexpr int PPC = WPC / 2;     // activation pair registers per chunk
  static constexpr float OFF = (float)(1 << (BITS - 1));
};

// Which two weights of a chunk (lo, hi) land in pair register `pi`, and by what power of two their
// activations are pre-divided so that the masked code field needs no shift of its own.
template <int BITS>
__device__ __forceinline__ void pair_pos(int pi, int& lo, int& hi, float& prescale) {
  if (BITS == 8) {           // dword d, bytes (0,2) then (1,3)
    const int d = pi >> 1, k = pi & 1;
    lo = 4 * d + k; hi = lo + 2; prescale = 1.0f;
  } else if (BITS == 4) {    // dword d, nibbles (0,4) (1,5) (2,6) (3,7); odd nibbles sit 4 bits up
    const int d = pi >> 2, k = pi & 3;
    lo = 8 * d + k; hi = lo + 4; prescale = (k & 1) ? 0.0625f : 1.0f;
  } else {                   // dword d, fields (j, j+8); fields 0..4 masked in place, 5..7 after >> 10
    const int d = pi >> 3, j = pi & 7;
    lo = 16 * d + j; hi = lo + 8;
    const int e = j < 5 ? j : j - 5;
    prescale = 1.0f / (float)(1 << (2 * e));
  }
}

__device__ __forceinline__ float dot2(uint32_t codes, uint32_t xpair, float acc) {
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, codes), __builtin_bit_cast(half2_t, xpair), acc, false);
}

// One dword of codes against its pair registers xr[0 .. 32/BITS/2).
template <int BITS>
__device__ __forceinline__ float dword_dot(uint32_t w, const uint32_t* xr, float acc) {
  if (BITS == 8) {
    acc = dot2(w & 0x00ff00ffu, xr[0], acc);
    acc = dot2((w >> 8) & 0x00ff00ffu, xr[1], acc);
  } else if (BITS == 4) {
    const uint32_t w8 = w >> 8;
    acc = dot2(w & 0x000f000fu, xr[0], acc);
    acc = dot2(w & 0x00f000f0u, xr[1], acc);
    acc = dot2(w8 & 0x000f000fu, xr[2], acc);
    acc = dot2(w8 & 0x00f000f0u, xr[3], acc);
  } else {
    const uint32_t w10 = w >> 10;
    acc = dot2(w & 0x00030003u, xr[0], acc);
    acc = dot2(w & 0x000c000cu, xr[1], acc);
    acc = dot2(w & 0x00300030u, xr[2], acc);
    acc = dot2(w & 0x00c000c0u, xr[3], acc);
    acc = dot2(w & 0x03000300u, xr[4], acc);
    acc = dot2(w10 & 0x00030003u, xr[5], acc);
    acc = dot2(w10 & 0x000c000cu, xr[6], acc);
    acc = dot2(w10 & 0x00300030u, xr[7], acc);
  }
  return acc;
}

// Stage `cols` activations into LDS for BITS: pair register pi of chunk c goes to word
// ((pi/4) * C + c) * 4 + pi%4, so a lane's 128-bit reads of consecutive chunks are conflict-free.
// XK[c * spc + j] = 2^(b-1) * 2^-24 * (sum of the binary16-rounded activations of scale slice j of chunk c).
template <int BITS, typename LoadX>
__device__ __forceinline__ void stage_x(LoadX load, int cols, int group, uint32_t* XP, float* XK) {
  constexpr int WPC = Fmt<BITS>::WPC, PPC = Fmt<BITS>::PPC;
  const int C = cols / WPC;
  for (int i = threadIdx.x; i < cols / 2; i += blockDim.x) {
    const int c = i / PPC, pi = i % PPC;
    int lo, hi;
    float ps;
    pair_pos<BITS>(pi, lo, hi, ps);
    const float xl = __half2float(__float2half_rn(load(c * WPC + lo)));
    const float xh = __half2float(__float2half_rn(load(c * WPC + hi)));
    const uint32_t bl = __half_as_ushort(__float2half_rn(xl * ps));
    const uint32_t bh = __half_as_ushort(__float2half_rn(xh * ps));
    XP[((pi >> 2) * C + c) * 4 + (pi & 3)] = bl | (bh << 16);
  }
  const int sub = group < WPC ? group : WPC;
  const int spc = WPC / sub;  // scale slices per chunk: 1, or 2 for INT2 with group 32
  for (int s = threadIdx.x; s < C * spc; s += blockDim.x) {
    float acc = 0.f;
    for (int i = 0; i < sub; ++i) acc += __half2float(__float2half_rn(load(s * sub + i)));
    XK[s] = acc * (Fmt<BITS>::OFF * 5.9604644775390625e-08f);
  }
  __syncthreads();
}

struct Tile {
  uint4 w;
  uint32_t s;  // one binary16 scale, or two adjacent ones (INT2 with group 32)
};

// Sum over the P lanes of a row group (P a power of two, lanes of a group are contiguous) of NM*NRM row
// totals per lane; v = m*NRM + i. Needs NRM <= P. Afterwards every lane holds, in v[m*NRM] (m < NM), the
// group totals of row i = lane & (NRM-1) of matrix m.
template <int NRM, int NM>
__device__ __forceinline__ void fold_rows(float (&v)[NRM * NM], int P, int lane) {
  int off = 1;
#pragma unroll
  for (int n = NRM; n > 1; n >>= 1) {  // transposing steps: halve the number of live rows per lane
    const bool upper = (lane & off) != 0;
#pragma unroll
    for (int m = 0; m < NM; ++m)
#pragma unroll
      for (int i = 0; i < n / 2; ++i) {
        const float a = v[m * NRM + 2 * i], b = v[m * NRM + 2 * i + 1];
        const float keep = upper ? b : a, send = upper ? a : b;
        v[m * NRM + i] = keep + __shfl_xor(send, off, 64);
      }
    off <<= 1;
  }
  for (; off < P; off <<= 1) {
#pragma unroll
    for (int m = 0; m < NM; ++m) v[m * NRM] += __shfl_xor(v[m * NRM], off, 64);
  }
}

// A pointer that is the same in every lane, moved to scalar registers so that loads can use the
// "scalar base + 32-bit lane offset" addressing mode instead of 64-bit per-lane addresses.
template <typename T>
__device__ __forceinline__ const T* uniform_ptr(const T* ptr) {
  const uint64_t v = (uint64_t)ptr;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const T*)(((uint64_t)hi << 32) | lo);
}

// One wavefront task: NRM rows (per lane group) of each of NM matrices, all chunks of those rows.
// row0 = first row of this lane's group; rows are row0 + i*RW, clamped to nrows-1 for the loads.
// Tiles (one 16-byte chunk of one row + its scale) are processed in blocks of kBlock; the loads of the
// next block are issued before the arithmetic of the current one (double buffering in registers).
constexpr int kBlock = 4;

template <int BITS, int NRM, int NM, bool TWO>
__device__ __forceinline__ void gemv_task(const uint8_t* const (&q)[NM], const uint16_t* const (&s)[NM], int cols,
                                          int group, int P, int p, int row0, int RW, int nrows,
                                          const uint32_t* XP, const float* XK, float (&tot)[NRM * NM]) {
  constexpr int WPC = Fmt<BITS>::WPC, PPC = Fmt<BITS>::PPC;
  constexpr int NR = NRM * NM;
  static_assert(NR <= kBlock && kBlock % NR == 0, "rows in flight must divide the block");
  constexpr int CPB = kBlock / NR;  // chunks per block
  const int C = cols / WPC;
  const int J = C / P;
  const int ng = cols / group;
  const uint4* XP4 = (const uint4*)XP;

  uint32_t qoff[NR], soff[NR];
#pragma unroll
  for (int v = 0; v < NR; ++v) {
    int row = row0 + (v % NRM) * RW;
    row = row < nrows ? row : nrows - 1;
    qoff[v] = (uint32_t)row * (uint32_t)(C * 16) + (uint32_t)p * 16u;
    soff[v] = ((uint32_t)row * (uint32_t)ng) * 2u;   // bytes
    tot[v] = 0.f;
  }
  const uint32_t jstride = (uint32_t)P * 16u;
  auto load_tile = [&](int j, int v) {
    Tile t;
    const int m = v / NRM;
    t.w = *(const uint4*)(q[m] + (qoff[v] + (uint32_t)j * jstride));
    const uint32_t g0 = (uint32_t)((p + j * P) * WPC) / (uint32_t)group;
    const uint8_t* sb = (const uint8_t*)s[m];
    if (TWO) t.s = *(const uint32_t*)(sb + (soff[v] + g0 * 2u));
    else t.s = *(const uint16_t*)(sb + (soff[v] + g0 * 2u));
    return t;
  };
  auto load_block = [&](Tile (&t)[kBlock], int blk) {
#pragma unroll
    for (int u = 0; u < kBlock; ++u) {
      const int j = blk * CPB + u / NR;
      if (j < J) t[u] = load_tile(j, u % NR);
    }
  };
  uint32_t xr[PPC];
  float k0 = 0.f, k1 = 0.f;
  auto compute_block = [&](const Tile (&t)[kBlock], int blk) {
#pragma unroll
    for (int u = 0; u < kBlock; ++u) {
      const int j = blk * CPB + u / NR;
      const int v = u % NR;
      if (j < J) {
        if (v == 0) {  // new chunk: fetch its activation pairs and offset terms
          const int c = p + j * P;
#pragma unroll
          for (int qq = 0; qq < PPC / 4; ++qq) {
            const uint4 t4 = XP4[qq * C + c];
            xr[4 * qq] = t4.x; xr[4 * qq + 1] = t4.y; xr[4 * qq + 2] = t4.z; xr[4 * qq + 3] = t4.w;
          }
          if (TWO) { k0 = XK[2 * c]; k1 = XK[2 * c + 1]; }
          else k0 = XK[c];
        }
        const uint4 w = t[u].w;
        const uint32_t sraw = t[u].s;
        if (TWO) {
          float a0 = dword_dot<BITS>(w.x, &xr[0], 0.f);
          a0 = dword_dot<BITS>(w.y, &xr[PPC / 4], a0);
          float a1 = dword_dot<BITS>(w.z, &xr[PPC / 2], 0.f);
          a1 = dword_dot<BITS>(w.w, &xr[3 * PPC / 4], a1);
          const float s0 = __half2float(__ushort_as_half((uint16_t)(sraw & 0xffffu))) * 16777216.0f;
          const float s1 = __half2float(__ushort_as_half((uint16_t)(sraw >> 16))) * 16777216.0f;
          tot[v] = fmaf(s0, a0 - k0, tot[v]);
          tot[v] = fmaf(s1, a1 - k1, tot[v]);
        } else {
          float a = dword_dot<BITS>(w.x, &xr[0], 0.f);
          a = dword_dot<BITS>(w.y, &xr[PPC / 4], a);
          a = dword_dot<BITS>(w.z, &xr[PPC / 2], a);
          a = dword_dot<BITS>(w.w, &xr[3 * PPC / 4], a);
          const float s0 = __half2float(__ushort_as_half((uint16_t)(sraw & 0xffffu))) * 16777216.0f;
          tot[v] = fmaf(s0, a - k0, tot[v]);
        }
      }
    }
  };

  const int nblocks = (J + CPB - 1) / CPB;
  Tile bufA[kBlock], bufB[kBlock];
  load_block(bufA, 0);
  for (int blk = 0; blk < nblocks; blk += 2) {
    if (blk + 1 < nblocks) load_block(bufB, blk + 1);
    compute_block(bufA, blk);
    if (blk + 1 < nblocks) {
      if (blk + 2 < nblocks) load_block(bufA, blk + 2);
      compute_block(bufB, blk + 1);
    }
  }
}

__host__ __device__ inline int lanes_per_row(int chunks) {
  int P = 1;
  while (P < 64 && chunks % (P * 2) == 0) P *= 2;
  return P;
}

// Rows per lane group and matrix in one task: as many (1, 2 or 4) as still leave every wavefront of the
// workgroup a task, and never more than P (the fold needs NRM <= P).
__host__ __device__ inline int pick_nrm(int rows_in_wg, int RW, int nwaves, int P, int nrm_max) {
  int nrm = nrm_max;
  while (nrm > 1 && (nrm > P || rows_in_wg < RW * nrm * nwaves)) nrm >>= 1;
  return nrm;
}

// ---------------------------------------------------------------------------------------------
// softmax + top-k of one token from its logits, by wavefront 0 of a workgroup. E <= 1024.
// Writes sel_e[0..k), sel_g[0..k) (LDS or global) from lane 0; probs (global, may be null) from all lanes.
__device__ __forceinline__ void topk_from_logits(const float* __restrict__ lg, int E, int k, int renorm, int lane,
                                                 int* sel_e, float* sel_g, float* __restrict__ probs) {
  constexpr int kMaxPerLane = 16;
  float v[kMaxPerLane];
  float m = -INFINITY;
#pragma unroll
  for (int j = 0; j < kMaxPerLane; ++j) {
    const int e = lane + 64 * j;
    v[j] = e < E ? lg[e] : -INFINITY;
    m = fmaxf(m, v[j]);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  float z = 0.f;
#pragma unroll
  for (int j = 0; j < kMaxPerLane; ++j)
    if (lane + 64 * j < E) z += expf(v[j] - m);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) z += __shfl_xor(z, off, 64);
  const float inv_z = 1.0f / z;
  if (probs) {
#pragma unroll
    for (int j = 0; j < kMaxPerLane; ++j)
      if (lane + 64 * j < E) probs[lane + 64 * j] = expf(v[j] - m) * inv_z;
  }
  // k selection passes on the logits (same order as on the probabilities): largest value, ties to the
  // lowest expert index.
  float sp[8];
  int se[8];
  float sum = 0.f;
  for (int r = 0; r < k; ++r) {
    float bv = -INFINITY;
    int be = 0x7fffffff;
#pragma unroll
    for (int j = 0; j < kMaxPerLane; ++j) {
      const int e = lane + 64 * j;
      if (e < E && (v[j] > bv)) { bv = v[j]; be = e; }  // ascending e per lane: '>' keeps the lowest
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const float ov = __shfl_xor(bv, off, 64);
      const int oe = __shfl_xor(be, off, 64);
      if (ov > bv || (ov == bv && oe < be)) { bv = ov; be = oe; }
    }
#pragma unroll
    for (int j = 0; j < kMaxPerLane; ++j)
      if (lane + 64 * j == be) v[j] = -INFINITY;
    sp[r] = expf(bv - m) * inv_z;
    se[r] = be;
    sum += sp[r];
  }
  if (lane == 0)
    for (int r = 0; r < k; ++r) {
      sel_e[r] = se[r];
      sel_g[r] = renorm ? sp[r] / sum : sp[r];
    }
}

__global__ __launch_bounds__(64) void k_topk(LayerDims L, const float* __restrict__ logits, int32_t* __restrict__ idx,
                                             float* __restrict__ gate, float* __restrict__ probs) {
  const int t = blockIdx.x;
  topk_from_logits(logits + (size_t)t * L.n_experts, L.n_experts, L.top_k, L.renorm, threadIdx.x,
                   idx + (size_t)t * L.top_k, gate + (size_t)t * L.top_k,
                   probs ? probs + (size_t)t * L.n_experts : nullptr);
}

// ---------------------------------------------------------------------------------------------
template <int BITS, bool SWIGLU>
__device__ __forceinline__ void ffn_in_tasks(const DevExpert& ex, int tid, int d, int f, int group, int row_begin,
                                             int row_end, float* __restrict__ h_out, const uint32_t* XP,
                                             const float* XK) {
  const int C = d / Fmt<BITS>::WPC;
  const int P = lanes_per_row(C), RW = 64 / P;
  const int lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
  const int p = lane % P, rsub = lane / P;
  constexpr int NM = SWIGLU ? 2 : 1;
  const int nrm = pick_nrm(row_end - row_begin, RW, nwaves, P, kBlock / NM);
  const bool two = (BITS == 2) && (group == 32);
  const uint8_t* q_in = uniform_ptr(ex.q_in);
  const uint16_t* s_in = uniform_ptr(ex.s_in);
  const uint8_t* q_gate = SWIGLU ? uniform_ptr(ex.q_gate) : nullptr;
  const uint16_t* s_gate = SWIGLU ? uniform_ptr(ex.s_gate) : nullptr;
  auto run = [&](auto nrm_tag, auto two_tag) {
    constexpr int NRM = decltype(nrm_tag)::value;
    constexpr bool TWO = decltype(two_tag)::value;
    const int task_rows = RW * NRM;
    for (int r0 = row_begin + wave * task_rows; r0 < row_end; r0 += nwaves * task_rows) {
      float tot[NRM * NM];
      if constexpr (SWIGLU) {
        const uint8_t* const qq[2] = {q_in, q_gate};
        const uint16_t* const ss[2] = {s_in, s_gate};
        gemv_task<BITS, NRM, 2, TWO>(qq, ss, d, group, P, p, r0 + rsub, RW, f, XP, XK, tot);
      } else {
        const uint8_t* const qq[1] = {q_in};
        const uint16_t* const ss[1] = {s_in};
        gemv_task<BITS, NRM, 1, TWO>(qq, ss, d, group, P, p, r0 + rsub, RW, f, XP, XK, tot);
      }
      fold_rows<NRM, NM>(tot, P, lane);
      if (p < NRM) {
        const int row = r0 + p * RW + rsub;
        if (row < row_end) {
          float v;
          if constexpr (SWIGLU) {
            const float a = tot[0];
            v = a / (1.0f + __expf(-a)) * tot[NRM];
          } else {
            v = fmaxf(tot[0], 0.f);
          }
          h_out[row] = v;
        }
      }
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

// Phase 1 for one token: (optionally) top-k from the router logits, then for each chosen expert
// h[slot][r] = act(W_in[r] . x [, W_gate[r] . x]) for the rows r this workgroup owns.
__global__ __launch_bounds__(768) void k_ffn_in(LayerDims L, const DevExpert* __restrict__ table,
                                                 const float* __restrict__ logits, int32_t* __restrict__ idx_out,
                                                 float* __restrict__ gate_out, int32_t fixed_expert,
                                                 const void* __restrict__ x, float* __restrict__ h,
                                                 int32_t rows_per_wg) {
  extern __shared__ uint32_t smem[];
  __shared__ int sel_e[8];
  __shared__ float sel_g[8];
  const int d = L.d_model, f = L.d_ff;
  const int token = blockIdx.y;
  uint32_t* XP = smem;                    // d/2 words
  float* XK = (float*)(smem + d / 2);     // at most d/16 words
  const int k = fixed_expert >= 0 ? 1 : L.top_k;
  if (fixed_expert < 0) {
    if (threadIdx.x < 64) topk_from_logits(logits + (size_t)token * L.n_experts, L.n_experts, k, L.renorm,
                                           threadIdx.x, sel_e, sel_g, nullptr);
    __syncthreads();
    if (blockIdx.x == 0 && threadIdx.x < k) {
      idx_out[(size_t)token * k + threadIdx.x] = sel_e[threadIdx.x];
      gate_out[(size_t)token * k + threadIdx.x] = sel_g[threadIdx.x];
    }
  }
  const int row_begin = blockIdx.x * rows_per_wg;
  const int row_end = min(f, row_begin + rows_per_wg);
  const bool sw = L.act == MOEQ_ACT_SWIGLU;
  int staged_bits = 0;
  for (int j = 0; j < k; ++j) {
    const int slot = fixed_expert >= 0 ? token : token * k + j;
    const int e = fixed_expert >= 0 ? fixed_expert : sel_e[j];
    const DevExpert ex = table[e];
    float* h_out = h + (size_t)slot * f;
    // Opaque copy of the thread index: keeps the per-variant lane arithmetic inside this iteration
    // instead of being hoisted (and spilled) ahead of the loop for every bitwidth at once.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    auto run = [&](auto bits_tag) {
      constexpr int BITS = decltype(bits_tag)::value;
      if (staged_bits != BITS) {   // the activation layout depends on the bitwidth only
        if (staged_bits != 0) __syncthreads();
        if (L.x_bf16) {
          const uint16_t* xr = (const uint16_t*)x + (size_t)token * d;
          stage_x<BITS>([&](int i) { return bf16_bits_to_f32(xr[i]); }, d, L.group, XP, XK);
        } else {
          const float* xr = (const float*)x + (size_t)token * d;
          stage_x<BITS>([&](int i) { return xr[i]; }, d, L.group, XP, XK);
        }
        staged_bits = BITS;
      }
      if (sw) ffn_in_tasks<BITS, true>(ex, tid, d, f, L.group, row_begin, row_end, h_out, XP, XK);
      else ffn_in_tasks<BITS, false>(ex, tid, d, f, L.group, row_begin, row_end, h_out, XP, XK);
    };
    switch (ex.bits) {
      case 2: run(std::integral_constant<int, 2>{}); break;
      case 4: run(std::integral_constant<int, 4>{}); break;
      default: run(std::integral_constant<int, 8>{}); break;
    }
  }
}

// ---------------------------------------------------------------------------------------------
template <int BITS>
__device__ __forceinline__ void ffn_out_tasks(const DevExpert& ex, int tid, int d, int f, int group, float g,
                                              int row_begin, int row_end, float* ybuf, const uint32_t* XP,
                                              const float* XK) {
  const int C = f / Fmt<BITS>::WPC;
  const int P = lanes_per_row(C), RW = 64 / P;
  const int lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
  const int p = lane % P, rsub = lane / P;
  const int nrm = pick_nrm(row_end - row_begin, RW, nwaves, P, kBlock);
  const bool two = (BITS == 2) && (group == 32);
  const uint8_t* const qq[1] = {uniform_ptr(ex.q_out)};
  const uint16_t* const ss[1] = {uniform_ptr(ex.s_out)};
  auto run = [&](auto nrm_tag, auto two_tag) {
    constexpr int NRM = decltype(nrm_tag)::value;
    constexpr bool TWO = decltype(two_tag)::value;
    const int task_rows = RW * NRM;
    for (int r0 = row_begin + wave * task_rows; r0 < row_end; r0 += nwaves * task_rows) {
      float tot[NRM];
      gemv_task<BITS, NRM, 1, TWO>(qq, ss, f, group, P, p, r0 + rsub, RW, d, XP, XK, tot);
      fold_rows<NRM, 1>(tot, P, lane);
      if (p < NRM) {
        const int row = r0 + p * RW + rsub;
        if (row < row_end) ybuf[row - row_begin] = fmaf(g, tot[0], ybuf[row - row_begin]);
      }
    }
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

// Phase 2 + combine for one token: y[t][r] (+)= sum_j gate_j * W_out_j[r] . h[slot_j], summed in top-k
// order in LDS for the rows this workgroup owns, each output written once.
__global__ __launch_bounds__(768) void k_ffn_out(LayerDims L, const DevExpert* __restrict__ table,
                                                  const int32_t* __restrict__ idx, const float* __restrict__ gate,
                                                  int32_t fixed_expert, int32_t accumulate,
                                                  const float* __restrict__ h, float* __restrict__ y,
                                                  int32_t rows_per_wg) {
  extern __shared__ uint32_t smem[];
  const int d = L.d_model, f = L.d_ff;
  const int token = blockIdx.y;
  uint32_t* XP = smem;                      // f/2 words
  float* XK = (float*)(smem + f / 2);       // at most f/16 words
  float* ybuf = XK + f / 16;                // rows_per_wg words
  float* y_out = y + (size_t)token * d;
  const int row_begin = blockIdx.x * rows_per_wg;
  const int row_end = min(d, row_begin + rows_per_wg);
  for (int i = threadIdx.x; i < rows_per_wg; i += blockDim.x) ybuf[i] = 0.f;
  const int k = fixed_expert >= 0 ? 1 : L.top_k;
  for (int j = 0; j < k; ++j) {
    const int slot = fixed_expert >= 0 ? token : token * k + j;
    const int e = fixed_expert >= 0 ? fixed_expert : idx[slot];
    const float g = gate ? gate[slot] : 1.0f;
    const DevExpert ex = table[e];
    const float* hr = h + (size_t)slot * f;
    int tid = threadIdx.x;       // opaque copy, see k_ffn_in
    asm volatile("" : "+v"(tid));
    if (j > 0) __syncthreads();  // everyone is done with the previous choice's activations and sums
    auto run = [&](auto bits_tag) {
      constexpr int BITS = decltype(bits_tag)::value;
      stage_x<BITS>([&](int i) { return hr[i]; }, f, L.group, XP, XK);
      ffn_out_tasks<BITS>(ex, tid, d, f, L.group, g, row_begin, row_end, ybuf, XP, XK);
    };
    switch (ex.bits) {
      case 2: run(std::integral_constant<int, 2>{}); break;
      case 4: run(std::integral_constant<int, 4>{}); break;
      default: run(std::integral_constant<int, 8>{}); break;
    }
  }
  __syncthreads();
  for (int i = row_begin + (int)threadIdx.x; i < row_end; i += blockDim.x)
    y_out[i] = accumulate ? y_out[i] + ybuf[i - row_begin] : ybuf[i - row_begin];
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

inline size_t lds_bytes(int cols) {
  // activation pairs (2 bytes per weight position) + offset terms (at most one per 16 weights)
  return (size_t)cols * 2 + (size_t)(cols / 16) * 4;
}

// Rows per workgroup and wavefronts per workgroup for a GEMV over `rows` output rows whose packed row
// has at least `min_chunks` 16-byte chunks. About one workgroup per compute unit when there is enough
// work; row ranges are multiples of 64 rows/P so that tasks never straddle workgroups.
struct Split { int rows_per_wg, gx, threads; };
Split plan_rows(int rows, int min_P, int T, int nrm_max) {
  const int RWmax = 64 / min_P;                       // rows a wavefront covers per step, worst bitwidth
  const int cus = num_cus();
  int target = cus / (T < 1 ? 1 : (T > cus ? cus : T));  // workgroups per token
  if (target < 1) target = 1;
  int rpw = (rows + target - 1) / target;
  rpw = (rpw + RWmax - 1) / RWmax * RWmax;
  if (rpw < RWmax) rpw = RWmax;
  Split s;
  s.rows_per_wg = rpw;
  s.gx = (rows + rpw - 1) / rpw;
  // wavefronts per workgroup: the count in [4, 12] that leaves the fewest idle task slots, more on ties
  int best_w = 4;
  double best_eff = -1.0;
  for (int w = 12; w >= 4; --w) {
    const int nrm = pick_nrm(rpw, RWmax, w, min_P, nrm_max);
    const int tasks = (rpw + RWmax * nrm - 1) / (RWmax * nrm);
    const int rounds = (tasks + w - 1) / w;
    const double eff = (double)tasks / ((double)rounds * w);
    if (eff > best_eff + 1e-9) { best_eff = eff; best_w = w; }
  }
  s.threads = best_w * 64;
  return s;
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

}  // namespace

hipError_t launch_topk(const LayerDims& L, const float* logits, int32_t T, int32_t* idx, float* gate, float* probs,
                       hipStream_t st) {
  hipLaunchKernelGGL(k_topk, dim3(T), dim3(64), 0, st, L, logits, idx, gate, probs);
  return hipGetLastError();
}

hipError_t launch_ffn_in(const LayerDims& L, const DevExpert* table, const float* logits, int32_t* idx_out,
                         float* gate_out, int32_t fixed_expert, const void* x, int32_t T, float* h, hipStream_t st) {
  const Split sp = plan_rows(L.d_ff, min_lanes_per_row(L.d_model), T, L.act == MOEQ_ACT_SWIGLU ? kBlock / 2 : kBlock);
  const size_t lds = lds_bytes(L.d_model);
  static size_t lds_set = 0;
  if (lds > 48 * 1024 && lds > lds_set) {
    hipError_t e = hipFuncSetAttribute((const void*)k_ffn_in, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    lds_set = lds;
  }
  hipLaunchKernelGGL(k_ffn_in, dim3(sp.gx, T), dim3(sp.threads), lds, st, L, table, logits, idx_out, gate_out,
                     fixed_expert, x, h, sp.rows_per_wg);
  return hipGetLastError();
}

hipError_t launch_ffn_out(const LayerDims& L, const DevExpert* table, const int32_t* idx, const float* gate,
                          int32_t fixed_expert, int32_t accumulate, const float* h, int32_t T, float* y,
                          hipStream_t st) {
  const Split sp = plan_rows(L.d_model, min_lanes_per_row(L.d_ff), T, kBlock);
  const size_t lds = lds_bytes(L.d_ff) + (size_t)sp.rows_per_wg * sizeof(float);
  static size_t lds_set = 0;
  if (lds > 48 * 1024 && lds > lds_set) {
    hipError_t e = hipFuncSetAttribute((const void*)k_ffn_out, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    lds_set = lds;
  }
  hipLaunchKernelGGL(k_ffn_out, dim3(sp.gx, T), dim3(sp.threads), lds, st, L, table, idx, gate, fixed_expert,
                     accumulate, h, y, sp.rows_per_wg);
  return hipGetLastError();
}

}  // namespace moeq
