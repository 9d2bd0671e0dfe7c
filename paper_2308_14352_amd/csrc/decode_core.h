// Device-side building blocks shared by the decode kernels: the unpack arithmetic on packed INT2/INT4/INT8
// rows, activation staging in LDS, DPP reductions, the streaming GEMV core and the softmax + top-k of one
// token. Everything is in an unnamed namespace: each translation unit gets its own copy.
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
// activation registers (for SwiGLU the rows of w1 and w3 count as separate "virtual rows"). The
// loads of the next block of tiles are issued before the arithmetic of the current one, across task
// boundaries, so a wavefront always has 4 to 8 loads in flight. Row totals are folded across the P
// lanes with a transposing butterfly on DPP. A workgroup owns a fixed range of output rows for all
// k chosen experts of its token, so the gate-weighted sum over the experts is ordered and needs no
// atomics.
#pragma once
#include <hip/hip_fp16.h>

#include <type_traits>

#include "moeq_internal.h"

namespace moeq {
namespace {


typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// Loads through pointers that are known to point to device memory. A pointer that was itself read from
// memory (an expert record) has no address space the compiler can see; without the cast it would emit
// FLAT loads, which count on the LDS counter as well, so that every wait for an LDS read would also wait
// for all weight loads in flight.
#define MOEQ_GLOBAL __attribute__((address_space(1)))
// 16-byte load with the non-temporal hint: packed weights are read once per call and should not
// displace the activations and scales that are reused from the caches.
__device__ __forceinline__ uint4 load_stream16(const uint8_t* ptr) {
  const u32x4_t v = __builtin_nontemporal_load((const MOEQ_GLOBAL u32x4_t*)ptr);
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint4 gload_u32x4(const uint8_t* ptr) {
  const u32x4_t v = *(const MOEQ_GLOBAL u32x4_t*)ptr;
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint32_t gload_u16(const uint8_t* ptr) { return *(const MOEQ_GLOBAL uint16_t*)ptr; }
__device__ __forceinline__ uint32_t gload_u32(const uint8_t* ptr) { return *(const MOEQ_GLOBAL uint32_t*)ptr; }
__device__ __forceinline__ uint2 gload_u32x2_nt(const uint8_t* ptr) {
  typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
  const u32x2_t v = __builtin_nontemporal_load((const MOEQ_GLOBAL u32x2_t*)ptr);
  return make_uint2(v.x, v.y);
}
__device__ __forceinline__ uint2 gload_u32x2(const uint8_t* ptr) {
  typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
  const u32x2_t v = *(const MOEQ_GLOBAL u32x2_t*)ptr;
  return make_uint2(v.x, v.y);
}

// v / group for a per-lane v: a shift when the group size is a power of two (gsh = its log2, else -1), the
// (40-instruction) division otherwise. gsh is uniform, so this is a branch, not a select.
__device__ __forceinline__ int group_shift(int group) { return (group & (group - 1)) == 0 ? __builtin_ctz(group) : -1; }
__device__ __forceinline__ uint32_t div_group(uint32_t v, int group, int gsh) {
  if (gsh >= 0) return v >> gsh;
  return v / (uint32_t)group;
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint32_t f32_to_f16_bits(float v) { return (uint32_t)__half_as_ushort(__float2half_rn(v)); }
__device__ __forceinline__ float f16_bits_to_f32(uint32_t h) { return __half2float(__ushort_as_half((uint16_t)h)); }

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

// Inverse of pair_pos: where activation number `col` of a vector of C chunks lives in the staged
// layout (index in units of binary16 values) and its pre-division.
template <int BITS>
__device__ __forceinline__ int staged_index(int col, int C, float& prescale) {
  constexpr int WPC = Fmt<BITS>::WPC;
  const int c = col / WPC, pos = col % WPC;
  int pi, half;
  if (BITS == 8) {
    const int d = pos >> 2, b = pos & 3;
    pi = 2 * d + (b & 1); half = b >> 1; prescale = 1.0f;
  } else if (BITS == 4) {
    const int d = pos >> 3, n = pos & 7, k = n & 3;
    pi = 4 * d + k; half = n >> 2; prescale = (k & 1) ? 0.0625f : 1.0f;
  } else {
    const int d = pos >> 4, jj = pos & 15, j = jj & 7;
    pi = 8 * d + j; half = jj >> 3;
    const int e = j < 5 ? j : j - 5;
    prescale = 1.0f / (float)(1 << (2 * e));
  }
  return (((pi >> 2) * C + c) * 4 + (pi & 3)) * 2 + half;
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

// ---------------------------------------------------------------------------------------------
// Matrix-core operands (v_mfma_f32_16x16x32_f16). B-operand lane l holds 8 consecutive k of column n = l%16
// (k block l/16); A-operand lane l holds 8 consecutive k of row m = l%16; D element i of lane l is
// D[4*(l/16) + i][l%16].
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4v_t __attribute__((ext_vector_type(4)));

// Eight codes as the four pair registers dword_dot<BITS> would consume: INT4: the 8 codes of w0; INT2: the
// lower (HH = 0) or upper (HH = 1) half of the 16 codes of w0; INT8: the 4 + 4 codes of w0 and w1.
template <int BITS, int HH>
__device__ __forceinline__ half8_t codes8(uint32_t w0, uint32_t w1) {
  u32x4v_t r;
  if (BITS == 4) {
    const uint32_t w8 = w0 >> 8;
    r = {w0 & 0x000f000fu, w0 & 0x00f000f0u, w8 & 0x000f000fu, w8 & 0x00f000f0u};
  } else if (BITS == 8) {
    // bytes 1 and 3 of a word into the low bytes of the two halves: one byte permute (selector 0x0c = zero byte)
    r = {w0 & 0x00ff00ffu, __builtin_amdgcn_perm(0u, w0, 0x0c030c01u), w1 & 0x00ff00ffu,
         __builtin_amdgcn_perm(0u, w1, 0x0c030c01u)};
  } else if (HH == 0) {
    r = {w0 & 0x00030003u, w0 & 0x000c000cu, w0 & 0x00300030u, w0 & 0x00c000c0u};
  } else {
    const uint32_t w10 = w0 >> 10;
    r = {w0 & 0x03000300u, w10 & 0x00030003u, w10 & 0x000c000cu, w10 & 0x00300030u};
  }
  return __builtin_bit_cast(half8_t, r);
}
__device__ __forceinline__ half8_t as_half8(const uint4& v) {
  const u32x4v_t r = {v.x, v.y, v.z, v.w};
  return __builtin_bit_cast(half8_t, r);
}
__device__ __forceinline__ float4_t mfma16(half8_t a, half8_t b, float4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// ---------------------------------------------------------------------------------------------
// Activation staging. An activation vector (hidden states, or the intermediate h of an FFN) enters the
// multipliers as binary16, so it is first brought into binary16's range: the vector is multiplied by the power
// of two 2^-e that puts its largest magnitude into [2^14, 2^15), converted (round to nearest even), and the
// consumer multiplies its fp32 results by 2^e again. Both scalings are exact, so the staged values carry
// 11 significant bits at every magnitude a float can hold, and elements down to 2^-29 of the largest one stay
// normal numbers even after the pre-divisions of the pair order (Section 4.1, "Baselines": the decompressed
// weights are used in FP32 arithmetic - the input range of the path is fp32's, not binary16's).
// Step 1 (stage_normalised): the vector goes to LDS as linear binary16 (RAW) with 16-byte accesses. Step 2
// (permute_x): pair register pi of chunk c goes to word ((pi/4) * C + c) * 4 + pi%4 of XP, so a lane's
// 128-bit reads of consecutive chunks are conflict-free, and XK[c * spc + j] = 2^(b-1) * 2^-24 * (sum of the
// activations of scale slice j of chunk c). Callers put a barrier between the steps and after step 2.
enum XKind { X_F32 = 0, X_BF16 = 1 };

__device__ __forceinline__ float wave_max(float v);   // defined with the other cross-lane helpers below

struct XItem { float v[8]; };

__device__ __forceinline__ XItem load_x_item(const void* __restrict__ x, int kind, int i) {
  XItem it;
  if (kind == X_BF16) {
    const uint4 v = ((const uint4*)x)[i];
    const uint32_t in[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      it.v[2 * k] = bf16_bits_to_f32(in[k] & 0xffffu);
      it.v[2 * k + 1] = bf16_bits_to_f32(in[k] >> 16);
    }
  } else {
    const float4 a = ((const float4*)x)[2 * i], b = ((const float4*)x)[2 * i + 1];
    it.v[0] = a.x; it.v[1] = a.y; it.v[2] = a.z; it.v[3] = a.w;
    it.v[4] = b.x; it.v[5] = b.y; it.v[6] = b.z; it.v[7] = b.w;
  }
  return it;
}
__device__ __forceinline__ float item_absmax(const XItem& it) {
  float m = 0.f;
#pragma unroll
  for (int k = 0; k < 8; ++k) m = fmaxf(m, fabsf(it.v[k]));      // a NaN element is skipped by fmaxf
  return m;
}
__device__ __forceinline__ uint4 item_to_f16(const XItem& it, float dn) {
  uint32_t o[4];
#pragma unroll
  for (int k = 0; k < 4; ++k)
    o[k] = f32_to_f16_bits(it.v[2 * k] * dn) | (f32_to_f16_bits(it.v[2 * k + 1] * dn) << 16);
  return make_uint4(o[0], o[1], o[2], o[3]);
}

// The exponent e of the normalisation for a vector whose largest magnitude is m: m * 2^-e lies in
// [2^14, 2^15). e is kept inside [-110, 110] so that both 2^e and 2^-e are normal floats: vectors whose
// largest magnitude is below 2^-96 lose precision gradually, above 2^124 they overflow to infinity. m == 0,
// infinite or NaN gives e = 0.
__device__ __forceinline__ int norm_exponent(float m) {
  int e = 0;
  if (m > 0.f && m < INFINITY) e = __builtin_amdgcn_frexp_expf(m) - 1 - 14;   // frexp: m = f * 2^exp, f in [0.5, 1)
  return min(max(e, -110), 110);
}
__device__ __forceinline__ float pow2f(int e) { return __uint_as_float((uint32_t)(e + 127) << 23); }   // |e| <= 126

// Step 1, called by EVERY thread of the workgroup at one place (it holds a barrier): x (cols values in the
// format `kind`) -> RAW (cols binary16 values, normalised). Returns 2^e, the factor that undoes the
// normalisation. red: nthreads/64 floats of LDS. The first 8 values of a thread stay in registers across the
// barrier, further ones (long vectors on small workgroups) are read again from the caches.
__device__ __forceinline__ float stage_normalised(const void* __restrict__ x, int kind, int cols, int tid, int nthreads,
                                                  uint16_t* RAW, float* red) {
  uint4* RAW4 = (uint4*)RAW;
  const int n = cols / 8;
  XItem first;
#pragma unroll
  for (int k = 0; k < 8; ++k) first.v[k] = 0.f;
  if (tid < n) first = load_x_item(x, kind, tid);
  float m = item_absmax(first);
  for (int i = tid + nthreads; i < n; i += nthreads) m = fmaxf(m, item_absmax(load_x_item(x, kind, i)));
  m = wave_max(m);
  if ((tid & 63) == 0) red[tid >> 6] = m;
  __syncthreads();
  float M = 0.f;
  for (int w = 0; w < (nthreads >> 6); ++w) M = fmaxf(M, red[w]);
  const int e = norm_exponent(M);
  const float dn = pow2f(-e);
  if (tid < n) RAW4[tid] = item_to_f16(first, dn);
  for (int i = tid + nthreads; i < n; i += nthreads) RAW4[i] = item_to_f16(load_x_item(x, kind, i), dn);
  return pow2f(e);
}

// XK from a linear binary16 vector (LDS or global memory).
template <int BITS>
__device__ __forceinline__ void offset_terms(const uint16_t* lin, int cols, int group, int tid, int nthreads,
                                             float* XK) {
  constexpr int WPC = Fmt<BITS>::WPC;
  const int sub = group < WPC ? group : WPC;   // 16, 32 or 64 weights share a scale inside a chunk
  const uint4* lin4 = (const uint4*)lin;
  for (int s = tid; s < cols / sub; s += nthreads) {
    float acc = 0.f;
    for (int i = 0; i < sub / 8; ++i) {
      const uint4 v = lin4[s * (sub / 8) + i];
      acc += (f16_bits_to_f32(v.x & 0xffffu) + f16_bits_to_f32(v.x >> 16)) + (f16_bits_to_f32(v.y & 0xffffu) + f16_bits_to_f32(v.y >> 16));
      acc += (f16_bits_to_f32(v.z & 0xffffu) + f16_bits_to_f32(v.z >> 16)) + (f16_bits_to_f32(v.w & 0xffffu) + f16_bits_to_f32(v.w >> 16));
    }
    XK[s] = acc * (Fmt<BITS>::OFF * 5.9604644775390625e-08f);
  }
}

// The negated offset terms of whole lane-column ranges (128 columns, 64 at 8 bits) of a linear binary16
// vector in LDS: KS[r] = -2^(b-1) * 2^-24 * (sum of the activations of range r). Four threads share a range.
template <int BITS>
__device__ __forceinline__ void range_offset_terms(const uint16_t* lin, int cols, int tid, int nthreads, float* KS,
                                                   int stride = 1);

// Where permute_x puts 16-byte item i of the pair order: by default item i itself.
struct PairOrderLinear {
  __device__ __forceinline__ int operator()(int i) const { return i; }
};

// Two binary16 halves of two registers as one pair register: (lo of a, lo of b) or (hi of a, hi of b).
__device__ __forceinline__ uint32_t pair_lo(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ uint32_t pair_hi(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }
// Both halves of a pair register times a power of two (one packed multiply; exact, or the single rounding to
// a binary16 subnormal that a widened multiply followed by a conversion gives as well).
__device__ __forceinline__ uint32_t pair_scale(uint32_t p, float s) {
  const half2_t v = __builtin_bit_cast(half2_t, p) * (half2_t){(_Float16)s, (_Float16)s};
  return __builtin_bit_cast(uint32_t, v);
}

// The staged layout, written with 16-byte accesses: the four pair registers of a quad (pair_pos) are made of
// eight (2-bit codes: sixteen) consecutive activations, so one work item turns one or two 16-byte reads of
// RAW into one or two 16-byte writes: quad q of chunk c goes to XP4[q * C + c].
template <int BITS, bool RANGES = false, typename Map = PairOrderLinear>
__device__ __forceinline__ void permute_x(const uint16_t* RAW, int cols, int group, int tid, int nthreads,
                                          uint32_t* XP, float* XK, Map at = Map()) {
  constexpr int WPC = Fmt<BITS>::WPC;
  const int C = cols / WPC;
  const uint4* R4 = (const uint4*)RAW;
  uint4* X4 = (uint4*)XP;
  if constexpr (BITS == 4) {
    // chunk = 32 activations = 4 reads; quad d = dword d of the codes: pairs (k, k+4), odd k pre-divided by 16
    for (int i = tid; i < 4 * C; i += nthreads) {
      const int q = i / C, c = i - q * C;
      const uint4 v = R4[c * 4 + q];
      X4[at(i)] = make_uint4(pair_lo(v.x, v.z), pair_scale(pair_hi(v.x, v.z), 0.0625f), pair_lo(v.y, v.w),
                             pair_scale(pair_hi(v.y, v.w), 0.0625f));
    }
  } else if constexpr (BITS == 8) {
    // chunk = 16 activations = 2 reads; quad q = dwords 2q, 2q+1 of the codes: pairs (k, k+2)
    for (int i = tid; i < 2 * C; i += nthreads) {
      const int q = i / C, c = i - q * C;
      const uint4 v = R4[c * 2 + q];
      X4[at(i)] = make_uint4(pair_lo(v.x, v.y), pair_hi(v.x, v.y), pair_lo(v.z, v.w), pair_hi(v.z, v.w));
    }
  } else {
    // chunk = 64 activations = 8 reads; dword d of the codes: pairs (j, j+8), j = 0..7, in the quads 2d
    // (j = 0..3, pre-divided by 1, 4, 16, 64) and 2d+1 (j = 4..7, pre-divided by 256, 1, 4, 16)
    for (int i = tid; i < 4 * C; i += nthreads) {
      const int dd = i / C, c = i - dd * C;
      const uint4 a = R4[c * 8 + 2 * dd], b = R4[c * 8 + 2 * dd + 1];
      X4[at((2 * dd) * C + c)] = make_uint4(pair_lo(a.x, b.x), pair_scale(pair_hi(a.x, b.x), 0.25f),
                                            pair_scale(pair_lo(a.y, b.y), 0.0625f), pair_scale(pair_hi(a.y, b.y), 0.015625f));
      X4[at((2 * dd + 1) * C + c)] = make_uint4(pair_scale(pair_lo(a.z, b.z), 0.00390625f), pair_hi(a.z, b.z),
                                                pair_scale(pair_lo(a.w, b.w), 0.25f), pair_scale(pair_hi(a.w, b.w), 0.0625f));
    }
  }
  if constexpr (RANGES) range_offset_terms<BITS>(RAW, cols, tid, nthreads, XK);
  else offset_terms<BITS>(RAW, cols, group, tid, nthreads, XK);
}

// ---------------------------------------------------------------------------------------------
// Cross-lane helpers on DPP (data-parallel primitives: one instruction, no LDS round trip).
template <int CTRL>
__device__ __forceinline__ float dpp(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
constexpr int kDppXor1 = 0xB1;   // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;   // quad_perm [2,3,0,1]
constexpr int kDppRor4 = 0x124;  // row_ror:4  (rotation inside a 16-lane row)
constexpr int kDppRor8 = 0x128;  // row_ror:8

template <int BITS>
__device__ __forceinline__ void range_offset_terms(const uint16_t* lin, int cols, int tid, int nthreads, float* KS,
                                                   int stride) {
  constexpr int R = BITS == 8 ? 64 : 128;    // columns of a range
  constexpr int V = R / 32;                  // 128-bit loads per thread
  const uint4* lin4 = (const uint4*)lin;
  const int n4 = (cols / R) * 4;             // a multiple of 4: whole quads of lanes run the loop together
  for (int i = tid; i < n4; i += nthreads) {
    float acc = 0.f;
#pragma unroll
    for (int v4 = 0; v4 < V; ++v4) {
      const uint4 v = lin4[i * V + v4];
      acc += (f16_bits_to_f32(v.x & 0xffffu) + f16_bits_to_f32(v.x >> 16)) + (f16_bits_to_f32(v.y & 0xffffu) + f16_bits_to_f32(v.y >> 16));
      acc += (f16_bits_to_f32(v.z & 0xffffu) + f16_bits_to_f32(v.z >> 16)) + (f16_bits_to_f32(v.w & 0xffffu) + f16_bits_to_f32(v.w >> 16));
    }
    acc += dpp<kDppXor1>(acc);
    acc += dpp<kDppXor2>(acc);
    if ((i & 3) == 0) KS[(i >> 2) * stride] = acc * (-Fmt<BITS>::OFF * 5.9604644775390625e-08f);
  }
}

// Sum over the P lanes of a row group (P a power of two, groups are contiguous lanes) of NM*NRM row
// totals per lane; v = m*NRM + i, NRM <= min(P, 4). Afterwards every lane holds, in v[m*NRM] (m < NM),
// the group total of row i = lane & (NRM-1) of matrix m.
template <int NRM, int NM>
__device__ __forceinline__ void fold_rows(float (&v)[NRM * NM], int P, int lane) {
  static_assert(NRM == 1 || NRM == 2 || NRM == 4, "transposing steps use the two quad permutes only");
  if (NRM >= 2) {  // transposing step on lane bit 0
    const bool upper = (lane & 1) != 0;
#pragma unroll
    for (int m = 0; m < NM; ++m)
#pragma unroll
      for (int i = 0; i < NRM / 2; ++i) {
        const float a = v[m * NRM + 2 * i], b = v[m * NRM + 2 * i + 1];
        v[m * NRM + i] = (upper ? b : a) + dpp<kDppXor1>(upper ? a : b);
      }
  }
  if (NRM >= 4) {  // transposing step on lane bit 1
    const bool upper = (lane & 2) != 0;
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      const float a = v[m * NRM], b = v[m * NRM + 1];
      v[m * NRM] = (upper ? b : a) + dpp<kDppXor2>(upper ? a : b);
    }
  }
#pragma unroll
  for (int m = 0; m < NM; ++m) {
    float t = v[m * NRM];
    if (NRM < 2 && P >= 2) t += dpp<kDppXor1>(t);
    if (NRM < 4 && P >= 4) t += dpp<kDppXor2>(t);
    if (P >= 16) {
      t += dpp<kDppRor4>(t);
      t += dpp<kDppRor8>(t);
    } else if (P == 8) {
      t += __shfl_xor(t, 4, 64);
    }
    if (P >= 32) t += __shfl_xor(t, 16, 64);
    if (P >= 64) t += __shfl_xor(t, 32, 64);
    v[m * NRM] = t;
  }
}

__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp<kDppXor1>(v));
  v = fmaxf(v, dpp<kDppXor2>(v));
  v = fmaxf(v, dpp<kDppRor4>(v));
  v = fmaxf(v, dpp<kDppRor8>(v));
  const int b = __builtin_bit_cast(int, v);
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
  return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp<kDppXor1>(v);
  v += dpp<kDppXor2>(v);
  v += dpp<kDppRor4>(v);
  v += dpp<kDppRor8>(v);
  const int b = __builtin_bit_cast(int, v);
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
  return (r0 + r1) + (r2 + r3);
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

// ---------------------------------------------------------------------------------------------
struct Tile {
  uint4 w;
  uint32_t s;  // one binary16 scale, or two adjacent ones (INT2 with group 32)
};
constexpr int kBlock = 4;  // tiles per block; one block is computed while the next is in flight
constexpr int kMaxKs = 4;  // at most this many wavefront teams split a row along its length

// All tasks of one wavefront for one expert. A task is NRM rows (per lane group) of each of NM
// matrices: rows r0 + i*RW + rsub, i < NRM, with r0 = row_begin + (wave + k*nwaves) * RW*NRM.
// epilogue(row, totals[NM]) is called by one lane per finished row (row < row_end guaranteed).
// stage() is called exactly once by EVERY thread of the workgroup (it may contain barriers), after the
// wavefront's first block of weight loads has been issued and before any activation is read from
// XP/XK: whatever it takes to get the activations into LDS overlaps with the first loads' latency.
template <int BITS, int NRM, int NM, bool TWO, typename Epilogue, typename Stage>
__device__ __forceinline__ void gemv_stream(const uint8_t* const (&q)[NM], const uint16_t* const (&s)[NM], int cols,
                                            int group, int nrows, int row_begin, int row_end, int lane, int wave,
                                            int nwaves, int ks_parts, const uint32_t* XP, const float* XK,
                                            Epilogue epilogue, Stage stage) {
  constexpr int WPC = Fmt<BITS>::WPC, PPC = Fmt<BITS>::PPC;
  constexpr int NR = NRM * NM;
  static_assert(NR <= kBlock && kBlock % NR == 0, "rows in flight must divide the block");
  constexpr int CPB = kBlock / NR;  // chunk steps per block
  const int C = cols / WPC;
  int P = 1;
  while (P < 64 && C % (P * 2) == 0) P *= 2;
  const int RW = 64 / P;
  const int p = lane % P, rsub = lane / P;
  // The nwaves wavefronts form ks_parts teams; team `part` covers the chunk steps
  // [jb, jb + J) of every row, and its wavefronts share the tasks. epilogue gets partial sums then.
  const int wpp = nwaves / ks_parts;            // wavefronts per team
  const int part = wave / wpp, tw = wave - part * wpp;
  const int Jfull = C / P;
  const int jb = (part * Jfull) / ks_parts;
  const int J = (wave < nwaves) ? ((part + 1) * Jfull) / ks_parts - jb : 0;
  const int ng = cols / group;
  const int gsh = group_shift(group);
  const int task_rows = RW * NRM;
  const int n_tasks = (row_end - row_begin + task_rows - 1) / task_rows;
  const int n_my = (wave < nwaves && tw < n_tasks) ? (n_tasks - tw + wpp - 1) / wpp : 0;
  const int S = n_my * J;  // chunk steps of this wavefront (0: it only takes part in stage())
  const uint4* XP4 = (const uint4*)XP;
  const uint32_t jstride = (uint32_t)P * 16u;
  const uint32_t row_bytes = (uint32_t)C * 16u;

  // prefetch cursor
  int pk = 0, pj = 0;
  uint32_t qoff[NR], soff[NR];
  auto load_step = [&](Tile (&t)[kBlock], int u0) {
    if (pj == 0) {
      const int r0 = row_begin + (tw + pk * wpp) * task_rows + rsub;
#pragma unroll
      for (int v = 0; v < NR; ++v) {
        int row = r0 + (v % NRM) * RW;
        row = row < nrows ? row : nrows - 1;
        qoff[v] = (uint32_t)row * row_bytes + (uint32_t)p * 16u;
        soff[v] = ((uint32_t)row * (uint32_t)ng) * 2u;
      }
    }
    const uint32_t g0 = div_group((uint32_t)((p + (jb + pj) * P) * WPC), group, gsh) * 2u;
#pragma unroll
    for (int v = 0; v < NR; ++v) {
      const int m = v / NRM;
      t[u0 + v].w = load_stream16(q[m] + (qoff[v] + (uint32_t)(jb + pj) * jstride));
      const uint8_t* sb = (const uint8_t*)s[m];
      if (TWO) t[u0 + v].s = gload_u32(sb + (soff[v] + g0));
      else t[u0 + v].s = gload_u16(sb + (soff[v] + g0));
    }
    if (++pj == J) { pj = 0; ++pk; }
  };
  auto load_block = [&](Tile (&t)[kBlock], int blk) {
#pragma unroll
    for (int c = 0; c < CPB; ++c)
      if (blk * CPB + c < S) load_step(t, c * NR);
  };

  // compute cursor
  int ck = 0, cj = 0;
  float tot[NR];
  auto compute_step = [&](const Tile (&t)[kBlock], int u0) {
    if (cj == 0) {
#pragma unroll
      for (int v = 0; v < NR; ++v) tot[v] = 0.f;
    }
    uint32_t xr[PPC];
    const int c = p + (jb + cj) * P;
#pragma unroll
    for (int qq = 0; qq < PPC / 4; ++qq) {
      const uint4 t4 = XP4[qq * C + c];
      xr[4 * qq] = t4.x; xr[4 * qq + 1] = t4.y; xr[4 * qq + 2] = t4.z; xr[4 * qq + 3] = t4.w;
    }
    float k0, k1 = 0.f;
    if (TWO) { k0 = XK[2 * c]; k1 = XK[2 * c + 1]; }
    else k0 = XK[c];
#pragma unroll
    for (int v = 0; v < NR; ++v) {
      const uint4 w = t[u0 + v].w;
      const uint32_t sraw = t[u0 + v].s;
      if (TWO) {
        float a0 = dword_dot<BITS>(w.x, &xr[0], 0.f);
        a0 = dword_dot<BITS>(w.y, &xr[PPC / 4], a0);
        float a1 = dword_dot<BITS>(w.z, &xr[PPC / 2], 0.f);
        a1 = dword_dot<BITS>(w.w, &xr[3 * PPC / 4], a1);
        tot[v] = fmaf(f16_bits_to_f32(sraw & 0xffffu) * 16777216.0f, a0 - k0, tot[v]);
        tot[v] = fmaf(f16_bits_to_f32(sraw >> 16) * 16777216.0f, a1 - k1, tot[v]);
      } else {
        float a = dword_dot<BITS>(w.x, &xr[0], 0.f);
        a = dword_dot<BITS>(w.y, &xr[PPC / 4], a);
        a = dword_dot<BITS>(w.z, &xr[PPC / 2], a);
        a = dword_dot<BITS>(w.w, &xr[3 * PPC / 4], a);
        tot[v] = fmaf(f16_bits_to_f32(sraw & 0xffffu) * 16777216.0f, a - k0, tot[v]);
      }
    }
    if (++cj == J) {
      fold_rows<NRM, NM>(tot, P, lane);
      if (p < NRM) {
        const int row = row_begin + (tw + ck * wpp) * task_rows + p * RW + rsub;
        if (row < row_end) {
          float r[NM];
#pragma unroll
          for (int m = 0; m < NM; ++m) r[m] = tot[m * NRM];
          epilogue(row, r, part);
        }
      }
      cj = 0;
      ++ck;
    }
  };
  auto compute_block = [&](const Tile (&t)[kBlock], int blk) {
#pragma unroll
    for (int c = 0; c < CPB; ++c)
      if (blk * CPB + c < S) compute_step(t, c * NR);
  };

  const int nblocks = (S + CPB - 1) / CPB;
  Tile bufA[kBlock], bufB[kBlock];
  load_block(bufA, 0);
  stage();
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

// Rows per lane group and matrix in one task: as many (up to nrm_max) as still leave every wavefront of
// the workgroup a task, and never more than P (the fold needs NRM <= P).
__host__ __device__ inline int pick_nrm(int rows_in_wg, int RW, int nwaves, int P, int nrm_max) {
  int nrm = nrm_max;
  while (nrm > 1 && (nrm > P || rows_in_wg < RW * nrm * nwaves)) nrm >>= 1;
  return nrm;
}

// ---------------------------------------------------------------------------------------------
// softmax + top-k of one token from its logits, by ONE wavefront (all 64 lanes call this). E <= 64*MPL.
// Lane 0 writes sel_e[0..k), sel_g[0..k); all lanes write probs (may be null).
// The selection is total: every index it writes lies in [0, E) and the k indices are distinct, whatever the
// logits hold (the kernels behind use them as addresses). When the softmax is undefined (a NaN or +Inf
// logit, or no finite logit at all) the token takes the experts 0 .. k-1 with NaN gates; logits of -Inf
// have probability zero and are chosen, in index order, only when fewer than k other experts remain.
template <int MPL>
__device__ __forceinline__ void topk_impl(const float* __restrict__ lg, int E, int k, int renorm, int lane, int* sel_e,
                                          float* sel_g, float* __restrict__ probs) {
  float v[MPL];
  float m = -INFINITY;
#pragma unroll
  for (int j = 0; j < MPL; ++j) {
    const int e = lane + 64 * j;
    v[j] = e < E ? lg[e] : -INFINITY;
    m = fmaxf(m, v[j]);
  }
  m = wave_max(m);
  float z = 0.f;
#pragma unroll
  for (int j = 0; j < MPL; ++j)
    if (lane + 64 * j < E) z += expf(v[j] - m);
  z = wave_sum(z);
  const bool defined = z >= 1.0f && z < INFINITY;      // the largest logit contributes exp(0) = 1
  const float inv_z = 1.0f / z;
  if (probs) {
#pragma unroll
    for (int j = 0; j < MPL; ++j)
      if (lane + 64 * j < E) probs[lane + 64 * j] = expf(v[j] - m) * inv_z;
  }
  // k selection passes on the logits (same order as on the probabilities): the largest value among the
  // experts not yet taken, ties to the lowest expert index = the lowest (j, lane) holding that value.
  float sp[8];
  int se[8];
  float sum = 0.f;
  uint32_t taken = 0;                                  // bit j: this lane's expert lane + 64*j is chosen
  for (int r = 0; r < k; ++r) {
    float bv = -INFINITY;
#pragma unroll
    for (int j = 0; j < MPL; ++j)
      if (!((taken >> j) & 1u)) bv = fmaxf(bv, v[j]);
    bv = wave_max(bv);
    int be = -1;
#pragma unroll
    for (int j = 0; j < MPL; ++j) {
      const unsigned long long mask = __ballot(v[j] == bv && (lane + 64 * j) < E && !((taken >> j) & 1u));
      if (be < 0 && mask != 0ull) be = 64 * j + (__ffsll((long long)mask) - 1);
    }
    if (be < 0) {                                      // only with undefined values: the lowest free expert
#pragma unroll
      for (int j = 0; j < MPL; ++j) {
        const unsigned long long mask = __ballot((lane + 64 * j) < E && !((taken >> j) & 1u));
        if (be < 0 && mask != 0ull) be = 64 * j + (__ffsll((long long)mask) - 1);
      }
    }
#pragma unroll
    for (int j = 0; j < MPL; ++j)
      if (lane + 64 * j == be) taken |= 1u << j;
    sp[r] = expf(bv - m) * inv_z;
    se[r] = be;
    sum += sp[r];
  }
  if (lane == 0)
    for (int r = 0; r < k; ++r) {
      sel_e[r] = defined ? se[r] : r;
      sel_g[r] = defined ? (renorm ? sp[r] / sum : sp[r]) : __builtin_nanf("");
    }
}

// The same for at most 64 experts (one logit per lane), written as one short dependent chain: the kernels
// that route inside a streaming workgroup wait for exactly this. The probabilities use the hardware
// exponential (relative error of a few 1e-7, far inside what the gates are compared with); the order of the
// experts is decided on the logits, so it is exact.
__device__ __forceinline__ void topk_small(const float* __restrict__ lg, int E, int k, int renorm, int lane, int* sel_e,
                                           float* sel_g, float* __restrict__ probs) {
  float v = lane < E ? lg[lane] : -INFINITY;
  const float m = wave_max(v);
  const float p = lane < E ? __expf(v - m) : 0.f;
  const float z = wave_sum(p);
  const bool defined = z >= 1.0f && z < INFINITY;      // false: NaN or +Inf among the logits, or none finite
  if (probs && lane < E) probs[lane] = p / z;
  float sum = 0.f, my_p = 0.f;
  int my_e = 0;
  unsigned long long avail = E >= 64 ? ~0ull : ((1ull << E) - 1ull);   // experts not yet taken
  for (int r = 0; r < k; ++r) {                              // lane r keeps the r-th choice
    const float bv = wave_max(v);
    unsigned long long mask = __ballot(v == bv) & avail;
    if (mask == 0ull) mask = avail;                          // only with undefined values; k <= E keeps avail non-empty
    const int be = __ffsll((long long)mask) - 1;             // ties: the lowest expert index
    avail &= ~(1ull << be);
    const float pe = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, p), be));
    if (lane == be) v = -INFINITY;
    my_e = lane == r ? be : my_e;
    my_p = lane == r ? pe : my_p;
    sum += pe;
  }
  const float inv = 1.0f / (renorm ? sum : z);
  if (lane < k) {
    sel_e[lane] = defined ? my_e : lane;
    sel_g[lane] = defined ? my_p * inv : __builtin_nanf("");
  }
}

// The same for at most EMAX (8 or 16) experts and at most 2 choices, with no cross-lane step at all: every lane reads the
// logits (broadcast reads) and selects in its own registers, so the chain is a few dozen dependent vector
// instructions instead of a dozen DPP / readlane round trips. Same rules: order on the logits, ties to the
// lowest index, an undefined softmax takes the experts 0 .. k-1 with NaN gates.
template <int EMAX>
__device__ __forceinline__ void topk_tiny(const float* __restrict__ lg, int E, int k, int renorm, int lane, int* sel_e,
                                          float* sel_g) {
  float v[EMAX];
  float m = -INFINITY;
#pragma unroll
  for (int e = 0; e < EMAX; ++e) {
    v[e] = e < E ? lg[e] : -INFINITY;
    m = fmaxf(m, v[e]);
  }
  float z = 0.f;
#pragma unroll
  for (int e = 0; e < EMAX; ++e) z += e < E ? __expf(v[e] - m) : 0.f;
  const bool defined = z >= 1.0f && z < INFINITY;
  // first choice: the largest, lowest index on ties (strict comparison while walking up)
  float b0 = v[0];
  int i0 = 0;
#pragma unroll
  for (int e = 1; e < EMAX; ++e) {
    const bool better = e < E && v[e] > b0;
    b0 = better ? v[e] : b0;
    i0 = better ? e : i0;
  }
  float b1 = -INFINITY;
  int i1 = -1;
#pragma unroll
  for (int e = 0; e < EMAX; ++e) {
    const bool ok = e < E && e != i0 && (i1 < 0 || v[e] > b1);
    b1 = ok ? v[e] : b1;
    i1 = ok ? e : i1;
  }
  const float p0 = __expf(b0 - m), p1 = k > 1 ? __expf(b1 - m) : 0.f;
  const float inv = 1.0f / (renorm ? p0 + p1 : z);
  if (lane == 0) {
    sel_e[0] = defined ? i0 : 0;
    sel_g[0] = defined ? p0 * inv : __builtin_nanf("");
    if (k > 1) {
      sel_e[1] = defined ? i1 : 1;
      sel_g[1] = defined ? p1 * inv : __builtin_nanf("");
    }
  }
}

__device__ __forceinline__ void topk_from_logits(const float* __restrict__ lg, int E, int k, int renorm, int lane,
                                                 int* sel_e, float* sel_g, float* __restrict__ probs) {
  if (E <= 64) topk_small(lg, E, k, renorm, lane, sel_e, sel_g, probs);
  else if (E <= 128) topk_impl<2>(lg, E, k, renorm, lane, sel_e, sel_g, probs);
  else topk_impl<16>(lg, E, k, renorm, lane, sel_e, sel_g, probs);
}



}  // namespace
}  // namespace moeq
