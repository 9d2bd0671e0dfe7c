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
// activation registers (for SwiGLU the rows of w1 and w3 count as separate "virtual rows"). The
// loads of the next block of tiles are issued before the arithmetic of the current one, across task
// boundaries, so a wavefront always has 4 to 8 loads in flight. Row totals are folded across the P
// lanes with a transposing butterfly on DPP. A workgroup owns a fixed range of output rows for all
// k chosen experts of its token, so the gate-weighted sum over the experts is ordered and needs no
// atomics.
#include <hip/hip_fp16.h>

#include <type_traits>

#include "moeq_internal.h"

namespace moeq {
namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// 16-byte load with the non-temporal hint: packed weights are read once per call and should not
// displace the activations and scales that are reused from the caches.
__device__ __forceinline__ uint4 load_stream16(const uint8_t* ptr) {
  const u32x4_t v = __builtin_nontemporal_load((const u32x4_t*)ptr);
  return make_uint4(v.x, v.y, v.z, v.w);
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
// Activation staging. Phase 1 (copy_x_to_lds): the activation vector goes to LDS as linear binary16
// (RAW) with 16-byte accesses. Phase 2 (permute_x): pair register pi of chunk c goes to word
// ((pi/4) * C + c) * 4 + pi%4 of XP, so a lane's 128-bit reads of consecutive chunks are
// conflict-free, and XK[c * spc + j] = 2^(b-1) * 2^-24 * (sum of the activations of scale slice j of
// chunk c). Callers put a barrier between the phases and after phase 2.
enum XKind { X_F32 = 0, X_BF16 = 1, X_F16 = 2 };

__device__ __forceinline__ void copy_x_to_lds(const void* __restrict__ x, int kind, int cols, int tid, int nthreads,
                                              uint16_t* RAW) {
  uint4* RAW4 = (uint4*)RAW;
  for (int i = tid; i < cols / 8; i += nthreads) {
    uint4 o;
    if (kind == X_F16) {
      o = ((const uint4*)x)[i];
    } else if (kind == X_BF16) {
      const uint4 v = ((const uint4*)x)[i];
      const uint32_t in[4] = {v.x, v.y, v.z, v.w};
      uint32_t out[4];
#pragma unroll
      for (int k = 0; k < 4; ++k)
        out[k] = f32_to_f16_bits(bf16_bits_to_f32(in[k] & 0xffffu)) | (f32_to_f16_bits(bf16_bits_to_f32(in[k] >> 16)) << 16);
      o = make_uint4(out[0], out[1], out[2], out[3]);
    } else {
      const float4 a = ((const float4*)x)[2 * i], b = ((const float4*)x)[2 * i + 1];
      o = make_uint4(f32_to_f16_bits(a.x) | (f32_to_f16_bits(a.y) << 16), f32_to_f16_bits(a.z) | (f32_to_f16_bits(a.w) << 16),
                     f32_to_f16_bits(b.x) | (f32_to_f16_bits(b.y) << 16), f32_to_f16_bits(b.z) | (f32_to_f16_bits(b.w) << 16));
    }
    RAW4[i] = o;
  }
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

template <int BITS>
__device__ __forceinline__ void permute_x(const uint16_t* RAW, int cols, int group, int tid, int nthreads,
                                          uint32_t* XP, float* XK) {
  constexpr int WPC = Fmt<BITS>::WPC, PPC = Fmt<BITS>::PPC;
  const int C = cols / WPC;
  for (int i = tid; i < cols / 2; i += nthreads) {
    const int c = i / PPC, pi = i % PPC;
    int lo, hi;
    float ps;
    pair_pos<BITS>(pi, lo, hi, ps);
    const uint32_t bl = f32_to_f16_bits(f16_bits_to_f32(RAW[c * WPC + lo]) * ps);
    const uint32_t bh = f32_to_f16_bits(f16_bits_to_f32(RAW[c * WPC + hi]) * ps);
    XP[((pi >> 2) * C + c) * 4 + (pi & 3)] = bl | (bh << 16);
  }
  offset_terms<BITS>(RAW, cols, group, tid, nthreads, XK);
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
    const uint32_t g0 = ((uint32_t)((p + (jb + pj) * P) * WPC) / (uint32_t)group) * 2u;
#pragma unroll
    for (int v = 0; v < NR; ++v) {
      const int m = v / NRM;
      t[u0 + v].w = load_stream16(q[m] + (qoff[v] + (uint32_t)(jb + pj) * jstride));
      const uint8_t* sb = (const uint8_t*)s[m];
      if (TWO) t[u0 + v].s = *(const uint32_t*)(sb + (soff[v] + g0));
      else t[u0 + v].s = *(const uint16_t*)(sb + (soff[v] + g0));
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
  const float inv_z = 1.0f / z;
  if (probs) {
#pragma unroll
    for (int j = 0; j < MPL; ++j)
      if (lane + 64 * j < E) probs[lane + 64 * j] = expf(v[j] - m) * inv_z;
  }
  // k selection passes on the logits (same order as on the probabilities): the largest value, ties to
  // the lowest expert index = the lowest (j, lane) holding that value.
  float sp[8];
  int se[8];
  float sum = 0.f;
  for (int r = 0; r < k; ++r) {
    float bv = -INFINITY;
#pragma unroll
    for (int j = 0; j < MPL; ++j) bv = fmaxf(bv, v[j]);
    bv = wave_max(bv);
    int be = -1;
#pragma unroll
    for (int j = 0; j < MPL; ++j) {
      const unsigned long long mask = __ballot(v[j] == bv && (lane + 64 * j) < E);
      if (be < 0 && mask != 0ull) be = 64 * j + (__ffsll((long long)mask) - 1);
    }
#pragma unroll
    for (int j = 0; j < MPL; ++j)
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

__device__ __forceinline__ void topk_from_logits(const float* __restrict__ lg, int E, int k, int renorm, int lane,
                                                 int* sel_e, float* sel_g, float* __restrict__ probs) {
  if (E <= 64) topk_impl<1>(lg, E, k, renorm, lane, sel_e, sel_g, probs);
  else if (E <= 128) topk_impl<2>(lg, E, k, renorm, lane, sel_e, sel_g, probs);
  else topk_impl<16>(lg, E, k, renorm, lane, sel_e, sel_g, probs);
}

__global__ __launch_bounds__(64) void k_topk(LayerDims L, const float* __restrict__ logits, int32_t* __restrict__ idx,
                                             float* __restrict__ gate, float* __restrict__ probs) {
  const int t = blockIdx.x;
  topk_from_logits(logits + (size_t)t * L.n_experts, L.n_experts, L.top_k, L.renorm, threadIdx.x,
                   idx + (size_t)t * L.top_k, gate + (size_t)t * L.top_k,
                   probs ? probs + (size_t)t * L.n_experts : nullptr);
}

// ---------------------------------------------------------------------------------------------
template <int BITS, bool SWIGLU, typename Stage>
__device__ __forceinline__ void ffn_in_tasks(const DevExpert& ex, int tid, int nwaves, int d, int f, int group,
                                             int row_begin, int row_end, uint16_t* __restrict__ h_out,
                                             uint16_t* __restrict__ hp_out, const uint32_t* XP, const float* XK,
                                             Stage stage) {
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
    // linear copy (for the offset terms of phase 2) and the copy already in phase 2's staged order
    const uint32_t hb = f32_to_f16_bits(v);
    h_out[row] = (uint16_t)hb;
    float ps;
    const int si = staged_index<BITS>(row, f / Fmt<BITS>::WPC, ps);
    hp_out[si] = (uint16_t)f32_to_f16_bits(f16_bits_to_f32(hb) * ps);
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
                                              const int* src_idx, int fixed, int k) {
  const int t = threadIdx.x;
  if (t < k * 4) {
    const int j = t >> 2, part = t & 3;
    const int e = src_idx ? src_idx[j] : fixed;
    ((uint4*)&sel_x[j])[part] = ((const uint4*)&table[e])[part];
  }
}

// Phase 1 of one token for the rows [row_begin, row_end) of d_ff: for each chosen expert
// h[slot][r] = act(W_in[r] . x [, W_gate[r] . x]); h is kept as binary16 (it is the activation vector
// of phase 2), once in linear order and once in the staged order phase 2 reads (hp). The activations
// are already in RAW (LDS, linear binary16) and the chosen experts' records in sel_x (LDS). The k
// experts are handled in passes of `spp`: the activation layouts a pass needs (one per distinct
// bitwidth) are staged together, then every wavefront streams its tasks of all the pass's experts
// without a barrier. Called by every thread of the workgroup; the first barrier inside also orders
// RAW and sel_x.
__device__ __forceinline__ void phase1_body(const LayerDims& L, const DevExpert* sel_x, int k, size_t slot0,
                                            uint16_t* __restrict__ h, uint16_t* __restrict__ hp, int row_begin,
                                            int row_end, int spp, const uint16_t* RAW, uint32_t* LAY, int nwaves) {
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
      uint16_t* h_out = h + (slot0 + j) * f;
      uint16_t* hp_out = hp + (slot0 + j) * f;
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
        if (sw) ffn_in_tasks<BITS, true>(ex, tid, nwaves, d, f, L.group, row_begin, row_end, h_out, hp_out, XP, XK, stage);
        else ffn_in_tasks<BITS, false>(ex, tid, nwaves, d, f, L.group, row_begin, row_end, h_out, hp_out, XP, XK, stage);
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
                                                 uint16_t* __restrict__ h, uint16_t* __restrict__ hp,
                                                 int32_t rows_per_wg, int32_t slots_per_pass) {
  extern __shared__ uint32_t smem[];
  __shared__ int sel_e[8];
  __shared__ float sel_g[8];
  __shared__ DevExpert sel_x[8];
  const int d = L.d_model, f = L.d_ff;
  const int token = blockIdx.y;
  uint16_t* RAW = (uint16_t*)smem;              // d halfs, then the layouts
  uint32_t* LAY = smem + d / 2;
  const int k = fixed_expert >= 0 ? 1 : L.top_k;
  const size_t xbytes = L.x_bf16 ? 2 : 4;
  copy_x_to_lds((const char*)x + (size_t)token * d * xbytes, L.x_bf16 ? X_BF16 : X_F32, d, threadIdx.x, blockDim.x, RAW);
  if (fixed_expert < 0) {
    if (threadIdx.x < 64) topk_from_logits(logits + (size_t)token * L.n_experts, L.n_experts, k, L.renorm,
                                           threadIdx.x, sel_e, sel_g, nullptr);
    __syncthreads();
    load_selected(sel_x, table, sel_e, -1, k);
    if (blockIdx.x == 0 && threadIdx.x < k) {
      idx_out[(size_t)token * k + threadIdx.x] = sel_e[threadIdx.x];
      gate_out[(size_t)token * k + threadIdx.x] = sel_g[threadIdx.x];
    }
    if (blockIdx.x == 0) {
      __syncthreads();
      if (threadIdx.x < k * 4)
        ((uint4*)&sel_tab[(size_t)token * k])[threadIdx.x] = ((const uint4*)sel_x)[threadIdx.x];
    }
  } else {
    load_selected(sel_x, table, nullptr, fixed_expert, 1);
  }
  const int row_begin = blockIdx.x * rows_per_wg;
  const int row_end = min(f, row_begin + rows_per_wg);
  phase1_body(L, sel_x, k, fixed_expert >= 0 ? (size_t)token : (size_t)token * k, h, hp, row_begin, row_end,
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
                                              float g, int row_begin, int row_end, int rows_per_wg, float* ybuf,
                                              const uint32_t* XP, const float* XK, Stage stage) {
  const int C = f / Fmt<BITS>::WPC;
  const int P = lanes_per_row(C), RW = 64 / P;
  const int lane = tid & 63, wave = tid >> 6;
  const int ks = pick_ks(row_end - row_begin, RW, nwaves, C / P);
  const int nrm = pick_nrm(row_end - row_begin, RW, nwaves / ks, P, kBlock);
  const bool two = (BITS == 2) && (group == 32);
  const uint8_t* const qq[1] = {uniform_ptr(ex.q_out)};
  const uint16_t* const ss[1] = {uniform_ptr(ex.s_out)};
  // ybuf: [kMaxKs][rows_per_wg] partial sums of this expert; teams beyond ks are zeroed by the caller
  auto epi = [&](int row, const float (&r)[1], int part) { ybuf[part * rows_per_wg + (row - row_begin)] = g * r[0]; };
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
// activation vectors (already in staged order in hp) are copied to LDS together, the offset terms are
// summed from the linear copy h, every wavefront streams its tasks of all of them without a barrier,
// each expert's contribution lands in its own LDS row buffer, and the buffers are summed in top-k order
// at the end: ordered, no atomics, every output written once.
// sel_x: the k chosen experts' records (LDS); gate_tok: their gates (LDS or global), may be null (= 1).
__device__ __forceinline__ void phase2_body(const LayerDims& L, const DevExpert* sel_x, const float* gate_tok, int k,
                                            int accumulate, size_t slot0, const uint16_t* __restrict__ h,
                                            const uint16_t* __restrict__ hp, float* __restrict__ y_out,
                                            int row_begin, int row_end, int rows_per_wg, int spp, uint32_t* smem,
                                            int nwaves) {
  const int d = L.d_model, f = L.d_ff;
  const int lay_words = f / 2 + f / 16;          // pair words + offset terms of one activation vector
  float* ybuf = (float*)smem;                    // [k][kMaxKs][rows_per_wg]
  uint32_t* LAY = smem + k * kMaxKs * rows_per_wg;   // [spp][lay_words]
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
      // The first expert of a pass brings, behind its first weight loads, the activation vectors of all
      // the pass's experts into LDS (already in staged order) and sums their offset terms.
      const bool do_stage = (j == j0);
      auto stage = [&]() {
        if (!do_stage) return;
        const int per = f / 8, n = (j1 - j0) * per;
        for (int i = tid; i < n; i += blockDim.x) {
          const int jj = i / per, r = i - jj * per;
          ((uint4*)(LAY + jj * lay_words))[r] = ((const uint4*)(hp + (slot0 + j0 + jj) * f))[r];
        }
        for (int jj = j0; jj < j1; ++jj) {
          float* XKs = (float*)(LAY + (jj - j0) * lay_words + f / 2);
          const uint16_t* lin = h + (slot0 + jj) * f;
          const int bits = sel_x[jj].bits;
          if (bits == 2) offset_terms<2>(lin, f, L.group, tid, blockDim.x, XKs);
          else if (bits == 4) offset_terms<4>(lin, f, L.group, tid, blockDim.x, XKs);
          else offset_terms<8>(lin, f, L.group, tid, blockDim.x, XKs);
        }
        __syncthreads();
      };
      auto run = [&](auto bits_tag) {
        constexpr int BITS = decltype(bits_tag)::value;
        ffn_out_tasks<BITS>(ex, tid, nwaves, d, f, L.group, g, row_begin, row_end, rows_per_wg,
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
                                                  const uint16_t* __restrict__ h, const uint16_t* __restrict__ hp,
                                                  float* __restrict__ y, int32_t rows_per_wg, int32_t slots_per_pass) {
  extern __shared__ uint32_t smem[];
  __shared__ DevExpert sel_x[8];
  __shared__ float sel_g[8];
  const int d = L.d_model;
  const int token = blockIdx.y;
  const int k = fixed_expert >= 0 ? 1 : L.top_k;
  const size_t slot0 = fixed_expert >= 0 ? (size_t)token : (size_t)token * k;
  if (fixed_expert >= 0) {
    load_selected(sel_x, table, nullptr, fixed_expert, 1);
  } else if (threadIdx.x < k * 4) {
    ((uint4*)sel_x)[threadIdx.x] = ((const uint4*)&sel_tab[slot0])[threadIdx.x];
  }
  if (threadIdx.x < k) sel_g[threadIdx.x] = gate ? gate[slot0 + threadIdx.x] : 1.0f;
  const int row_begin = blockIdx.x * rows_per_wg;
  const int row_end = min(d, row_begin + rows_per_wg);
  phase2_body(L, sel_x, sel_g, k, accumulate, slot0, h, hp, y + (size_t)token * d, row_begin, row_end, rows_per_wg,
              slots_per_pass, smem, (int)(blockDim.x >> 6));
}

// ---------------------------------------------------------------------------------------------
// The whole layer of a few tokens in ONE launch: router partial sums -> grid barrier -> top-k ->
// phase 1 -> grid barrier -> phase 2 + combine. gridDim.x workgroups per token, all resident at once
// (the host checks the occupancy), so a counter in device memory can act as a barrier between them.
//
// Barrier words (per token: arrive_a, arrive_b, done, unused) live in the layer's device table, are
// zero between calls, and are reset by the last workgroup to finish. A wait is bounded: a workgroup
// that does not see its peers in kSpinLimit polls raises the sticky error word and stops waiting, and
// every later wait returns at once, so the kernel always terminates (with invalid output and the
// error word set, which moe_layer_forward's caller can read back with moe_layer_health).
constexpr uint32_t kSpinLimit = 1u << 22;

__device__ __forceinline__ void grid_barrier(uint32_t* counter, uint32_t target, uint32_t* err) {
  __syncthreads();
  if (threadIdx.x == 0) {
    __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    uint32_t spins = 0;
    while (__hip_atomic_load(counter, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < target) {
      if (__hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
      if (++spins > kSpinLimit) {
        __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
      __builtin_amdgcn_s_sleep(2);
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "agent");  // see what the other workgroups wrote before arriving
  }
  __syncthreads();
}

template <bool BF16>
__global__ __launch_bounds__(1024) void k_layer_decode(LayerDims L, const DevExpert* __restrict__ table,
                                                       const float* __restrict__ Wr, const float* __restrict__ bias,
                                                       const void* __restrict__ x, float* __restrict__ y,
                                                       int32_t* __restrict__ idx_out, float* __restrict__ gate_out,
                                                       float* __restrict__ part, uint16_t* __restrict__ h,
                                                       uint16_t* __restrict__ hp, uint32_t* __restrict__ bar,
                                                       int32_t n_slices, int32_t slice_cols,
                                                       int32_t rpw1, int32_t nw1, int32_t spp1, int32_t rpw2,
                                                       int32_t nw2, int32_t spp2) {
  extern __shared__ uint32_t smem[];
  __shared__ int sel_e[8];
  __shared__ float sel_g[8];
  __shared__ DevExpert sel_x[8];
  __shared__ float red[16];
  __shared__ float lg[1024];
  const int d = L.d_model, f = L.d_ff, E = L.n_experts, k = L.top_k;
  const int G = gridDim.x, b = blockIdx.x, token = blockIdx.y;
  const int tid0 = threadIdx.x, lane0 = tid0 & 63, wave0 = tid0 >> 6, nwaves = blockDim.x >> 6;
  uint32_t* bar_t = bar + 4 * token;
  uint32_t* err = bar + 4 * gridDim.y;

  // ---- phase 0: partial router logits, one (expert, column slice) unit at a time
  float* part_t = part + (size_t)token * n_slices * E;
  for (int u = b; u < E * n_slices; u += G) {
    const int e = u / n_slices, sl = u % n_slices;
    const int c0 = sl * slice_cols, c1 = min(d, c0 + slice_cols);
    float acc = 0.f;
    for (int i = c0 + tid0 * 4; i < c1; i += blockDim.x * 4) {
      const float4 w = *(const float4*)(Wr + (size_t)e * d + i);
      float4 v;
      if (BF16) {
        const ushort4 q = *(const ushort4*)((const uint16_t*)x + (size_t)token * d + i);
        v = make_float4(bf16_bits_to_f32(q.x), bf16_bits_to_f32(q.y), bf16_bits_to_f32(q.z), bf16_bits_to_f32(q.w));
      } else {
        v = *(const float4*)((const float*)x + (size_t)token * d + i);
      }
      acc = fmaf(w.x, v.x, acc); acc = fmaf(w.y, v.y, acc); acc = fmaf(w.z, v.z, acc); acc = fmaf(w.w, v.w, acc);
    }
    acc = wave_sum(acc);
    __syncthreads();                 // red[] from the previous unit has been consumed
    if (lane0 == 0) red[wave0] = acc;
    __syncthreads();
    if (tid0 == 0) {
      float t = 0.f;
      for (int w = 0; w < nwaves; ++w) t += red[w];
      part_t[sl * E + e] = t;
    }
  }
  // the activations of phase 1 travel to LDS while the barrier settles
  uint16_t* RAW = (uint16_t*)smem;
  uint32_t* LAY = smem + d / 2;
  const size_t xbytes = BF16 ? 2 : 4;
  copy_x_to_lds((const char*)x + (size_t)token * d * xbytes, BF16 ? X_BF16 : X_F32, d, tid0, blockDim.x, RAW);
  grid_barrier(&bar_t[0], (uint32_t)G, err);

  // ---- logits = ordered sum of the slices (+ bias); softmax + top-k by wavefront 0
  for (int e = tid0; e < E; e += blockDim.x) {
    float t = 0.f;
    for (int sl = 0; sl < n_slices; ++sl) t += part_t[sl * E + e];
    lg[e] = t + (bias ? bias[e] : 0.f);
  }
  __syncthreads();
  if (tid0 < 64) topk_from_logits(lg, E, k, L.renorm, tid0, sel_e, sel_g, nullptr);
  __syncthreads();
  load_selected(sel_x, table, sel_e, -1, k);
  if (b == 0 && tid0 < k) {
    if (idx_out) idx_out[(size_t)token * k + tid0] = sel_e[tid0];
    if (gate_out) gate_out[(size_t)token * k + tid0] = sel_g[tid0];
  }

  // ---- phase 1
  {
    const int row_begin = b * rpw1;
    const int row_end = min(f, row_begin + rpw1);
    phase1_body(L, sel_x, k, (size_t)token * k, h, hp, row_begin, row_end, spp1, RAW, LAY, nw1);
  }
  grid_barrier(&bar_t[1], (uint32_t)G, err);

  // ---- phase 2 + combine
  {
    const int row_begin = b * rpw2;
    const int row_end = min(d, row_begin + rpw2);
    phase2_body(L, sel_x, sel_g, k, 0, (size_t)token * k, h, hp, y + (size_t)token * d, row_begin, row_end, rpw2,
                spp2, smem, nw2);
  }

  // ---- the last workgroup to get here re-arms the barrier words for the next call
  __syncthreads();
  if (tid0 == 0) {
    const uint32_t old = __hip_atomic_fetch_add(&bar_t[2], 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    if (old == (uint32_t)G - 1u) {
      __hip_atomic_store(&bar_t[0], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(&bar_t[1], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(&bar_t[2], 0u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
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
  const size_t per_slot = ((size_t)L.d_ff / 2 + (size_t)L.d_ff / 16) * 4;
  int spp = (int)((kLdsBudget - ybuf) / per_slot);
  if (spp > k) spp = k;
  if (spp < 1) spp = 1;
  return {ybuf + (size_t)spp * per_slot, spp};
}

template <typename K>
hipError_t allow_lds(K kernel, size_t lds, size_t& granted) {
  if (lds > 48 * 1024 && lds > granted) {
    hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    granted = lds;
  }
  return hipSuccess;
}

}  // namespace

hipError_t launch_topk(const LayerDims& L, const float* logits, int32_t T, int32_t* idx, float* gate, float* probs,
                       hipStream_t st) {
  hipLaunchKernelGGL(k_topk, dim3(T), dim3(64), 0, st, L, logits, idx, gate, probs);
  return hipGetLastError();
}

hipError_t launch_ffn_in(const LayerDims& L, const DevExpert* table, const float* logits, int32_t* idx_out,
                         float* gate_out, DevExpert* sel_tab, int32_t fixed_expert, const void* x, int32_t T,
                         uint16_t* h, uint16_t* hp, hipStream_t st) {
  const Split sp = plan_rows(L.d_ff, min_lanes_per_row(L.d_model), wgs_per_token(T),
                             L.act == MOEQ_ACT_SWIGLU ? kBlock / 2 : kBlock);
  const PhaseLds pl = phase1_lds(L, fixed_expert >= 0 ? 1 : L.top_k);
  static size_t granted = 0;
  if (hipError_t e = allow_lds(k_ffn_in, pl.bytes, granted); e != hipSuccess) return e;
  hipLaunchKernelGGL(k_ffn_in, dim3(sp.gx, T), dim3(sp.threads), pl.bytes, st, L, table, logits, idx_out, gate_out,
                     sel_tab, fixed_expert, x, h, hp, sp.rows_per_wg, pl.spp);
  return hipGetLastError();
}

hipError_t launch_ffn_out(const LayerDims& L, const DevExpert* table, const DevExpert* sel_tab, const float* gate,
                          int32_t fixed_expert, int32_t accumulate, const uint16_t* h, const uint16_t* hp, int32_t T,
                          float* y, hipStream_t st) {
  Split sp = plan_rows(L.d_model, min_lanes_per_row(L.d_ff), wgs_per_token(T), kBlock);
  sp.threads = phase2_threads(sp.threads);
  const PhaseLds pl = phase2_lds(L, fixed_expert >= 0 ? 1 : L.top_k, sp.rows_per_wg);
  static size_t granted = 0;
  if (hipError_t e = allow_lds(k_ffn_out, pl.bytes, granted); e != hipSuccess) return e;
  hipLaunchKernelGGL(k_ffn_out, dim3(sp.gx, T), dim3(sp.threads), pl.bytes, st, L, table, sel_tab, gate, fixed_expert,
                     accumulate, h, hp, y, sp.rows_per_wg, pl.spp);
  return hipGetLastError();
}

// One-launch layer. Returns hipErrorNotSupported (and launches nothing) when the shape does not fit
// the resident-grid scheme; the caller then uses the three-kernel path.
hipError_t launch_layer_decode(const LayerDims& L, const DevExpert* table, const float* router_w,
                               const float* router_bias, const void* x, int32_t T, float* y, int32_t* idx_out,
                               float* gate_out, float* part, uint16_t* h, uint16_t* hp, uint32_t* bar,
                               hipStream_t st) {
  if (T < 1 || T > kFusedMaxTokens) return hipErrorNotSupported;
  const int G = wgs_per_token(T);
  if (G < 8) return hipErrorNotSupported;
  const Split s1 = plan_rows(L.d_ff, min_lanes_per_row(L.d_model), G, L.act == MOEQ_ACT_SWIGLU ? kBlock / 2 : kBlock);
  Split s2 = plan_rows(L.d_model, min_lanes_per_row(L.d_ff), G, kBlock);
  s2.threads = phase2_threads(s2.threads);
  const PhaseLds p1 = phase1_lds(L, L.top_k), p2 = phase2_lds(L, L.top_k, s2.rows_per_wg);
  const size_t lds = p1.bytes > p2.bytes ? p1.bytes : p2.bytes;
  if (lds > kLdsBudget) return hipErrorNotSupported;
  // column slices of the router GEMV: enough (expert, slice) units to give every workgroup one
  int n_slices = G / L.n_experts;
  if (n_slices < 1) n_slices = 1;
  if (n_slices > kFusedMaxSlices) n_slices = kFusedMaxSlices;
  int slice_cols = (L.d_model + n_slices - 1) / n_slices;
  slice_cols = (slice_cols + 63) / 64 * 64;
  n_slices = (L.d_model + slice_cols - 1) / slice_cols;
  const int threads = 1024;
  auto kernel = L.x_bf16 ? k_layer_decode<true> : k_layer_decode<false>;
  static size_t granted[2] = {0, 0};
  if (hipError_t e = allow_lds(kernel, lds, granted[L.x_bf16 ? 1 : 0]); e != hipSuccess) return e;
  // every workgroup must be resident at once: the barrier between them is a spin on a counter
  static int resident[2] = {-1, -1};
  static size_t resident_lds[2] = {0, 0};
  int& res = resident[L.x_bf16 ? 1 : 0];
  if (res < 0 || resident_lds[L.x_bf16 ? 1 : 0] != lds) {
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)kernel, threads, lds) != hipSuccess)
      return hipErrorNotSupported;
    res = per_cu * num_cus();
    resident_lds[L.x_bf16 ? 1 : 0] = lds;
  }
  if (G * T > res) return hipErrorNotSupported;
  hipLaunchKernelGGL(kernel, dim3(G, T), dim3(threads), lds, st, L, table, router_w, router_bias, x, y, idx_out,
                     gate_out, part, h, hp, bar, n_slices, slice_cols, s1.rows_per_wg, s1.threads / 64, p1.spp,
                     s2.rows_per_wg, s2.threads / 64, p2.spp);
  return hipGetLastError();
}

}  // namespace moeq
