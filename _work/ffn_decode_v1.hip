// Dequantize-fused expert FFN for decode (one to a few tokens): bandwidth-bound GEMVs that stream the
// packed INT2/INT4/INT8 rows of the activated expert with 128-bit loads, unpack the codes in
// registers and accumulate in fp32 (Section 3.2: the weights are decompressed by the mirror of the
// linear quantization before use; here that mirror map is applied on the fly and the fp32 copy of
// the expert is never written).
//
// Work split. A packed row is a run of 16-byte chunks (128/b weights each). P lanes of a wavefront
// share a row (P = a power of two chosen from the row length), so a wavefront works on 64/P rows at
// once and each lane keeps R such rows in flight. The activation vector sits in LDS in a
// chunk-interleaved order that makes every lane's 128-bit LDS read conflict-free. Per chunk a lane
// forms t = sum_i u_i * x_i over the unsigned codes and applies the group's scale and the code
// offset once: acc += s * (t - 2^(b-1) * sum_i x_i), the per-group sums of x being computed once per
// workgroup. Partial sums are folded across the P lanes with cross-lane shuffles.
#include <hip/hip_fp16.h>

#include "moeq_internal.h"

namespace moeq {
namespace {

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ float half_bits_to_f32(uint16_t h) { return __half2float(__ushort_as_half(h)); }

__device__ __forceinline__ float ub0(uint32_t v) { return (float)(v & 0xffu); }
__device__ __forceinline__ float ub1(uint32_t v) { return (float)((v >> 8) & 0xffu); }
__device__ __forceinline__ float ub2(uint32_t v) { return (float)((v >> 16) & 0xffu); }
__device__ __forceinline__ float ub3(uint32_t v) { return (float)(v >> 24); }

template <int BITS>
struct Fmt {
  static constexpr int WPC = 128 / BITS;          // weights per 16-byte chunk
  static constexpr int QPC = WPC / 4;             // float4 of x per chunk
  static constexpr float OFF = (float)(1 << (BITS - 1));
};

// sum_i u_i * x_i over the 32 weights held in two dwords (INT2), one dword (INT4: 8 weights) ...
// Each helper consumes one dword of codes and the matching x values.
__device__ __forceinline__ float dot_dword8(uint32_t w, const float4& a, float t) {  // 4 x INT8
  t = fmaf(ub0(w), a.x, t); t = fmaf(ub1(w), a.y, t); t = fmaf(ub2(w), a.z, t); t = fmaf(ub3(w), a.w, t);
  return t;
}
__device__ __forceinline__ float dot_dword4(uint32_t w, const float4& a, const float4& b, float t) {  // 8 x INT4
  const uint32_t lo = w & 0x0f0f0f0fu, hi = (w >> 4) & 0x0f0f0f0fu;  // lo: elements 0,2,4,6; hi: 1,3,5,7
  t = fmaf(ub0(lo), a.x, t); t = fmaf(ub0(hi), a.y, t); t = fmaf(ub1(lo), a.z, t); t = fmaf(ub1(hi), a.w, t);
  t = fmaf(ub2(lo), b.x, t); t = fmaf(ub2(hi), b.y, t); t = fmaf(ub3(lo), b.z, t); t = fmaf(ub3(hi), b.w, t);
  return t;
}
__device__ __forceinline__ float dot_dword2(uint32_t w, const float4& a, const float4& b, const float4& c,
                                            const float4& d, float t) {  // 16 x INT2
  const uint32_t m0 = w & 0x03030303u, m1 = (w >> 2) & 0x03030303u, m2 = (w >> 4) & 0x03030303u,
                 m3 = (w >> 6) & 0x03030303u;  // m_j byte n = element 4n + j
  t = fmaf(ub0(m0), a.x, t); t = fmaf(ub0(m1), a.y, t); t = fmaf(ub0(m2), a.z, t); t = fmaf(ub0(m3), a.w, t);
  t = fmaf(ub1(m0), b.x, t); t = fmaf(ub1(m1), b.y, t); t = fmaf(ub1(m2), b.z, t); t = fmaf(ub1(m3), b.w, t);
  t = fmaf(ub2(m0), c.x, t); t = fmaf(ub2(m1), c.y, t); t = fmaf(ub2(m2), c.z, t); t = fmaf(ub2(m3), c.w, t);
  t = fmaf(ub3(m0), d.x, t); t = fmaf(ub3(m1), d.y, t); t = fmaf(ub3(m2), d.z, t); t = fmaf(ub3(m3), d.w, t);
  return t;
}

// Stage `cols` activations into LDS, chunk-interleaved for BITS: float4 number q of chunk c goes to
// X4[q * C + c]. Then the sums of x over every scale group slice of a chunk go to XS.
// sub = min(WPC, group) weights share one scale inside a chunk; XS[c * (WPC/sub) + j].
template <int BITS, typename LoadX>
__device__ __forceinline__ void stage_x(LoadX load4, int cols, int group, float* X, float* XS) {
  constexpr int WPC = Fmt<BITS>::WPC, QPC = Fmt<BITS>::QPC;
  const int C = cols / WPC;
  float4* X4 = (float4*)X;
  for (int i4 = threadIdx.x; i4 < cols / 4; i4 += blockDim.x) {
    const int c = i4 / QPC, q = i4 % QPC;
    X4[q * C + c] = load4(i4);
  }
  __syncthreads();
  const int sub = group < WPC ? group : WPC;
  const int spc = WPC / sub;        // scale slices per chunk: 1, or 2 for INT2 with group 32
  const int qps = sub / 4;
  for (int s = threadIdx.x; s < C * spc; s += blockDim.x) {
    const int c = s / spc, j = s % spc;
    float acc = 0.f;
    for (int q = j * qps; q < (j + 1) * qps; ++q) {
      const float4 v = X4[q * C + c];
      acc += (v.x + v.y) + (v.z + v.w);
    }
    XS[s] = acc;
  }
  __syncthreads();
}

// One pass over the chunks of R rows (per lane) of NM matrices that share the activation vector.
// rows[r] are already clamped to valid rows. Returns per-lane partial sums in acc[m][r].
template <int BITS, int R, int NM>
__device__ __forceinline__ void rows_dot(const uint8_t* const (&q)[NM], const uint16_t* const (&s)[NM], int cols,
                                         int group, const int (&rows)[R], int P, int p, const float* X,
                                         const float* XS, float (&acc)[NM][R]) {
  constexpr int WPC = Fmt<BITS>::WPC, QPC = Fmt<BITS>::QPC;
  constexpr float OFF = Fmt<BITS>::OFF;
  const int C = cols / WPC;
  const size_t row_bytes = (size_t)C * 16;
  const int ng = cols / group;
  const float4* X4 = (const float4*)X;
  const bool two_scales = (BITS == 2) && (group == 32);
#pragma unroll
  for (int m = 0; m < NM; ++m)
#pragma unroll
    for (int r = 0; r < R; ++r) acc[m][r] = 0.f;

  for (int c = p; c < C; c += P) {
    uint4 w[NM][R];
    float sc0[NM][R], sc1[NM][R];
#pragma unroll
    for (int m = 0; m < NM; ++m)
#pragma unroll
      for (int r = 0; r < R; ++r) {
        w[m][r] = *(const uint4*)(q[m] + (size_t)rows[r] * row_bytes + (size_t)c * 16);
        const int g0 = (c * WPC) / group;
        sc0[m][r] = half_bits_to_f32(s[m][(size_t)rows[r] * ng + g0]);
        sc1[m][r] = two_scales ? half_bits_to_f32(s[m][(size_t)rows[r] * ng + g0 + 1]) : 0.f;
      }
    float4 xv[QPC];
#pragma unroll
    for (int qq = 0; qq < QPC; ++qq) xv[qq] = X4[qq * C + c];
    if (BITS == 2 && two_scales) {
      const float xs0 = XS[2 * c], xs1 = XS[2 * c + 1];
#pragma unroll
      for (int m = 0; m < NM; ++m)
#pragma unroll
        for (int r = 0; r < R; ++r) {
          float t0 = 0.f, t1 = 0.f;
          if constexpr (BITS == 2) {
            t0 = dot_dword2(w[m][r].x, xv[0], xv[1], xv[2], xv[3], t0);
            t0 = dot_dword2(w[m][r].y, xv[4], xv[5], xv[6], xv[7], t0);
            t1 = dot_dword2(w[m][r].z, xv[8], xv[9], xv[10], xv[11], t1);
            t1 = dot_dword2(w[m][r].w, xv[12], xv[13], xv[14], xv[15], t1);
          }
          acc[m][r] = fmaf(sc0[m][r], t0 - OFF * xs0, acc[m][r]);
          acc[m][r] = fmaf(sc1[m][r], t1 - OFF * xs1, acc[m][r]);
        }
    } else {
      const float xs0 = XS[c];
#pragma unroll
      for (int m = 0; m < NM; ++m)
#pragma unroll
        for (int r = 0; r < R; ++r) {
          float t = 0.f;
          if constexpr (BITS == 8) {
            t = dot_dword8(w[m][r].x, xv[0], t); t = dot_dword8(w[m][r].y, xv[1], t);
            t = dot_dword8(w[m][r].z, xv[2], t); t = dot_dword8(w[m][r].w, xv[3], t);
          } else if constexpr (BITS == 4) {
            t = dot_dword4(w[m][r].x, xv[0], xv[1], t); t = dot_dword4(w[m][r].y, xv[2], xv[3], t);
            t = dot_dword4(w[m][r].z, xv[4], xv[5], t); t = dot_dword4(w[m][r].w, xv[6], xv[7], t);
          } else {
            t = dot_dword2(w[m][r].x, xv[0], xv[1], xv[2], xv[3], t);
            t = dot_dword2(w[m][r].y, xv[4], xv[5], xv[6], xv[7], t);
            t = dot_dword2(w[m][r].z, xv[8], xv[9], xv[10], xv[11], t);
            t = dot_dword2(w[m][r].w, xv[12], xv[13], xv[14], xv[15], t);
          }
          acc[m][r] = fmaf(sc0[m][r], t - OFF * xs0, acc[m][r]);
        }
    }
  }
  // fold the P lanes of a row together
#pragma unroll
  for (int m = 0; m < NM; ++m)
#pragma unroll
    for (int r = 0; r < R; ++r) {
      float v = acc[m][r];
      for (int off = P >> 1; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
      acc[m][r] = v;
    }
}

__host__ __device__ inline int lanes_per_row(int chunks) {
  // largest power of two that divides the chunk count, capped at a full wavefront; short odd rows
  // fall back to the next power of two above the count.
  int P = 1;
  while (P < 64 && chunks % (P * 2) == 0) P *= 2;
  if (P < 4) {
    P = 1;
    while (P < 64 && P < chunks) P *= 2;
  }
  return P;
}

constexpr int kRowsInFlight = 4;  // R for single-matrix passes; two-matrix (SwiGLU) passes use R/2

// ---------------------------------------------------------------------------------------------
// Phase 1: h[slot][r] = act(W_in[r] . x [, W_gate[r] . x]) for every row r of the slot's expert.
template <int BITS, bool SWIGLU>
__device__ __forceinline__ void ffn_in_body(const DevExpert& ex, int d, int f, int group, float* __restrict__ h_out,
                                            const float* X, const float* XS) {
  constexpr int R = SWIGLU ? kRowsInFlight / 2 : kRowsInFlight;
  constexpr int NM = SWIGLU ? 2 : 1;
  const int C = d / Fmt<BITS>::WPC;
  const int P = lanes_per_row(C), RW = 64 / P;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
  const int p = lane % P, rsub = lane / P;
  const int rows_per_pass = RW * R;
  const int n_pass = (f + rows_per_pass - 1) / rows_per_pass;
  for (int pass = blockIdx.x * nwaves + wave; pass < n_pass; pass += gridDim.x * nwaves) {
    int rows[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int row = pass * rows_per_pass + r * RW + rsub;
      rows[r] = row < f ? row : f - 1;
    }
    float acc[NM][R];
    if constexpr (SWIGLU) {
      const uint8_t* const qq[2] = {ex.q_in, ex.q_gate};
      const uint16_t* const ss[2] = {ex.s_in, ex.s_gate};
      rows_dot<BITS, R, 2>(qq, ss, d, group, rows, P, p, X, XS, acc);
    } else {
      const uint8_t* const qq[1] = {ex.q_in};
      const uint16_t* const ss[1] = {ex.s_in};
      rows_dot<BITS, R, 1>(qq, ss, d, group, rows, P, p, X, XS, acc);
    }
    if (p == 0) {
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const int row = pass * rows_per_pass + r * RW + rsub;
        if (row < f) {
          float v;
          if constexpr (SWIGLU) {
            const float a = acc[0][r];
            v = a / (1.0f + __expf(-a)) * acc[1][r];
          } else {
            v = fmaxf(acc[0][r], 0.f);
          }
          h_out[row] = v;
        }
      }
    }
  }
}

__global__ __launch_bounds__(256) void k_ffn_in(LayerDims L, const DevExpert* __restrict__ table,
                                                const int32_t* __restrict__ idx, int32_t fixed_expert,
                                                const void* __restrict__ x, float* __restrict__ h) {
  extern __shared__ float smem[];
  const int d = L.d_model, f = L.d_ff;
  const int slot = blockIdx.y;
  const int token = fixed_expert >= 0 ? slot : slot / L.top_k;
  const int e = fixed_expert >= 0 ? fixed_expert : idx[slot];
  const DevExpert ex = table[e];
  float* X = smem;
  float* XS = smem + d;   // d/16 entries at most
  float* h_out = h + (size_t)slot * f;
  const bool sw = L.act == MOEQ_ACT_SWIGLU;
  auto run = [&](auto bits_tag) {
    constexpr int BITS = decltype(bits_tag)::value;
    if (L.x_bf16) {
      const uint16_t* xr = (const uint16_t*)x + (size_t)token * d;
      stage_x<BITS>([&](int i4) {
        const ushort4 v = *(const ushort4*)(xr + 4 * i4);
        return make_float4(bf16_bits_to_f32(v.x), bf16_bits_to_f32(v.y), bf16_bits_to_f32(v.z), bf16_bits_to_f32(v.w));
      }, d, L.group, X, XS);
    } else {
      const float* xr = (const float*)x + (size_t)token * d;
      stage_x<BITS>([&](int i4) { return *(const float4*)(xr + 4 * i4); }, d, L.group, X, XS);
    }
    if (sw) ffn_in_body<BITS, true>(ex, d, f, L.group, h_out, X, XS);
    else ffn_in_body<BITS, false>(ex, d, f, L.group, h_out, X, XS);
  };
  switch (ex.bits) {
    case 2: run(std::integral_constant<int, 2>{}); break;
    case 4: run(std::integral_constant<int, 4>{}); break;
    default: run(std::integral_constant<int, 8>{}); break;
  }
}

// ---------------------------------------------------------------------------------------------
// Phase 2 + combine: y[t][r] (+)= sum_j gate_j * W_out_j[r] . h[slot_j]. A workgroup owns a fixed
// range of rows of y for all k choices of the token (whatever their bitwidths), sums the k
// contributions in LDS in top-k order and writes each output once: ordered, no atomics.
template <int BITS>
__device__ __forceinline__ void ffn_out_body(const DevExpert& ex, int f, int group, float g, int row_begin,
                                             int row_end, int d, float* ybuf, const float* X, const float* XS) {
  constexpr int R = kRowsInFlight;
  const int C = f / Fmt<BITS>::WPC;
  const int P = lanes_per_row(C), RW = 64 / P;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
  const int p = lane % P, rsub = lane / P;
  const int rows_per_pass = RW * R;
  const uint8_t* const qq[1] = {ex.q_out};
  const uint16_t* const ss[1] = {ex.s_out};
  for (int base = row_begin + wave * rows_per_pass; base < row_end; base += nwaves * rows_per_pass) {
    int rows[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int row = base + r * RW + rsub;
      rows[r] = row < d ? row : d - 1;
    }
    float acc[1][R];
    rows_dot<BITS, R, 1>(qq, ss, f, group, rows, P, p, X, XS, acc);
    if (p == 0) {
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const int row = base + r * RW + rsub;
        if (row < row_end) ybuf[row - row_begin] = fmaf(g, acc[0][r], ybuf[row - row_begin]);
      }
    }
  }
}

__global__ __launch_bounds__(512) void k_ffn_out(LayerDims L, const DevExpert* __restrict__ table,
                                                  const int32_t* __restrict__ idx, const float* __restrict__ gate,
                                                  int32_t fixed_expert, int32_t accumulate,
                                                  const float* __restrict__ h, float* __restrict__ y,
                                                  int32_t rows_per_wg) {
  extern __shared__ float smem[];
  const int d = L.d_model, f = L.d_ff;
  const int token = blockIdx.y;
  float* X = smem;
  float* XS = smem + f;
  float* ybuf = XS + f / 16;
  float* y_out = y + (size_t)token * d;
  const int row_begin = blockIdx.x * rows_per_wg;
  const int row_end = min(d, row_begin + rows_per_wg);
  for (int i = threadIdx.x; i < rows_per_wg; i += blockDim.x) ybuf[i] = 0.f;
  const int k = fixed_expert >= 0 ? 1 : L.top_k;
  for (int j = 0; j < k; ++j) {
    const int slot = fixed_expert >= 0 ? token : token * L.top_k + j;
    const int e = fixed_expert >= 0 ? fixed_expert : idx[slot];
    const float g = gate ? gate[slot] : 1.0f;
    const DevExpert ex = table[e];
    const float* hr = h + (size_t)slot * f;
    if (j > 0) __syncthreads();  // everyone is done with the previous choice's activations and sums
    auto run = [&](auto bits_tag) {
      constexpr int BITS = decltype(bits_tag)::value;
      stage_x<BITS>([&](int i4) { return *(const float4*)(hr + 4 * i4); }, f, L.group, X, XS);
      ffn_out_body<BITS>(ex, f, L.group, g, row_begin, row_end, d, ybuf, X, XS);
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
  // activations + per-scale-slice sums (at most one per 16 weights: an INT8 chunk)
  return ((size_t)cols + (size_t)cols / 16) * sizeof(float);
}

}  // namespace

hipError_t launch_ffn_in(const LayerDims& L, const DevExpert* table, const int32_t* idx, int32_t fixed_expert,
                         const void* x, int32_t slots, float* h, hipStream_t st) {
  const int threads = 256, nwaves = threads / 64;
  // enough workgroups that every wavefront gets at least one pass even for the widest rows-per-pass
  const int min_rows_per_pass = L.act == MOEQ_ACT_SWIGLU ? kRowsInFlight / 2 : kRowsInFlight;
  int gx = (L.d_ff + min_rows_per_pass * nwaves - 1) / (min_rows_per_pass * nwaves);
  const int cap = num_cus() * 8;
  if (gx * slots > cap) gx = (cap + slots - 1) / slots;
  if (gx < 1) gx = 1;
  const size_t lds = lds_bytes(L.d_model);
  static size_t lds_set = 0;
  if (lds > 64 * 1024 && lds > lds_set) {
    hipError_t e = hipFuncSetAttribute((const void*)k_ffn_in, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    lds_set = lds;
  }
  hipLaunchKernelGGL(k_ffn_in, dim3(gx, slots), dim3(threads), lds, st, L, table, idx, fixed_expert, x, h);
  return hipGetLastError();
}

hipError_t launch_ffn_out(const LayerDims& L, const DevExpert* table, const int32_t* idx, const float* gate,
                          int32_t fixed_expert, int32_t accumulate, const float* h, int32_t T, float* y,
                          hipStream_t st) {
  // large activation vectors: fewer, fatter workgroups so that staging them is amortised
  const int threads = lds_bytes(L.d_ff) > 32 * 1024 ? 512 : 256;
  const int nwaves = threads / 64;
  int gx = (L.d_model + kRowsInFlight * nwaves - 1) / (kRowsInFlight * nwaves);
  const int cap = num_cus() * (threads == 512 ? 2 : 8);
  if ((int64_t)gx * T > cap) gx = (cap + T - 1) / T;
  if (gx < 1) gx = 1;
  const int rows_per_wg = (L.d_model + gx - 1) / gx;
  gx = (L.d_model + rows_per_wg - 1) / rows_per_wg;
  const size_t lds = lds_bytes(L.d_ff) + (size_t)rows_per_wg * sizeof(float);
  static size_t lds_set = 0;
  if (lds > 64 * 1024 && lds > lds_set) {
    hipError_t e = hipFuncSetAttribute((const void*)k_ffn_out, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    lds_set = lds;
  }
  hipLaunchKernelGGL(k_ffn_out, dim3(gx, T), dim3(threads), lds, st, L, table, idx, gate, fixed_expert, accumulate, h,
                     y, rows_per_wg);
  return hipGetLastError();
}

}  // namespace moeq
