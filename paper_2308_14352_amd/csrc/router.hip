// Router GEMV (Section 1; Section 2.1: a small router scores the experts for every token).
// logits[t][e] = router_w[e] . x[t] (+ bias[e]) in fp32. One workgroup per (expert, group of up to 8
// tokens): the expert's row is read once with 128-bit loads and dotted with each token of the group;
// partial sums are folded with DPP inside each wavefront, then across the wavefronts through LDS.
// The softmax and the top-k selection run where the result is needed (see the FFN kernels).
#include "moeq_internal.h"

namespace moeq {
namespace {

constexpr int kThreads = 256;
constexpr int kTokensPerWg = 8;

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// Sum over the 64 lanes: DPP inside the 16-lane rows, then the four row totals through scalar reads.
template <int CTRL>
__device__ __forceinline__ float dpp(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp<0x124>(v);   // row_ror:4
  v += dpp<0x128>(v);   // row_ror:8
  const int b = __builtin_bit_cast(int, v);
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
  return (r0 + r1) + (r2 + r3);
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void k_router_logits(LayerDims L, const float* __restrict__ Wr,
                                                            const float* __restrict__ bias,
                                                            const void* __restrict__ x, int32_t T,
                                                            float* __restrict__ logits) {
  __shared__ float part[kThreads / 64][kTokensPerWg];
  const int d = L.d_model, E = L.n_experts;
  const int e = blockIdx.x;
  const int t0 = blockIdx.y * kTokensPerWg;
  const int nt = min(kTokensPerWg, T - t0);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* wr = Wr + (size_t)e * d;
  float acc[kTokensPerWg];
#pragma unroll
  for (int tt = 0; tt < kTokensPerWg; ++tt) acc[tt] = 0.f;
  for (int i = tid * 4; i < d; i += kThreads * 4) {
    const float4 w = *(const float4*)(wr + i);
#pragma unroll
    for (int tt = 0; tt < kTokensPerWg; ++tt) {
      if (tt < nt) {
        float4 v;
        if (BF16) {
          const ushort4 b = *(const ushort4*)((const uint16_t*)x + (size_t)(t0 + tt) * d + i);
          v = make_float4(bf16_bits_to_f32(b.x), bf16_bits_to_f32(b.y), bf16_bits_to_f32(b.z), bf16_bits_to_f32(b.w));
        } else {
          v = *(const float4*)((const float*)x + (size_t)(t0 + tt) * d + i);
        }
        acc[tt] = fmaf(w.x, v.x, acc[tt]); acc[tt] = fmaf(w.y, v.y, acc[tt]);
        acc[tt] = fmaf(w.z, v.z, acc[tt]); acc[tt] = fmaf(w.w, v.w, acc[tt]);
      }
    }
  }
#pragma unroll
  for (int tt = 0; tt < kTokensPerWg; ++tt) {
    if (tt < nt) {   // uniform over the workgroup
      const float v = wave_sum(acc[tt]);
      if (lane == 0) part[wave][tt] = v;
    }
  }
  __syncthreads();
  if (tid < nt) {
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) v += part[w][tid];
    logits[(size_t)(t0 + tid) * E + e] = v + (bias ? bias[e] : 0.f);
  }
}

}  // namespace

hipError_t launch_router_logits(const LayerDims& L, const float* router_w, const float* router_bias, const void* x,
                                int32_t T, float* logits, hipStream_t st) {
  const dim3 grid(L.n_experts, (T + kTokensPerWg - 1) / kTokensPerWg);
  if (L.x_bf16)
    hipLaunchKernelGGL(k_router_logits<true>, grid, dim3(kThreads), 0, st, L, router_w, router_bias, x, T, logits);
  else
    hipLaunchKernelGGL(k_router_logits<false>, grid, dim3(kThreads), 0, st, L, router_w, router_bias, x, T, logits);
  return hipGetLastError();
}

}  // namespace moeq
