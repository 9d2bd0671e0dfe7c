// Router GEMV + softmax + top-k (Section 1; Section 2.1: a small router picks the top-K experts
// of every token). One workgroup per token: the hidden vector is staged in LDS, each wavefront
// owns a strided subset of experts and reduces its dot products with cross-lane shuffles;
// wavefront 0 then does the softmax and the k selection passes.
#include "moeq_internal.h"

namespace moeq {
namespace {

constexpr int kRouterThreads = 256;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// logits live in LDS; E <= 1024 so a lane holds at most 16 of them.
constexpr int kMaxPerLane = 16;

template <bool BF16>
__global__ __launch_bounds__(kRouterThreads) void k_router_topk(LayerDims L, const float* __restrict__ Wr,
                                                                const float* __restrict__ bias,
                                                                const void* __restrict__ x, int32_t* __restrict__ idx,
                                                                float* __restrict__ gate, float* __restrict__ probs) {
  extern __shared__ float smem[];
  const int d = L.d_model, E = L.n_experts, k = L.top_k;
  float* xs = smem;       // [d]
  float* lg = smem + d;   // [E]
  const int t = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;

  if (BF16) {
    const uint16_t* xr = (const uint16_t*)x + (size_t)t * d;
    for (int i = tid * 4; i < d; i += blockDim.x * 4) {
      const ushort4 v = *(const ushort4*)(xr + i);
      xs[i] = bf16_bits_to_f32(v.x); xs[i + 1] = bf16_bits_to_f32(v.y);
      xs[i + 2] = bf16_bits_to_f32(v.z); xs[i + 3] = bf16_bits_to_f32(v.w);
    }
  } else {
    const float* xr = (const float*)x + (size_t)t * d;
    for (int i = tid * 4; i < d; i += blockDim.x * 4) *(float4*)(xs + i) = *(const float4*)(xr + i);
  }
  __syncthreads();

  for (int e = wave; e < E; e += nwaves) {
    const float* wr = Wr + (size_t)e * d;
    float acc = 0.f;
    for (int i = lane * 4; i < d; i += 256) {
      const float4 w = *(const float4*)(wr + i);
      const float4 v = *(const float4*)(xs + i);
      acc = fmaf(w.x, v.x, acc); acc = fmaf(w.y, v.y, acc);
      acc = fmaf(w.z, v.z, acc); acc = fmaf(w.w, v.w, acc);
    }
    acc = wave_sum(acc);
    if (lane == 0) lg[e] = acc + (bias ? bias[e] : 0.f);
  }
  __syncthreads();
  if (wave != 0) return;

  float v[kMaxPerLane];
  float m = -INFINITY;
#pragma unroll
  for (int j = 0; j < kMaxPerLane; ++j) {
    const int e = lane + 64 * j;
    v[j] = e < E ? lg[e] : -INFINITY;
    m = fmaxf(m, v[j]);
  }
  m = wave_max(m);
  float z = 0.f;
#pragma unroll
  for (int j = 0; j < kMaxPerLane; ++j)
    if (lane + 64 * j < E) z += expf(v[j] - m);
  z = wave_sum(z);
  const float inv_z = 1.0f / z;
  if (probs) {
#pragma unroll
    for (int j = 0; j < kMaxPerLane; ++j)
      if (lane + 64 * j < E) probs[(size_t)t * E + lane + 64 * j] = expf(v[j] - m) * inv_z;
  }

  // k selection passes on the logits (same order as on the probabilities): largest value, ties to
  // the lowest expert index.
  float sel_p[8];
  int sel_e[8];
  float sel_sum = 0.f;
  for (int r = 0; r < k; ++r) {
    float bv = -INFINITY;
    int be = 0x7fffffff;
#pragma unroll
    for (int j = 0; j < kMaxPerLane; ++j) {
      const int e = lane + 64 * j;
      if (e < E && (v[j] > bv)) { bv = v[j]; be = e; }   // ascending e per lane: '>' keeps the lowest
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const float ov = __shfl_xor(bv, off, 64);
      const int oe = __shfl_xor(be, off, 64);
      if (ov > bv || (ov == bv && oe < be)) { bv = ov; be = oe; }
    }
    // every lane now holds the same (bv, be); retire it
#pragma unroll
    for (int j = 0; j < kMaxPerLane; ++j)
      if (lane + 64 * j == be) v[j] = -INFINITY;
    const float p = expf(bv - m) * inv_z;
    sel_p[r] = p;
    sel_e[r] = be;
    sel_sum += p;
  }
  if (lane == 0) {
    for (int r = 0; r < k; ++r) {
      idx[(size_t)t * k + r] = sel_e[r];
      gate[(size_t)t * k + r] = L.renorm ? sel_p[r] / sel_sum : sel_p[r];
    }
  }
}

}  // namespace

hipError_t launch_router_topk(const LayerDims& L, const float* router_w, const float* router_bias, const void* x,
                              int32_t T, int32_t* idx, float* gate, float* probs, hipStream_t st) {
  const size_t lds = ((size_t)L.d_model + (size_t)L.n_experts) * sizeof(float);
  if (L.x_bf16) {
    if (lds > 64 * 1024)
      (void)hipFuncSetAttribute((const void*)k_router_topk<true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL(k_router_topk<true>, dim3(T), dim3(kRouterThreads), lds, st, L, router_w, router_bias, x, idx,
                       gate, probs);
  } else {
    if (lds > 64 * 1024)
      (void)hipFuncSetAttribute((const void*)k_router_topk<false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL(k_router_topk<false>, dim3(T), dim3(kRouterThreads), lds, st, L, router_w, router_bias, x, idx,
                       gate, probs);
  }
  return hipGetLastError();
}

}  // namespace moeq
