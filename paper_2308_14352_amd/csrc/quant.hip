// Compression primitives on the device (Section 3.2): group-wise linear quantization with float16
// scales, packing into the boundary format, and the two mirror maps (packed -> signed codes,
// packed -> fp32). These are the offline side of the path; they are written for exactness, and
// only coalesced enough to quantize tens of gigabytes of synthetic weights in seconds.
#include "moeq_internal.h"

namespace moeq {
namespace {

// fp32 -> binary16 bits, round to nearest even, for a finite input >= 0.
// Normal results: the exponent is re-biased and the 13 dropped mantissa bits are rounded by adding 0xfff plus
// the lowest kept bit, one integer addition whose carry runs into the exponent where it must (so values that
// round up to 65536 come out as the infinity pattern 0x7c00). Results below 2^-14 are multiples of 2^-24:
// adding 0.5f puts the float's last mantissa bit exactly there, the addition itself rounds to nearest even
// (the wavefront's default mode), and the low bits of the sum are the binary16 pattern.
__device__ __forceinline__ uint32_t f32_to_f16_bits_rne(float f) {
  const uint32_t x = __float_as_uint(f);
  if (x >= 0x47800000u) return 0x7c00u;                            // 65536 and above
  if (x < 0x38800000u) return __float_as_uint(f + 0.5f) - 0x3f000000u;
  return (x + 0xc8000fffu + ((x >> 13) & 1u)) >> 13;               // 0xc8000000 = -(112 << 23): exponent bias 127 -> 15
}

// binary16 bits (finite, non-negative) -> fp32, exact.
__device__ __forceinline__ float f16_bits_to_f32(uint32_t h) {
  const uint32_t e = (h >> 10) & 0x1fu, m = h & 0x3ffu;
  if (e == 0) return (float)m * 5.9604644775390625e-08f;  // m * 2^-24, exact
  return __uint_as_float(((e + 112u) << 23) | (m << 13));
}

// One group of `group` weights is handled by LPG lanes (a power of two <= 64); each lane walks the
// group's float4 slots with stride LPG, twice: once for the max magnitude, once to emit codes.
template <int BITS>
__global__ __launch_bounds__(256) void k_quantize_pack(const float* __restrict__ w, int64_t n_groups, int group,
                                                       int lpg, uint8_t* __restrict__ q, uint16_t* __restrict__ s) {
  constexpr int QMAX = (1 << (BITS - 1)) - 1;
  constexpr int OFF = 1 << (BITS - 1);
  const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t G = gtid / lpg;
  const int l = (int)(gtid % lpg);
  const bool live = G < n_groups;
  if (!live) G = n_groups - 1;  // keep the lane in the shuffles; it writes nothing
  const float4* wg = (const float4*)(w + G * group);
  const int n4 = group / 4;
  float a = 0.f;
  for (int i = l; i < n4; i += lpg) {
    const float4 v = wg[i];
    a = fmaxf(a, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
  }
  for (int off = lpg >> 1; off >= 1; off >>= 1) a = fmaxf(a, __shfl_xor(a, off, 64));
  uint32_t sh = 0;
  float sf = 0.f;
  if (a > 0.f) {
    const float s32 = __fdiv_rn(a, (float)QMAX);
    sh = f32_to_f16_bits_rne(s32);
    if (sh >= 0x7c00u) sh = 0x7bffu;
    else if (f16_bits_to_f32(sh) * (float)QMAX < a) sh += 1;  // next half up: the max element must not clamp
    if (sh >= 0x7c00u) sh = 0x7bffu;
    sf = f16_bits_to_f32(sh);
  }
  if (live && l == 0) s[G] = (uint16_t)sh;
  // 4 weights -> 4*BITS bits: one byte (INT2), two bytes (INT4), four bytes (INT8)
  uint8_t* qg = q + G * group * BITS / 8;
  for (int i = l; i < n4; i += lpg) {
    const float4 v = wg[i];
    const float e[4] = {v.x, v.y, v.z, v.w};
    uint32_t packed = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float r = 0.f;
      if (a > 0.f) {
        r = rintf(__fdiv_rn(e[j], sf));
        r = fminf(fmaxf(r, (float)-QMAX), (float)QMAX);
      }
      packed |= (uint32_t)((int)r + OFF) << (j * BITS);
    }
    if (!live) continue;
    if (BITS == 8) ((uint32_t*)qg)[i] = packed;
    else if (BITS == 4) ((uint16_t*)qg)[i] = (uint16_t)packed;
    else qg[i] = (uint8_t)packed;
  }
}

__global__ __launch_bounds__(256) void k_unpack_codes(const uint8_t* __restrict__ q, int64_t n, int bits,
                                                      int8_t* __restrict__ codes) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // weight index (rows are whole bytes)
  if (i >= n) return;
  const int64_t bit = i * bits;
  const uint32_t u = (q[bit >> 3] >> (bit & 7)) & ((1u << bits) - 1u);
  codes[i] = (int8_t)((int)u - (1 << (bits - 1)));
}

// One weight per thread: any byte-aligned row length and any pointer alignment.
__global__ __launch_bounds__(256) void k_dequantize_any(const uint8_t* __restrict__ q, const uint16_t* __restrict__ s,
                                                        int64_t n, int64_t cols, int bits, int group,
                                                        float* __restrict__ w) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int64_t bit = i * bits;
  const uint32_t u = (q[bit >> 3] >> (bit & 7)) & ((1u << bits) - 1u);
  const int64_t row = i / cols, col = i % cols;
  const float sc = f16_bits_to_f32(s[row * (cols / group) + col / group]);
  w[i] = sc * (float)((int)u - (1 << (bits - 1)));
}

// W^[row][col] = scale[row][col / group] * (code - 2^(bits-1)) as fp32 (Section 3.2: the decompression of
// an activated expert). A thread takes one 32-bit word of codes (32 / bits weights of one row: rows are
// multiples of 16 bytes) and writes its weights as 16-byte stores; one scale serves the word when the group
// size is a multiple of the weights per word, else every weight looks its scale up.
template <int BITS>
__global__ __launch_bounds__(256) void k_dequantize(const uint32_t* __restrict__ q, const uint16_t* __restrict__ s,
                                                    int64_t n_words, uint32_t words_per_row, uint32_t group,
                                                    float* __restrict__ w) {
  constexpr int WPW = 32 / BITS;                  // weights per word
  constexpr uint32_t MASK = (1u << BITS) - 1u;
  constexpr int OFF = 1 << (BITS - 1);
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_words) return;
  const int64_t row = i / words_per_row;
  const uint32_t wc = (uint32_t)(i - row * words_per_row), col0 = wc * WPW;
  const uint32_t cols = words_per_row * WPW, groups = cols / group;
  const uint16_t* srow = s + row * groups;
  const uint32_t u = q[i];
  float v[WPW];
  if (group % WPW == 0) {
    const float sc = f16_bits_to_f32(srow[col0 / group]);
#pragma unroll
    for (int e = 0; e < WPW; ++e) v[e] = sc * (float)((int)((u >> (e * BITS)) & MASK) - OFF);
  } else {
#pragma unroll
    for (int e = 0; e < WPW; ++e)
      v[e] = f16_bits_to_f32(srow[(col0 + e) / group]) * (float)((int)((u >> (e * BITS)) & MASK) - OFF);
  }
  float4* o = (float4*)(w + row * cols + col0);
#pragma unroll
  for (int e = 0; e < WPW; e += 4) o[e / 4] = make_float4(v[e], v[e + 1], v[e + 2], v[e + 3]);
}

}  // namespace

hipError_t launch_quantize_pack(const float* w, int64_t rows, int64_t cols, int bits, int group, uint8_t* q,
                                uint16_t* s, hipStream_t st) {
  const int64_t n_groups = rows * (cols / group);
  int lpg = 1;
  while (lpg < 64 && lpg * 2 <= group / 4) lpg *= 2;
  const int64_t threads = n_groups * lpg;
  const int64_t blocks = (threads + 255) / 256;
  if (blocks > 0x7fffffff) return hipErrorInvalidValue;
  const dim3 grid((unsigned)blocks), block(256);
  switch (bits) {
    case 2: hipLaunchKernelGGL(k_quantize_pack<2>, grid, block, 0, st, w, n_groups, group, lpg, q, s); break;
    case 4: hipLaunchKernelGGL(k_quantize_pack<4>, grid, block, 0, st, w, n_groups, group, lpg, q, s); break;
    default: hipLaunchKernelGGL(k_quantize_pack<8>, grid, block, 0, st, w, n_groups, group, lpg, q, s); break;
  }
  return hipGetLastError();
}

hipError_t launch_unpack_codes(const uint8_t* q, int64_t rows, int64_t cols, int bits, int8_t* codes,
                               hipStream_t st) {
  const int64_t n = rows * cols, blocks = (n + 255) / 256;
  if (blocks > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_unpack_codes, dim3((unsigned)blocks), dim3(256), 0, st, q, n, bits, codes);
  return hipGetLastError();
}

hipError_t launch_dequantize(const uint8_t* q, const uint16_t* s, int64_t rows, int64_t cols, int bits, int group,
                             float* w, hipStream_t st) {
  if ((cols * bits) % 32 || ((uintptr_t)q & 3u) || ((uintptr_t)w & 15u)) {
    const int64_t n = rows * cols, nb = (n + 255) / 256;
    if (nb > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_dequantize_any, dim3((unsigned)nb), dim3(256), 0, st, q, s, n, cols, bits, group, w);
    return hipGetLastError();
  }
  const int64_t words_per_row = cols * bits / 32, n_words = rows * words_per_row, blocks = (n_words + 255) / 256;
  if (blocks > 0x7fffffff || words_per_row > 0x7fffffff) return hipErrorInvalidValue;
  const dim3 grid((unsigned)blocks), block(256);
  const uint32_t* qw = (const uint32_t*)q;
  switch (bits) {
    case 2: hipLaunchKernelGGL(k_dequantize<2>, grid, block, 0, st, qw, s, n_words, (uint32_t)words_per_row, (uint32_t)group, w); break;
    case 4: hipLaunchKernelGGL(k_dequantize<4>, grid, block, 0, st, qw, s, n_words, (uint32_t)words_per_row, (uint32_t)group, w); break;
    default: hipLaunchKernelGGL(k_dequantize<8>, grid, block, 0, st, qw, s, n_words, (uint32_t)words_per_row, (uint32_t)group, w); break;
  }
  return hipGetLastError();
}

}  // namespace moeq
