// CPU oracle for the mixed-bitwidth MoE layer forward (EdgeMoE, arxiv 2308.14352).
//
// THIS IS TEST INFRASTRUCTURE. It defines what the GPU library must compute and is
// timed as the reported host baseline; nothing in the product path may call it.
// It shares no code with the HIP kernels: its own fp16 conversion, its own packer,
// its own loops. Plain C++17, double accumulation, no blocking or fusion.
//
// What it follows:
//   * Section 3.2 ("Choosing the algorithm"): linear, scale-only quantization; the
//     scale of a channel (here: of a group of `g` consecutive input indices of one
//     output channel; g = cols is the paper's per-channel case) comes from the
//     largest magnitude in it and the integer range of the bitwidth; scales are
//     kept as float16. Decompression is the mirror map, and the decompressed
//     weights are used as FP32 (Section 4.1, baselines paragraph).
//   * Section 1 / Section 2.1: a router sends each token to its top-K experts
//     (K = 1 or 2), each expert an independent FFN.
//
// Readings taken where the paper is silent:
//   qmax = 2^(b-1)-1, codes symmetric in [-qmax, qmax], stored offset-binary
//   u = q + 2^(b-1); element i of a row sits in byte floor(i*b/8) at bit offset
//   (i*b mod 8); scale = fp16(absmax/qmax) rounded to nearest even and moved one
//   fp16 step up when it would make the largest element clamp; q = rint(w/scale)
//   with fp32 division and ties to even; gates are the softmax probabilities of
//   the chosen experts, optionally renormalised over the chosen ones; ties in the
//   top-k go to the lowest expert index.
//
// Pins (tests/test_oracle_*.py): fp16 conversion against an independent
// implementation, hand-computed packed bytes, |w - dequant| <= scale/2, lossless
// cases against numpy matmul, softmax/top-k against sorting, one-hot routing
// against a single dense FFN, tiny brute force. Numeric layer outputs on real
// checkpoints are "parity unpinned": the paper prints none.

#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

extern "C" {

// ---------------------------------------------------------------- fp16 <-> fp32
// IEEE binary16, round to nearest even, subnormals kept, overflow to infinity.
uint16_t orc_f32_to_f16(float f) {
  uint32_t x;
  std::memcpy(&x, &f, 4);
  const uint32_t sign = (x >> 16) & 0x8000u;
  const uint32_t expo = (x >> 23) & 0xffu;
  uint32_t mant = x & 0x7fffffu;
  if (expo == 0xffu) return (uint16_t)(sign | 0x7c00u | (mant ? 0x200u : 0u));
  const int e = (int)expo - 127;  // unbiased
  if (e > 15) return (uint16_t)(sign | 0x7c00u);
  if (e >= -14) {  // normal half
    uint32_t h = ((uint32_t)(e + 15) << 10) | (mant >> 13);
    const uint32_t rem = mant & 0x1fffu;
    if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) h += 1;  // may carry into exponent/inf: correct
    return (uint16_t)(sign | h);
  }
  if (e < -25) return (uint16_t)sign;  // below half the smallest subnormal
  // subnormal half: value = m * 2^-24 with m in [0, 1023]
  mant |= 0x800000u;                    // implicit one, value = mant * 2^(e-23)
  const int shift = -e - 1;             // mant * 2^(e-23) / 2^-24 = mant >> (-e-1)
  uint32_t h = mant >> shift;
  const uint32_t rem = mant & ((1u << shift) - 1u);
  const uint32_t half = 1u << (shift - 1);
  if (rem > half || (rem == half && (h & 1u))) h += 1;
  return (uint16_t)(sign | h);
}

float orc_f16_to_f32(uint16_t h) {
  const int sign = (h >> 15) & 1;
  const int expo = (h >> 10) & 0x1f;
  const int mant = h & 0x3ff;
  double v;
  if (expo == 0) v = std::ldexp((double)mant, -24);
  else if (expo == 31) v = mant ? NAN : INFINITY;
  else v = std::ldexp((double)(mant | 0x400), expo - 25);
  return (float)(sign ? -v : v);
}

static inline int qmax_of(int bits) { return (1 << (bits - 1)) - 1; }
static inline bool bits_ok(int bits) { return bits == 2 || bits == 4 || bits == 8; }

// ---------------------------------------------------------------- quantize
// Section 3.2: per group, scale from max-abs and the bitwidth's range, fp16 scale.
// w [rows][cols] fp32 -> q [rows][cols] signed codes, s [rows][cols/g] fp16 bits.
int orc_quantize(const float* w, int64_t rows, int64_t cols, int bits, int group,
                 int8_t* q, uint16_t* s) {
  if (!bits_ok(bits) || group <= 0 || cols % group) return 1;
  const int qmax = qmax_of(bits);
  const int64_t ng = cols / group;
#pragma omp parallel for schedule(static)
  for (int64_t o = 0; o < rows; ++o) {
    for (int64_t G = 0; G < ng; ++G) {
      const float* wg = w + o * cols + G * group;
      int8_t* qg = q + o * cols + G * group;
      float a = 0.0f;
      for (int i = 0; i < group; ++i) a = std::fmax(a, std::fabs(wg[i]));
      if (a == 0.0f) {
        s[o * ng + G] = 0;
        for (int i = 0; i < group; ++i) qg[i] = 0;
        continue;
      }
      const float s32 = a / (float)qmax;
      uint16_t sh = orc_f32_to_f16(s32);
      if (sh >= 0x7c00u) sh = 0x7bffu;                          // saturate at the largest finite half
      else if (orc_f16_to_f32(sh) * (float)qmax < a) sh += 1;   // next half up: the max element must not clamp
      if (sh >= 0x7c00u) sh = 0x7bffu;
      const float sf = orc_f16_to_f32(sh);
      s[o * ng + G] = sh;
      for (int i = 0; i < group; ++i) {
        float r = std::nearbyintf(wg[i] / sf);  // default rounding mode: ties to even
        if (r > (float)qmax) r = (float)qmax;
        if (r < (float)-qmax) r = (float)-qmax;
        qg[i] = (int8_t)r;
      }
    }
  }
  return 0;
}

// ---------------------------------------------------------------- pack / unpack
// Offset-binary code u = q + 2^(b-1); element i of a row occupies bits
// [(i*b) mod 8, (i*b) mod 8 + b) of byte floor(i*b/8). Row length cols*b/8 bytes.
int orc_pack(const int8_t* q, int64_t rows, int64_t cols, int bits, uint8_t* out) {
  if (!bits_ok(bits) || (cols * bits) % 8) return 1;
  const int64_t rb = cols * bits / 8;
  std::memset(out, 0, (size_t)(rows * rb));
  const int off = 1 << (bits - 1);
  for (int64_t o = 0; o < rows; ++o)
    for (int64_t i = 0; i < cols; ++i) {
      const unsigned u = (unsigned)((int)q[o * cols + i] + off) & ((1u << bits) - 1u);
      out[o * rb + (i * bits) / 8] |= (uint8_t)(u << ((i * bits) % 8));
    }
  return 0;
}

int orc_unpack(const uint8_t* packed, int64_t rows, int64_t cols, int bits, int8_t* q) {
  if (!bits_ok(bits) || (cols * bits) % 8) return 1;
  const int64_t rb = cols * bits / 8;
  const int off = 1 << (bits - 1);
  for (int64_t o = 0; o < rows; ++o)
    for (int64_t i = 0; i < cols; ++i) {
      const unsigned u = (packed[o * rb + (i * bits) / 8] >> ((i * bits) % 8)) & ((1u << bits) - 1u);
      q[o * cols + i] = (int8_t)((int)u - off);
    }
  return 0;
}

// ---------------------------------------------------------------- dequantize
// Mirror of compression (Section 3.2): w^[o,i] = scale[o, i/g] * q[o,i], as fp32.
int orc_dequant(const uint8_t* packed, const uint16_t* s, int64_t rows, int64_t cols,
                int bits, int group, float* w) {
  if (!bits_ok(bits) || group <= 0 || cols % group || (cols * bits) % 8) return 1;
  const int64_t rb = cols * bits / 8, ng = cols / group;
  const int off = 1 << (bits - 1);
#pragma omp parallel for schedule(static)
  for (int64_t o = 0; o < rows; ++o)
    for (int64_t i = 0; i < cols; ++i) {
      const unsigned u = (packed[o * rb + (i * bits) / 8] >> ((i * bits) % 8)) & ((1u << bits) - 1u);
      w[o * cols + i] = orc_f16_to_f32(s[o * ng + i / group]) * (float)((int)u - off);
    }
  return 0;
}

// ---------------------------------------------------------------- router + top-k
// logits = Wr x (+bias); p = softmax(logits); the k experts with the largest scores,
// ties to the lowest index, in descending order; gate = p[idx], divided by the sum
// of the selected probabilities when renorm != 0. The order is taken on the logits:
// softmax is strictly increasing, so this IS the order of the probabilities, and it
// stays so where exp() underflows and would make distinct scores look tied.
// When the softmax is undefined (a NaN or +Inf logit, or no finite logit) the token
// takes the experts 0 .. k-1 with NaN gates, so that the indices stay valid.
int orc_router_topk(const float* x, int32_t T, int32_t d, const float* Wr, const float* bias,
                    int32_t E, int32_t k, int32_t renorm, int32_t* idx, float* gate,
                    float* probs_opt, double* logits_opt) {
  if (k < 1 || k > E) return 1;
  std::vector<double> lg(E), p(E);
  std::vector<char> taken(E);
  for (int32_t t = 0; t < T; ++t) {
    for (int32_t e = 0; e < E; ++e) {
      double acc = 0.0;
      for (int32_t i = 0; i < d; ++i) acc += (double)x[(int64_t)t * d + i] * (double)Wr[(int64_t)e * d + i];
      if (bias) acc += (double)bias[e];
      lg[e] = acc;
      if (logits_opt) logits_opt[(int64_t)t * E + e] = acc;
    }
    double m = lg[0];
    for (int32_t e = 1; e < E; ++e) m = std::fmax(m, lg[e]);
    double Z = 0.0;
    for (int32_t e = 0; e < E; ++e) { p[e] = std::exp(lg[e] - m); Z += p[e]; }
    for (int32_t e = 0; e < E; ++e) { p[e] /= Z; taken[e] = 0; }
    if (probs_opt) for (int32_t e = 0; e < E; ++e) probs_opt[(int64_t)t * E + e] = (float)p[e];
    if (!(Z >= 1.0 && Z < INFINITY)) {  // undefined softmax (the largest logit alone contributes exp(0) = 1)
      for (int32_t j = 0; j < k; ++j) { idx[(int64_t)t * k + j] = j; gate[(int64_t)t * k + j] = NAN; }
      continue;
    }
    double sel = 0.0;
    for (int32_t j = 0; j < k; ++j) {
      int32_t best = -1;
      for (int32_t e = 0; e < E; ++e)
        if (!taken[e] && (best < 0 || lg[e] > lg[best])) best = e;  // strict '>' keeps the lowest index on ties
      taken[best] = 1;
      idx[(int64_t)t * k + j] = best;
      sel += p[best];
    }
    for (int32_t j = 0; j < k; ++j) {
      const double g = p[idx[(int64_t)t * k + j]];
      gate[(int64_t)t * k + j] = (float)(renorm ? g / sel : g);
    }
  }
  return 0;
}

// ---------------------------------------------------------------- expert FFN
// One expert's packed weights (host pointers). act 0: ReLU (w_in = wi, w_out = wo);
// act 1: SwiGLU (w_in = w1, w_gate = w3, w_out = w2).
struct orc_expert {
  int32_t bits;
  const uint8_t* q_in;   const uint16_t* s_in;    // [f][d*b/8], [f][d/g]
  const uint8_t* q_gate; const uint16_t* s_gate;  // SwiGLU only
  const uint8_t* q_out;  const uint16_t* s_out;   // [d][f*b/8], [d][f/g]
};

// y_e[t] = W_out^ act(W_in^ x[t]) in the paper's order: decompress the expert to
// fp32 buffers first, then run the FFN on them (double accumulation).
// x [T][d] fp32, y [T][d] fp32, h_opt [T][f] fp32 (intermediate, may be null).
int orc_expert_ffn(const orc_expert* ex, int32_t d, int32_t f, int32_t g, int32_t act,
                   const float* x, int32_t T, float* y, float* h_opt) {
  if (!bits_ok(ex->bits) || (act != 0 && act != 1)) return 1;
  std::vector<float> Win((size_t)f * d), Wout((size_t)d * f), Wg;
  if (orc_dequant(ex->q_in, ex->s_in, f, d, ex->bits, g, Win.data())) return 1;
  if (orc_dequant(ex->q_out, ex->s_out, d, f, ex->bits, g, Wout.data())) return 1;
  if (act == 1) {
    Wg.resize((size_t)f * d);
    if (orc_dequant(ex->q_gate, ex->s_gate, f, d, ex->bits, g, Wg.data())) return 1;
  }
  std::vector<double> h(f);
  for (int32_t t = 0; t < T; ++t) {
    const float* xt = x + (int64_t)t * d;
#pragma omp parallel for schedule(static)
    for (int32_t o = 0; o < f; ++o) {
      double a = 0.0;
      for (int32_t i = 0; i < d; ++i) a += (double)Win[(size_t)o * d + i] * (double)xt[i];
      if (act == 0) {
        h[o] = a > 0.0 ? a : 0.0;
      } else {
        double b = 0.0;
        for (int32_t i = 0; i < d; ++i) b += (double)Wg[(size_t)o * d + i] * (double)xt[i];
        h[o] = (a / (1.0 + std::exp(-a))) * b;  // silu(a) * b
      }
    }
    if (h_opt) for (int32_t o = 0; o < f; ++o) h_opt[(int64_t)t * f + o] = (float)h[o];
#pragma omp parallel for schedule(static)
    for (int32_t o = 0; o < d; ++o) {
      double a = 0.0;
      for (int32_t i = 0; i < f; ++i) a += (double)Wout[(size_t)o * f + i] * h[i];
      y[(int64_t)t * d + o] = (float)a;
    }
  }
  return 0;
}

// ---------------------------------------------------------------- given routing
// Static-routing layers (Section 3.1, "Applicability"): the experts of a token are known from the
// input, no router runs.
// y[t] = sum_j gate[t,j] * FFN_{idx[t,j]}(x[t]) for a routing that is already decided. A pair whose
// index is outside [0, E) contributes nothing.
int orc_layer_forward_routed(const orc_expert* experts, int32_t E, int32_t d, int32_t f, int32_t g,
                             int32_t act, int32_t k, const float* x, int32_t T, const int32_t* idx,
                             const float* gate, float* y) {
  std::vector<float> ye((size_t)T * k * d, 0.0f);  // ye[(t*k+j)*d + i] = FFN_{idx[t,j]}(x[t])[i]
  for (int32_t e = 0; e < E; ++e) {
    std::vector<int64_t> slots;
    for (int64_t s = 0; s < (int64_t)T * k; ++s)
      if (idx[s] == e) slots.push_back(s);
    if (slots.empty()) continue;
    const int32_t n = (int32_t)slots.size();
    std::vector<float> xe((size_t)n * d), yo((size_t)n * d);
    for (int32_t r = 0; r < n; ++r)
      std::memcpy(&xe[(size_t)r * d], x + (slots[r] / k) * d, sizeof(float) * d);
    if (orc_expert_ffn(&experts[e], d, f, g, act, xe.data(), n, yo.data(), nullptr)) return 1;
    for (int32_t r = 0; r < n; ++r)
      std::memcpy(&ye[(size_t)slots[r] * d], &yo[(size_t)r * d], sizeof(float) * d);
  }
  for (int32_t t = 0; t < T; ++t)
    for (int32_t i = 0; i < d; ++i) {
      double acc = 0.0;
      for (int32_t j = 0; j < k; ++j) {
        const int64_t s = (int64_t)t * k + j;
        if (idx[s] < 0 || idx[s] >= E) continue;
        acc += (double)gate[s] * (double)ye[(size_t)s * d + i];
      }
      y[(int64_t)t * d + i] = (float)acc;
    }
  return 0;
}

// ---------------------------------------------------------------- whole layer
// router -> top-k -> each chosen expert's FFN -> y[t] = sum_j gate[t,j] * y_{idx[t,j]}[t].
// Each activated expert is decompressed once per call and applied to the tokens
// routed to it (for one token this is exactly: decompress the chosen expert, run
// it); the k results of a token are then summed in top-k order.
int orc_layer_forward(const orc_expert* experts, int32_t E, int32_t d, int32_t f, int32_t g,
                      int32_t act, int32_t k, int32_t renorm, const float* Wr, const float* bias,
                      const float* x, int32_t T, float* y, int32_t* idx, float* gate) {
  if (orc_router_topk(x, T, d, Wr, bias, E, k, renorm, idx, gate, nullptr, nullptr)) return 1;
  return orc_layer_forward_routed(experts, E, d, f, g, act, k, x, T, idx, gate, y);
}

// Harness knob for the timed baseline (1 thread against all): no effect on any result.
void orc_set_num_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

int orc_num_threads() {
  int n = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp single
    n = __builtin_omp_get_num_threads();
  }
#endif
  return n;
}

}  // extern "C"
