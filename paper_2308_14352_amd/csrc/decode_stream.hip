// The MoE layer of a decode call as ONE streaming kernel on integer dot products, for layers whose W_in / W_gate
// are held in the "row-block stream" layout and W_out in the dword-column-major layout
// (Section 1, Section 2.1: router, top-k, the chosen experts' FFNs, gate-weighted combine; Section 3.2: the
// experts' weights are decompressed by the mirror of the linear quantization before use - here the codes stay
// integers all the way into the multiplier and the group scale is applied to each group's integer sum).
//
// Arithmetic. The activations of a scale group (128 columns) are turned into block-floating-point integers:
// x_int = rint(x * 2^-e) with e chosen per group so that the largest magnitude lands in [2^13, 2^14], and each
// x_int is split into four signed 4-bit digits (x_int = d0 + 16 d1 + 256 d2 + 4096 d3, d in [-8, 7]). A 32-bit
// word of eight 4-bit codes (offset-binary; one XOR makes them two's complement) then meets the four digit
// words of its eight columns in four v_dot8_i32_i4, which is the exact integer sum of code * x_int; 2-bit
// codes are masked into the low bits of nibbles (even and odd columns apart) and keep their offset, which is
// removed with the group's sum of x_int; 8-bit codes use v_dot4_i32_i8 against two signed byte digits. Per
// row and group: sum * scale * 2^e in fp32. Nothing is rounded except x (to 14 bits per group, like binary16's
// 11 bits per element) and the fp32 sums, at any scale of x that fp32 can hold.
//
// Work split (as in decode_fused.hip): workgroup (slice, token) takes a slice of 64 columns of d_ff through
// both FFN matrices of every chosen expert and writes a partial output vector; k_reduce_partials sums the
// partial vectors in a fixed order. 8 wavefronts; wavefront w owns rows 8w .. 8w+7 of the slice in phase 1 and
// the output rows 4 * (64 * (2w + q) + lane) + {0..3}, q = 0, 1, in phase 2, and keeps its outputs in registers.
//
// Memory. A wavefront reads blocks of eight 1 KB tiles (16 bytes per lane, consecutive lanes consecutive
// addresses) plus the block's scales, kNSets register sets in rotation over ONE list of blocks, so ten loads
// per lane and set are in flight from the first block to the last. The list is ordered so that the memory side
// never waits for the arithmetic of a phase: phase 1 of expert 0, then phase 1 of expert j interleaved with
// phase 2 of expert j-1, then phase 2 of the last expert; the barrier pair in front of an expert's first
// phase-2 block (h of that expert is staged between them) is passed with the other sets' loads in flight.
// In the stream layout a block is contiguous in memory with its scales right behind its tiles; lane l always
// holds columns 64 l .. 64 l + 63, so its digit words stay in registers.
#include <hip/hip_ext.h>

#include "decode_core.h"

namespace moeq {
namespace {

constexpr int kSD = 4096;        // d_model the kernel is written for (64 lanes x 64 columns)
constexpr int kSSlice = 64;      // columns of d_ff per workgroup
constexpr int kSWaves = 8;
constexpr int kSThreads = kSWaves * 64;
constexpr int kSGroup = 128;     // scale group: the columns of two lanes
constexpr int kSInlineMaxE = 64;
constexpr int kNSets = 2;        // register sets in rotation
constexpr int kMaxBlocks = 8 * 12; // blocks of a wavefront's list: 8 experts x (8 of phase 1 + 4 of phase 2) at most

__device__ __forceinline__ int sdot8(uint32_t a, uint32_t b, int c) { return __builtin_amdgcn_sdot8((int)a, (int)b, c, false); }
__device__ __forceinline__ int sdot4(uint32_t a, uint32_t b, int c) { return __builtin_amdgcn_sdot4((int)a, (int)b, c, false); }

template <int CTRL>
__device__ __forceinline__ int dppi(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true); }

// Rows of one block of the stream layout: a block is eight tiles.
__host__ __device__ constexpr int stream_rows_per_block(int bits) { return 16 / bits; }          // 8, 4, 2
__host__ __device__ constexpr uint32_t stream_block_bytes(int bits) { return 8192u + 64u * (16u / (uint32_t)bits); }

// ---------------------------------------------------------------------------------------------
// e for a block whose largest magnitude is m: m * 2^-e in [2^13, 2^14); kept inside [-120, 120].
__device__ __forceinline__ int block_exponent(float m) {
  int e = 0;
  if (m > 0.f && m < INFINITY) e = __builtin_amdgcn_frexp_expf(m) - 1 - 13;
  return min(max(e, -120), 120);
}
// nibble k of the signed-digit expansion; advances v to the remaining quotient
__device__ __forceinline__ uint32_t next_digit(int& v) {
  const uint32_t n = (uint32_t)v & 15u;
  v = (v + 8) >> 4;
  return n;
}

struct StreamParams {
  LayerDims L;
  const DevExpert* table;
  const float* Wr;
  const float* bias;
  const float* logits;        // non-null: router logits [T][E] computed beforehand
  int32_t fixed_expert;       // >= 0: every token uses this expert
  const float* gate_in;       // fixed-expert mode: [T] or null (= 1)
  const int32_t* route_idx;   // non-null: the routing is given ([T][k], validated)
  const float* route_gate;
  const void* x;
  float* part;                // [T][n_slices][d]
  int32_t* idx_out;
  float* gate_out;
};

struct BlkSet { uint4 t[8]; uint2 s[2]; };

enum BlkKind { B_NONE = 0, B_P1 = 1, B_P2 = 2 };
struct BlkTag { int kind, j, bits, mat, rb, q, first; };   // what a requested set holds; first: the expert's first phase-2 block

// BM: the bitwidths the layer's experts have, or-ed (2 | 4 | 8): code and registers for the others are left out.
template <bool SWIGLU, int BM>
__global__ __launch_bounds__(kSThreads) void k_moe_stream(StreamParams P) {
  constexpr int NM = SWIGLU ? 2 : 1;
  __shared__ uint4 XD4[8][64];            // digits for 4-bit codes: [word j of the lane][lane] = digit words k = 0..3
  __shared__ uint4 XD2[8][64];            // for 2-bit codes: [2 * word + (0: even, 1: odd columns)][lane]
  __shared__ uint4 XD8[8][64];            // for 8-bit codes: [2 * tile + half][lane] = (lo, hi) byte digits of words 2*half, 2*half+1
  __shared__ float XS[32];                // 2^e of every scale group of x (NaN: the group holds a non-finite value)
  __shared__ int SXL[64];                 // sum of x_int over a lane's 64 columns
  __shared__ float rpart[kSWaves * kSInlineMaxE];   // router: every wavefront's part of every logit
  __shared__ float lgw[kSWaves][kSInlineMaxE];
  __shared__ int sel_ew[kSWaves][8];
  __shared__ float sel_gw[kSWaves][8];
  __shared__ float HF[8][kSSlice];        // h of every chosen expert, fp32
  __shared__ uint4 HD[8][8];              // digits of h for phase 2: per expert 8 x (4 words)
  __shared__ float uph[8];                // 2^e of an expert's h slice (NaN: non-finite)
  __shared__ int SH[8];                   // sum of h_int
  __shared__ DevExpert tab[kSInlineMaxE]; // the expert table, when it fits
  const LayerDims& L = P.L;
  const int E = L.n_experts;
  const int token = blockIdx.y;
  const int slice = (gridDim.x & 7u) == 0 ? (int)((blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3))
                                          : (int)blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int k = P.fixed_expert >= 0 ? 1 : L.top_k;
  const bool bf16 = L.x_bf16 != 0;
  const char* xt = (const char*)P.x + (size_t)token * kSD * (bf16 ? 2 : 4);
  const bool routed = P.fixed_expert < 0;
  const bool given = routed && P.route_idx != nullptr;
  const bool inline_router = routed && !P.logits && !given;

  // ---- the activations: thread t holds columns 8t .. 8t+7; a scale group is the 16 threads of a DPP row
  XItem xit = load_x_item(xt, bf16 ? X_BF16 : X_F32, tid);
  const bool tab_in_lds = E <= kSInlineMaxE;
  if (tab_in_lds && tid < E * 4) ((uint4*)tab)[tid] = ((const uint4*)P.table)[tid];
  const DevExpert* tabp = tab_in_lds ? tab : P.table;
  // ---- digits of the activations, for every bitwidth the layer has, straight from the registers
  auto stage_digits = [&]() __attribute__((always_inline)) {
    float m = 0.f;
    bool bad = false;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      m = fmaxf(m, fabsf(xit.v[i]));
      bad = bad || !(fabsf(xit.v[i]) < INFINITY);
    }
    m = bad ? INFINITY : m;
    m = fmaxf(m, dpp<kDppXor1>(m));
    m = fmaxf(m, dpp<kDppXor2>(m));
    m = fmaxf(m, dpp<kDppRor4>(m));
    m = fmaxf(m, dpp<kDppRor8>(m));
    const int e = block_exponent(m);
    const float dn = pow2f(-e);
    if ((tid & 15) == 0) XS[tid >> 4] = m < INFINITY ? pow2f(e) : __builtin_nanf("");
    int xi[8];
    int sum = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      xi[i] = m < INFINITY ? __float2int_rn(xit.v[i] * dn) : 0;
      sum += xi[i];
    }
    // sum over the 8 threads of a lane's columns
    sum += dppi<kDppXor1>(sum);
    sum += dppi<kDppXor2>(sum);
    sum += __shfl_xor(sum, 4);
    if ((tid & 7) == 0) SXL[tid >> 3] = sum;
    // 8-bit codes: two signed byte digits, x_int = lo + 256 * hi; a word of four codes meets (lo word, hi word)
    if constexpr ((BM & 8) != 0) {
      uint32_t lo[2] = {0u, 0u}, hi[2] = {0u, 0u};
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int v = xi[i];
        const uint32_t l8 = (uint32_t)v & 255u;
        const int h8 = (v + 128) >> 8;
        lo[i >> 2] |= l8 << (8 * (i & 3));
        hi[i >> 2] |= ((uint32_t)h8 & 255u) << (8 * (i & 3));
      }
      // thread t: lane t/8; its 8 columns are the words 2*(t%2), 2*(t%2)+1 of tile (t%8)/2
      XD8[tid & 7][tid >> 3] = make_uint4(lo[0], hi[0], lo[1], hi[1]);
    }
    uint32_t d4[4] = {0u, 0u, 0u, 0u};       // 4-bit layout: nibble i of digit word k = digit k of column i
    uint32_t he[4] = {0u, 0u, 0u, 0u};       // 2-bit layout: half words of the even and of the odd columns
    uint32_t ho[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int v = xi[i];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const uint32_t n = next_digit(v);
        d4[kk] |= n << (4 * i);
        if (i & 1) ho[kk] |= n << (4 * (i >> 1));
        else he[kk] |= n << (4 * (i >> 1));
      }
    }
    if constexpr ((BM & 4) != 0) XD4[tid & 7][tid >> 3] = make_uint4(d4[0], d4[1], d4[2], d4[3]);
    // a word of 2-bit codes covers 16 columns = this thread and its neighbour (tid ^ 1)
    uint32_t full[4];
    const bool upper = (tid & 1) != 0;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      // the even thread assembles the even-column word, the odd thread the odd-column word
      const uint32_t mine = upper ? ho[kk] : he[kk];
      const uint32_t give = upper ? he[kk] : ho[kk];
      const uint32_t got = (uint32_t)dppi<kDppXor1>((int)give);   // neighbour's half of MY word
      full[kk] = upper ? (got | (mine << 16)) : (mine | (got << 16));
    }
    if constexpr ((BM & 2) != 0) XD2[2 * ((tid & 7) >> 1) + (tid & 1)][tid >> 3] = make_uint4(full[0], full[1], full[2], full[3]);
  };
  // ---- router: thread t dots ITS 8 columns (already in registers) with the same columns of every expert's
  // router row, eight experts at a time: all loads of a pass are requested at once, right behind the
  // activations', and the digits of the activations are made while they are in flight. Wavefront sums go to
  // rpart[wave][e]; the logits are the sums of the eight wavefronts' parts, in order.
  bool staged = false;
  if (inline_router) {
    for (int e0 = 0; e0 < E; e0 += 8) {
      float4 w[8][2];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float* wr = P.Wr + (size_t)min(e0 + i, E - 1) * kSD + 8 * tid;     // rows past E repeat the last one
        w[i][0] = *(const float4*)wr;
        w[i][1] = *(const float4*)(wr + 4);
      }
      if (!staged) { stage_digits(); staged = true; }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float acc = w[i][0].x * xit.v[0];
        acc = fmaf(w[i][0].y, xit.v[1], acc); acc = fmaf(w[i][0].z, xit.v[2], acc); acc = fmaf(w[i][0].w, xit.v[3], acc);
        acc = fmaf(w[i][1].x, xit.v[4], acc); acc = fmaf(w[i][1].y, xit.v[5], acc);
        acc = fmaf(w[i][1].z, xit.v[6], acc); acc = fmaf(w[i][1].w, xit.v[7], acc);
        acc = wave_sum(acc);
        if (lane == 0 && e0 + i < E) rpart[wave * kSInlineMaxE + e0 + i] = acc;
      }
    }
  }
  if (!staged) stage_digits();
  __syncthreads();   // digits, XS, SXL, rpart, tab are complete


  // ---- routing, by every wavefront for itself (identical arithmetic, identical result): no second barrier
  int* sel_e = sel_ew[wave];
  float* sel_g = sel_gw[wave];
  if (given) {
    if (lane < k) {
      sel_e[lane] = P.route_idx[(size_t)token * k + lane];
      sel_g[lane] = P.route_gate[(size_t)token * k + lane];
    }
  } else if (routed) {
    if (inline_router) {
      float* lg = lgw[wave];
      if (lane < E) {
        float t = rpart[lane];
#pragma unroll
        for (int wv = 1; wv < kSWaves; ++wv) t += rpart[wv * kSInlineMaxE + lane];
        lg[lane] = t + (P.bias ? P.bias[lane] : 0.f);
      }
      if (E <= 8 && k <= 2) topk_tiny<8>(lg, E, k, L.renorm, lane, sel_e, sel_g);
      else if (E <= 16 && k <= 2) topk_tiny<16>(lg, E, k, L.renorm, lane, sel_e, sel_g);
      else topk_from_logits(lg, E, k, L.renorm, lane, sel_e, sel_g, nullptr);
    } else {
      topk_from_logits(P.logits + (size_t)token * E, E, k, L.renorm, lane, sel_e, sel_g, nullptr);
    }
  } else if (lane == 0) {
    sel_e[0] = P.fixed_expert;
    sel_g[0] = P.gate_in ? P.gate_in[token] : 1.0f;
  }
  if (lane < k) sel_e[lane] = min(max(sel_e[lane], 0), E - 1);
  if (routed && !given && slice == 0 && wave == 0 && lane < k) {
    if (P.idx_out) P.idx_out[(size_t)token * k + lane] = sel_e[lane];
    if (P.gate_out) P.gate_out[(size_t)token * k + lane] = sel_g[lane];
  }

  // ---- the list of blocks of a wavefront (the same for every wavefront): lane g computes entries g and g + 64
  // and keeps them in two registers, read with v_readlane when a block is requested. Entry: kind | first << 2 |
  // j << 3 | bits << 6 | index << 10, index = rb * NM + mat in phase 1, q in phase 2. Segment j (0 .. k) holds
  // phase 1 of expert j interleaved with phase 2 of expert j - 1, alternating while both have blocks left.
  const DevExpert* tabq = tabp;
  int n_total = 0, bm = 0;
  int ent_lo = 0, ent_hi = 0;
  {
    int start = 0, b2 = 0;                                      // b2: bits of expert j - 1
    for (int j = 0; j <= k; ++j) {
      {
        const int b1 = j < k ? __builtin_amdgcn_readfirstlane(tabq[sel_e[j]].bits) : 0;   // bits of expert j
        bm |= b1;
        const int n1 = (b1 >> 1) * NM, n2 = b2 == 0 ? 0 : (b2 == 2 ? 1 : (b2 == 4 ? 2 : 4));
        const int m = min(n1, n2);
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const int i = lane + 64 * half - start;
          if (i >= 0 && i < n1 + n2) {
            int kind, idx;
            if (i < 2 * m) { kind = (i & 1) ? B_P2 : B_P1; idx = i >> 1; }
            else { kind = n1 > n2 ? B_P1 : B_P2; idx = m + (i - 2 * m); }
            const int ent = kind == B_P1 ? (B_P1 | (j << 3) | (b1 << 6) | (idx << 10))
                                         : (B_P2 | ((idx == 0 ? 1 : 0) << 2) | ((j - 1) << 3) | (b2 << 6) | (idx << 10));
            if (half == 0) ent_lo = ent; else ent_hi = ent;
          }
        }
        start += n1 + n2;
        b2 = b1;
      }
    }
    n_total = start;
  }
  const uint8_t* idle = (const uint8_t*)xt;       // at least 8 KB of readable, cached bytes
  // Requests block g of the list into S and notes in tag what it is.
  auto issue = [&](BlkSet& S, BlkTag& tag, int g) __attribute__((always_inline)) {
    const int ent = g >= n_total ? 0 : (g < 64 ? __builtin_amdgcn_readlane(ent_lo, g) : __builtin_amdgcn_readlane(ent_hi, g - 64));
    tag.kind = ent & 3; tag.first = (ent >> 2) & 1; tag.j = (ent >> 3) & 7; tag.bits = (ent >> 6) & 15;
    const int index = ent >> 10;
    tag.mat = 0; tag.rb = 0; tag.q = index;
    const uint8_t* base = idle;
    uint32_t tstride = 0u, qstride = 0u, lane_t = (uint32_t)lane * 16u, soff0 = 0u, soff1 = 0u;
    const uint8_t* sbase = idle;
    int qshift = 3;                                  // tiles i >> qshift select the second row quad
    if (tag.kind != B_NONE) {
      const DevExpert* ex = tabq + sel_e[tag.j];
      if (tag.kind == B_P1) {
        tag.mat = SWIGLU ? (index & 1) : 0;
        tag.rb = SWIGLU ? (index >> 1) : index;
        const int rbsh = tag.bits == 2 ? 3 : (tag.bits == 4 ? 2 : 1);
        const uint32_t RB = 1u << rbsh, BB = 8192u + 64u * RB;
        const uint32_t blk = (((uint32_t)slice * 64u + (uint32_t)wave * 8u) >> rbsh) + (uint32_t)tag.rb;
        base = uniform_ptr(tag.mat ? ex->q_gate : ex->q_in) + (size_t)blk * BB;
        tstride = 1024u;
        sbase = base + 8192u;
        // the aligned 8 bytes that hold the lane's RB bytes of scales (always inside the block's scale area)
        soff0 = soff1 = ((uint32_t)lane * RB) & ~7u;
      } else {
        // phase 2: tile i = word column (first + i % wpb) of row quad (q0 + i / wpb)
        const uint32_t DW = 2u * (uint32_t)tag.bits;                           // word columns of the slice
        const uint32_t wpb = tag.bits == 2 ? 4u : 8u;                          // word columns per block
        const uint32_t first = tag.bits == 8 ? (uint32_t)(tag.q & 1) * 8u : 0u; // 8-bit: two blocks per row quad
        const uint32_t q0 = tag.bits == 2 ? 0u : (tag.bits == 4 ? (uint32_t)tag.q : (uint32_t)(tag.q >> 1));
        qshift = tag.bits == 2 ? 2 : 3;
        base = uniform_ptr(ex->q_out) + ((size_t)slice * DW + first) * ((size_t)kSD * 4);
        tstride = (uint32_t)kSD * 4u;
        qstride = 1024u - wpb * tstride;                                       // from the last word of quad 0 to quad 1
        lane_t = (uint32_t)(64 * (2 * wave + (int)q0) + lane) * 16u;
        sbase = (const uint8_t*)uniform_ptr(ex->s_out) + (size_t)(slice >> 1) * ((size_t)kSD * 2);
        soff0 = (uint32_t)(64 * (2 * wave + (int)q0) + lane) * 8u;
        soff1 = tag.bits == 2 ? soff0 + 512u : soff0;
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t off = (uint32_t)i * tstride + ((i >> qshift) ? qstride : 0u) + lane_t;
      S.t[i] = load_stream16(base + off);
    }
    S.s[0] = gload_u32x2(sbase + soff0);
    S.s[1] = gload_u32x2(sbase + soff1);
  };

  // ---- per-lane constants of phase 1 (read after the digits are staged)
  uint32_t xd4[(BM & 4) ? 8 : 1][4], xd2[(BM & 2) ? 8 : 1][4], xd8[(BM & 8) ? 8 : 1][4];
  float xs = 0.f;
  int sxl = 0;
  // the digit words of the lane's columns, for the bitwidths the chosen experts have (bm: their bitwidths or-ed)
  auto load_digits = [&](int bm_) __attribute__((always_inline)) {
    xs = XS[lane >> 1];
    sxl = SXL[lane];
    if constexpr ((BM & 4) != 0) if (bm_ & 4) {
#pragma unroll
      for (int j = 0; j < 8; ++j) { const uint4 v = XD4[j][lane]; xd4[j][0] = v.x; xd4[j][1] = v.y; xd4[j][2] = v.z; xd4[j][3] = v.w; }
    }
    if constexpr ((BM & 2) != 0) if (bm_ & 2) {
#pragma unroll
      for (int j = 0; j < 8; ++j) { const uint4 v = XD2[j][lane]; xd2[j][0] = v.x; xd2[j][1] = v.y; xd2[j][2] = v.z; xd2[j][3] = v.w; }
    }
    if constexpr ((BM & 8) != 0) if (bm_ & 8) {
#pragma unroll
      for (int j = 0; j < 8; ++j) { const uint4 v = XD8[j][lane]; xd8[j][0] = v.x; xd8[j][1] = v.y; xd8[j][2] = v.z; xd8[j][3] = v.w; }
    }
  };
  // sum over the 32 lanes of one parity (a lane pair is a scale group)
  auto parity_sum = [&](float t) __attribute__((always_inline)) {
    t += dpp<kDppXor2>(t);
    t += dpp<kDppRor4>(t);
    t += dpp<kDppRor8>(t);
    t += __shfl_xor(t, 16);
    t += __shfl_xor(t, 32);
    return t;
  };
  const bool odd = (lane & 1) != 0;
  float pa[4];                   // pre-activations of W_in waiting for W_gate (SwiGLU)
  // Phase 1 block: RB rows; lane pair (l, l^1) = scale group l/2; the even lane finishes the first RB/2 rows, the
  // odd lane the others. s: the lane's RB/2 scales (binary16) in s.x / s.y.
  auto consume_p1 = [&](const BlkSet& S, const BlkTag& tag) __attribute__((always_inline)) {
    float f[4] = {0.f, 0.f, 0.f, 0.f};
    int nrow = 0;                                     // rows this lane finishes
    if ((BM & 4) && tag.bits == 4) {
      int pv[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        int a[4] = {0, 0, 0, 0};
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          const uint4 t = S.t[2 * r + hf];
          const uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const uint32_t c = w[j] ^ 0x88888888u;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) a[kk] = sdot8(c, xd4[4 * hf + j][kk], a[kk]);
          }
        }
        const int v = a[0] + (a[1] << 4) + (a[2] << 8) + (a[3] << 12);
        pv[r] = v + dppi<kDppXor1>(v);
      }
      nrow = 2;
      const uint32_t s2 = odd ? S.s[0].y : S.s[0].x;      // the lane's 4 bytes of the aligned 8
      f[0] = (float)(odd ? pv[2] : pv[0]) * (f16_bits_to_f32(s2 & 0xffffu) * xs);
      f[1] = (float)(odd ? pv[3] : pv[1]) * (f16_bits_to_f32(s2 >> 16) * xs);
    } else if ((BM & 2) && tag.bits == 2) {
      int pv[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        int a[4] = {0, 0, 0, 0};
        const uint4 t = S.t[r];
        const uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint32_t ce = w[j] & 0x33333333u, co = (w[j] >> 2) & 0x33333333u;
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) {
            a[kk] = sdot8(ce, xd2[2 * j][kk], a[kk]);
            a[kk] = sdot8(co, xd2[2 * j + 1][kk], a[kk]);
          }
        }
        const int v = a[0] + (a[1] << 4) + (a[2] << 8) + (a[3] << 12) - 2 * sxl;   // codes carry the offset 2
        pv[r] = v + dppi<kDppXor1>(v);
      }
      nrow = 4;
      f[0] = (float)(odd ? pv[4] : pv[0]) * (f16_bits_to_f32(S.s[0].x & 0xffffu) * xs);
      f[1] = (float)(odd ? pv[5] : pv[1]) * (f16_bits_to_f32(S.s[0].x >> 16) * xs);
      f[2] = (float)(odd ? pv[6] : pv[2]) * (f16_bits_to_f32(S.s[0].y & 0xffffu) * xs);
      f[3] = (float)(odd ? pv[7] : pv[3]) * (f16_bits_to_f32(S.s[0].y >> 16) * xs);
    } else if ((BM & 8) && tag.bits == 8) {
      int pv[2];
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        int alo = 0, ahi = 0;
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
          const uint4 t = S.t[4 * r + tt];
          const uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const uint32_t c = w[j] ^ 0x80808080u;
            alo = sdot4(c, xd8[2 * tt + (j >> 1)][2 * (j & 1)], alo);
            ahi = sdot4(c, xd8[2 * tt + (j >> 1)][2 * (j & 1) + 1], ahi);
          }
        }
        const int v = alo + (ahi << 8);
        pv[r] = v + dppi<kDppXor1>(v);
      }
      nrow = 1;
      const uint32_t s2 = (lane & 2) ? S.s[0].y : S.s[0].x;   // the lane's 2 bytes of the aligned 8
      f[0] = (float)(odd ? pv[1] : pv[0]) * (f16_bits_to_f32((s2 >> (16 * (lane & 1))) & 0xffffu) * xs);
    }
    const int RB = 16 / tag.bits;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (i < nrow) {
        const float tot = parity_sum(f[i]);
        if (SWIGLU && tag.mat == 0) {
          pa[i] = tot;
        } else {
          float hv;
          if constexpr (SWIGLU) hv = pa[i] / (1.0f + __expf(-pa[i])) * tot;
          else hv = fmaxf(tot, 0.f);
          if (lane < 2) HF[tag.j][wave * 8 + tag.rb * RB + lane * (RB / 2) + i] = hv;
        }
      }
    }
  };

  // ---- phase 2 state: the lane's 8 output rows
  float y[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  int acc8[4][2] = {{0, 0}, {0, 0}, {0, 0}, {0, 0}};   // 8-bit experts: a row quad's sums run over two blocks
  auto consume_p2 = [&](const BlkSet& S, const BlkTag& tag) __attribute__((always_inline)) {
    const float gu = sel_g[tag.j] * uph[tag.j];
    const uint4* hd = HD[tag.j];
    if ((BM & 4) && tag.bits == 4) {
      int a[4][4];
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) a[r][kk] = 0;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint4 h4 = hd[i];
        const uint32_t hk[4] = {h4.x, h4.y, h4.z, h4.w};
        const uint32_t w[4] = {S.t[i].x, S.t[i].y, S.t[i].z, S.t[i].w};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const uint32_t c = w[r] ^ 0x88888888u;
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) a[r][kk] = sdot8(c, hk[kk], a[r][kk]);
        }
      }
      const uint32_t sc[4] = {S.s[0].x & 0xffffu, S.s[0].x >> 16, S.s[0].y & 0xffffu, S.s[0].y >> 16};
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int v = a[r][0] + (a[r][1] << 4) + (a[r][2] << 8) + (a[r][3] << 12);
        const float c = (float)v * (f16_bits_to_f32(sc[r]) * gu);
        // both candidates with static indices (a run-time index would move y out of the registers)
        y[r] += tag.q == 0 ? c : 0.f;
        y[4 + r] += tag.q == 0 ? 0.f : c;
      }
    } else if ((BM & 2) && tag.bits == 2) {
      const int sh2 = 2 * SH[tag.j];
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        int a[4][4];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) a[r][kk] = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const uint4 he4 = hd[2 * i], ho4 = hd[2 * i + 1];
          const uint32_t hek[4] = {he4.x, he4.y, he4.z, he4.w}, hok[4] = {ho4.x, ho4.y, ho4.z, ho4.w};
          const uint4 t = S.t[4 * q + i];
          const uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const uint32_t ce = w[r] & 0x33333333u, co = (w[r] >> 2) & 0x33333333u;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
              a[r][kk] = sdot8(ce, hek[kk], a[r][kk]);
              a[r][kk] = sdot8(co, hok[kk], a[r][kk]);
            }
          }
        }
        const uint2 s2 = S.s[q];
        const uint32_t sc[4] = {s2.x & 0xffffu, s2.x >> 16, s2.y & 0xffffu, s2.y >> 16};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int v = a[r][0] + (a[r][1] << 4) + (a[r][2] << 8) + (a[r][3] << 12) - sh2;
          y[4 * q + r] += (float)v * (f16_bits_to_f32(sc[r]) * gu);
        }
      }
    } else if ((BM & 8) && tag.bits == 8) {
      // 8-bit: word columns 8 * (q & 1) .. + 7 of row quad q >> 1; the digits of h: word i -> HD[j][i / 2], (lo, hi) pairs
      const int half = tag.q & 1;
      if (half == 0) {
#pragma unroll
        for (int r = 0; r < 4; ++r) acc8[r][0] = acc8[r][1] = 0;
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint4 h4 = hd[4 * half + (i >> 1)];
        const uint32_t lo = (i & 1) ? h4.z : h4.x, hi = (i & 1) ? h4.w : h4.y;
        const uint32_t w[4] = {S.t[i].x, S.t[i].y, S.t[i].z, S.t[i].w};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const uint32_t c = w[r] ^ 0x80808080u;
          acc8[r][0] = sdot4(c, lo, acc8[r][0]);
          acc8[r][1] = sdot4(c, hi, acc8[r][1]);
        }
      }
      if (half == 1) {
        const uint32_t sc[4] = {S.s[0].x & 0xffffu, S.s[0].x >> 16, S.s[0].y & 0xffffu, S.s[0].y >> 16};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int v = acc8[r][0] + (acc8[r][1] << 8);
          const float c = (float)v * (f16_bits_to_f32(sc[r]) * gu);
          y[r] += (tag.q >> 1) == 0 ? c : 0.f;
          y[4 + r] += (tag.q >> 1) == 0 ? 0.f : c;
        }
      }
    }
  };

  // ---- between the phases of expert j: digits of its h slice (one wavefront)
  auto stage_h = [&](int j) __attribute__((always_inline)) {
    if (wave == (j & (kSWaves - 1))) {
      const int bits = __builtin_amdgcn_readfirstlane(tabp[sel_e[j]].bits);
      const float hv = HF[j][lane];
      float m = !(fabsf(hv) < INFINITY) ? INFINITY : fabsf(hv);
      m = wave_max(m);
      const int e = block_exponent(m);
      const int hi = m < INFINITY ? __float2int_rn(hv * pow2f(-e)) : 0;
      if (lane == 0) uph[j] = m < INFINITY ? pow2f(e) : __builtin_nanf("");
      int s = hi;
      s += dppi<kDppXor1>(s); s += dppi<kDppXor2>(s); s += dppi<kDppRor4>(s); s += dppi<kDppRor8>(s);
      s += __shfl_xor(s, 16); s += __shfl_xor(s, 32);
      if (lane == 0) SH[j] = s;
      uint32_t* HDw = (uint32_t*)HD[j];
      if (bits == 8) {
        // word i (4 columns) -> HD word 2i (lo bytes), 2i+1 (hi bytes); lane c: word c/4, byte c%4
        const uint32_t l8 = (uint32_t)hi & 255u, h8 = (uint32_t)((hi + 128) >> 8) & 255u;
        uint32_t lo = l8 << (8 * (lane & 3)), hh = h8 << (8 * (lane & 3));
        lo |= (uint32_t)dppi<kDppXor1>((int)lo); lo |= (uint32_t)dppi<kDppXor2>((int)lo);
        hh |= (uint32_t)dppi<kDppXor1>((int)hh); hh |= (uint32_t)dppi<kDppXor2>((int)hh);
        if ((lane & 3) == 0) { HDw[2 * (lane >> 2)] = lo; HDw[2 * (lane >> 2) + 1] = hh; }
      } else {
        int v = hi;
        uint32_t n[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) n[kk] = next_digit(v);
        if (bits == 4) {
          // word i = columns 8i .. 8i+7 -> HD[j][i] = digit words k
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) {
            uint32_t d = n[kk] << (4 * (lane & 7));
            d |= (uint32_t)dppi<kDppXor1>((int)d); d |= (uint32_t)dppi<kDppXor2>((int)d);
            d |= (uint32_t)__shfl_xor((int)d, 4);
            if ((lane & 7) == 0) HDw[4 * (lane >> 3) + kk] = d;
          }
        } else {
          // word i = columns 16i .. 16i+15 -> HD[j][2i] (even columns), HD[j][2i+1] (odd columns)
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) {
            uint32_t d = n[kk] << (4 * ((lane & 15) >> 1));
            d |= (uint32_t)dppi<kDppXor2>((int)d); d |= (uint32_t)dppi<kDppRor4>((int)d); d |= (uint32_t)dppi<kDppRor8>((int)d);
            if ((lane & 15) < 2) HDw[4 * (2 * (lane >> 4) + (lane & 1)) + kk] = d;
          }
        }
      }
    }
  };

  // ---- the stream: kNSets register sets in rotation over the list
  BlkSet S[kNSets];
  BlkTag tg[kNSets];
#pragma unroll
  for (int i = 0; i < kNSets; ++i) issue(S[i], tg[i], i);
  load_digits(bm);     // behind the first requests
  auto consume = [&](const BlkSet& St, const BlkTag& tag) __attribute__((always_inline)) {
    if (tag.kind == B_P1) {
      consume_p1(St, tag);
    } else if (tag.kind == B_P2) {
      if (tag.first) {          // uniform over the workgroup: every wavefront walks the same list
        __syncthreads();        // the h slice of expert tag.j is complete (fp32)
        stage_h(tag.j);
        __syncthreads();
      }
      consume_p2(St, tag);
    }
  };
  for (int g = 0; g < n_total; g += kNSets) {
#pragma unroll
    for (int i = 0; i < kNSets; ++i) {
      consume(S[i], tg[i]);
      issue(S[i], tg[i], g + kNSets + i);
    }
  }
  // ---- the partial output vector, straight from the registers
  float* out = P.part + ((size_t)token * gridDim.x + slice) * kSD;
#pragma unroll
  for (int q = 0; q < 2; ++q)
    *(float4*)(out + 4 * (64 * (2 * wave + q) + lane)) = make_float4(y[4 * q], y[4 * q + 1], y[4 * q + 2], y[4 * q + 3]);
}

// ---------------------------------------------------------------------------------------------
// Canonical <-> row-block stream layout of a [rows][4096] matrix with scale groups of 128 columns. One thread
// per 16-byte piece of codes; the threads of a block's first 64 pieces also move the block's scales.
//   block (RB = 16/bits rows): [8 tiles x 1 KB][64 lanes x RB bytes of scales]
//   tile t = row t / TPR, part t % TPR (TPR = bits/2 tiles per row); lane l's 16 bytes = canonical bytes
//   [16 * (TPR * l + part), +16) of that row, i.e. 32 / 64 / 16 consecutive columns inside [64 l, 64 l + 64)
//   scales: lane l's RB/2 values = canonical scale[row0 + (l & 1) * RB/2 + i][l >> 1], i < RB/2
template <bool TO_STREAM>
__global__ __launch_bounds__(256) void k_relayout_in(const uint8_t* __restrict__ q, const uint16_t* __restrict__ s,
                                                     int64_t rows, int bits, uint8_t* __restrict__ stream) {
  const int TPR = bits / 2, RB = 16 / bits;
  const uint32_t BB = stream_block_bytes(bits);
  const int64_t piece = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;     // 16-byte piece of the stream's tiles
  const int64_t n_pieces = rows * TPR * 64;
  if (piece >= n_pieces) return;
  const int64_t blk = piece / 512;
  const int in_blk = (int)(piece % 512), t = in_blk / 64, l = in_blk % 64;
  const int64_t row = blk * RB + t / TPR;
  const int part = t % TPR;
  uint4* dst_s = (uint4*)(stream + blk * BB + (size_t)t * 1024 + (size_t)l * 16);
  uint4* src_c = (uint4*)(q + row * (int64_t)(TPR * 1024) + (int64_t)(TPR * l + part) * 16);
  if (TO_STREAM) *dst_s = *src_c; else *src_c = *dst_s;
  if (t == 0) {
    uint16_t* sc = (uint16_t*)(stream + blk * BB + 8192 + (size_t)l * RB);
    for (int i = 0; i < RB / 2; ++i) {
      uint16_t* canon = (uint16_t*)s + (blk * RB + (l & 1) * (RB / 2) + i) * 32 + (l >> 1);
      if (TO_STREAM) sc[i] = *canon; else *canon = sc[i];
    }
  }
}

}  // namespace

bool stream_supported(const LayerDims& L) {
  return L.d_model == kSD && L.group == kSGroup && L.group_out == kSGroup && L.d_ff % kSSlice == 0 && L.top_k <= 8;
}
int stream_inline_router_max() { return kSInlineMaxE; }
int stream_slices(const LayerDims& L) { return L.d_ff / kSSlice; }

hipError_t launch_moe_stream(const LayerDims& L, const DevExpert* table, const float* router_w, const float* router_bias,
                             const float* logits, int32_t fixed_expert, const float* gate_in, const int32_t* route_idx,
                             const float* route_gate, int32_t bits_mask, const void* x, int32_t T, float* part,
                             int32_t* idx_out, float* gate_out, hipStream_t st, hipEvent_t ev_start,
                             hipEvent_t ev_stop) {
  if (!stream_supported(L) || T < 1 || T > 65535 || !(bits_mask & 14)) return hipErrorInvalidValue;
  if (!logits && !route_idx && fixed_expert < 0 && L.n_experts > kSInlineMaxE) return hipErrorInvalidValue;
  if ((route_idx != nullptr) != (route_gate != nullptr)) return hipErrorInvalidValue;
  StreamParams P{L, table, router_w, router_bias, logits, fixed_expert, gate_in, route_idx, route_gate, x, part,
                 idx_out, gate_out};
  // the variant for the bitwidths the layer holds (2 | 4 | 8 or-ed); the mixes without their own variant take the full one
  const bool sw = L.act == MOEQ_ACT_SWIGLU;
  void (*kernel)(StreamParams) = nullptr;
  switch (bits_mask & 14) {
    case 2: kernel = sw ? k_moe_stream<true, 2> : k_moe_stream<false, 2>; break;
    case 4: kernel = sw ? k_moe_stream<true, 4> : k_moe_stream<false, 4>; break;
    case 6: kernel = sw ? k_moe_stream<true, 6> : k_moe_stream<false, 6>; break;
    case 8: kernel = sw ? k_moe_stream<true, 8> : k_moe_stream<false, 8>; break;
    default: kernel = sw ? k_moe_stream<true, 14> : k_moe_stream<false, 14>; break;
  }
  const dim3 grid(stream_slices(L), T), block(kSThreads);
  if (ev_start && ev_stop) hipExtLaunchKernelGGL(kernel, grid, block, 0, st, ev_start, ev_stop, 0, P);
  else hipLaunchKernelGGL(kernel, grid, block, 0, st, P);
  return hipGetLastError();
}

hipError_t launch_relayout_in(const void* q, const void* s, int64_t rows, int bits, void* stream_buf, bool to_stream,
                              hipStream_t st) {
  const int64_t n_pieces = rows * (bits / 2) * 64, blocks = (n_pieces + 255) / 256;
  if (blocks > 0x7fffffff || blocks < 1) return hipErrorInvalidValue;
  if (to_stream)
    hipLaunchKernelGGL(k_relayout_in<true>, dim3((unsigned)blocks), dim3(256), 0, st, (const uint8_t*)q,
                       (const uint16_t*)s, rows, bits, (uint8_t*)stream_buf);
  else
    hipLaunchKernelGGL(k_relayout_in<false>, dim3((unsigned)blocks), dim3(256), 0, st, (const uint8_t*)q,
                       (const uint16_t*)s, rows, bits, (uint8_t*)stream_buf);
  return hipGetLastError();
}

}  // namespace moeq
