// Batched (prefill) path of the MoE layer: the (token, choice) pairs are grouped by expert and every
// expert's FFN runs as two GEMMs on the matrix cores over its own tokens (Section 2.1: only the chosen
// experts work on a token; Section 3.2: their weights are decompressed by the mirror of the linear
// quantization before use - here inside the GEMM, on the way from the packed tile to the instruction).
//
//   grouping : histogram of the pairs per expert, offsets, a list of (expert, block of 64 tokens) work
//              items, a stable scatter of the pairs into expert order (and its inverse)
//   staging  : per pair, the token's activations, normalised by a power of two of their own, as binary16 in
//              the pair order of its expert's bitwidth (the order dword_dot / codes8 consume), plus the
//              offset term of every K step
//   GEMM 1   : H[pair][row] = act(W_in x [, W_gate x]) (fp32) for 64 tokens x 128 or 256 rows per workgroup
//   staging  : the same for every pair's h
//   GEMM 2   : Ypair[pair][row] = W_out h for 64 tokens x 256 rows per workgroup
//   combine  : y[t] = sum_j gate[t][j] * Ypair[pair(t, j)], in top-k order
//
// The GEMMs never form floating-point weights: a wavefront reads 16-byte pieces of packed rows, masks
// the code fields into binary16 subnormals (codes8) and feeds them to v_mfma_f32_16x16x32_f16 as the B
// operand; the A operand (activations pre-divided by the fields' powers of two) comes from LDS. One K
// step (128 columns, 64 at 8 bits) lies inside one scale group, so the group scale and the code offset
// are applied to the step's partial product: acc += s * (D - 2^(b-1) * sum(x_step)).
#include "decode_core.h"

namespace moeq {
namespace {

constexpr int kTB = 64;        // tokens per work item
constexpr int kGemmThreads = 512;
constexpr int kGemmWaves = kGemmThreads / 64;

// ---------------------------------------------------------------------------------------------
// grouping
__global__ __launch_bounds__(1024) void k_count_pairs(const int32_t* __restrict__ idx, int M, int E,
                                                      int32_t* __restrict__ poff, int2* __restrict__ blocks,
                                                      int32_t* __restrict__ n_blocks) {
  __shared__ int h[1024];
  for (int e = threadIdx.x; e < E; e += blockDim.x) h[e] = 0;
  __syncthreads();
  for (int p = threadIdx.x; p < M; p += blockDim.x) atomicAdd(&h[min(max(idx[p], 0), E - 1)], 1);
  __syncthreads();
  if (threadIdx.x == 0) {
    int off = 0, nb = 0;
    for (int e = 0; e < E; ++e) {
      poff[e] = off;
      const int c = h[e];
      for (int tb = 0; tb * kTB < c; ++tb) blocks[nb++] = make_int2(e, tb);
      off += c;
    }
    poff[E] = off;
    *n_blocks = nb;
  }
}

// Workgroup e writes the pairs routed to expert e, in increasing pair order, behind poff[e].
__global__ __launch_bounds__(256) void k_scatter_pairs(const int32_t* __restrict__ idx, int M,
                                                       const int32_t* __restrict__ poff, int32_t* __restrict__ gpair,
                                                       int32_t* __restrict__ ginv, int32_t* __restrict__ gexp) {
  __shared__ int wcnt[4];
  const int e = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int base = poff[e];
  for (int p0 = 0; p0 < M; p0 += 256) {
    const int p = p0 + threadIdx.x;
    const bool hit = p < M && min(max(idx[p], 0), (int)gridDim.x - 1) == e;   // the same clamp as the histogram
    const unsigned long long mask = __ballot(hit);
    const int before = __popcll(mask & ((1ull << lane) - 1ull));
    if (lane == 0) wcnt[wave] = __popcll(mask);
    __syncthreads();
    int wbase = 0;
    for (int w = 0; w < wave; ++w) wbase += wcnt[w];
    const int total = wcnt[0] + wcnt[1] + wcnt[2] + wcnt[3];
    if (hit) {
      const int g = base + wbase + before;
      gpair[g] = p;
      ginv[p] = g;
      gexp[g] = e;
    }
    base += total;
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------------
// Staging of the activation vector of one pair for a GEMM. Per pair: [K/2 words in pair order][K/64 floats:
// the negated offset term of every K step][the factor 2^e that undoes the normalisation, then 3 unused words].
// FROM_H = false: the pair's token row of x (GEMM 1); true: row g of the fp32 h that GEMM 1 wrote (GEMM 2).
// The vector is normalised by its own power of two before the conversion to binary16 (stage_normalised).
template <bool FROM_H>
__global__ __launch_bounds__(256) void k_stage(LayerDims L, const DevExpert* __restrict__ table,
                                               const void* __restrict__ src, const int32_t* __restrict__ gpair,
                                               const int32_t* __restrict__ gexp, uint32_t* __restrict__ OUT,
                                               int64_t pair_words) {
  extern __shared__ uint32_t smem[];
  __shared__ float red[4];
  const int cols = FROM_H ? L.d_ff : L.d_model;
  uint16_t* RAW = (uint16_t*)smem;
  const int g = blockIdx.x;
  const int bits = table[gexp[g]].bits;
  const char* row;
  int kind;
  if (FROM_H) {
    row = (const char*)src + (size_t)g * cols * 4;
    kind = X_F32;
  } else {
    row = (const char*)src + (size_t)(gpair[g] / L.top_k) * cols * (L.x_bf16 ? 2 : 4);
    kind = L.x_bf16 ? X_BF16 : X_F32;
  }
  const float up = stage_normalised(row, kind, cols, threadIdx.x, blockDim.x, RAW, red);
  __syncthreads();
  uint32_t* XP = OUT + (size_t)g * pair_words;
  float* KS = (float*)(XP + cols / 2);
  float* scratch = (float*)(smem + cols / 2);     // the per-chunk offset terms permute_x also makes; not kept
  const int group = FROM_H ? L.group_out : L.group;
  if (bits == 2) { permute_x<2>(RAW, cols, group, threadIdx.x, blockDim.x, XP, scratch); range_offset_terms<2>(RAW, cols, threadIdx.x, blockDim.x, KS); }
  else if (bits == 4) { permute_x<4>(RAW, cols, group, threadIdx.x, blockDim.x, XP, scratch); range_offset_terms<4>(RAW, cols, threadIdx.x, blockDim.x, KS); }
  else { permute_x<8>(RAW, cols, group, threadIdx.x, blockDim.x, XP, scratch); range_offset_terms<8>(RAW, cols, threadIdx.x, blockDim.x, KS); }
  if (threadIdx.x == 0) KS[cols / 64] = up;
}

// ---------------------------------------------------------------------------------------------
// The quantized GEMM. Workgroup = 8 wavefronts = 64 tokens x (8 wavefronts x NS streams x 16 rows); a
// stream is (matrix, block of 16 rows): with two matrices (SwiGLU phase 1) a wavefront owns 32 rows of both,
// else 64 rows. Lane (n, kb) of a wavefront holds, per K step, the 16-byte piece 4*step + kb of row n of
// each stream (8 bytes at 2 bits): four k blocks along one scale group.
struct GemmArgs {
  LayerDims L;
  const DevExpert* table;
  const int2* blocks;
  const int32_t* n_blocks;
  const int32_t* poff;
  const uint32_t* A;        // staged activations: per pair [K/2 pair words][K/64 offset terms][2^e ...]
  int64_t a_pair_words;
  float* Hf;                // GEMM 1 out: h per pair, fp32 [pairs][d_ff]
  float* Y;                 // GEMM 2 out: [pairs][d_model]
};

// uint4 index, inside a pair's staged words, of A operand q of a K step for k block kb
template <int BITS>
__device__ __forceinline__ int a_src_index(int C, int step, int q, int kb) {
  if (BITS == 2) return (2 * (2 * (kb & 1) + (q >> 1)) + (q & 1)) * C + 2 * step + (kb >> 1);
  return q * C + 4 * step + kb;
}

template <int BITS, int NM, int PHASE, bool COLS>
__device__ __forceinline__ void gemm_body(const GemmArgs& G, const DevExpert& ex, int e, int tb, uint4* As, float* Ks) {
  constexpr int WPC = 128 / BITS;
  constexpr int SC = BITS == 8 ? 64 : 128;        // columns per K step
  constexpr int NQ = BITS == 8 ? 2 : 4;           // instructions per step, stream and token block
  // streams (row blocks of 16 rows) per wavefront; GEMM 2 has few rows (d_model): with two streams per
  // wavefront its grid has twice the workgroups and fills the compute units more evenly
  constexpr int NS = PHASE == 1 ? 2 : 4;
  constexpr int RBW = NS / NM;                    // row blocks per wavefront and matrix
  constexpr int BN = kGemmWaves * RBW * 16;       // rows per workgroup
  constexpr int APAD = 65;                        // tokens per (q, kb) line of the LDS tile, padded
  using TileT = std::conditional_t<BITS == 2, uint2, uint4>;
  const int K = PHASE == 0 ? G.L.d_model : G.L.d_ff;
  const int N = PHASE == 0 ? G.L.d_ff : G.L.d_model;
  const int group = PHASE == 0 ? G.L.group : G.L.group_out;
  const int C = K / WPC, n_steps = K / SC;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 15, kb = lane >> 4;
  const int g0 = G.poff[e] + tb * kTB;
  const int ntok = min(kTB, G.poff[e + 1] - g0);
  const int R0 = blockIdx.x * BN + wave * (RBW * 16);
  const uint32_t row_bytes = (uint32_t)C * 16u;
  const uint32_t ng2 = (uint32_t)(K / group) * 2u;

  const uint8_t* qs[NM];
  const uint8_t* ss[NM];
  if (PHASE == 0) {
    qs[0] = ex.q_in; ss[0] = (const uint8_t*)ex.s_in;
    if (NM == 2) { qs[NM - 1] = ex.q_gate; ss[NM - 1] = (const uint8_t*)ex.s_gate; }
  } else {
    qs[0] = ex.q_out; ss[0] = (const uint8_t*)ex.s_out;
  }
  uint32_t qrow[NS], srow[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    const uint32_t row = (uint32_t)min(R0 + (s % RBW) * 16 + n, N - 1);
    // COLS (GEMM 2 on a W_out in the dword-column-major layout): word w of row r is the 32-bit word
    // w * N + r, the scale of group g of row r the binary16 value g * N + r
    qrow[s] = COLS ? row * 4u : row * row_bytes;
    srow[s] = COLS ? row * 2u : row * ng2;
  }
  struct BSet { TileT t[NS]; };
  auto load_b = [&](BSet& B, int step) __attribute__((always_inline)) {
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const uint8_t* q = qs[s / RBW];
      if constexpr (COLS) {
        const uint32_t col_bytes = (uint32_t)N * 4u;
        if constexpr (BITS == 2) {
          const uint32_t w0 = ((uint32_t)step * 4u + (uint32_t)kb) * 2u;
          B.t[s].x = gload_u32(q + (w0 * col_bytes + qrow[s]));
          B.t[s].y = gload_u32(q + ((w0 + 1u) * col_bytes + qrow[s]));
        } else {
          const uint32_t w0 = ((uint32_t)step * 4u + (uint32_t)kb) * 4u;
          B.t[s].x = gload_u32(q + (w0 * col_bytes + qrow[s]));
          B.t[s].y = gload_u32(q + ((w0 + 1u) * col_bytes + qrow[s]));
          B.t[s].z = gload_u32(q + ((w0 + 2u) * col_bytes + qrow[s]));
          B.t[s].w = gload_u32(q + ((w0 + 3u) * col_bytes + qrow[s]));
        }
      } else if constexpr (BITS == 2) {
        B.t[s] = gload_u32x2(q + (qrow[s] + (uint32_t)step * 32u + (uint32_t)kb * 8u));
      } else {
        B.t[s] = gload_u32x4(q + (qrow[s] + (uint32_t)step * 64u + (uint32_t)kb * 16u));
      }
    }
  };
  // A tile of a step: thread -> (kb, token, q) items; 4 consecutive threads read 64 contiguous bytes
  constexpr int AITEMS = NQ * 4 * kTB / kGemmThreads;     // 16-byte items per thread and step
  struct ASet { uint4 v[AITEMS]; float ks; };
  auto load_a = [&](ASet& A, int step) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < AITEMS; ++r) {
      const int item = threadIdx.x + r * kGemmThreads;
      const int akb = item & 3, tok = (item >> 2) & 63, q = item >> 8;
      A.v[r] = make_uint4(0u, 0u, 0u, 0u);
      if (tok < ntok) {
        const uint4* src = (const uint4*)(G.A + (size_t)(g0 + tok) * G.a_pair_words);
        A.v[r] = src[a_src_index<BITS>(C, step, q, akb)];
      }
    }
    A.ks = 0.f;
    if ((int)threadIdx.x < ntok)
      A.ks = ((const float*)(G.A + (size_t)(g0 + threadIdx.x) * G.a_pair_words + K / 2))[step];
  };
  auto store_a = [&](const ASet& A, int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < AITEMS; ++r) {
      const int item = threadIdx.x + r * kGemmThreads;
      const int akb = item & 3, tok = (item >> 2) & 63, q = item >> 8;
      As[(buf * NQ * 4 + q * 4 + akb) * APAD + tok] = A.v[r];
    }
    if (threadIdx.x < kTB) Ks[buf * kTB + threadIdx.x] = A.ks;    // already negated: the accumulations start there
  };

  float4_t acc[NS][4];
  const float4_t zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < NS; ++s)
#pragma unroll
    for (int t4 = 0; t4 < 4; ++t4) acc[s][t4] = zero;

  // The arithmetic of a step is split in two so that the raw tiles' registers can take the next step's
  // loads as soon as the codes are unpacked: one set of tile registers serves the whole loop.
  half8_t Bop[NS][NQ];
  float sc[NS];
  uint32_t scx[NS], scy[NS];                      // a stream's scales of the current block of four groups
#pragma unroll
  for (int s = 0; s < NS; ++s) scx[s] = scy[s] = 0u;
  auto unpack = [&](const BSet& B, int step) __attribute__((always_inline)) {
    // the step's scale among the four of the block held in scb
    const uint32_t gi = ((uint32_t)step * (uint32_t)SC) / (uint32_t)group;
    const bool sel = (gi & 2u) != 0;
    const uint32_t sh = (gi & 1u) * 16u;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      if constexpr (BITS == 4) {
        Bop[s][0] = codes8<4, 0>(B.t[s].x, 0u); Bop[s][1] = codes8<4, 0>(B.t[s].y, 0u);
        Bop[s][2] = codes8<4, 0>(B.t[s].z, 0u); Bop[s][3] = codes8<4, 0>(B.t[s].w, 0u);
      } else if constexpr (BITS == 8) {
        Bop[s][0] = codes8<8, 0>(B.t[s].x, B.t[s].y); Bop[s][1] = codes8<8, 0>(B.t[s].z, B.t[s].w);
      } else {
        Bop[s][0] = codes8<2, 0>(B.t[s].x, 0u); Bop[s][1] = codes8<2, 1>(B.t[s].x, 0u);
        Bop[s][2] = codes8<2, 0>(B.t[s].y, 0u); Bop[s][3] = codes8<2, 1>(B.t[s].y, 0u);
      }
      sc[s] = f16_bits_to_f32((sel ? scy[s] : scx[s]) >> sh);   // (the conversion takes the low 16 bits)
    }
  };
  // The A operands of a step are read from LDS two instructions groups ahead of the matrix-core instructions
  // that use them (three register slots): the latency of a read is covered by the eight to sixteen
  // instructions in between instead of being waited for in front of every group.
  constexpr int NI = 4 * NQ;                      // (token block, q) items of a step
  auto read_a = [&](int buf, int idx) __attribute__((always_inline)) {
    return As[(buf * NQ * 4 + (idx % NQ) * 4 + kb) * APAD + 16 * (idx / NQ) + n];
  };
  auto read_k = [&](int buf, int t4) __attribute__((always_inline)) {
    // the accumulation starts at the negated offset terms of the lane's four tokens
    const float4 k4 = *(const float4*)(Ks + buf * kTB + 16 * t4 + 4 * kb);
    const float4_t kv = {k4.x, k4.y, k4.z, k4.w};
    return kv;
  };
  // Without this the compiler sinks the unpacking below the next tiles' loads (its results are used only
  // by the multiplications): the raw tiles then stay live beside the new ones and are copied at the end of
  // every step. An empty statement that names the operands keeps the unpacking where it is written, so the
  // loads reuse the raw tiles' registers.
  auto pin_operands = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
      for (int q = 0; q < NQ; ++q) asm volatile("" : "+v"(Bop[s][q]));
  };
  // two result sets where the registers allow it (not for GEMM 1 with one matrix: it would spill)
  constexpr bool DBL = NM == 2 || PHASE == 1;
  auto multiply = [&](int buf) __attribute__((always_inline)) {
    uint4 af[3];
    af[0] = read_a(buf, 0);
    af[1] = read_a(buf, 1);
    float4_t kv = read_k(buf, 0);
    // two sets of results: the scaling of a token block's results waits for its last matrix-core
    // instructions, so it is issued behind the first instructions of the next token block
    float4_t D[2][NS];
#pragma unroll
    for (int idx = 0; idx < NI; ++idx) {
      const int t4 = idx / NQ, q = idx % NQ, d = DBL ? (t4 & 1) : 0;
      if (idx + 2 < NI) af[(idx + 2) % 3] = read_a(buf, idx + 2);
      if (q == 0) {
#pragma unroll
        for (int s = 0; s < NS; ++s) D[d][s] = kv;
        if (t4 + 1 < 4) kv = read_k(buf, t4 + 1);
      }
      const half8_t A = as_half8(af[idx % 3]);
#pragma unroll
      for (int s = 0; s < NS; ++s) D[d][s] = mfma16(A, Bop[s][q], D[d][s]);
      if (DBL && q == 0 && t4 > 0) {
#pragma unroll
        for (int s = 0; s < NS; ++s) acc[s][t4 - 1] += sc[s] * D[d ^ 1][s];
      }
      if (!DBL && q == NQ - 1) {
#pragma unroll
        for (int s = 0; s < NS; ++s) acc[s][t4] += sc[s] * D[0][s];
      }
    }
    if (DBL) {
#pragma unroll
      for (int s = 0; s < NS; ++s) acc[s][3] += sc[s] * D[1][s];
    }
  };

  // Step s multiplies the A tile in LDS buffer s & 1 with the B tiles unpacked at its start. The A tile of
  // step s + 1 was requested during step s - 1 and goes to the other LDS buffer at the start of step s (all
  // wavefronts are past the barrier that ended the last reads of that buffer); then the B tiles of step
  // s + 1 and the A tile of step s + 2 are requested: every load has a whole step to arrive. The last two
  // steps are peeled so that the loop body holds no condition on the step number.
  // The scales are not fetched with every tile: a 2-byte read per lane from 16 different rows costs the
  // memory system as much as the tile itself. A stream's scales of four consecutive groups are 8 contiguous
  // bytes (the plan makes rows of scales multiples of 8 bytes); they are read together, once per block of
  // blk_steps = 4 * group / SC steps, right after the last step of the previous block has taken its scale.
  const int blk_steps = 4 * group / SC;
  auto load_scales = [&](int step) __attribute__((always_inline)) {
    const uint32_t gi = ((uint32_t)step * (uint32_t)SC) / (uint32_t)group;     // a multiple of 4 here
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      if constexpr (COLS) {
        const uint8_t* sb = ss[s / RBW];
        const uint32_t g_bytes = (uint32_t)N * 2u;
        const uint32_t a0 = gload_u16(sb + (gi * g_bytes + srow[s])), a1 = gload_u16(sb + ((gi + 1u) * g_bytes + srow[s]));
        const uint32_t a2 = gload_u16(sb + ((gi + 2u) * g_bytes + srow[s])), a3 = gload_u16(sb + ((gi + 3u) * g_bytes + srow[s]));
        scx[s] = a0 | (a1 << 16);
        scy[s] = a2 | (a3 << 16);
      } else {
        const uint2 v = gload_u32x2(ss[s / RBW] + (srow[s] + gi * 2u));
        scx[s] = v.x;
        scy[s] = v.y;
      }
    }
  };
  BSet B;
  ASet A0;
  load_scales(0);
  load_a(A0, 0);
  load_b(B, 0);
  store_a(A0, 0);
  if (n_steps > 1) load_a(A0, 1);
  __syncthreads();
  int step = 0;
  for (; step + 2 < n_steps; ++step) {
    const int buf = step & 1;
    unpack(B, step);
    pin_operands();
    if ((step + 1) % blk_steps == 0) load_scales(step + 1);
    load_b(B, step + 1);
    store_a(A0, buf ^ 1);
    load_a(A0, step + 2);
    multiply(buf);
    __syncthreads();
  }
  if (step + 1 < n_steps) {
    const int buf = step & 1;
    unpack(B, step);
    if ((step + 1) % blk_steps == 0) load_scales(step + 1);
    load_b(B, step + 1);
    store_a(A0, buf ^ 1);
    multiply(buf);
    __syncthreads();
    ++step;
  }
  unpack(B, step);
  multiply(step & 1);

  // D element i of lane (n, kb) belongs to token 16*t4 + 4*kb + i and row n of the stream. The factor of the
  // subnormal code fields (2^24) and the one that undoes the normalisation of the token's activations are
  // applied here, in that order.
  float upt[4][4];
#pragma unroll
  for (int t4 = 0; t4 < 4; ++t4)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int tok = min(16 * t4 + 4 * kb + i, ntok - 1);
      upt[t4][i] = ((const float*)(G.A + (size_t)(g0 + tok) * G.a_pair_words + K / 2))[K / 64];
    }
  if constexpr (PHASE == 0) {
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) {
      const int row = R0 + rb * 16 + n;
#pragma unroll
      for (int t4 = 0; t4 < 4; ++t4)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int tok = 16 * t4 + 4 * kb + i;
          if (tok < ntok && row < N) {
            float v;
            const float a = acc[rb][t4][i] * 16777216.0f * upt[t4][i];
            if constexpr (NM == 2) v = a / (1.0f + __expf(-a)) * (acc[RBW + rb][t4][i] * 16777216.0f * upt[t4][i]);
            else v = fmaxf(a, 0.f);
            G.Hf[(size_t)(g0 + tok) * N + row] = v;
          }
        }
    }
  } else {
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int row = R0 + s * 16 + n;
#pragma unroll
      for (int t4 = 0; t4 < 4; ++t4)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int tok = 16 * t4 + 4 * kb + i;
          if (tok < ntok && row < N) G.Y[(size_t)(g0 + tok) * N + row] = acc[s][t4][i] * 16777216.0f * upt[t4][i];
        }
    }
  }
}

template <int NM, int PHASE, bool COLS = false>
__global__ __launch_bounds__(kGemmThreads) void k_gemm_q(GemmArgs G) {
  __shared__ uint4 As[2 * 4 * 4 * 65];
  __shared__ float Ks[2 * kTB];
  if ((int)blockIdx.y >= *G.n_blocks) return;
  const int2 blk = G.blocks[blockIdx.y];
  const DevExpert ex = G.table[blk.x];
  switch (ex.bits) {
    case 2: gemm_body<2, NM, PHASE, COLS>(G, ex, blk.x, blk.y, As, Ks); break;
    case 4: gemm_body<4, NM, PHASE, COLS>(G, ex, blk.x, blk.y, As, Ks); break;
    default: gemm_body<8, NM, PHASE, COLS>(G, ex, blk.x, blk.y, As, Ks); break;
  }
}

// y[t][r] = sum_j gate[t][j] * Ypair[ginv[t*k + j]][r], j in top-k order
__global__ __launch_bounds__(256) void k_combine(const float* __restrict__ Ypair, const int32_t* __restrict__ ginv,
                                                 const float* __restrict__ gate, int k, int d, float* __restrict__ y) {
  const int t = blockIdx.x;
  for (int r = threadIdx.x * 4; r < d; r += blockDim.x * 4) {
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int j = 0; j < k; ++j) {
      const float g = gate[(size_t)t * k + j];
      const float4 v = *(const float4*)(Ypair + (size_t)ginv[(size_t)t * k + j] * d + r);
      a.x = fmaf(g, v.x, a.x); a.y = fmaf(g, v.y, a.y); a.z = fmaf(g, v.z, a.z); a.w = fmaf(g, v.w, a.w);
    }
    *(float4*)(y + (size_t)t * d + r) = a;
  }
}

inline size_t up256(size_t v) { return (v + 255) / 256 * 256; }

}  // namespace

bool prefill_supported(const LayerDims& L) {
  return L.group % 128 == 0 && L.group_out % 128 == 0 && L.d_model % 256 == 0 && L.d_ff % 256 == 0 &&
         (L.d_model / L.group) % 4 == 0 && (L.d_ff / L.group_out) % 4 == 0 && L.d_model <= 16384 &&
         L.d_ff <= 32768 && L.n_experts <= 1024;
}

hipError_t init_attrs_prefill() {
  // the staging kernels keep one activation vector (up to 32768 values) in LDS
  const int lds = 32768 * 2 + 32768 / 16 * 4 + 64;
  if (hipError_t e = hipFuncSetAttribute((const void*)k_stage<false>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
      e != hipSuccess)
    return e;
  return hipFuncSetAttribute((const void*)k_stage<true>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
}

PrefillWs prefill_ws(const LayerDims& L, int64_t T) {
  PrefillWs w{};
  const size_t M = (size_t)T * L.top_k;
  const size_t max_blocks = M / kTB + (size_t)L.n_experts;
  w.a_pair_words = (size_t)L.d_model / 2 + (size_t)L.d_model / 64 + 4;
  w.h_pair_words = (size_t)L.d_ff / 2 + (size_t)L.d_ff / 64 + 4;
  size_t off = 0;
  w.poff = off;    off += up256(((size_t)L.n_experts + 1) * 4);
  w.nblk = off;    off += 256;
  w.blocks = off;  off += up256(max_blocks * 8);
  w.gpair = off;   off += up256(M * 4);
  w.ginv = off;    off += up256(M * 4);
  w.gexp = off;    off += up256(M * 4);
  w.xa = off;      off += up256(M * w.a_pair_words * 4);
  w.ha = off;      off += up256(M * w.h_pair_words * 4);
  w.hf = off;      off += up256(M * (size_t)L.d_ff * 4);
  w.ypair = off;   off += up256(M * (size_t)L.d_model * 4);
  w.total = off;
  w.max_blocks = max_blocks;
  return w;
}

hipError_t launch_prefill(const LayerDims& L, const DevExpert* table, const void* x, int32_t T, const int32_t* idx,
                          const float* gate, char* ws, const PrefillWs& w, float* y, bool out_columns,
                          hipStream_t st) {
  const int M = T * L.top_k;
  int32_t* poff = (int32_t*)(ws + w.poff);
  int32_t* nblk = (int32_t*)(ws + w.nblk);
  int2* blocks = (int2*)(ws + w.blocks);
  int32_t* gpair = (int32_t*)(ws + w.gpair);
  int32_t* ginv = (int32_t*)(ws + w.ginv);
  int32_t* gexp = (int32_t*)(ws + w.gexp);
  uint32_t* XA = (uint32_t*)(ws + w.xa);
  uint32_t* HA = (uint32_t*)(ws + w.ha);
  float* Ypair = (float*)(ws + w.ypair);
  hipLaunchKernelGGL(k_count_pairs, dim3(1), dim3(1024), 0, st, idx, M, L.n_experts, poff, blocks, nblk);
  hipLaunchKernelGGL(k_scatter_pairs, dim3(L.n_experts), dim3(256), 0, st, idx, M, poff, gpair, ginv, gexp);
  float* Hf = (float*)(ws + w.hf);
  auto stage_lds = [](int cols) { return (size_t)cols * 2 + (size_t)cols / 16 * 4 + 64; };
  hipLaunchKernelGGL(k_stage<false>, dim3(M), dim3(256), stage_lds(L.d_model), st, L, table, x, gpair, gexp, XA,
                     (int64_t)w.a_pair_words);
  GemmArgs G{L, table, blocks, nblk, poff, XA, (int64_t)w.a_pair_words, Hf, Ypair};
  const unsigned nb = (unsigned)w.max_blocks;
  if (L.act == MOEQ_ACT_SWIGLU)
    hipLaunchKernelGGL((k_gemm_q<2, 0>), dim3((L.d_ff + kGemmWaves * 32 - 1) / (kGemmWaves * 32), nb), dim3(kGemmThreads), 0, st, G);
  else
    hipLaunchKernelGGL((k_gemm_q<1, 0>), dim3((L.d_ff + kGemmWaves * 64 - 1) / (kGemmWaves * 64), nb), dim3(kGemmThreads), 0, st, G);
  hipLaunchKernelGGL(k_stage<true>, dim3(M), dim3(256), stage_lds(L.d_ff), st, L, table, (const void*)Hf, gpair, gexp, HA,
                     (int64_t)w.h_pair_words);
  G.A = HA;
  G.a_pair_words = (int64_t)w.h_pair_words;
  const dim3 grid2((L.d_model + kGemmWaves * 32 - 1) / (kGemmWaves * 32), nb);
  if (out_columns) hipLaunchKernelGGL((k_gemm_q<1, 1, true>), grid2, dim3(kGemmThreads), 0, st, G);
  else hipLaunchKernelGGL((k_gemm_q<1, 1, false>), grid2, dim3(kGemmThreads), 0, st, G);
  hipLaunchKernelGGL(k_combine, dim3(T), dim3(256), 0, st, Ypair, ginv, gate, L.top_k, L.d_model, y);
  return hipGetLastError();
}

}  // namespace moeq
