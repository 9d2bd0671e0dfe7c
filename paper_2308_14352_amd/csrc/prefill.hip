// Batched (prefill) path of the MoE layer: the (token, choice) pairs are grouped by expert and every
// expert's FFN runs as two GEMMs on the matrix cores over its own tokens (Section 2.1: only the chosen
// experts work on a token; Section 3.2: their weights are decompressed by the mirror of the linear
// quantization before use - here inside the GEMM, on the way from the packed tile to the instruction).
//
//   grouping : histogram of the pairs per expert, offsets, a list of (expert, block of 128 tokens) work
//              items, a stable scatter of the pairs into expert order (and its inverse)
//   staging  : per 64 tokens of an expert (a token tile), the tokens' activations - each normalised by a power
//              of two of its own - as binary16 in the pair order of the expert's bitwidth (the order codes8
//              produces), laid out as the 1 KB lines (64 tokens x 16 bytes) the GEMM's LDS tiles are made of,
//              plus the offset term of every (token, K step) and the tokens' factors 2^e
//   GEMM 1   : H[pair][row] = act(W_in x [, W_gate x]) (fp32) for 128 tokens x 128 or 256 rows per workgroup
//   staging  : the same for every pair's h
//   GEMM 2   : Ypair[pair][row] = W_out h for 128 tokens x 128 rows per workgroup
//   combine  : y[t] = sum_j gate[t][j] * Ypair[pair(t, j)], in top-k order
//
// The GEMMs never form floating-point weights: a wavefront takes 16-byte pieces of packed rows, masks
// the code fields into binary16 subnormals (codes8) and feeds them to v_mfma_f32_16x16x32_f16 as the B
// operand; the A operand (activations pre-divided by the fields' powers of two) comes from LDS. One K
// step (128 columns, 64 at 8 bits) lies inside one scale group, so the group scale and the code offset
// are applied to the step's partial product: acc += s * (D - 2^(b-1) * sum(x_step)).
//
// Every operand of the main loop travels HBM -> LDS directly (global_load_lds: no registers in between), into
// rings of two or three stages, so that the loads of the next steps are in flight while a step is multiplied; the loop
// holds no other memory instruction, and its waits are the hand-written s_waitcnt of stage_wait.
#include "decode_core.h"

namespace moeq {
namespace {

constexpr int kTB = 64;        // tokens per staged tile
constexpr int kItemTiles = 2;  // token tiles per GEMM work item (128 tokens)
// Wavefronts of a GEMM workgroup (template parameter WV): 16 (four per SIMD, two streams per wavefront: 123 registers),
// or 8 with two per SIMD (GEMM 2 on a W_out in columns, whose gathers need more registers). Wavefront = (token tile,
// row group); WV / kItemTiles row groups.
__host__ __device__ constexpr int gemm_streams(int phase, int wv) { return (phase == 1 || wv == 16) ? 2 : 4; }

#define MOEQ_LDS __attribute__((address_space(3)))

// Staged operand of one GEMM (x for GEMM 1, h for GEMM 2; K = its length), per token tile (64 tokens of an expert):
//   [K / 128 tiles of 16 KB]  tile = the 1 KB lines of one 128-column range: line (q, kb) holds, for each of the
//                             64 tokens, the 16 bytes that are A operand q of k block kb (at 8 bits a K step is
//                             64 columns = 8 lines: two steps per tile)
//   [K / 64 x 64 floats]      the negated offset term of every (K step, token)
//   [64 floats]               2^e of every token (undoes its normalisation)
struct Staged { size_t ks_off, up_off, block_bytes; };
__host__ __device__ inline Staged staged_layout(int K) {
  Staged s;
  s.ks_off = (size_t)K * 128;
  s.up_off = s.ks_off + (size_t)(K / 64) * 256;
  s.block_bytes = s.up_off + 256;
  return s;
}

// ---------------------------------------------------------------------------------------------
// grouping
__global__ __launch_bounds__(1024) void k_count_pairs(const int32_t* __restrict__ idx, int M, int E,
                                                      int32_t* __restrict__ poff, int32_t* __restrict__ boff,
                                                      int2* __restrict__ blocks, int32_t* __restrict__ n_blocks) {
  __shared__ int h[1024];
  for (int e = threadIdx.x; e < E; e += blockDim.x) h[e] = 0;
  __syncthreads();
  for (int p = threadIdx.x; p < M; p += blockDim.x) atomicAdd(&h[min(max(idx[p], 0), E - 1)], 1);
  __syncthreads();
  if (threadIdx.x == 0) {
    int off = 0, nb = 0, nt = 0;
    for (int e = 0; e < E; ++e) {
      poff[e] = off;
      boff[e] = nt;                 // token tile tb of expert e is tile number boff[e] + tb
      const int c = h[e];
      for (int tb = 0; tb * (kTB * kItemTiles) < c; ++tb) blocks[nb++] = make_int2(e, tb);
      nt += (c + kTB - 1) / kTB;
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
// Staging of the activation vector of one pair for a GEMM, into the tiles of its work item (see Staged).
// FROM_H = false: the pair's token row of x (GEMM 1); true: row g of the fp32 h that GEMM 1 wrote (GEMM 2).
// The vector is normalised by its own power of two before the conversion to binary16 (stage_normalised).

// 16-byte item i of the pair order of a vector (permute_x) -> its place in the work item's tiles, for token t:
// item i is A operand q of k block kb of K step `step`; line = 4 q + kb; a K step has NQ * 4 lines of 64 x 16 bytes.
template <int BITS>
struct TilePlace {
  int C, t;
  __device__ __forceinline__ int operator()(int i) const {
    constexpr int NQ = BITS == 8 ? 2 : 4;
    const int r = i / C, c = i - r * C;
    int step, q, kb;
    if (BITS == 2) {          // item (2 (2 (kb & 1) + (q >> 1)) + (q & 1)) * C + 2 step + (kb >> 1)
      step = c >> 1;
      kb = (c & 1) * 2 + (r >> 2);
      q = ((r >> 1) & 1) * 2 + (r & 1);
    } else {                  // item q * C + 4 step + kb
      step = c >> 2;
      kb = c & 3;
      q = r;
    }
    return (step * (NQ * 4) + q * 4 + kb) * 64 + t;
  }
};

template <bool FROM_H>
__global__ __launch_bounds__(256) void k_stage(LayerDims L, const DevExpert* __restrict__ table,
                                               const void* __restrict__ src, const int32_t* __restrict__ gpair,
                                               const int32_t* __restrict__ gexp, const int32_t* __restrict__ poff,
                                               const int32_t* __restrict__ boff, char* __restrict__ OUT, int M) {
  extern __shared__ uint32_t smem[];
  __shared__ float red[4];
  const int cols = FROM_H ? L.d_ff : L.d_model;
  uint16_t* RAW = (uint16_t*)smem;
  // consecutive pairs go to workgroups on the same XCD (workgroup i runs on XCD i % 8), so that the 16-byte pieces
  // eight neighbouring tokens write into one 128-byte line meet in one L2
  const int per = ((int)gridDim.x + 7) / 8;
  const int g = ((int)blockIdx.x & 7) * per + ((int)blockIdx.x >> 3);
  if (g >= M) return;
  const int e = gexp[g];
  const int bits = table[e].bits;
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
  const Staged lay = staged_layout(cols);
  const int rank = g - poff[e];
  const int t = rank & (kTB - 1);
  char* blk = OUT + (size_t)(boff[e] + rank / kTB) * lay.block_bytes;
  uint32_t* XP = (uint32_t*)blk;
  float* KS = (float*)(blk + lay.ks_off) + t;
  float* scratch = (float*)(smem + cols / 2);     // the per-chunk offset terms permute_x also makes; not kept
  const int group = FROM_H ? L.group_out : L.group;
  const int tid = threadIdx.x, nt = blockDim.x;
  if (bits == 2) {
    permute_x<2>(RAW, cols, group, tid, nt, XP, scratch, TilePlace<2>{cols / 64, t});
    range_offset_terms<2>(RAW, cols, tid, nt, KS, kTB);
  } else if (bits == 4) {
    permute_x<4>(RAW, cols, group, tid, nt, XP, scratch, TilePlace<4>{cols / 32, t});
    range_offset_terms<4>(RAW, cols, tid, nt, KS, kTB);
  } else {
    permute_x<8>(RAW, cols, group, tid, nt, XP, scratch, TilePlace<8>{cols / 16, t});
    range_offset_terms<8>(RAW, cols, tid, nt, KS, kTB);
  }
  if (threadIdx.x == 0) ((float*)(blk + lay.up_off))[t] = up;
}

// ---------------------------------------------------------------------------------------------
// The quantized GEMM. Workgroup = 8 wavefronts = 128 tokens (two token tiles) x 4 row groups; wavefront
// (tile th, row group rg) multiplies the 64 tokens of its tile with the NS streams of its row group; a stream is
// (matrix, block of 16 rows): NS = 2 per row group with 16 wavefronts (with two matrices a row group is 16 rows of
// both), NS = 4 with 8. The two wavefronts of a row group share its packed pieces (each requests half of the streams), so
// a weight byte comes from memory once per 128 tokens. Lane (n, kb) takes, per K step, the 16-byte piece
// 4*step + kb of row n of each stream (8 bytes at 2 bits): four k blocks along one scale group.
struct GemmArgs {
  LayerDims L;
  const DevExpert* table;
  const int2* blocks;
  const int32_t* n_blocks;
  const int32_t* poff;
  const int32_t* boff;      // first token tile of every expert
  const char* A;            // staged activations of every token tile (Staged)
  float* Hf;                // GEMM 1 out: h per pair, fp32 [pairs][d_ff]
  float* Y;                 // GEMM 2 out: [pairs][d_model]
};

// Direct HBM -> LDS loads: lane l's 16 (4) bytes land at lds_base + 16 l (4 l); lds_base (an LDS byte address) is
// wave-uniform and goes through M0. They are issued through asm statements: the compiler's wait-count pass would
// otherwise make every later LDS read wait for all of them, which would serialise the ring. stage_wait states how
// many of the wavefront's youngest loads may still be in flight. (M0 is a register the compiler reserves and never
// keeps a value in across other code in these kernels, which use it nowhere else.)
__device__ __forceinline__ void dma16(const uint8_t* g, uint32_t lds_base) {
  const uint32_t base = __builtin_amdgcn_readfirstlane(lds_base);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(g), "s"(base) : "memory");
}
__device__ __forceinline__ void dma4(const uint8_t* g, uint32_t lds_base) {
  const uint32_t base = __builtin_amdgcn_readfirstlane(lds_base);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" : : "v"(g), "s"(base) : "memory");
}
template <int N>
__device__ __forceinline__ void stage_wait() {
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

// COLS: GEMM 2 on a W_out in the dword-column-major layout. SIN: GEMM 1 on W_in / W_gate in the row-block stream
// layout (blocks of RB = 16 / bits rows: 8 tiles of 1 KB, then 64 * RB bytes of scales; 16-byte piece c of row r is
// piece c / TPR of tile (r % RB) * TPR + c % TPR of block r / RB, TPR = bits / 2).
template <int BITS, int NM, int PHASE, bool COLS, int WV, bool SIN>
__device__ __forceinline__ void gemm_body(const GemmArgs& G, const DevExpert& ex, int e, int tb, int rb, char* smem) {
  constexpr int SC = 128;                         // columns per K step: one scale group (or a part of one)
  constexpr int NQ = 4;                           // instructions per step, stream and token block
  // at 8 bits a step is two half steps of 64 columns (the unit of the staged tiles and of the pair order): each
  // has its own lines, offset terms and 16-byte pieces, both accumulate into the same results
  constexpr int NH = BITS == 8 ? 2 : 1;
  // ring depth: the stage being multiplied + those in flight. A step at 8 bits moves twice the bytes per stream,
  // so two stages of it take the LDS that three stages take otherwise.
  constexpr int STAGES = BITS == 8 ? 2 : 3;
  constexpr int AHEAD = STAGES - 1;
  // streams (row blocks of 16 rows) per row group: two with 16 wavefronts per workgroup, four with 8
  constexpr int NS = gemm_streams(PHASE, WV);
  constexpr int HS = NS / kItemTiles;             // streams whose pieces one wavefront of the pair requests
  constexpr int RBW = NS / NM;                    // row blocks per row group and matrix
  constexpr int kRowGroups = WV / kItemTiles;
  constexpr int kGemmWaves = WV;
  constexpr int BN = kRowGroups * RBW * 16;       // rows per workgroup
  constexpr int LINES = NQ * 4;                   // 1 KB lines of a token tile's A stage
  constexpr int A_TILE = LINES * 1024 + NH * 256; // + the 64 offset terms of the step (of each half step)
  constexpr int A_STAGE = kItemTiles * A_TILE;
  constexpr int B_STREAM = NH * 1024;             // a stream's pieces of a step (2-bit codes use half of it)
  constexpr int B_STAGE = NS * B_STREAM;          // per row group
  constexpr int NSCW = (COLS || SIN) ? 4 : 2;     // dwords of a row's scale block (four groups)
  constexpr int SC_SLOT = NS * NSCW * 64;         // per row group: NSCW areas of 16 dwords per stream
  // loads a wavefront issues per stage, counted by stage_wait: its half of the row group's pieces + its lines
  // of the two A tiles
  constexpr int B_OPS = HS * (BITS == 2 ? 2 : (COLS ? 4 * NH : NH));
  constexpr int A_OPS = kItemTiles * LINES / kGemmWaves;
  constexpr int OPS = B_OPS + A_OPS;
  const int K = PHASE == 0 ? G.L.d_model : G.L.d_ff;
  const int N = PHASE == 0 ? G.L.d_ff : G.L.d_model;
  const int group = PHASE == 0 ? G.L.group : G.L.group_out;
  const int n_steps = K / SC;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int th = wave / kRowGroups, rg = wave % kRowGroups;
  const int n = lane & 15, kb = lane >> 4;
  const int g0 = G.poff[e] + (tb * kItemTiles + th) * kTB;       // first pair of this wavefront's token tile
  const int ntok = min(kTB, G.poff[e + 1] - g0);                 // <= 0: the work item's second tile does not exist
  const int R0 = rb * BN + rg * (RBW * 16);
  const uint32_t row_bytes = (uint32_t)(K / (128 / BITS)) * 16u;
  const uint32_t ng2 = (uint32_t)(K / group) * 2u;
  const Staged lay = staged_layout(K);
  // the work item's token tiles are consecutive; the tile behind an expert's last one belongs to the next expert
  // (or is the spare tile at the end of the buffer): it is loaded like the others and its results are dropped
  const uint8_t* Aitem = (const uint8_t*)G.A + (size_t)(G.boff[e] + tb * kItemTiles) * lay.block_bytes;

  // LDS: [A ring: stages x two tiles][B ring of every row group][scale blocks of every row group, two slots]
  const uint32_t lds0 = (uint32_t)(uintptr_t)(MOEQ_LDS char*)smem;
  char* const Aring = smem;
  char* const Bring = smem + STAGES * A_STAGE + rg * (STAGES * B_STAGE);
  char* const Sring = smem + STAGES * A_STAGE + kRowGroups * (STAGES * B_STAGE) + rg * (2 * SC_SLOT);
  const uint32_t a_lds = lds0, b_lds = lds0 + (uint32_t)(Bring - smem), s_lds = lds0 + (uint32_t)(Sring - smem);

  const uint8_t* qs[NM];
  const uint8_t* ss[NM];
  if (PHASE == 0) {
    qs[0] = ex.q_in; ss[0] = SIN ? ex.q_in : (const uint8_t*)ex.s_in;
    if (NM == 2) { qs[NM - 1] = ex.q_gate; ss[NM - 1] = SIN ? ex.q_gate : (const uint8_t*)ex.s_gate; }
  } else {
    qs[0] = ex.q_out; ss[0] = (const uint8_t*)ex.s_out;
  }
  // the streams this wavefront requests: s = th * HS + i
  constexpr uint32_t RB = 16 / BITS, TPR = BITS / 2, BB = 8192u + 64u * RB;   // stream layout: rows, tiles per row, bytes of a block
  // scale of group g of row r: COLS the binary16 value g * N + r (fetched as the dword of rows r & ~1, r | 1); SIN
  // value (r % RB) % (RB / 2) of lane 2 g + ((r % RB) >= RB / 2) of its block's scale area (RB bytes per lane),
  // fetched as the dword around it; sgrp = bytes from a group's dword to the next group's
  const uint32_t sgrp = COLS ? (uint32_t)N * 2u : (SIN ? 2u * RB : 0u);
  auto scale_half = [&](uint32_t row) __attribute__((always_inline)) {       // which half of the fetched dword
    if (COLS) return (row & 1u) * 16u;
    if (SIN) { const uint32_t rr = row % RB; return (BITS == 8 ? rr : (rr % (RB / 2)) & 1u) * 16u; }
    return 0u;
  };
  uint32_t qrow[HS], srow[HS];
#pragma unroll
  for (int i = 0; i < HS; ++i) {
    const int s = th * HS + i;
    const uint32_t row = (uint32_t)min(R0 + (s % RBW) * 16 + n, N - 1);
    if (SIN) {
      const uint32_t blk = row / RB, rr = row % RB, hi2 = rr >= RB / 2 ? 1u : 0u, ii = rr % (RB / 2 ? RB / 2 : 1);
      // the lane's piece of (half) step 0: 4 bits: tile part kb & 1, piece kb >> 1; 8 bits: tile part kb, piece 0;
      // 2 bits: the 8 bytes kb of the row's first 32
      const uint32_t koff = BITS == 4 ? (uint32_t)(kb & 1) * 1024u + (uint32_t)(kb >> 1) * 16u
                          : (BITS == 8 ? (uint32_t)kb * 1024u : (uint32_t)kb * 8u);
      qrow[i] = blk * BB + rr * TPR * 1024u + koff;
      srow[i] = blk * BB + 8192u + (BITS == 8 ? 0u : hi2 * RB + (ii >> 1) * 4u);
    } else {
      // COLS: word w of row r is the 32-bit word w * N + r
      qrow[i] = COLS ? row * 4u : row * row_bytes + (uint32_t)kb * (BITS == 2 ? 8u : 16u);
      srow[i] = COLS ? (row & ~1u) * 2u : row * ng2;
    }
  }
  // bytes from the lane's piece of one (half) step to that of the next
  constexpr uint32_t hstep = SIN ? (BITS == 8 ? 16u : 32u) : (BITS == 2 ? 32u : 64u);
  uint32_t rodd[NS];        // which half of a fetched scale dword is row n of stream s
#pragma unroll
  for (int s = 0; s < NS; ++s) rodd[s] = scale_half((uint32_t)min(R0 + (s % RBW) * 16 + n, N - 1));
  // The scales of a stream's row for four consecutive groups (8 contiguous bytes in the canonical layout; the
  // plan makes rows of scales multiples of 8 bytes), fetched once per block of blk_steps = 4 * group / SC steps
  // by the sixteen lanes with kb = 0 into slot (block & 1).
  const int blk_steps = 4 * group / SC;
  auto issue_scales = [&](int step) __attribute__((always_inline)) {
    const uint32_t gi = ((uint32_t)step * (uint32_t)SC) / (uint32_t)group;     // a multiple of 4 here
    const uint32_t slot = s_lds + (uint32_t)((step / blk_steps) & 1) * (uint32_t)SC_SLOT;
    if (kb == 0) {
#pragma unroll
      for (int i = 0; i < HS; ++i) {
        const int s = th * HS + i;
        const uint8_t* sb = ss[s / RBW];
#pragma unroll
        for (int j = 0; j < NSCW; ++j) {
          const uint8_t* sp = (COLS || SIN) ? sb + ((gi + (uint32_t)j) * sgrp + srow[i])
                                            : sb + (srow[i] + gi * 2u + (uint32_t)j * 4u);
          dma4(sp, slot + (uint32_t)((s * NSCW + j) * 64));
        }
      }
    }
  };
  // One stage = the pieces of the row group's streams for a K step (half of them from this wavefront) + this
  // wavefront's share of the lines of the two A tiles.
  auto issue_stage = [&](int step) __attribute__((always_inline)) {
    const int st = step % STAGES;
    if (wave >= kGemmWaves - kItemTiles) {     // the step's offset terms, first (stage_wait counts the youngest loads)
      const int tile = wave - (kGemmWaves - kItemTiles);
      if (lane < 16 * NH)
        dma16(Aitem + (size_t)tile * lay.block_bytes + lay.ks_off + (size_t)step * (NH * 256) + (size_t)lane * 16,
              a_lds + (uint32_t)(st * A_STAGE + tile * A_TILE + LINES * 1024));
    }
    const uint32_t bst = b_lds + (uint32_t)(st * B_STAGE);
#pragma unroll
    for (int i = 0; i < HS; ++i) {
      const int s = th * HS + i;
      const uint8_t* q = qs[s / RBW];
      if constexpr (COLS) {
        const uint32_t col_bytes = (uint32_t)N * 4u;
        constexpr int NW = BITS == 2 ? 2 : 4;
#pragma unroll
        for (int h = 0; h < NH; ++h) {
          const uint32_t w0 = (((uint32_t)step * NH + h) * 4u + (uint32_t)kb) * (uint32_t)NW;
#pragma unroll
          for (int j = 0; j < NW; ++j)
            dma4(q + ((w0 + (uint32_t)j) * col_bytes + qrow[i]), bst + (uint32_t)(s * B_STREAM + h * 1024 + j * 256));
        }
      } else if constexpr (BITS == 2) {
        const uint8_t* p = q + (qrow[i] + (uint32_t)step * hstep);
        dma4(p, bst + (uint32_t)(s * B_STREAM));
        dma4(p + 4, bst + (uint32_t)(s * B_STREAM + 256));
      } else {
#pragma unroll
        for (int h = 0; h < NH; ++h)
          dma16(q + (qrow[i] + ((uint32_t)step * NH + h) * hstep), bst + (uint32_t)(s * B_STREAM + h * 1024));
      }
    }
#pragma unroll
    for (int r = 0; r < A_OPS; ++r) {
      const int l2 = wave * A_OPS + r;                 // line of the stage: (tile, line)
      const int tile = l2 / LINES, line = l2 % LINES;
      dma16(Aitem + (size_t)tile * lay.block_bytes + (size_t)step * (LINES * 1024) + line * 1024 + lane * 16,
            a_lds + (uint32_t)(st * A_STAGE + tile * A_TILE + line * 1024));
    }
  };

  float4_t acc[NS][4];
  const float4_t zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < NS; ++s)
#pragma unroll
    for (int t4 = 0; t4 < 4; ++t4) acc[s][t4] = zero;

  half8_t Bop[NS][NQ];
  float sc[NS];
  auto unpack = [&](int step) __attribute__((always_inline)) {
    const char* bst = Bring + (step % STAGES) * B_STAGE;
    const uint32_t gi = ((uint32_t)step * (uint32_t)SC) / (uint32_t)group;
    const char* slot = Sring + ((step / blk_steps) & 1) * SC_SLOT;
    auto piece = [&](int s, int h) __attribute__((always_inline)) {
      const char* b = bst + s * B_STREAM + h * 1024;
      uint4 t;
      if constexpr (COLS) {
        t.x = *(const uint32_t*)(b + lane * 4); t.y = *(const uint32_t*)(b + 256 + lane * 4);
        t.z = *(const uint32_t*)(b + 512 + lane * 4); t.w = *(const uint32_t*)(b + 768 + lane * 4);
      } else {
        t = *(const uint4*)(b + lane * 16);
      }
      return t;
    };
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      if constexpr (BITS == 2) {
        const uint32_t x = *(const uint32_t*)(bst + s * B_STREAM + lane * 4), y = *(const uint32_t*)(bst + s * B_STREAM + 256 + lane * 4);
        Bop[s][0] = codes8<2, 0>(x, 0u); Bop[s][1] = codes8<2, 1>(x, 0u);
        Bop[s][2] = codes8<2, 0>(y, 0u); Bop[s][3] = codes8<2, 1>(y, 0u);
      } else if constexpr (BITS == 4) {
        const uint4 t = piece(s, 0);
        Bop[s][0] = codes8<4, 0>(t.x, 0u); Bop[s][1] = codes8<4, 0>(t.y, 0u);
        Bop[s][2] = codes8<4, 0>(t.z, 0u); Bop[s][3] = codes8<4, 0>(t.w, 0u);
      } else {
        const uint4 t0 = piece(s, 0), t1 = piece(s, 1);
        Bop[s][0] = codes8<8, 0>(t0.x, t0.y); Bop[s][1] = codes8<8, 0>(t0.z, t0.w);
        Bop[s][2] = codes8<8, 0>(t1.x, t1.y); Bop[s][3] = codes8<8, 0>(t1.z, t1.w);
      }
      // the step's scale among the four of the block
      uint32_t w;
      if constexpr (COLS || SIN) w = *(const uint32_t*)(slot + (s * NSCW + (int)(gi & 3u)) * 64 + n * 4) >> rodd[s];
      else w = *(const uint32_t*)(slot + (s * NSCW + (int)((gi >> 1) & 1u)) * 64 + n * 4) >> ((gi & 1u) * 16u);
      sc[s] = f16_bits_to_f32(w);   // (the conversion takes the low 16 bits)
    }
  };
  // The A operands of a step are read from LDS two instruction groups ahead of the matrix-core instructions
  // that use them (three register slots): the latency of a read is covered by the eight to sixteen
  // instructions in between instead of being waited for in front of every group.
  constexpr int NI = 4 * NQ;                      // (token block, q) items of a step
  // two result sets where the registers allow it (not for GEMM 1 with one matrix: it would spill)
  constexpr bool DBL = NM == 2 || PHASE == 1;
  auto multiply = [&](int st) __attribute__((always_inline)) {
    const uint4* As = (const uint4*)(Aring + st * A_STAGE + th * A_TILE);
    const float* Ks = (const float*)(Aring + st * A_STAGE + th * A_TILE + LINES * 1024);
    auto read_a = [&](int idx) __attribute__((always_inline)) {
      // operand q of the step: at 8 bits operand q & 1 of half step q >> 1 (a half step's lines are 8 in a row)
      const int q = idx % NQ, line = BITS == 8 ? (q >> 1) * 8 + (q & 1) * 4 + kb : q * 4 + kb;
      return As[line * 64 + 16 * (idx / NQ) + n];
    };
    auto read_k = [&](int t4) __attribute__((always_inline)) {
      // the accumulation starts at the negated offset terms of the lane's four tokens (of both half steps)
      const float4 k4 = *(const float4*)(Ks + 16 * t4 + 4 * kb);
      float4_t kv = {k4.x, k4.y, k4.z, k4.w};
      if constexpr (NH == 2) {
        const float4 k5 = *(const float4*)(Ks + 64 + 16 * t4 + 4 * kb);
        kv += (float4_t){k5.x, k5.y, k5.z, k5.w};
      }
      return kv;
    };
    uint4 af[3];
    af[0] = read_a(0);
    af[1] = read_a(1);
    float4_t kv = read_k(0);
    // two sets of results: the scaling of a token block's results waits for its last matrix-core
    // instructions, so it is issued behind the first instructions of the next token block
    float4_t D[2][NS];
#pragma unroll
    for (int idx = 0; idx < NI; ++idx) {
      const int t4 = idx / NQ, q = idx % NQ, d = DBL ? (t4 & 1) : 0;
      if (idx + 2 < NI) af[(idx + 2) % 3] = read_a(idx + 2);
      if (q == 0) {
#pragma unroll
        for (int s = 0; s < NS; ++s) D[d][s] = kv;
        if (t4 + 1 < 4) kv = read_k(t4 + 1);
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

  // Stage s + AHEAD is requested at the start of step s, into the ring slot that step s - 1 read: every wavefront
  // is past the barrier of step s by then, so nobody reads that slot any more. At the top of step s a wavefront waits
  // until only the loads of the stages behind s (its youngest (AHEAD - 1) * OPS) are still in flight, which means
  // its own parts of stage s have landed; the barrier then says the same of every wavefront's part of the shared
  // tiles. Scale blocks are requested in front of the first stage that uses them, so they are older than that
  // stage's loads.
  issue_scales(0);
#pragma unroll
  for (int i = 0; i < AHEAD; ++i)
    if (i < n_steps) issue_stage(i);
  for (int step = 0; step < n_steps; ++step) {
    if (AHEAD == 2 && step + 1 < n_steps) stage_wait<OPS>();
    else stage_wait<0>();
    __syncthreads();
    if (step + AHEAD < n_steps) {
      if ((step + AHEAD) % blk_steps == 0) issue_scales(step + AHEAD);
      issue_stage(step + AHEAD);
    }
    if (ntok > 0) {                 // (a wavefront without tokens still requests its share and keeps the barriers)
      unpack(step);
      multiply(step % STAGES);
    }
  }
  if (ntok <= 0) return;

  // D element i of lane (n, kb) belongs to token 16*t4 + 4*kb + i and row n of the stream. The factor of the
  // subnormal code fields (2^24) and the one that undoes the normalisation of the token's activations are
  // applied here, in that order.
  const float* UP = (const float*)(Aitem + (size_t)th * lay.block_bytes + lay.up_off);
  float upt[4][4];
#pragma unroll
  for (int t4 = 0; t4 < 4; ++t4)
#pragma unroll
    for (int i = 0; i < 4; ++i) upt[t4][i] = UP[min(16 * t4 + 4 * kb + i, ntok - 1)];
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

// LDS of a GEMM workgroup: the largest carve over the bitwidths
template <int PHASE, bool WIDE, int WV>      // WIDE: four dwords per row and scale block (columns and stream layouts)
constexpr int gemm_lds_bytes() {
  constexpr int NS = gemm_streams(PHASE, WV);
  constexpr int RG = WV / kItemTiles;
  constexpr int scales = RG * 2 * NS * (WIDE ? 4 : 2) * 64;
  constexpr int b24 = 3 * kItemTiles * (16 * 1024 + 256) + RG * 3 * NS * 1024 + scales;    // 2 and 4 bits
  constexpr int b8 = 2 * kItemTiles * (16 * 1024 + 512) + RG * 2 * NS * 2048 + scales;     // 8 bits
  return b24 > b8 ? b24 : b8;
}
// rows of the GEMM's output a workgroup covers
template <int NM, int PHASE, int WV>
constexpr int gemm_rows() { return (WV / kItemTiles) * (gemm_streams(PHASE, WV) / NM) * 16; }

// Grid: one dimension, n_rb * (upper bound of the work items) workgroups, n_rb = row blocks of the GEMM; the row
// blocks of a work item are consecutive workgroups (they share the item's activation tiles in the L2s).
template <int NM, int PHASE, bool COLS, int WV, bool SIN = false>
__global__ __launch_bounds__(WV * 64) void k_gemm_q(GemmArgs G, int n_rb) {
  extern __shared__ __attribute__((aligned(16))) char gsmem[];
  const int it0 = (int)blockIdx.x / n_rb;
  if (it0 >= *G.n_blocks) return;
  const int2 blk0 = G.blocks[it0];
  const int e = blk0.x, tb = blk0.y;
  const int rb = (int)blockIdx.x - it0 * n_rb;
  const DevExpert ex = G.table[e];
  switch (ex.bits) {
    case 2: gemm_body<2, NM, PHASE, COLS, WV, SIN>(G, ex, e, tb, rb, gsmem); break;
    case 4: gemm_body<4, NM, PHASE, COLS, WV, SIN>(G, ex, e, tb, rb, gsmem); break;
    default: gemm_body<8, NM, PHASE, COLS, WV, SIN>(G, ex, e, tb, rb, gsmem); break;
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

constexpr int kWaves1 = 16;    // wavefronts of a GEMM 1 workgroup
constexpr int kWaves2 = 16;    // wavefronts of a GEMM 2 workgroup on the canonical W_out

hipError_t init_attrs_prefill() {
  // the staging kernels keep one activation vector (up to 32768 values) in LDS
  const int lds = 32768 * 2 + 32768 / 16 * 4 + 64;
  if (hipError_t e = hipFuncSetAttribute((const void*)k_stage<false>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
      e != hipSuccess)
    return e;
  if (hipError_t e = hipFuncSetAttribute((const void*)k_stage<true>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
      e != hipSuccess)
    return e;
  // the GEMMs' rings
  if (hipError_t e = hipFuncSetAttribute((const void*)k_gemm_q<2, 0, false, kWaves1>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                         gemm_lds_bytes<0, false, kWaves1>());
      e != hipSuccess)
    return e;
  if (hipError_t e = hipFuncSetAttribute((const void*)k_gemm_q<1, 0, false, kWaves1>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                         gemm_lds_bytes<0, false, kWaves1>());
      e != hipSuccess)
    return e;
  if (hipError_t e = hipFuncSetAttribute((const void*)k_gemm_q<2, 0, false, kWaves1, true>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, gemm_lds_bytes<0, true, kWaves1>());
      e != hipSuccess)
    return e;
  if (hipError_t e = hipFuncSetAttribute((const void*)k_gemm_q<1, 0, false, kWaves1, true>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, gemm_lds_bytes<0, true, kWaves1>());
      e != hipSuccess)
    return e;
  if (hipError_t e = hipFuncSetAttribute((const void*)k_gemm_q<1, 1, false, kWaves2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                         gemm_lds_bytes<1, false, kWaves2>());
      e != hipSuccess)
    return e;
  return hipFuncSetAttribute((const void*)k_gemm_q<1, 1, true, 8>, hipFuncAttributeMaxDynamicSharedMemorySize,
                             gemm_lds_bytes<1, true, 8>());
}

PrefillWs prefill_ws(const LayerDims& L, int64_t T) {
  PrefillWs w{};
  const size_t M = (size_t)T * L.top_k;
  const size_t max_blocks = M / (kTB * kItemTiles) + (size_t)L.n_experts;   // GEMM work items
  const size_t max_tiles = M / kTB + (size_t)L.n_experts + 1;               // token tiles, + the spare one a work item
                                                                            // whose second tile does not exist reads
  size_t off = 0;
  w.poff = off;    off += up256(((size_t)L.n_experts + 1) * 4);
  w.boff = off;    off += up256((size_t)L.n_experts * 4);
  w.nblk = off;    off += 256;
  w.blocks = off;  off += up256(max_blocks * 8);
  w.gpair = off;   off += up256(M * 4);
  w.ginv = off;    off += up256(M * 4);
  w.gexp = off;    off += up256(M * 4);
  w.xa = off;      off += up256(max_tiles * staged_layout(L.d_model).block_bytes);
  w.ha = off;      off += up256(max_tiles * staged_layout(L.d_ff).block_bytes);
  w.hf = off;      off += up256(M * (size_t)L.d_ff * 4);
  w.ypair = off;   off += up256(M * (size_t)L.d_model * 4);
  w.total = off;
  w.max_blocks = max_blocks;
  return w;
}

hipError_t launch_prefill(const LayerDims& L, const DevExpert* table, const void* x, int32_t T, const int32_t* idx,
                          const float* gate, char* ws, const PrefillWs& w, float* y, bool out_columns, bool in_stream,
                          hipStream_t st) {
  const int M = T * L.top_k;
  int32_t* poff = (int32_t*)(ws + w.poff);
  int32_t* boff = (int32_t*)(ws + w.boff);
  int32_t* nblk = (int32_t*)(ws + w.nblk);
  int2* blocks = (int2*)(ws + w.blocks);
  int32_t* gpair = (int32_t*)(ws + w.gpair);
  int32_t* ginv = (int32_t*)(ws + w.ginv);
  int32_t* gexp = (int32_t*)(ws + w.gexp);
  char* XA = ws + w.xa;
  char* HA = ws + w.ha;
  float* Ypair = (float*)(ws + w.ypair);
  hipLaunchKernelGGL(k_count_pairs, dim3(1), dim3(1024), 0, st, idx, M, L.n_experts, poff, boff, blocks, nblk);
  hipLaunchKernelGGL(k_scatter_pairs, dim3(L.n_experts), dim3(256), 0, st, idx, M, poff, gpair, ginv, gexp);
  float* Hf = (float*)(ws + w.hf);
  auto stage_lds = [](int cols) { return (size_t)cols * 2 + (size_t)cols / 16 * 4 + 64; };
  const unsigned stage_grid = (unsigned)((M + 7) / 8 * 8);
  hipLaunchKernelGGL(k_stage<false>, dim3(stage_grid), dim3(256), stage_lds(L.d_model), st, L, table, x, gpair, gexp,
                     poff, boff, XA, M);
  GemmArgs G{L, table, blocks, nblk, poff, boff, XA, Hf, Ypair};
  const unsigned nb = (unsigned)w.max_blocks;
  constexpr int lds1 = gemm_lds_bytes<0, false, kWaves1>(), lds2 = gemm_lds_bytes<1, false, kWaves2>(),
                lds2c = gemm_lds_bytes<1, true, 8>();
  constexpr int lds1s = gemm_lds_bytes<0, true, kWaves1>();
  if (L.act == MOEQ_ACT_SWIGLU) {
    constexpr int BN = gemm_rows<2, 0, kWaves1>();
    const int n_rb = (L.d_ff + BN - 1) / BN;
    const dim3 grid((unsigned)n_rb * nb), block(kWaves1 * 64);
    if (in_stream) hipLaunchKernelGGL((k_gemm_q<2, 0, false, kWaves1, true>), grid, block, lds1s, st, G, n_rb);
    else hipLaunchKernelGGL((k_gemm_q<2, 0, false, kWaves1>), grid, block, lds1, st, G, n_rb);
  } else {
    constexpr int BN = gemm_rows<1, 0, kWaves1>();
    const int n_rb = (L.d_ff + BN - 1) / BN;
    const dim3 grid((unsigned)n_rb * nb), block(kWaves1 * 64);
    if (in_stream) hipLaunchKernelGGL((k_gemm_q<1, 0, false, kWaves1, true>), grid, block, lds1s, st, G, n_rb);
    else hipLaunchKernelGGL((k_gemm_q<1, 0, false, kWaves1>), grid, block, lds1, st, G, n_rb);
  }
  hipLaunchKernelGGL(k_stage<true>, dim3(stage_grid), dim3(256), stage_lds(L.d_ff), st, L, table, (const void*)Hf, gpair,
                     gexp, poff, boff, HA, M);
  G.A = HA;
  if (out_columns) {
    constexpr int BN = gemm_rows<1, 1, 8>();
    const int n_rb = (L.d_model + BN - 1) / BN;
    hipLaunchKernelGGL((k_gemm_q<1, 1, true, 8>), dim3((unsigned)n_rb * nb), dim3(512), lds2c, st, G, n_rb);
  } else {
    constexpr int BN = gemm_rows<1, 1, kWaves2>();
    const int n_rb = (L.d_model + BN - 1) / BN;
    hipLaunchKernelGGL((k_gemm_q<1, 1, false, kWaves2>), dim3((unsigned)n_rb * nb), dim3(kWaves2 * 64), lds2, st, G, n_rb);
  }
  hipLaunchKernelGGL(k_combine, dim3(T), dim3(256), 0, st, Ypair, ginv, gate, L.top_k, L.d_model, y);
  return hipGetLastError();
}

}  // namespace moeq
