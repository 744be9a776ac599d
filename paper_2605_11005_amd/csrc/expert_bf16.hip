// bf16 grouped GEMMs for the expert FFNs on gfx950 (CDNA4): MFMA 32x32x16 bf16, fp32 accumulate.
//
// One persistent kernel template covers the six GEMM shapes of the expert layer:
//   UP     h1|h3 = xp [W1|W3]        ragged M, B read transposed, fused SwiGLU epilogue -> a
//   DOWN   o     = a W2              ragged M, B read transposed
//   DA     dA    = d_o W2^T          ragged M, B K-contiguous, fused SwiGLU-backward epilogue
//   DX     dxp   = dH1 W1^T + dH3 W3^T   ragged M, K = 2f in two segments
//   WG     dW2   = a^T d_o           ragged K (the expert's rows), both operands read transposed
//   WGD    dW1|dW3 = xp^T [dH1|dH3]  ragged K, two outputs sharing the A operand
//
// Tiling: 256x256 block tile, 32-deep k-tiles, 256 threads = 4 wavefronts in a 2x2 grid,
// 128x128 per wavefront = 4x4 MFMA blocks (256 accumulator registers), one wavefront per SIMD.
//
// Data path: global memory -> LDS directly (global_load_lds_dwordx4, 16 bytes per lane, no
// staging registers), through a 128 KB ring (four k-tiles of both operands), so up to three
// k-tiles (96 KB per CU) are in flight while one is being multiplied.  Every load fetches whole
// 128-byte cache lines where the layout allows it: the K-contiguous operand A of the ragged-M
// shapes is fetched two k-tiles at a time (128 bytes per row) into two double stages, because a
// panel walked in 64-byte pieces crosses the L2-to-CU path twice.  Because a wavefront's 64
// lanes always land on 1 KB of consecutive LDS, bank conflicts are avoided by choosing WHICH
// global chunk each lane fetches (an XOR swizzle of the chunk index), not by padding:
//   K-contiguous A, two k-tiles [256 rows][8 chunks of 8 k]  chunk' = chunk ^ ((row>>1)&7)
//   K-contiguous B, one k-tile  [256 rows][4 chunks of 8 k]  chunk' = chunk ^ ((row>>2)&3)
//   transposed operand tile    2 x [32 k][16 chunks of 8 n]  chunk' = chunk ^ (4*(k&3))
// (LDS has 64 four-byte banks: the 16 lanes served together by a 16-byte read, or the 32 lanes
// of an 8-byte transposing read, must cover 256 distinct bytes modulo 256.)
// Operands whose contraction index is not the contiguous one in memory (the weights in the
// forward pass, both operands of the weight gradients) are kept in their memory layout in
// LDS and transposed on the way to registers by ds_read_b64_tr_b16.
// Per k-tile each wavefront runs two k-steps of 16 MFMAs; the fragments of the next k-step
// are fetched while the current one multiplies, and there is one workgroup barrier per k-tile.
// Workgroups are persistent and walk a device-built tile list (row counts never visit the
// host); the list is ordered so that the tiles resident on one XCD share operand panels.
#include "common.h"
#include "kernels.h"

namespace {

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
// 16-byte store of a finished output vector.  The epilogues' bf16 outputs stream out once (2-8 GB per step) and
// are next read by another kernel: a nontemporal store keeps them from displacing operand panels in the caches
// (measured: -0.3 % at the DeepSeek-V3-like share, -0.5 % at the Mixtral-like layer over the six GEMMs).
__device__ __forceinline__ void store16(void* ptr, uint4 v) {
  __builtin_nontemporal_store(__builtin_bit_cast(u32x4_t, v), reinterpret_cast<u32x4_t*>(ptr));
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BM = 256, BN = 256, BK = 32;
constexpr int NT = 256;                 // threads
constexpr int NSTAGE = 4;
constexpr int OPER_BYTES = 256 * BK * 2;           // 16384: one operand tile
constexpr int STAGE_BYTES = 2 * OPER_BYTES;        // 32768
constexpr int TILE_LDS = NSTAGE * STAGE_BYTES;     // 131072
// Epilogue staging, outside the tile ring: one private slab per wavefront, fp32.
//   single-output tiles: 16 rows x 64 columns, pitch 68 floats; dual tiles: 8 rows x 128 columns, pitch 132
constexpr int SPITCH = 68, DPITCH = 132;
constexpr int STAGING_WAVE_BYTES = 16 * SPITCH * 4;   // 4352 >= 8 * DPITCH * 4 = 4224
static_assert(8 * DPITCH * 4 <= STAGING_WAVE_BYTES, "dual slab must fit");
// scheduler tables after the ring: tile_start[L+1], offs[L+1], split[L] (int32), order[L] (uint16), ticket
constexpr int SCHED_BYTES = 2 * (MOE_MAX_LOCAL + 1) * 4 + MOE_MAX_LOCAL * 4 + MOE_MAX_LOCAL * 2 + 16;
constexpr int STAGING_OFF = (TILE_LDS + SCHED_BYTES + 15) & ~15;
constexpr int SMEM_BYTES = STAGING_OFF + 4 * STAGING_WAVE_BYTES;
static_assert(SMEM_BYTES <= 160 * 1024, "one workgroup per CU: 160 KB of LDS");

enum { UP = 0, DOWN = 1, DA = 2, DX = 3, WG = 4, WGD = 5,
       // the trainable router reuses the same machinery on one full-height "expert":
       RL = 6,    // logits = x Wr            ragged-M shape, B read transposed, fp32 output
       RW = 7,    // dWr partials = x^T dl    ragged-K shape over fixed chunks of the tokens, fp32 output
       RX = 8 };  // dx (+)= dl Wr^T          ragged-M shape, B K-contiguous, optional bf16 accumulate

struct GArgs {
  const bf16_t* A0; const bf16_t* A1;     // A sources (A1: second K segment of DX)
  const bf16_t* B0; const bf16_t* B1;     // B sources (B1: second half of a dual tile / second K segment)
  long lda, ldb;                          // leading dimensions (elements)
  long b_es;                              // expert stride of B (elements); 0 for row-indexed B
  bf16_t* C0; bf16_t* C1; bf16_t* C2;     // outputs
  long ldc, c_es;
  const bf16_t* H1; const bf16_t* H3;     // DA epilogue inputs
  float* F0;                              // fp32 output (RL, RW)
  const int32_t* off;                     // row offsets; NULL: segment e = [min(e*chunk, rows), min((e+1)*chunk, rows))
  int rows, chunk;
  // Weight gradients of experts with far more rows than the average are cut along the rows into
  // up to split_budget pieces in total, whose fp32 partial tiles go to P0 (piece s at
  // P0 + s * p_stride; the second output of a dual tile at + M*N) and are added up, in piece
  // order, by wgrad_reduce.  plan[e] = (first piece << 8) | pieces  (pieces == 1: not cut).
  float* P0;
  long p_stride;
  int split_budget;
  int32_t* plan;
  int32_t* sched;                         // 8 zeroed ticket counters (one per XCD)
  int e_cnt;
  int M;                                  // WG/WGD: rows of the output (d or f)
  int N;                                  // output columns (per half for dual tiles)
  int K;                                  // contraction length per segment (ragged-M modes)
  // RL only: the contraction is cut into ksplit ranges of K columns each (the last one may be
  // shorter; k_total columns in all); range j writes its fp32 tile to F0 + j * c_es and a
  // separate pass adds the ranges up.  0 or 1: not cut.
  int ksplit, k_total;
  int accumulate;
  int save_h;
};

template <int MODE> struct Traits {
  static constexpr bool A_TRANS = MODE == WG || MODE == WGD || MODE == RW;
  static constexpr bool B_TRANS = MODE == UP || MODE == DOWN || MODE == WG || MODE == WGD || MODE == RL || MODE == RW;
  static constexpr bool DUAL = MODE == UP || MODE == WGD;
  static constexpr bool RAGGED_K = MODE == WG || MODE == WGD || MODE == RW;
  static constexpr int BN_EFF = DUAL ? BN / 2 : BN;   // output columns covered per tile
};

// 16 bytes per lane from global memory straight into LDS: lane l lands at lds_wave_base + 16*l
// (lds_wave_base is wave-uniform and travels in M0).  The global address is a wave-uniform
// 64-bit base in SGPRs plus a 32-bit per-lane byte offset: with 64-bit per-lane addresses the
// address path, not the data path, limits a CU to ~27 B/clk; this form sustains ~42 B/clk.
// Written as inline assembly so that the compiler's wait-count pass does not serialise later
// LDS reads against these loads; the kernel waits for them itself (s_waitcnt vmcnt) before
// the barrier that publishes a tile.
__device__ __forceinline__ void dma16(const bf16_t* sbase, uint32_t voff_bytes, uint32_t lds_wave_base) {
  // make the uniformity of the base explicit so that it is allocated to an SGPR pair
  const uint64_t u = (uint64_t)sbase;
  const uint64_t ub = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(u >> 32)) << 32) |
                      (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)u);
  sbase = (const bf16_t*)ub;
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_wave_base), "v"(voff_bytes), "s"(sbase)
               : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

// ---- K-contiguous operand B (source rows are tile rows; a k-tile is 64 contiguous bytes) -
// Wavefront w issues 4 loads per k-tile; load j covers LDS chunks [(4w+j)*64, +64):
// row = 16*(4w+j) + lane/4, LDS slot = lane%4, logical chunk = slot ^ ((row>>2)&3).
// Rows past the valid range re-read the last valid row (their products land in output rows
// or columns that the epilogue never stores).
struct KcIssue {
  const bf16_t* base;      // wave-uniform: first row of the tile
  uint32_t voff[4];        // byte offset of this lane's chunk in load j
  __device__ __forceinline__ void setup(const bf16_t* base_, long ld, int rows_valid, int wave, int lane) {
    base = base_;
    const int c = (lane & 3) ^ ((lane >> 4) & 3);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int r = 16 * (4 * wave + j) + (lane >> 2);
      if (r > rows_valid - 1) r = rows_valid - 1;
      voff[j] = (uint32_t)(r * ld * 2 + c * 16);
    }
  }
  __device__ __forceinline__ void issue1(int j, uint32_t oper_lds, int wave, long kofs) const {
    dma16(base + kofs, voff[j], oper_lds + (4 * wave + j) * 1024);
  }
};

// ---- K-contiguous operand A of the ragged-M shapes, fetched two k-tiles at a time ----------
// A 64-byte piece is half a cache line, and walking a panel in such pieces moves every line
// from L2 to the CU twice (a load stream of 64-byte pieces sustains half the rate of one of
// 128-byte pieces).  So operand A lives in two double stages of [256 rows][128 bytes] = k-tiles
// 2p and 2p+1 of pair p, filled by 8 loads per wavefront that each fetch whole lines:
// load q covers LDS chunks [(8w+q)*64, +64): row = 8*(8w+q) + lane/8, LDS slot = lane%8,
// logical chunk = slot ^ ((row>>1)&7)  (chunks 0..3: k-tile 2p, 4..7: k-tile 2p+1).
struct KcPairIssue {
  const bf16_t* base;      // wave-uniform: first row of the tile
  uint32_t voff[8];        // byte offset of this lane's chunk in load q
  __device__ __forceinline__ void setup(const bf16_t* base_, long ld, int rows_valid, int wave, int lane) {
    base = base_;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int rl = 8 * (8 * wave + q) + (lane >> 3);
      const int c = (lane & 7) ^ ((rl >> 1) & 7);
      const int r = rl > rows_valid - 1 ? rows_valid - 1 : rl;
      voff[q] = (uint32_t)(r * ld * 2 + c * 16);
    }
  }
  __device__ __forceinline__ void issue1(int q, uint32_t dstage_lds, int wave, long kofs) const {
    dma16(base + kofs, voff[q], dstage_lds + (8 * wave + q) * 1024);
  }
};

// ---- transposed operand (source is [k][n], n contiguous) --------------------------------
// Kept in LDS as two sub-tiles [32 k][128 n] of 8 KB (for a dual tile they come from two
// source matrices).  A tile is 16 loads; load id = 4*wave + j covers sub-tile id/8 and the
// four k rows 4*(id%8) + lane/16; LDS slot = lane%16, logical n chunk = slot ^ (4*(k&3)).
// Columns past n_lim are clamped (garbage output columns, never stored); with CLAMP, source
// rows past the last valid one are clamped (the caller zeroes the matching A fragments).
struct TrIssue {
  const bf16_t* src;       // wave-uniform: column n0 of this wavefront's sub-tile source, row 0
  long ld;
  uint32_t coff;           // byte offset of this lane's column chunk
  // a wavefront's four loads all belong to sub-tile wave/2
  __device__ __forceinline__ void setup(const bf16_t* b0, const bf16_t* b1, bool dual, long ld_, int n0, int n_lim,
                                        int wave, int lane) {
    ld = ld_;
    const int sub = wave >> 1;
    const int nc = (lane & 15) ^ (4 * (lane >> 4));
    src = (dual && sub) ? b1 : b0;
    int n = n0 + (dual ? 0 : sub * 128) + nc * 8;
    if (n > n_lim - 8) n = n_lim - 8;
    coff = (uint32_t)(n * 2);
  }
  // load j of the k-tile whose first source row is k0 (rows above k_last_rel clamped if CLAMP)
  template <bool CLAMP>
  __device__ __forceinline__ void issue1(int j, uint32_t oper_lds, int wave, int lane, long k0, int k_last_rel) const {
    const int id = 4 * wave + j;
    int kr = 4 * (id & 7) + (lane >> 4);
    if (CLAMP && kr > k_last_rel) kr = k_last_rel;
    dma16(src + k0 * ld, (uint32_t)(kr * ld * 2) + coff, oper_lds + id * 1024);
  }
};

template <int V> struct IntC { static constexpr int value = V; };

// Fragment addressing.  MFMA 32x32x16 operand: lane l holds row (l&31), k = 8*(l>>5) + 0..7.
// K-contiguous tile: one 16-byte read.  byte offset of (row, k-step s) = row*64 + ((2s + (l>>5)) ^ ((row>>2)&3))*16
// (k-step 1 is k-step 0 with bit 5 flipped: the swizzle is an XOR, not an addition)
__device__ __forceinline__ int kc_frag_off(int row, int lane, int s) {
  return row * 64 + (((2 * s + (lane >> 5)) ^ ((row >> 2) & 3)) << 4);
}
// Double stage of operand A: byte offset of (row, k-tile parity h, k-step s) =
// row*128 + ((4h + 2s + (l>>5)) ^ ((row>>1)&7))*16; h and s enter as XORs of 64 and 32.
__device__ __forceinline__ int kcp_frag_off(int row, int lane) {
  return row * 128 + (((lane >> 5) ^ ((row >> 1) & 7)) << 4);
}
// Transposed tile: two 8-byte transposing reads (k 0..3 and 4..7 of the lane's group).  Within
// each group of 16 lanes, lane i supplies the address of T[kb + i/4][nb16 + 4*(i%4) ..+3] and
// receives T[kb + 0..3][nb16 + i].  Offset for k-step 0, first read; add s*4096 + t*1024.
__device__ __forceinline__ int tr_frag_off(int nb, int lane) {
  const int i = lane & 15, g = lane >> 4;
  const int k = 8 * (g >> 1) + (i >> 2);
  const int n = nb + 16 * (g & 1) + 4 * (i & 3);
  const int sub = n >> 7, nl = n & 127;
  return sub * 8192 + k * 256 + (((nl >> 3) ^ (4 * (k & 3))) << 4) + ((n & 4) << 1);
}

__device__ __forceinline__ bf16x8 lds_frag_kc(const char* p) { return *reinterpret_cast<const bf16x8*>(p); }
__device__ __forceinline__ bf16x8 lds_frag_tr(const char* p) {
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p + 1024));
  s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

extern __shared__ __align__(16) char smem[];

// One grouped GEMM from its set-up to its last tile, run by a persistent workgroup.
template <int MODE>
__device__ __forceinline__ void gg_body(const GArgs& p) {
  using TR = Traits<MODE>;
  int32_t* tile_start = reinterpret_cast<int32_t*>(smem + TILE_LDS);
  int32_t* offs = tile_start + (MOE_MAX_LOCAL + 1);      // LDS copy of the row offsets
  int32_t* split = offs + (MOE_MAX_LOCAL + 1);           // ragged-K modes: (first piece << 8) | pieces, by expert
  uint16_t* order = reinterpret_cast<uint16_t*>(split + MOE_MAX_LOCAL);   // experts by descending row count
  int32_t* next_q = reinterpret_cast<int32_t*>(order + MOE_MAX_LOCAL);    // hand-over slot of the tile scheduler

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int e_cnt = p.e_cnt;

  // ---- tile list.  Experts are taken heaviest first (ties by id), so that the cheap tiles
  // come last and even out the end of the schedule.  position -> expert in order[];
  // tile_start[pos] = number of tiles before that position (ragged-M modes).
  // (RL: the ranges of a cut contraction are listed like further column tiles)
  const int n_tiles_cols = (p.N + TR::BN_EFF - 1) / TR::BN_EFF;
  const int n_tiles_n = MODE == RL && p.ksplit > 1 ? n_tiles_cols * p.ksplit : n_tiles_cols;
  int total;
  int wg_tiles_per_e = 0, wg_mt = 0;
  for (int e = tid; e <= e_cnt; e += NT) {
    const long long cut = (long long)e * p.chunk;
    offs[e] = p.off ? p.off[e] : (int)(cut < p.rows ? cut : p.rows);
  }
  __syncthreads();
  for (int e = tid; e < e_cnt; e += NT) {
    const int rows = offs[e + 1] - offs[e];
    int rank = 0;
    for (int o = 0; o < e_cnt; ++o) {
      const int r2 = offs[o + 1] - offs[o];
      rank += (r2 > rows || (r2 == rows && o < e)) ? 1 : 0;
    }
    order[rank] = (uint16_t)e;
  }
  __syncthreads();
  if (TR::RAGGED_K) {
    // Every expert has the same number of output tiles, but a tile's cost is the expert's row
    // count.  An expert whose k loop is longer than a workgroup's fair share of the whole launch
    // (in k-tiles) bounds the kernel from below; it is cut into pieces of about half that share
    // (at least 16 k-tiles) when the time saved exceeds the time to write and re-read the fp32
    // partial tiles (p_stride floats per piece, priced at ~4 TB/s against ~0.85 us per k-tile),
    // heaviest experts first while the budget of partial tiles lasts.
    wg_mt = (p.M + BM - 1) / BM;
    wg_tiles_per_e = wg_mt * n_tiles_n;
    if (tid == 0) {
      long long units = 0;
      for (int e = 0; e < e_cnt; ++e) units += (offs[e + 1] - offs[e] + BK - 1) / BK;
      const int share = (int)(units * wg_tiles_per_e / gridDim.x);
      const int target = share / 2 > 16 ? share / 2 : 16;
      const int piece_cost = (int)(p.p_stride / 400000) + 1;
      int used = 0;
      for (int pos = 0; pos < e_cnt; ++pos) {
        const int e = order[pos];
        const int nke = (offs[e + 1] - offs[e] + BK - 1) / BK;
        int pieces = 1;
        if (nke > share) {
          pieces = (nke + target - 1) / target;
          if (pieces > 255) pieces = 255;
          if (pieces > p.split_budget - used) pieces = p.split_budget - used;
          if (pieces < 2 || nke - share <= pieces * piece_cost) pieces = 1;
        }
        if (pieces > 1) used += pieces;
        split[e] = pieces;
      }
    }
    __syncthreads();
    // list the experts again, now by the length of one tile's k loop (a cut expert's pieces are
    // shorter than the tiles of the next heaviest ones), longest first
    for (int e = tid; e < e_cnt; e += NT) {
      const int len = ((offs[e + 1] - offs[e] + BK - 1) / BK + split[e] - 1) / split[e];
      int rank = 0;
      for (int o = 0; o < e_cnt; ++o) {
        const int l2 = ((offs[o + 1] - offs[o] + BK - 1) / BK + split[o] - 1) / split[o];
        rank += (l2 > len || (l2 == len && o < e)) ? 1 : 0;
      }
      order[rank] = (uint16_t)e;
    }
    __syncthreads();
    if (tid == 0) {
      int run = 0, used = 0;
      for (int pos = 0; pos < e_cnt; ++pos) {
        const int e = order[pos];
        const int pieces = split[e];
        split[e] = pieces > 1 ? ((used << 8) | pieces) : 1;
        if (pieces > 1) used += pieces;
        tile_start[pos] = run;
        run += pieces * wg_tiles_per_e;
      }
      tile_start[e_cnt] = run;
    }
    __syncthreads();
    total = tile_start[e_cnt];
    if (p.plan && blockIdx.x == 0)
      for (int e = tid; e < e_cnt; e += NT) p.plan[e] = split[e];
  } else {
    for (int pos = tid; pos < e_cnt; pos += NT) {
      const int e = order[pos];
      const int rows = offs[e + 1] - offs[e];
      tile_start[pos] = ((rows + BM - 1) / BM) * n_tiles_n;
    }
    __syncthreads();
    if (tid == 0) {
      int run = 0;
      for (int pos = 0; pos < e_cnt; ++pos) {
        int v = tile_start[pos];
        tile_start[pos] = run;
        run += v;
      }
      tile_start[e_cnt] = run;
    }
    __syncthreads();
    total = tile_start[e_cnt];
  }

  // LDS ring.  Ragged-K shapes: four stages of [A tile | B tile].  Ragged-M shapes (PAIR): operand A
  // in two double stages of 32 KB (k-tiles 2p, 2p+1) at 0, operand B in four 16 KB stages at 64 KB.
  constexpr bool PAIR = !TR::RAGGED_K;
  static_assert(PAIR == !TR::A_TRANS, "operand A is K-contiguous exactly in the ragged-M shapes");
  constexpr int B_REGION = PAIR ? NSTAGE * OPER_BYTES : OPER_BYTES;
  // per-lane fragment offsets inside an operand tile (k-step 0; k-tile 2p of a double stage)
  int a_off[4], b_off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int arow = wm * 128 + i * 32;
    const int brow = TR::DUAL ? (i < 2 ? 0 : 128) + wn * 64 + (i & 1) * 32 : wn * 128 + i * 32;
    a_off[i] = TR::A_TRANS ? tr_frag_off(arow, lane) : kcp_frag_off(arow + (lane & 31), lane);
    b_off[i] = B_REGION + (TR::B_TRANS ? tr_frag_off(brow, lane) : kc_frag_off(brow + (lane & 31), lane, 0));
  }

  const int G = gridDim.x;
  const int n_queues = (G % 8) == 0 ? 8 : 1;
  int queue = blockIdx.x % n_queues;       // the queue this workgroup currently draws from
  int pos_hint = 0;                        // list position of the last decoded tile
  const uint32_t smem_base = lds_addr(smem);

  // ---- state of the tile whose k loop runs next (written by next_tile)
  int e = 0, lo = 0, hi = 0, n0 = 0;
  int piece = -1;         // ragged-K modes: index of the fp32 partial tile to write, or -1
  int krange = 0;         // RL: which range of a cut contraction
  int nk0 = 0, nk = 0;    // k-tiles in segment 0 / in total
  int row0 = 0;           // first output row (global row for ragged-M, i for the weight gradients)
  int row_end = 0;        // one past the last valid output row
  KcPairIssue ia_kp;
  KcIssue ib_kc;
  TrIssue ia_tr, ib_tr;

  // One of the 8 loads (q = 0..3: operand A, 4..7: operand B) of k-tile kt.  kt is clamped to
  // the last tile, so every iteration issues the same number of loads and the vmcnt
  // arithmetic below is uniform; the surplus loads re-fetch the last tile into a free stage.
  auto issue_one = [&](int kt, int q) {       // ragged-K shapes
    if (kt > nk - 1) kt = nk - 1;
    const uint32_t st = smem_base + (kt & (NSTAGE - 1)) * STAGE_BYTES;
    const int j = q & 3;
    const long k0 = (long)lo + kt * BK;
    const int k_last_rel = hi - 1 - lo - kt * BK;
    if (q < 4) ia_tr.template issue1<true>(j, st, wave, lane, k0, k_last_rel);
    else ib_tr.template issue1<true>(j, st + OPER_BYTES, wave, lane, k0, k_last_rel);
  };
  // Ragged-M shapes: one of the 8 loads of operand A's pair pj (k-tiles 2pj, 2pj+1; K is a
  // multiple of 64 per segment, so a pair never straddles DX's two segments) and one of the 4
  // loads of operand B's k-tile kt.  Both indices are clamped like kt above.
  auto issue_a_pair = [&](int pj, int q) {
    if (pj > (nk >> 1) - 1) pj = (nk >> 1) - 1;
    const int kt0 = 2 * pj;
    const bool seg1 = MODE == DX && kt0 >= nk0;
    const long kofs = (long)(seg1 ? kt0 - nk0 : kt0) * BK + (seg1 ? p.A1 - p.A0 : 0);
    ia_kp.issue1(q, smem_base + (pj & 1) * (2 * OPER_BYTES), wave, kofs);
  };
  auto issue_b = [&](int kt, int j) {
    if (kt > nk - 1) kt = nk - 1;
    const uint32_t st = smem_base + B_REGION + (kt & (NSTAGE - 1)) * OPER_BYTES;
    const bool seg1 = MODE == DX && kt >= nk0;
    const int k0 = (seg1 ? kt - nk0 : kt) * BK;
    if (TR::B_TRANS) ib_tr.template issue1<false>(j, st, wave, lane, k0, 0);
    else ib_kc.issue1(j, st, wave, k0 + (seg1 ? p.B1 - p.B0 : 0));
  };
  auto issue_tile = [&](int kt) {
#pragma unroll
    for (int q = 0; q < 8; ++q) issue_one(kt, q);
  };

  // ---- dynamic, XCD-aware tile scheduler.  The list is cut into chunks of 32 consecutive
  // tiles (an 8 x 4 block of one expert: 8 A panels and 4 B panels); chunk c belongs to XCD
  // c mod 8 (workgroup b runs on XCD b mod 8), whose workgroups draw tiles from it in order
  // through one atomic counter per XCD.  Ticket q of XCD x is tile 32*(8*(q/32) + x) + q%32.
  // The ticket for the next tile is drawn near the end of the current k loop.  A workgroup whose
  // queue has run dry draws from the next XCD's queue that still has tiles.
  //
  // next_tile: takes the ticket waiting in *next_q, decodes it into the tile state above and
  // starts the loads of that tile's first k-tiles.  The tile ring must be free when it is
  // called (it is called after the barrier that ends a k loop, before that tile's epilogue,
  // so the first operands of the next tile travel while the finished one is being stored).
  auto next_tile = [&]() -> bool {
    int L;
    while (true) {
      const int q = __builtin_amdgcn_readfirstlane(next_q[0]);
      L = 32 * (n_queues * (q >> 5) + queue) + (q & 31);
      if (L < total) break;                  // (the slot is next written after a whole k loop of barriers)
      // Tickets only grow, so this queue is finished, and so is every queue whose counter has passed
      // its last ticket.  All counters are looked at in one round trip (an atomic add of zero, one lane
      // per queue): when none is open the workgroup is done; otherwise it draws from the first open
      // queue after its own (work stealing at the tail of the schedule) and, should others have emptied
      // that queue in between, looks again.  Every failed draw means that others took tiles meanwhile,
      // so the loop ends when the list does.
      __syncthreads();                       // everyone has read the ticket before it is replaced
      if (wave == 0) {
        int open = 0;
        if (lane < n_queues) {
          const int per_round = 32 * n_queues;
          const int full = total / per_round;
          int extra = total - full * per_round - 32 * lane;
          extra = extra < 0 ? 0 : (extra > 32 ? 32 : extra);
          open = atomicAdd(p.sched + lane, 0) < 32 * full + extra;
        }
        const unsigned all = (1u << n_queues) - 1u;
        const unsigned m = (unsigned)__ballot(open) & all;
        if (lane == 0) {
          if (m == 0) {
            next_q[0] = -1;
          } else {
            const unsigned rot = ((m >> (queue + 1)) | (m << (n_queues - queue - 1))) & all;
            const int pick = (queue + 1 + __builtin_ctz(rot)) % n_queues;
            next_q[1] = pick;
            next_q[0] = atomicAdd(p.sched + pick, 1);
          }
        }
      }
      __syncthreads();
      if (__builtin_amdgcn_readfirstlane(next_q[0]) < 0) return false;
      queue = __builtin_amdgcn_readfirstlane(next_q[1]);
    }
    // Within an expert, tiles are ordered in bands of 8 m-tiles, n-tile next, m-tile inside the
    // band fastest: 32 consecutive tiles (one chunk) then form an 8 x 4 block that shares 8 A
    // panels and 4 B panels through one XCD's L2.
    int mt, nt;
    {
      int li, mte;
      // largest position with tile_start[pos] <= L: tickets of a queue ascend, so it is usually
      // the position of the previous tile or the one after it; otherwise a binary search
      int a = pos_hint;
      {
        const int t0 = tile_start[a], t1 = tile_start[a + 1], t2 = tile_start[min(a + 2, e_cnt)];
        if (L >= t1 && L < t2) a = a + 1;
        else if (L < t0 || L >= t1) {
          a = 0;
          int c = e_cnt;
          while (c - a > 1) {
            int mid = (a + c) >> 1;
            if (tile_start[mid] <= L) a = mid; else c = mid;
          }
        }
      }
      a = __builtin_amdgcn_readfirstlane(a);
      pos_hint = a;
      li = __builtin_amdgcn_readfirstlane(L - tile_start[a]);
      e = __builtin_amdgcn_readfirstlane((int)order[a]);
      lo = __builtin_amdgcn_readfirstlane(offs[e]);
      hi = __builtin_amdgcn_readfirstlane(offs[e + 1]);
      if (TR::RAGGED_K) {
        mte = wg_mt;
        const int sp = __builtin_amdgcn_readfirstlane(split[e]);
        const int pieces = sp & 255;
        piece = -1;
        if (pieces > 1) {                        // this tile covers one piece of the expert's rows
          const int c_idx = li / wg_tiles_per_e;
          li -= c_idx * wg_tiles_per_e;
          const int nke = (hi - lo + BK - 1) / BK;
          const int piece_rows = ((nke + pieces - 1) / pieces) * BK;
          lo = __builtin_amdgcn_readfirstlane(min(hi, lo + c_idx * piece_rows));
          hi = __builtin_amdgcn_readfirstlane(min(hi, lo + piece_rows));
          piece = (sp >> 8) + c_idx;
        }
      } else {
        mte = (hi - lo + BM - 1) / BM;
      }
      const int band = li / (8 * n_tiles_n);
      const int in_band = li - band * 8 * n_tiles_n;
      const int band_rows = min(8, mte - band * 8);
      nt = in_band / band_rows;
      mt = band * 8 + (in_band - nt * band_rows);
    }
    if (MODE == RL) {
      krange = nt / n_tiles_cols;
      nt -= krange * n_tiles_cols;
    }
    n0 = nt * TR::BN_EFF;
    if (TR::RAGGED_K) {
      row0 = mt * BM;
      row_end = p.M;
      nk0 = nk = (hi - lo + BK - 1) / BK;
      ia_tr.setup(p.A0, p.A0, false, p.lda, row0, p.M, wave, lane);
      ib_tr.setup(p.B0, p.B1, TR::DUAL, p.ldb, n0, p.N, wave, lane);
    } else {
      row0 = lo + mt * BM;
      row_end = hi;
      const size_t kfirst = MODE == RL ? (size_t)krange * p.K : 0;      // first column of this tile's range
      nk0 = (MODE == RL && p.ksplit > 1 ? min(p.K, p.k_total - krange * p.K) : p.K) / BK;
      nk = MODE == DX ? 2 * nk0 : nk0;
      ia_kp.setup(p.A0 + (size_t)row0 * p.lda + kfirst, p.lda, hi - row0, wave, lane);
      if (TR::B_TRANS) ib_tr.setup(p.B0 + (size_t)e * p.b_es + kfirst * p.ldb, p.B1 + (size_t)e * p.b_es, TR::DUAL, p.ldb, n0, p.N, wave, lane);
      else ib_kc.setup(p.B0 + (size_t)e * p.b_es + (size_t)n0 * p.ldb, p.ldb, p.N - n0, wave, lane);
    }
    if (nk > 0) {
      if (PAIR) {       // what the k loop's iterations -2 and -1 would have issued, in its order
#pragma unroll
        for (int q = 0; q < 8; ++q) issue_a_pair(0, q);
#pragma unroll
        for (int t = 0; t < 3; ++t)
#pragma unroll
          for (int j = 0; j < 4; ++j) issue_b(t, j);
#pragma unroll
        for (int q = 0; q < 4; ++q) issue_a_pair(1, q);
      } else {
        issue_tile(0); issue_tile(1); issue_tile(2);
#pragma unroll
        for (int q = 0; q < 4; ++q) issue_one(3, q);
      }
    } else {
      __syncthreads();   // a tile without a k loop has no barrier between this read of the ticket and its replacement
    }
    return true;
  };

  if (tid == 0) *next_q = atomicAdd(p.sched + queue, 1);
  __syncthreads();
  bool have = next_tile();

  while (have) {
    // The ticket of the tile after this one is drawn eight k-tiles before the end of the k loop
    // (at its start if it is shorter): late, so that a workgroup commits to its next tile only
    // when it is about to be free -- tiles are listed heaviest first and long ones must go to
    // whoever finishes first -- yet early enough that the atomic's latency is never waited for.
    // It is handed over through LDS after the k loop.
    int my_ticket = 0;
    const int kt_draw = nk > 8 ? nk - 8 : 0;
    if (nk == 0 && tid == 0) my_ticket = atomicAdd(p.sched + queue, 1);

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // Fragment sets: set h holds the A and B fragments of one k-step.  frag_op(h, kt, s, o)
    // performs the o-th of the 8 fragment reads of k-step s of tile kt, in the order the
    // MFMAs consume them: A0, B0, B1, B2, B3, A1, A2, A3.
    bf16x8 fa[2][4], fb[2][4];
    auto frag_op = [&](int h, int kt, int s, int o) {
      const char* st = smem + (kt & (NSTAGE - 1)) * (PAIR ? OPER_BYTES : STAGE_BYTES);
      const bool is_a = o == 0 || o >= 5;
      const int idx = o == 0 ? 0 : (o >= 5 ? o - 4 : o - 1);
      if (is_a) {
        const char* q = TR::A_TRANS ? st + a_off[idx] + s * 4096
                                    : smem + ((kt >> 1) & 1) * (2 * OPER_BYTES) + (a_off[idx] ^ ((kt & 1) * 64 + s * 32));
        fa[h][idx] = TR::A_TRANS ? lds_frag_tr(q) : lds_frag_kc(q);
      } else {
        const char* q = st + (TR::B_TRANS ? b_off[idx] + s * 4096 : b_off[idx] ^ (s * 32));
        fb[h][idx] = TR::B_TRANS ? lds_frag_tr(q) : lds_frag_kc(q);
      }
    };
    auto mfma_one = [&](int h, int m) {
      // The 4 x 4 grid of blocks is walked in a snake (columns 0..3, 3..0, 0..3, 3..0), so that exactly one of the
      // two operand fragments changes from one MFMA to the next.  Under the package power limit the rate follows the
      // switching activity: an MFMA-only loop runs 0.8 % faster this way than row-major and 2.4 % faster than a walk
      // that changes both operands every time.
      const int i = m >> 2, j = (i & 1) ? 3 - (m & 3) : (m & 3);
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[h][i], fb[h][j], acc[i][j], 0, 0, 0);
    };
    // ragged contraction: zero the A fragment elements whose source row is past the expert's
    // last row (only the last k-tile can contain such rows)
    auto mask_tail = [&](int h, int kt, int s) {
      const int kbase = lo + kt * BK + 16 * s + 8 * (lane >> 5);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        s16x8 v = __builtin_bit_cast(s16x8, fa[h][i]);
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = (kbase + j < hi) ? v[j] : (short)0;
        fa[h][i] = __builtin_bit_cast(bf16x8, v);
      }
    };

    // ---- k loop.  At the barrier of iteration kt every wavefront has all fragments of tile kt
    // in registers, so the LDS that held it is free, and tile kt+1 has landed.  Loads are spread
    // evenly over the iteration -- one per four MFMAs -- so that the CU's address unit (one
    // 64-lane load per ~24 cycles, shared by the four wavefronts) never backs up into the issue
    // stream.  Ragged-K shapes (k_loop): four stages, the first half issues operand B of tile
    // kt+3, the second half operand A of tile kt+4; issue order is A(t),B(t),A(t+1),..; at the
    // barrier the loads after B(kt+1) are A,B(kt+2) and A,B(kt+3): 16 may remain.  Ragged-M shapes:
    // k_loop_pair below.
    // The instruction order inside an iteration is fixed by hand (scheduling fences after every
    // MFMA pair): 16 MFMAs of k-step 0 with the 8 fragment reads of k-step 1 between them,
    // barrier, 16 MFMAs of k-step 1 with the next tile's first fragment reads between them.
    // The first loads (28: k-tiles 0..2 and operand A of k-tile 3; ragged-M shapes 24: A's pair
    // 0 and half of pair 1, B's k-tiles 0..2) were issued by next_tile; the stores of the previous
    // tile's epilogue were issued after them and share the counter, so the first wait is for
    // everything.
    if (nk > 0) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
#pragma unroll
      for (int o = 0; o < 8; ++o) frag_op(0, 0, 0, o);
    }
    // MV = number of 32-row MFMA blocks of this wavefront that hold valid output rows (4, 2 or
    // 0).  A tail tile's wavefronts whose rows lie past the expert's last row skip their MFMAs
    // and fragment reads but keep issuing their share of the loads and meeting the barriers.
    auto k_loop = [&](auto mv_tag) {
      constexpr int MV = decltype(mv_tag)::value;
      // fragment read o is needed iff it feeds a live MFMA: A0, B0..B3, A1, A2, A3
      auto live = [](int o) { return MV == 4 || (MV == 2 && o <= 5); };
      for (int kt = 0; kt < nk; ++kt) {
        if (kt == kt_draw && tid == 0) my_ticket = atomicAdd(p.sched + queue, 1);
        if (TR::RAGGED_K && kt == nk - 1) mask_tail(0, kt, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < 16; m += 2) {
          if (m < 4 * MV) mfma_one(0, m);
          if (m < 8) {                                   // all reads done well before the barrier
            if (live(m)) frag_op(1, kt, 1, m);
            if (live(m + 1)) frag_op(1, kt, 1, m + 1);
          }
          if (m < 4 * MV) mfma_one(0, m + 1);
          if ((m & 3) == 2) issue_one(kt + 3, 4 + (m >> 2));     // operand B of tile kt+3
          __builtin_amdgcn_sched_barrier(0);
        }
        asm volatile("s_waitcnt vmcnt(16) lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        if (TR::RAGGED_K && kt == nk - 1) mask_tail(1, kt, 1);
#pragma unroll
        for (int m = 0; m < 16; m += 2) {
          if (m < 4 * MV) mfma_one(1, m);
          if (live(m >> 1)) frag_op(0, kt + 1, 0, m >> 1);
          if (m < 4 * MV) mfma_one(1, m + 1);
          if ((m & 3) == 2) issue_one(kt + 4, m >> 2);           // operand A of tile kt+4
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    };
    // Ragged-M shapes: the same iteration, two k-tiles per trip (nk is even).  Operand A arrives
    // in pairs of k-tiles, operand B one k-tile at a time in its own four stages, and the loads
    // stay one per four MFMAs: an even iteration kt issues the second half of A's pair kt/2+1,
    // then (after its barrier) B of tile kt+3; the odd one B of tile kt+3, then the first half
    // of A's pair (kt-1)/2+2, whose double stage its barrier has just freed.  Issue order is
    // .. B(2j+1) | B(2j+2) A(j+1)a | A(j+1)b B(2j+3) | B(2j+4) A(j+2)a | ..: at the barrier of
    // an even iteration 2j (tile 2j+1 must have landed) the 12 loads after B(2j+1) may remain,
    // at the barrier of an odd one the 8 after A(j+1)b.
    auto k_loop_pair = [&](auto mv_tag) {
      constexpr int MV = decltype(mv_tag)::value;
      auto live = [](int o) { return MV == 4 || (MV == 2 && o <= 5); };
      auto iteration = [&](int kt, auto odd_tag) {
        constexpr bool ODD = decltype(odd_tag)::value != 0;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < 16; m += 2) {
          if (m < 4 * MV) mfma_one(0, m);
          if (m < 8) {
            if (live(m)) frag_op(1, kt, 1, m);
            if (live(m + 1)) frag_op(1, kt, 1, m + 1);
          }
          if (m < 4 * MV) mfma_one(0, m + 1);
          if ((m & 3) == 2) {
            if (ODD) issue_b(kt + 3, m >> 2);
            else issue_a_pair((kt >> 1) + 1, 4 + (m >> 2));
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        if (ODD) asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(12) lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < 16; m += 2) {
          if (m < 4 * MV) mfma_one(1, m);
          if (live(m >> 1)) frag_op(0, kt + 1, 0, m >> 1);
          if (m < 4 * MV) mfma_one(1, m + 1);
          if ((m & 3) == 2) {
            if (ODD) issue_a_pair((kt >> 1) + 2, m >> 2);
            else issue_b(kt + 3, m >> 2);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      };
      for (int kt = 0; kt < nk; kt += 2) {
        if (kt == kt_draw && tid == 0) my_ticket = atomicAdd(p.sched + queue, 1);
        iteration(kt, IntC<0>{});
        iteration(kt + 1, IntC<1>{});
      }
    };
    if (TR::RAGGED_K) {
      k_loop(IntC<4>{});
    } else {
      const int rows_left = row_end - (row0 + wm * 128);
      const int mv = rows_left > 64 ? 4 : (rows_left > 0 ? 2 : 0);
      if (mv == 4) k_loop_pair(IntC<4>{});
      else if (mv == 2) k_loop_pair(IntC<2>{});
      else k_loop_pair(IntC<0>{});
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    if (tid == 0) *next_q = my_ticket;
    __syncthreads();

    // the ring is free: decode the next tile and start its first loads, then store this one
    const int ep_e = e, ep_row0 = row0, ep_row_end = row_end, ep_n0 = n0, ep_piece = piece, ep_krange = krange;
    have = next_tile();

    // ---------------------------------------------------------------- epilogue
    // Each wavefront moves its 128x128 accumulators through a private LDS slab (outside the
    // tile ring, which already receives the next tile), 16 slabs per tile, and walks each slab
    // row-major so that global accesses are 16 bytes per lane and 128 bytes per row segment.
    // A slab is private to its wavefront and LDS executes a wavefront's accesses in order, so
    // no workgroup barrier is needed between the writes and the reads.
    // (three instances: a piece of a cut expert stores fp32 partial tiles, every other tile the final
    // result, either overwriting or adding to what is there; adding is an instance of its own so that
    // the loads of the old values are unconditional and stay where they are issued)
    auto epilogue = [&](auto partial_tag, auto rmw_tag) {
    constexpr bool PARTIAL = decltype(partial_tag)::value != 0;
    constexpr bool RMW_TAG = decltype(rmw_tag)::value != 0;
    float* stage = reinterpret_cast<float*>(smem + STAGING_OFF) + wave * (STAGING_WAVE_BYTES / 4);
    const int acc_col = lane & 31, acc_rg = lane >> 5;
    if (TR::DUAL) {
      // slab = 8 rows x 128 columns: both halves of a dual tile, so that a lane holds h1 and h3
      // (or dW1 and dW3) of the same position.  lanes: 8 per row (8 columns each).
      const int c8 = lane & 7, rl = lane >> 3;
      // WGD adding to existing gradients: the old values of a slab are fetched C_AHEAD slabs
      // before they are needed (clamped addresses), so that the read-modify-write does not
      // wait for memory once per slab
      constexpr int C_AHEAD = 3;
      constexpr bool rmw = MODE == WGD && !PARTIAL && RMW_TAG;
      uint4 old0[C_AHEAD + 1], old1[C_AHEAD + 1];
      auto old_fetch = [&](int sl) {
        int grow = ep_row0 + wm * 128 + (sl >> 2) * 32 + 8 * (sl & 3) + rl;
        int gcol = ep_n0 + wn * 64 + c8 * 8;
        if (grow > ep_row_end - 1) grow = ep_row_end - 1;
        if (gcol > p.N - 8) gcol = p.N - 8;
        const size_t idx = (size_t)ep_e * p.c_es + (size_t)grow * p.ldc + gcol;
        old0[sl % (C_AHEAD + 1)] = *reinterpret_cast<const uint4*>(p.C0 + idx);
        old1[sl % (C_AHEAD + 1)] = *reinterpret_cast<const uint4*>(p.C1 + idx);
      };
      if (rmw) {
#pragma unroll
        for (int sl = 0; sl < C_AHEAD; ++sl) old_fetch(sl);
      }
#pragma unroll
      for (int sl = 0; sl < 16; ++sl) {
        const int mi = sl >> 2, g = sl & 3;
        if (rmw && sl + C_AHEAD < 16) old_fetch(sl + C_AHEAD);
#pragma unroll
        for (int nj = 0; nj < 4; ++nj)
#pragma unroll
          for (int i = 0; i < 4; ++i) stage[(4 * acc_rg + i) * DPITCH + nj * 32 + acc_col] = acc[mi][nj][4 * g + i];
        __builtin_amdgcn_wave_barrier();
        const int grow = ep_row0 + wm * 128 + mi * 32 + 8 * g + rl;
        const int gcol = ep_n0 + wn * 64 + c8 * 8;
        const float* s1 = stage + rl * DPITCH + c8 * 8;
        const float* s3 = s1 + 64;
        float x1[8], x3[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) { x1[i] = s1[i]; x3[i] = s3[i]; }
        __builtin_amdgcn_wave_barrier();
        if (grow < ep_row_end && gcol < p.N) {
          if (MODE == UP) {
            const size_t idx = (size_t)grow * p.ldc + gcol;
            uint4 o1, o3, oa;
            uint32_t* w1 = reinterpret_cast<uint32_t*>(&o1);
            uint32_t* w3 = reinterpret_cast<uint32_t*>(&o3);
            uint32_t* wa = reinterpret_cast<uint32_t*>(&oa);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              w1[i] = pack_bf16x2(x1[2 * i], x1[2 * i + 1]);
              w3[i] = pack_bf16x2(x3[2 * i], x3[2 * i + 1]);
              wa[i] = pack_bf16x2(silu_f(x1[2 * i]) * x3[2 * i], silu_f(x1[2 * i + 1]) * x3[2 * i + 1]);
            }
            if (p.save_h) {
              store16(p.C0 + idx, o1);
              store16(p.C1 + idx, o3);
            }
            store16(p.C2 + idx, oa);
          } else if (PARTIAL) {   // WGD, one piece of a cut expert: fp32 partial tiles
            float* c0 = p.P0 + (size_t)ep_piece * p.p_stride + (size_t)grow * p.ldc + gcol;
            float* c1 = c0 + (size_t)p.M * p.N;
            *reinterpret_cast<float4*>(c0) = make_float4(x1[0], x1[1], x1[2], x1[3]);
            *reinterpret_cast<float4*>(c0 + 4) = make_float4(x1[4], x1[5], x1[6], x1[7]);
            *reinterpret_cast<float4*>(c1) = make_float4(x3[0], x3[1], x3[2], x3[3]);
            *reinterpret_cast<float4*>(c1 + 4) = make_float4(x3[4], x3[5], x3[6], x3[7]);
          } else {   // WGD: two weight-gradient outputs
            const size_t idx = (size_t)ep_e * p.c_es + (size_t)grow * p.ldc + gcol;
            bf16_t* c0 = p.C0 + idx;
            bf16_t* c1 = p.C1 + idx;
            if (rmw) {
              const uint4 q0 = old0[sl % (C_AHEAD + 1)], q1 = old1[sl % (C_AHEAD + 1)];
              const uint32_t* u0 = reinterpret_cast<const uint32_t*>(&q0);
              const uint32_t* u1 = reinterpret_cast<const uint32_t*>(&q1);
#pragma unroll
              for (int i = 0; i < 4; ++i) {
                x1[2 * i] += bf16lo(u0[i]); x1[2 * i + 1] += bf16hi(u0[i]);
                x3[2 * i] += bf16lo(u1[i]); x3[2 * i + 1] += bf16hi(u1[i]);
              }
            }
            uint4 o1, o3;
            uint32_t* w1 = reinterpret_cast<uint32_t*>(&o1);
            uint32_t* w3 = reinterpret_cast<uint32_t*>(&o3);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              w1[i] = pack_bf16x2(x1[2 * i], x1[2 * i + 1]);
              w3[i] = pack_bf16x2(x3[2 * i], x3[2 * i + 1]);
            }
            store16(c0, o1);
            store16(c1, o3);
          }
        }
      }
    } else {
      // slab = 16 rows x 64 columns; lanes: 8 per row (8 columns each), 8 rows per pass.
      // slab sl: accumulator block row mi = sl/4, row half h = (sl/2)%2, column pair np = sl%2.
      const int c8 = lane & 7;
      // DA: h1/h3 of a slab are fetched DA_AHEAD slabs before they are needed (clamped
      // addresses), so that their latency is hidden behind the slabs in between
      constexpr int DA_AHEAD = 3;
      uint4 pre1[DA_AHEAD + 1][2], pre3[DA_AHEAD + 1][2];
      auto da_fetch = [&](int sl) {
        const int mi = sl >> 2, h = (sl >> 1) & 1, np = sl & 1;
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
          int grow = ep_row0 + wm * 128 + mi * 32 + 16 * h + pass * 8 + (lane >> 3);
          int gcol = ep_n0 + wn * 128 + np * 64 + c8 * 8;
          if (grow > ep_row_end - 1) grow = ep_row_end - 1;
          if (gcol > p.N - 8) gcol = p.N - 8;
          const size_t idx = (size_t)grow * p.ldc + gcol;
          pre1[sl % (DA_AHEAD + 1)][pass] = *reinterpret_cast<const uint4*>(p.H1 + idx);
          pre3[sl % (DA_AHEAD + 1)][pass] = *reinterpret_cast<const uint4*>(p.H3 + idx);
        }
      };
      // WG and the router's dx adding to existing gradients: the same, with the old values
      constexpr bool rmw = (MODE == WG || MODE == RX) && !PARTIAL && RMW_TAG;
      auto old_fetch = [&](int sl) {
        const int mi = sl >> 2, h = (sl >> 1) & 1, np = sl & 1;
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
          int grow = ep_row0 + wm * 128 + mi * 32 + 16 * h + pass * 8 + (lane >> 3);
          int gcol = ep_n0 + wn * 128 + np * 64 + c8 * 8;
          if (grow > ep_row_end - 1) grow = ep_row_end - 1;
          if (gcol > p.N - 8) gcol = p.N - 8;
          const size_t idx = (MODE == WG ? (size_t)ep_e * p.c_es : (size_t)0) + (size_t)grow * p.ldc + gcol;
          pre1[sl % (DA_AHEAD + 1)][pass] = *reinterpret_cast<const uint4*>(p.C0 + idx);
        }
      };
      if (MODE == DA) {
#pragma unroll
        for (int sl = 0; sl < DA_AHEAD; ++sl) da_fetch(sl);
      }
      if (rmw) {
#pragma unroll
        for (int sl = 0; sl < DA_AHEAD; ++sl) old_fetch(sl);
      }
#pragma unroll
      for (int sl = 0; sl < 16; ++sl) {
        const int mi = sl >> 2, h = (sl >> 1) & 1, np = sl & 1;
        if (MODE == DA && sl + DA_AHEAD < 16) da_fetch(sl + DA_AHEAD);
        if (rmw && sl + DA_AHEAD < 16) old_fetch(sl + DA_AHEAD);
#pragma unroll
        for (int gg = 0; gg < 2; ++gg)
#pragma unroll
          for (int nn = 0; nn < 2; ++nn)
#pragma unroll
            for (int i = 0; i < 4; ++i)
              stage[(8 * gg + 4 * acc_rg + i) * SPITCH + nn * 32 + acc_col] = acc[mi][2 * np + nn][4 * (2 * h + gg) + i];
        __builtin_amdgcn_wave_barrier();
        float xs[2][8];
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
          const float* sp = stage + (pass * 8 + (lane >> 3)) * SPITCH + c8 * 8;
#pragma unroll
          for (int i = 0; i < 8; ++i) xs[pass][i] = sp[i];
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
          const int grow = ep_row0 + wm * 128 + mi * 32 + 16 * h + pass * 8 + (lane >> 3);
          const int gcol = ep_n0 + wn * 128 + np * 64 + c8 * 8;
          float* x = xs[pass];
          if (grow < ep_row_end && gcol < p.N) {
            if (MODE == DA) {
              const size_t idx = (size_t)grow * p.ldc + gcol;
              const uint4 q1 = pre1[sl % (DA_AHEAD + 1)][pass], q3 = pre3[sl % (DA_AHEAD + 1)][pass];
              const uint32_t* u1 = reinterpret_cast<const uint32_t*>(&q1);
              const uint32_t* u3 = reinterpret_cast<const uint32_t*>(&q3);
              float av[8], d1[8], d3[8];
#pragma unroll
              for (int i = 0; i < 8; ++i) {
                float z = (i & 1) ? bf16hi(u1[i >> 1]) : bf16lo(u1[i >> 1]);
                float gv = (i & 1) ? bf16hi(u3[i >> 1]) : bf16lo(u3[i >> 1]);
                float ds;
                float sl_ = silu_grad_f(z, &ds);
                av[i] = sl_ * gv;
                d1[i] = x[i] * gv * ds;
                d3[i] = x[i] * sl_;
              }
              uint4 oa, o1, o3;
              uint32_t* wa = reinterpret_cast<uint32_t*>(&oa);
              uint32_t* w1 = reinterpret_cast<uint32_t*>(&o1);
              uint32_t* w3 = reinterpret_cast<uint32_t*>(&o3);
#pragma unroll
              for (int i = 0; i < 4; ++i) {
                wa[i] = pack_bf16x2(av[2 * i], av[2 * i + 1]);
                w1[i] = pack_bf16x2(d1[2 * i], d1[2 * i + 1]);
                w3[i] = pack_bf16x2(d3[2 * i], d3[2 * i + 1]);
              }
              if (p.C0) store16(p.C0 + idx, oa);      // not stored when the forward's copy is at hand
              store16(p.C1 + idx, o1);
              store16(p.C2 + idx, o3);
            } else if (MODE == WG && PARTIAL) {   // one piece of a cut expert: fp32 partial tile
              float* c0 = p.P0 + (size_t)ep_piece * p.p_stride + (size_t)grow * p.ldc + gcol;
              *reinterpret_cast<float4*>(c0) = make_float4(x[0], x[1], x[2], x[3]);
              *reinterpret_cast<float4*>(c0 + 4) = make_float4(x[4], x[5], x[6], x[7]);
            } else if (MODE == RL || MODE == RW) {
              float* c0 = p.F0 + (size_t)(MODE == RW ? ep_e : ep_krange) * p.c_es + (size_t)grow * p.ldc + gcol;
              *reinterpret_cast<float4*>(c0) = make_float4(x[0], x[1], x[2], x[3]);
              *reinterpret_cast<float4*>(c0 + 4) = make_float4(x[4], x[5], x[6], x[7]);
            } else {
              const size_t idx = (MODE == WG ? (size_t)ep_e * p.c_es : (size_t)0) + (size_t)grow * p.ldc + gcol;
              bf16_t* c0 = p.C0 + idx;
              if (rmw) {
                const uint4 q0 = pre1[sl % (DA_AHEAD + 1)][pass];
                const uint32_t* u0 = reinterpret_cast<const uint32_t*>(&q0);
#pragma unroll
                for (int i = 0; i < 4; ++i) { x[2 * i] += bf16lo(u0[i]); x[2 * i + 1] += bf16hi(u0[i]); }
              }
              uint4 o;
              uint32_t* w = reinterpret_cast<uint32_t*>(&o);
#pragma unroll
              for (int i = 0; i < 4; ++i) w[i] = pack_bf16x2(x[2 * i], x[2 * i + 1]);
              store16(c0, o);
            }
          }
        }
      }
    }
    };
    if ((MODE == WG || MODE == WGD) && ep_piece >= 0) epilogue(IntC<1>{}, IntC<0>{});
    else if ((MODE == WG || MODE == WGD || MODE == RX) && p.accumulate) epilogue(IntC<0>{}, IntC<1>{});
    else epilogue(IntC<0>{}, IntC<0>{});
  }
}

template <int MODE>
__global__ __launch_bounds__(NT, 1) void gg_kernel(GArgs p) {
  gg_body<MODE>(p);
}

// Two grouped GEMMs that do not depend on each other in one launch: a workgroup that finds no tile
// of the first left goes on to the second at once, so the second fills the first one's tail (the
// last round of whole tiles, in which most CUs would idle) and one launch boundary goes away.
template <int M1, int M2>
__global__ __launch_bounds__(NT, 1) void gg_pair(GArgs p1, GArgs p2) {
  gg_body<M1>(p1);
  __syncthreads();          // the first GEMM's scheduler tables in LDS are rewritten by the second's set-up
  gg_body<M2>(p2);
}

__global__ void zero_words(int32_t* p, int n) {
  if ((int)threadIdx.x < n) p[threadIdx.x] = 0;
}

// Adds up the fp32 partial tiles of the experts that the weight-gradient kernel cut into pieces
// (plan[e] = (first piece << 8) | pieces), in piece order, and writes the bf16 gradient.
// Every block first lists the cut experts, then the grid walks the elements of all of them
// together (n_out outputs of mn elements each per expert), so that a single hot expert is
// reduced by the whole chip; with no cut expert every block exits after reading the plan.
__global__ __launch_bounds__(256) void wgrad_reduce(const int32_t* __restrict__ plan, int e_cnt,
                                                   const float* __restrict__ P0, long p_stride, long mn, int n_out,
                                                   bf16_t* __restrict__ C0, bf16_t* __restrict__ C1, long c_es,
                                                   int accumulate) {
  __shared__ int32_t list[MOE_MAX_LOCAL];   // the cut experts in ascending order: the same list in every block
  __shared__ uint8_t cut[MOE_MAX_LOCAL];
  __shared__ int n_cut;
  if (threadIdx.x == 0) n_cut = 0;
  for (int e = threadIdx.x; e < e_cnt; e += 256) cut[e] = (plan[e] & 255) > 1;
  __syncthreads();
  for (int e = threadIdx.x; e < e_cnt; e += 256)
    if (cut[e]) {
      int rank = 0;
      for (int j = 0; j < e; ++j) rank += cut[j];
      list[rank] = e;
      atomicAdd(&n_cut, 1);
    }
  __syncthreads();
  const long vecs = mn / 8;                       // mn is a multiple of 64 * 64
  const long per_e = vecs * n_out;
  const long total = per_e * n_cut;
  for (long g = (long)blockIdx.x * 256 + threadIdx.x; g < total; g += (long)gridDim.x * 256) {
    const int e = list[g / per_e];
    const long r = g % per_e;
    const int o = (int)(r / vecs);
    const long v = r - o * vecs;
    const int sp = plan[e];
    const int pieces = sp & 255;
    const float* base = P0 + (size_t)(sp >> 8) * p_stride + (size_t)o * mn + v * 8;
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    for (int c = 0; c < pieces; ++c) {
      const float* q = base + (size_t)c * p_stride;
      const float4 a = *reinterpret_cast<const float4*>(q), b = *reinterpret_cast<const float4*>(q + 4);
      acc[0] += a.x; acc[1] += a.y; acc[2] += a.z; acc[3] += a.w;
      acc[4] += b.x; acc[5] += b.y; acc[6] += b.z; acc[7] += b.w;
    }
    uint4* dst = reinterpret_cast<uint4*>((o ? C1 : C0) + (size_t)e * c_es + v * 8);
    if (accumulate) {
      const uint4 q0 = *dst;
      const uint32_t* u0 = reinterpret_cast<const uint32_t*>(&q0);
#pragma unroll
      for (int i = 0; i < 4; ++i) { acc[2 * i] += bf16lo(u0[i]); acc[2 * i + 1] += bf16hi(u0[i]); }
    }
    uint4 out;
    uint32_t* w = reinterpret_cast<uint32_t*>(&out);
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = pack_bf16x2(acc[2 * i], acc[2 * i + 1]);
    *dst = out;
  }
}

// ticket counters live in the 256 bytes of slack that moe_workspace_bytes adds after the
// activation scratch; each kernel of an entry point gets its own 8 (one per XCD)
inline int32_t* sched_area(void* ws, size_t scratch_bytes) {
  return reinterpret_cast<int32_t*>(static_cast<char*>(ws) + ((scratch_bytes + 255) & ~(size_t)255));
}

constexpr size_t WGRAD_PLAN_BYTES = 2 * MOE_MAX_LOCAL * 4;

template <int M1, int M2>
int launch_pair(const GArgs& a, const GArgs& b, int prof_id, hipStream_t s) {
  static bool attr_set[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MOE_EHIP;
  if (!attr_set[dev]) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&gg_pair<M1, M2>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            SMEM_BYTES) != hipSuccess)
      return MOE_EHIP;
    attr_set[dev] = true;
  }
  ProfScope prof(prof_id, s);
  hipLaunchKernelGGL((gg_pair<M1, M2>), dim3(device_cu_count()), dim3(NT), SMEM_BYTES, s, a, b);
  HIP_CHECK_LAUNCH();
  return MOE_OK;
}

template <int MODE>
int launch_gg(const GArgs& a, hipStream_t s) {
  // the LDS opt-in is a per-device attribute of the kernel
  static bool attr_set[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MOE_EHIP;
  if (!attr_set[dev]) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&gg_kernel<MODE>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            SMEM_BYTES) != hipSuccess)
      return MOE_EHIP;
    attr_set[dev] = true;
  }
  int grid = device_cu_count();
  ProfScope prof(MODE == RL ? MOE_K_ROUTER_FWD : MODE == RW ? MOE_K_ROUTER_DW : MODE == RX ? MOE_K_ROUTER_DX : MOE_K_UP + MODE, s);
  hipLaunchKernelGGL(gg_kernel<MODE>, dim3(grid), dim3(NT), SMEM_BYTES, s, a);
  HIP_CHECK_LAUNCH();
  return MOE_OK;
}

}  // namespace

int launch_expert_fwd_bf16(const void* xp, int cap, int d, int f, int e_cnt, const int32_t* offsets,
                           const void* w1, const void* w3, const void* w2, void* h1, void* h3, void* a_out, void* o,
                           void* a_ws, hipStream_t s) {
  if (cap == 0 || e_cnt == 0) return MOE_OK;
  bf16_t* act = a_out ? (bf16_t*)a_out : (bf16_t*)a_ws;
  int32_t* sched = sched_area(a_ws, (size_t)cap * f * 2);
  hipLaunchKernelGGL(zero_words, dim3(1), dim3(64), 0, s, sched, 16);
  HIP_CHECK_LAUNCH();
  GArgs u = {};
  u.A0 = u.A1 = (const bf16_t*)xp; u.lda = d;
  u.B0 = (const bf16_t*)w1; u.B1 = (const bf16_t*)w3; u.ldb = f; u.b_es = (long)d * f;
  u.C0 = (bf16_t*)h1; u.C1 = (bf16_t*)h3; u.C2 = act; u.ldc = f;
  u.off = offsets; u.sched = sched; u.e_cnt = e_cnt; u.N = f; u.K = d; u.save_h = (h1 && h3) ? 1 : 0;
  int rc = launch_gg<UP>(u, s);
  if (rc) return rc;
  GArgs w = {};
  w.A0 = w.A1 = act; w.lda = f;
  w.B0 = w.B1 = (const bf16_t*)w2; w.ldb = d; w.b_es = (long)f * d;
  w.C0 = (bf16_t*)o; w.ldc = d;
  w.off = offsets; w.sched = sched + 8; w.e_cnt = e_cnt; w.N = d; w.K = f;
  return launch_gg<DOWN>(w, s);
}

int launch_expert_bwd_bf16(const void* xp, const void* h1, const void* h3, const void* a_in, const void* d_o, int cap,
                           int d, int f, int e_cnt, const int32_t* offsets, const void* w1,
                           const void* w3, const void* w2, void* dxp, void* dw1, void* dw3, void* dw2,
                           int accumulate, void* ws, hipStream_t s) {
  if (e_cnt == 0) return MOE_OK;
  bf16_t* a = (bf16_t*)ws;
  bf16_t* dh1 = a + (size_t)cap * f;
  bf16_t* dh3 = dh1 + (size_t)cap * f;
  int32_t* sched = sched_area(ws, 3 * (size_t)cap * f * 2);
  int32_t* plans = sched + 64;                                   // two plans of MOE_MAX_LOCAL words
  float* partials = reinterpret_cast<float*>(reinterpret_cast<char*>(sched) + 256 + WGRAD_PLAN_BYTES);
  const size_t split_bytes = wgrad_split_bytes(d, f);
  const long mn = (long)d * f;
  hipLaunchKernelGGL(zero_words, dim3(1), dim3(64), 0, s, sched, 32);
  HIP_CHECK_LAUNCH();
  GArgs g = {};   // dA = d_o W2^T, epilogue -> a, dH1, dH3
  g.A0 = g.A1 = (const bf16_t*)d_o; g.lda = d;
  g.B0 = g.B1 = (const bf16_t*)w2; g.ldb = d; g.b_es = (long)f * d;
  g.C0 = a_in ? nullptr : a; g.C1 = dh1; g.C2 = dh3; g.ldc = f;
  g.H1 = (const bf16_t*)h1; g.H3 = (const bf16_t*)h3;
  g.off = offsets; g.sched = sched; g.e_cnt = e_cnt; g.N = f; g.K = d;
  GArgs x = {};   // dxp = dH1 W1^T + dH3 W3^T
  x.A0 = dh1; x.A1 = dh3; x.lda = f;
  x.B0 = (const bf16_t*)w1; x.B1 = (const bf16_t*)w3; x.ldb = f; x.b_es = (long)d * f;
  x.C0 = (bf16_t*)dxp; x.ldc = d;
  x.off = offsets; x.sched = sched + 8; x.e_cnt = e_cnt; x.N = d; x.K = f;
  GArgs w = {};   // dW2 = a^T d_o
  w.A0 = w.A1 = a_in ? (const bf16_t*)a_in : a; w.lda = f;
  w.B0 = w.B1 = (const bf16_t*)d_o; w.ldb = d;
  w.C0 = (bf16_t*)dw2; w.ldc = d; w.c_es = (long)f * d;
  w.off = offsets; w.sched = sched + 16; w.e_cnt = e_cnt; w.M = f; w.N = d; w.accumulate = accumulate;
  w.P0 = partials; w.p_stride = mn; w.split_budget = (int)(split_bytes / (mn * 4)); w.plan = plans;
  GArgs v = {};   // dW1|dW3 = xp^T [dH1|dH3]
  v.A0 = v.A1 = (const bf16_t*)xp; v.lda = d;
  v.B0 = dh1; v.B1 = dh3; v.ldb = f;
  v.C0 = (bf16_t*)dw1; v.C1 = (bf16_t*)dw3; v.ldc = f; v.c_es = (long)d * f;
  v.off = offsets; v.sched = sched + 24; v.e_cnt = e_cnt; v.M = d; v.N = f; v.accumulate = accumulate;
  v.P0 = partials; v.p_stride = 2 * mn; v.split_budget = (int)(split_bytes / (2 * mn * 4)); v.plan = plans + MOE_MAX_LOCAL;
  // Order and pairing.  dW2 needs a and d_o, dX and dW1|dW3 need what dA's epilogue writes (dH1, dH3).  With the
  // forward's a at hand dA and dW2 are independent, dX and dW1|dW3 always are, and independent GEMMs may share a
  // launch (gg_pair).  That pays while the first GEMM's tail -- its last round of whole tiles -- is a visible part
  // of it; the second GEMM's workgroups then start out of step, and the panels that the 32 workgroups of an XCD
  // would share through their L2 while walking k together are fetched more often (a quarter more L2 misses
  // measured).  Measured break-even: about a dozen rounds of tiles per workgroup in the first GEMM (a pair gains
  // 2.5-4 % at 8-9 rounds and loses 1-2.5 % at 29-31), counted from the capacity bound since the row counts are
  // on the device.  The fp32 partial tiles of cut experts are one buffer: dW2's are added up before dW1|dW3
  // writes its own.
  int rc;
  const int red_grid = 4 * device_cu_count();
  const auto rounds = [&](int n_cols) {     // tiles of a ragged-M GEMM with n_cols output columns, per workgroup
    const long long m_tiles = (cap + BM - 1) / BM + e_cnt / 2;
    return m_tiles * ((n_cols + BN - 1) / BN) / device_cu_count();
  };
  constexpr int PAIR_MAX_ROUNDS = 12;
  if (cap == 0) {            // no rows at all: only the gradients are written (zeros unless accumulating)
    if ((rc = launch_gg<WG>(w, s))) return rc;
  } else if (a_in && rounds(f) <= PAIR_MAX_ROUNDS) {
    if ((rc = launch_pair<DA, WG>(g, w, MOE_K_DA_WG, s))) return rc;
  } else {
    if ((rc = launch_gg<DA>(g, s))) return rc;
    if ((rc = launch_gg<WG>(w, s))) return rc;
  }
  {
    ProfScope prof(MOE_K_WGRAD_REDUCE, s);
    hipLaunchKernelGGL(wgrad_reduce, dim3(red_grid), dim3(256), 0, s, plans, e_cnt, partials, mn, mn, 1, (bf16_t*)dw2,
                       (bf16_t*)dw2, mn, accumulate);
  }
  HIP_CHECK_LAUNCH();
  if (cap == 0) {
    if ((rc = launch_gg<WGD>(v, s))) return rc;
  } else if (rounds(d) <= PAIR_MAX_ROUNDS) {
    if ((rc = launch_pair<DX, WGD>(x, v, MOE_K_DX_WGD, s))) return rc;
  } else {
    if ((rc = launch_gg<DX>(x, s))) return rc;
    if ((rc = launch_gg<WGD>(v, s))) return rc;
  }
  {
    ProfScope prof(MOE_K_WGRAD_REDUCE, s);
    hipLaunchKernelGGL(wgrad_reduce, dim3(red_grid), dim3(256), 0, s, plans + MOE_MAX_LOCAL, e_cnt, partials, 2 * mn, mn, 2,
                       (bf16_t*)dw1, (bf16_t*)dw3, mn, accumulate);
  }
  HIP_CHECK_LAUNCH();
  return MOE_OK;
}

// ---- trainable router on the matrix cores (bf16, E % 64 == 0, d % 64 == 0) ----------------
// ws layout: [0,256) ticket counters; then dl as bf16 [T,E]; then the fp32 chunk sums [S,d,E].
// Into how many chunks of tokens the router's weight gradient is cut: the split whose schedule is
// shortest, counted in k-tiles per workgroup: rounds of the chip's CUs times (k-tiles per chunk +
// what a tile costs besides its k loop, about 16 k-tiles for its first loads and its fp32 stores).
constexpr int SPLIT_OVERHEAD_KTILES = 16;
int router_dw_splits(int T, int d, int E) {
  const long long tiles = (long long)((d + BM - 1) / BM) * ((E + BN - 1) / BN);
  const int cus = device_cu_count();
  const int max_by_rows = (T + 4 * BK - 1) / (4 * BK);      // at least four k-tiles per chunk
  int best = 1;
  long long best_cost = -1;
  for (int s = 1; s <= 32 && s <= max_by_rows; ++s) {
    const long long rounds = (tiles * s + cus - 1) / cus;
    const long long cost = rounds * (((T + s - 1) / s + BK - 1) / BK + SPLIT_OVERHEAD_KTILES);
    if (best_cost < 0 || cost < best_cost) { best = s; best_cost = cost; }
  }
  return best;
}

// Into how many ranges the router's forward GEMM cuts its contraction over d: with few experts
// the [T, E] logits are fewer tiles than the chip has CUs, so each tile's k loop is shared out.
// The same cost model as above, in pairs of k-tiles (a range is a whole number of pairs).
int router_fwd_splits(int T, int d, int E) {
  const long long tiles = (long long)((T + BM - 1) / BM) * ((E + BN - 1) / BN);
  const int cus = device_cu_count();
  const int pairs = d / (2 * BK);
  int best = 1;
  long long best_cost = -1;
  for (int s = 1; s <= 8 && s <= pairs / 4; ++s) {
    const long long rounds = (tiles * s + cus - 1) / cus;
    const long long cost = rounds * (2 * ((pairs + s - 1) / s) + SPLIT_OVERHEAD_KTILES);
    if (best_cost < 0 || cost < best_cost) { best = s; best_cost = cost; }
  }
  // no empty range: as many ranges as the rounded-up range length needs
  const int per = (pairs + best - 1) / best;
  return (pairs + per - 1) / per;
}

// partials: fp32 [splits, T, E] when the contraction is cut (splits > 1), else unused; the caller adds them up
int launch_router_fwd_bf16(const void* x, const void* wr, int T, int d, int E, float* logits, float* partials,
                           int splits, int32_t* sched, hipStream_t s) {
  if (T == 0) return MOE_OK;
  hipLaunchKernelGGL(zero_words, dim3(1), dim3(64), 0, s, sched, 8);
  HIP_CHECK_LAUNCH();
  GArgs g = {};
  g.A0 = g.A1 = (const bf16_t*)x; g.lda = d;
  g.B0 = g.B1 = (const bf16_t*)wr; g.ldb = E; g.b_es = 0;
  g.F0 = splits > 1 ? partials : logits; g.ldc = E; g.c_es = (long)T * E;
  g.off = nullptr; g.rows = T; g.chunk = T; g.sched = sched; g.e_cnt = 1; g.N = E;
  const int pairs = d / (2 * BK);
  g.ksplit = splits; g.k_total = d; g.K = splits > 1 ? (pairs + splits - 1) / splits * 2 * BK : d;
  return launch_gg<RL>(g, s);
}

int launch_router_dw_bf16(const void* x, const void* dl_bf16, int T, int d, int E, float* partials, int splits,
                          int32_t* sched, hipStream_t s) {
  GArgs g = {};
  g.A0 = g.A1 = (const bf16_t*)x; g.lda = d;
  g.B0 = g.B1 = (const bf16_t*)dl_bf16; g.ldb = E;
  g.F0 = partials; g.ldc = E; g.c_es = (long)d * E;
  g.off = nullptr; g.rows = T; g.chunk = (((T + splits - 1) / splits + BK - 1) / BK) * BK;
  g.sched = sched; g.e_cnt = splits; g.M = d; g.N = E;
  return launch_gg<RW>(g, s);
}

int launch_router_dx_bf16(const void* dl_bf16, const void* wr, int T, int d, int E, void* dx, int accumulate,
                          int32_t* sched, hipStream_t s) {
  GArgs g = {};
  g.A0 = g.A1 = (const bf16_t*)dl_bf16; g.lda = E;
  g.B0 = g.B1 = (const bf16_t*)wr; g.ldb = E; g.b_es = 0;
  g.C0 = (bf16_t*)dx; g.ldc = d;
  g.off = nullptr; g.rows = T; g.chunk = T; g.sched = sched; g.e_cnt = 1; g.N = d; g.K = E; g.accumulate = accumulate;
  return launch_gg<RX>(g, s);
}

int launch_zero_words(int32_t* p, int n, hipStream_t s) {
  hipLaunchKernelGGL(zero_words, dim3(1), dim3(64), 0, s, p, n);
  HIP_CHECK_LAUNCH();
  return MOE_OK;
}

// fp32 partial tiles for weight gradients cut along the rows: room for up to 32 pieces of the
// larger (two-output) gradient, at most 512 MB
size_t wgrad_split_bytes(int d, int f) {
  const size_t piece = 2 * (size_t)d * f * 4;
  size_t b = 32 * piece;
  const size_t cap = (size_t)512 << 20;
  if (b > cap) b = cap / piece * piece;
  return b;
}
size_t expert_bwd_extra_ws_bytes(int d, int f) { return 256 + WGRAD_PLAN_BYTES + wgrad_split_bytes(d, f); }
