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
// Tiling: 256x256x64 block tile, 256 threads = 4 wavefronts in a 2x2 grid, 128x128 per
// wavefront = 4x4 MFMA blocks (256 accumulator registers), one wavefront per SIMD.
// Operand tiles live in LDS as [row][64 k] with a 144-byte row pitch (conflict-free 16-byte
// fragment reads), double buffered: global loads of tile kt+1 are in flight while tile kt
// feeds the MFMAs; one barrier per k-tile.  Operands whose contraction index is not the
// contiguous one in memory (weights in the forward, everything in the weight gradients)
// are transposed in registers (8x8 bf16 blocks) on their way into LDS.
// Workgroups are persistent and walk a device-built tile list (row counts never visit the
// host); the list is ordered so that the tiles resident on one XCD share weight panels.
#include "common.h"
#include "kernels.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int NT = 256;                 // threads
constexpr int PITCH = 144;              // bytes per LDS tile row (64 bf16 + 16 B pad)
constexpr int A_BYTES = BM * PITCH;     // 36864
constexpr int STAGE_BYTES = (BM + BN) * PITCH;
constexpr int TILE_LDS = 2 * STAGE_BYTES;          // 147456
constexpr int SPITCH = 132;             // floats per staging row (128 + 4 pad)
constexpr int SMEM_BYTES = TILE_LDS + (MOE_MAX_LOCAL + 1) * 4;

enum { UP = 0, DOWN = 1, DA = 2, DX = 3, WG = 4, WGD = 5 };

struct GArgs {
  const bf16_t* A0; const bf16_t* A1;     // A sources (A1: second K segment of DX)
  const bf16_t* B0; const bf16_t* B1;     // B sources (B1: second half of a dual tile / second K segment)
  long lda, ldb;                          // leading dimensions (elements)
  long b_es;                              // expert stride of B (elements); 0 for row-indexed B
  bf16_t* C0; bf16_t* C1; bf16_t* C2;     // outputs
  long ldc, c_es;
  const bf16_t* H1; const bf16_t* H3;     // DA epilogue inputs
  const int32_t* off;
  int e_cnt;
  int M;                                  // WG/WGD: rows of the output (d or f)
  int N;                                  // output columns (per half for dual tiles)
  int K;                                  // contraction length per segment (ragged-M modes)
  int accumulate;
  int save_h;
};

template <int MODE> struct Traits {
  static constexpr bool A_TRANS = MODE == WG || MODE == WGD;
  static constexpr bool B_TRANS = MODE == UP || MODE == DOWN || MODE == WG || MODE == WGD;
  static constexpr bool DUAL = MODE == UP || MODE == WGD;
  static constexpr bool RAGGED_K = MODE == WG || MODE == WGD;
  static constexpr int BN_EFF = DUAL ? BN / 2 : BN;   // output columns covered per tile
};

__device__ __forceinline__ uint4 ld16(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }

// 8x8 transpose of bf16: r[i] holds 8 consecutive n at k=i; out[j] holds 8 consecutive k at n=j
__device__ __forceinline__ void transpose8x8(const uint4 (&r)[8], uint4 (&out)[8]) {
  const uint32_t* rv = reinterpret_cast<const uint32_t*>(r);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    uint32_t o[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      uint32_t lo = rv[(2 * p) * 4 + j / 2], hi = rv[(2 * p + 1) * 4 + j / 2];
      o[p] = (j & 1) ? ((lo >> 16) | (hi & 0xFFFF0000u)) : ((lo & 0xFFFFu) | (hi << 16));
    }
    out[j] = make_uint4(o[0], o[1], o[2], o[3]);
  }
}

// ---- K-contiguous operand: source rows are tile rows, 64 k = 128 contiguous bytes -------
struct KcLoader {
  const bf16_t* base;      // &src[row_first * ld]
  int roff[8];             // element offset of this thread's 8 rows (clamped into range)
  int kc;                  // 16-byte chunk within the k-tile
  int r_in;
  __device__ __forceinline__ void setup(const bf16_t* b, long ld, int rows_valid) {
    base = b;
    kc = threadIdx.x & 7;
    r_in = threadIdx.x >> 3;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int r = i * 32 + r_in;
      if (r > rows_valid - 1) r = rows_valid - 1;   // tail rows re-read the last valid row; never stored
      roff[i] = (int)(r * ld);
    }
  }
  __device__ __forceinline__ void g2r(uint4 (&v)[8], int k0) const {
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = ld16(base + roff[i] + k0 + kc * 8);
  }
  __device__ __forceinline__ void r2s(const uint4 (&v)[8], char* lds) const {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      *reinterpret_cast<uint4*>(lds + (i * 32 + r_in) * PITCH + kc * 16) = v[i];
  }
};

// ---- transposed operand: source is [k][n] with n contiguous; tile rows are n ------------
struct TrLoader {
  const bf16_t* base;      // &src[n_first] of this thread's 8-wide n group (already offset), or null
  long ld;
  int q;                   // k group (8 k rows) of this thread
  int g;                   // n group (8 columns) of this thread, 0..31
  bool n_ok;
  __device__ __forceinline__ void setup(const bf16_t* b0, const bf16_t* b1, bool dual, long ld_, int n0, int n_lim) {
    q = threadIdx.x & 7;
    g = threadIdx.x >> 3;
    ld = ld_;
    int gg = g;
    const bf16_t* b = b0;
    if (dual && g >= 16) { gg = g - 16; b = b1; }
    int n = n0 + gg * 8;
    n_ok = n < n_lim;
    base = b + (n_ok ? n : 0);
  }
  // k0 = first source row of the k-tile; rows >= k_lim read as zero
  __device__ __forceinline__ void g2r(uint4 (&v)[8], long k0, long k_lim) const {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      long kk = k0 + q * 8 + i;
      if (n_ok && kk < k_lim) v[i] = ld16(base + kk * ld);
      else v[i] = make_uint4(0, 0, 0, 0);
    }
  }
  __device__ __forceinline__ void r2s(const uint4 (&v)[8], char* lds) const {
    uint4 t[8];
    transpose8x8(v, t);
#pragma unroll
    for (int j = 0; j < 8; ++j)
      *reinterpret_cast<uint4*>(lds + (g * 8 + j) * PITCH + q * 16) = t[j];
  }
};

template <int MODE>
__global__ __launch_bounds__(NT, 1) void gg_kernel(GArgs p) {
  using TR = Traits<MODE>;
  extern __shared__ __align__(16) char smem[];
  int32_t* tile_start = reinterpret_cast<int32_t*>(smem + TILE_LDS);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int e_cnt = p.e_cnt;

  const int n_tiles_n = (p.N + TR::BN_EFF - 1) / TR::BN_EFF;
  int total;
  int wg_tiles_per_e = 0, wg_mt = 0;
  if (TR::RAGGED_K) {
    wg_mt = (p.M + BM - 1) / BM;
    wg_tiles_per_e = wg_mt * n_tiles_n;
    total = wg_tiles_per_e * e_cnt;
  } else {
    // tile_start[e] = number of tiles before expert e
    for (int e = tid; e < e_cnt; e += NT) {
      int rows = p.off[e + 1] - p.off[e];
      tile_start[e] = ((rows + BM - 1) / BM) * n_tiles_n;
    }
    __syncthreads();
    if (tid == 0) {
      int run = 0;
      for (int e = 0; e < e_cnt; ++e) {
        int v = tile_start[e];
        tile_start[e] = run;
        run += v;
      }
      tile_start[e_cnt] = run;
    }
    __syncthreads();
    total = tile_start[e_cnt];
  }

  // XCD-aware walk: workgroup b runs on XCD b%8; give each XCD a contiguous run of tiles
  const int G = gridDim.x;
  const bool xcd_ok = (G % 8) == 0;
  const int b = blockIdx.x;
  const int first = xcd_ok ? (b % 8) * (G / 8) + b / 8 : b;

  for (int L = first; L < total; L += G) {
    // ---------------------------------------------------------------- decode tile
    int e, lo, hi, mt, nt;
    if (TR::RAGGED_K) {
      e = L / wg_tiles_per_e;
      int li = L - e * wg_tiles_per_e;
      mt = li % wg_mt;
      nt = li / wg_mt;
      lo = p.off[e];
      hi = p.off[e + 1];
    } else {
      int a = 0, c = e_cnt;                    // largest e with tile_start[e] <= L
      while (c - a > 1) {
        int mid = (a + c) >> 1;
        if (tile_start[mid] <= L) a = mid; else c = mid;
      }
      e = a;
      lo = p.off[e];
      hi = p.off[e + 1];
      int mte = (hi - lo + BM - 1) / BM;
      int li = L - tile_start[e];
      mt = li % mte;
      nt = li / mte;
    }
    const int n0 = nt * TR::BN_EFF;

    int nk0, nk;            // k-tiles in segment 0 / in total
    int row0;               // first output row (global row for ragged-M, i for WG)
    int row_end;            // one past the last valid output row
    KcLoader la_kc, lb_kc;
    TrLoader la_tr, lb_tr;
    if (TR::RAGGED_K) {
      row0 = mt * BM;
      row_end = p.M;
      nk0 = nk = (hi - lo + BK - 1) / BK;
      la_tr.setup(p.A0, p.A0, false, p.lda, row0, p.M);
      lb_tr.setup(p.B0, p.B1, TR::DUAL, p.ldb, n0, p.N);
    } else {
      row0 = lo + mt * BM;
      row_end = hi;
      nk0 = p.K / BK;
      nk = MODE == DX ? 2 * nk0 : nk0;
      la_kc.setup(p.A0 + (size_t)row0 * p.lda, p.lda, hi - row0);
      if (TR::B_TRANS) lb_tr.setup(p.B0 + (size_t)e * p.b_es, p.B1 + (size_t)e * p.b_es, TR::DUAL, p.ldb, n0, p.N);
      else lb_kc.setup(p.B0 + (size_t)e * p.b_es + (size_t)n0 * p.ldb, p.ldb, p.N - n0);
    }

    auto g2r = [&](uint4 (&va)[8], uint4 (&vb)[8], int kt) {
      if (TR::RAGGED_K) {
        la_tr.g2r(va, (long)lo + (long)kt * BK, hi);
        lb_tr.g2r(vb, (long)lo + (long)kt * BK, hi);
      } else {
        const bool seg1 = MODE == DX && kt >= nk0;
        const int k0 = (seg1 ? kt - nk0 : kt) * BK;
        if (seg1) {
          // second K segment: same row layout, other pointers
          const long da = p.A1 - p.A0, db = p.B1 - p.B0;
#pragma unroll
          for (int i = 0; i < 8; ++i) va[i] = ld16(la_kc.base + da + la_kc.roff[i] + k0 + la_kc.kc * 8);
#pragma unroll
          for (int i = 0; i < 8; ++i) vb[i] = ld16(lb_kc.base + db + lb_kc.roff[i] + k0 + lb_kc.kc * 8);
        } else {
          la_kc.g2r(va, k0);
          if (TR::B_TRANS) lb_tr.g2r(vb, k0, p.K);
          else lb_kc.g2r(vb, k0);
        }
      }
    };
    auto r2s = [&](const uint4 (&va)[8], const uint4 (&vb)[8], int stage) {
      char* sa = smem + stage * STAGE_BYTES;
      char* sb = sa + A_BYTES;
      if (TR::A_TRANS) la_tr.r2s(va, sa); else la_kc.r2s(va, sa);
      if (TR::B_TRANS) lb_tr.r2s(vb, sb); else lb_kc.r2s(vb, sb);
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // LDS row of this lane's fragment for MFMA block mi / nj
    const int frag_row = lane & 31, frag_kc = lane >> 5;
    int a_row[4], b_row[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      a_row[i] = wm * 128 + i * 32 + frag_row;
      b_row[i] = (TR::DUAL ? (i < 2 ? 0 : 128) + wn * 64 + (i & 1) * 32 : wn * 128 + i * 32) + frag_row;
    }

    uint4 va[8], vb[8];
    if (nk > 0) {
      g2r(va, vb, 0);
      r2s(va, vb, 0);
    }
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
      const bool more = kt + 1 < nk;
      if (more) g2r(va, vb, kt + 1);
      const char* sa = smem + (kt & 1) * STAGE_BYTES;
      const char* sb = sa + A_BYTES;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        bf16x8 fa[4], fb[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          fa[i] = *reinterpret_cast<const bf16x8*>(sa + a_row[i] * PITCH + (ks * 2 + frag_kc) * 16);
          fb[i] = *reinterpret_cast<const bf16x8*>(sb + b_row[i] * PITCH + (ks * 2 + frag_kc) * 16);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
      }
      if (more) r2s(va, vb, (kt + 1) & 1);
      __syncthreads();
    }

    // ---------------------------------------------------------------- epilogue
    // Each wavefront stages one 32-row slab of its 128x128 tile in LDS as fp32, then walks it
    // row-major so that global accesses are 16 bytes per lane and contiguous along rows.
    float* stage = reinterpret_cast<float*>(smem) + wave * (32 * SPITCH);
    const int acc_col = lane & 31, acc_rg = lane >> 5;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
      for (int nj = 0; nj < 4; ++nj)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int rl = 8 * (r >> 2) + 4 * acc_rg + (r & 3);
          stage[rl * SPITCH + nj * 32 + acc_col] = acc[mi][nj][r];
        }
      __syncthreads();
      const int slab_row0 = row0 + wm * 128 + mi * 32;
      if (TR::DUAL) {
        // lanes: 8 per row (8 columns each), 8 rows per pass
        const int c8 = lane & 7;
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
          const int rl = pass * 8 + (lane >> 3);
          const int grow = slab_row0 + rl;
          const int gcol = n0 + wn * 64 + c8 * 8;
          const float* s1 = stage + rl * SPITCH + c8 * 8;
          const float* s3 = s1 + 64;
          float x1[8], x3[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) { x1[i] = s1[i]; x3[i] = s3[i]; }
          if (grow < row_end && gcol < p.N) {
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
                *reinterpret_cast<uint4*>(p.C0 + idx) = o1;
                *reinterpret_cast<uint4*>(p.C1 + idx) = o3;
              }
              *reinterpret_cast<uint4*>(p.C2 + idx) = oa;
            } else {   // WGD: two weight-gradient outputs
              const size_t idx = (size_t)e * p.c_es + (size_t)grow * p.ldc + gcol;
              bf16_t* c0 = p.C0 + idx;
              bf16_t* c1 = p.C1 + idx;
              if (p.accumulate) {
                uint4 q0 = *reinterpret_cast<const uint4*>(c0), q1 = *reinterpret_cast<const uint4*>(c1);
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
              *reinterpret_cast<uint4*>(c0) = o1;
              *reinterpret_cast<uint4*>(c1) = o3;
            }
          }
        }
      } else {
        // lanes: 16 per row (8 columns each), 4 rows per pass
        const int c8 = lane & 15;
#pragma unroll
        for (int pass = 0; pass < 8; ++pass) {
          const int rl = pass * 4 + (lane >> 4);
          const int grow = slab_row0 + rl;
          const int gcol = n0 + wn * 128 + c8 * 8;
          const float* sp = stage + rl * SPITCH + c8 * 8;
          float x[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) x[i] = sp[i];
          if (grow < row_end && gcol < p.N) {
            if (MODE == DA) {
              const size_t idx = (size_t)grow * p.ldc + gcol;
              uint4 q1 = *reinterpret_cast<const uint4*>(p.H1 + idx), q3 = *reinterpret_cast<const uint4*>(p.H3 + idx);
              const uint32_t* u1 = reinterpret_cast<const uint32_t*>(&q1);
              const uint32_t* u3 = reinterpret_cast<const uint32_t*>(&q3);
              float av[8], d1[8], d3[8];
#pragma unroll
              for (int i = 0; i < 8; ++i) {
                float z = (i & 1) ? bf16hi(u1[i >> 1]) : bf16lo(u1[i >> 1]);
                float g = (i & 1) ? bf16hi(u3[i >> 1]) : bf16lo(u3[i >> 1]);
                float ds;
                float sl = silu_grad_f(z, &ds);
                av[i] = sl * g;
                d1[i] = x[i] * g * ds;
                d3[i] = x[i] * sl;
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
              *reinterpret_cast<uint4*>(p.C0 + idx) = oa;
              *reinterpret_cast<uint4*>(p.C1 + idx) = o1;
              *reinterpret_cast<uint4*>(p.C2 + idx) = o3;
            } else {
              const size_t idx = (MODE == WG ? (size_t)e * p.c_es : (size_t)0) + (size_t)grow * p.ldc + gcol;
              bf16_t* c0 = p.C0 + idx;
              if (MODE == WG && p.accumulate) {
                uint4 q0 = *reinterpret_cast<const uint4*>(c0);
                const uint32_t* u0 = reinterpret_cast<const uint32_t*>(&q0);
#pragma unroll
                for (int i = 0; i < 4; ++i) { x[2 * i] += bf16lo(u0[i]); x[2 * i + 1] += bf16hi(u0[i]); }
              }
              uint4 o;
              uint32_t* w = reinterpret_cast<uint32_t*>(&o);
#pragma unroll
              for (int i = 0; i < 4; ++i) w[i] = pack_bf16x2(x[2 * i], x[2 * i + 1]);
              *reinterpret_cast<uint4*>(c0) = o;
            }
          }
        }
      }
      __syncthreads();
    }
  }
}

template <int MODE>
int launch_gg(const GArgs& a, hipStream_t s) {
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&gg_kernel<MODE>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            SMEM_BYTES) != hipSuccess)
      return MOE_EHIP;
    attr_set = true;
  }
  int grid = device_cu_count();
  ProfScope prof(MOE_K_UP + MODE, s);
  hipLaunchKernelGGL(gg_kernel<MODE>, dim3(grid), dim3(NT), SMEM_BYTES, s, a);
  HIP_CHECK_LAUNCH();
  return MOE_OK;
}

}  // namespace

int launch_expert_fwd_bf16(const void* xp, int cap, int d, int f, int e_cnt, const int32_t* offsets,
                           const void* w1, const void* w3, const void* w2, void* h1, void* h3, void* o,
                           void* a_ws, hipStream_t s) {
  if (cap == 0 || e_cnt == 0) return MOE_OK;
  GArgs u = {};
  u.A0 = u.A1 = (const bf16_t*)xp; u.lda = d;
  u.B0 = (const bf16_t*)w1; u.B1 = (const bf16_t*)w3; u.ldb = f; u.b_es = (long)d * f;
  u.C0 = (bf16_t*)h1; u.C1 = (bf16_t*)h3; u.C2 = (bf16_t*)a_ws; u.ldc = f;
  u.off = offsets; u.e_cnt = e_cnt; u.N = f; u.K = d; u.save_h = (h1 && h3) ? 1 : 0;
  int rc = launch_gg<UP>(u, s);
  if (rc) return rc;
  GArgs w = {};
  w.A0 = w.A1 = (const bf16_t*)a_ws; w.lda = f;
  w.B0 = w.B1 = (const bf16_t*)w2; w.ldb = d; w.b_es = (long)f * d;
  w.C0 = (bf16_t*)o; w.ldc = d;
  w.off = offsets; w.e_cnt = e_cnt; w.N = d; w.K = f;
  return launch_gg<DOWN>(w, s);
}

int launch_expert_bwd_bf16(const void* xp, const void* h1, const void* h3, const void* d_o, int cap,
                           int d, int f, int e_cnt, const int32_t* offsets, const void* w1,
                           const void* w3, const void* w2, void* dxp, void* dw1, void* dw3, void* dw2,
                           int accumulate, void* ws, hipStream_t s) {
  if (e_cnt == 0) return MOE_OK;
  bf16_t* a = (bf16_t*)ws;
  bf16_t* dh1 = a + (size_t)cap * f;
  bf16_t* dh3 = dh1 + (size_t)cap * f;
  int rc;
  if (cap > 0) {
    GArgs g = {};   // dA = d_o W2^T, epilogue -> a, dH1, dH3
    g.A0 = g.A1 = (const bf16_t*)d_o; g.lda = d;
    g.B0 = g.B1 = (const bf16_t*)w2; g.ldb = d; g.b_es = (long)f * d;
    g.C0 = a; g.C1 = dh1; g.C2 = dh3; g.ldc = f;
    g.H1 = (const bf16_t*)h1; g.H3 = (const bf16_t*)h3;
    g.off = offsets; g.e_cnt = e_cnt; g.N = f; g.K = d;
    if ((rc = launch_gg<DA>(g, s))) return rc;
    GArgs x = {};   // dxp = dH1 W1^T + dH3 W3^T
    x.A0 = dh1; x.A1 = dh3; x.lda = f;
    x.B0 = (const bf16_t*)w1; x.B1 = (const bf16_t*)w3; x.ldb = f; x.b_es = (long)d * f;
    x.C0 = (bf16_t*)dxp; x.ldc = d;
    x.off = offsets; x.e_cnt = e_cnt; x.N = d; x.K = f;
    if ((rc = launch_gg<DX>(x, s))) return rc;
  }
  GArgs w = {};     // dW2 = a^T d_o
  w.A0 = w.A1 = a; w.lda = f;
  w.B0 = w.B1 = (const bf16_t*)d_o; w.ldb = d;
  w.C0 = (bf16_t*)dw2; w.ldc = d; w.c_es = (long)f * d;
  w.off = offsets; w.e_cnt = e_cnt; w.M = f; w.N = d; w.accumulate = accumulate;
  if ((rc = launch_gg<WG>(w, s))) return rc;
  GArgs v = {};     // dW1|dW3 = xp^T [dH1|dH3]
  v.A0 = v.A1 = (const bf16_t*)xp; v.lda = d;
  v.B0 = dh1; v.B1 = dh3; v.ldb = f;
  v.C0 = (bf16_t*)dw1; v.C1 = (bf16_t*)dw3; v.ldc = f; v.c_es = (long)d * f;
  v.off = offsets; v.e_cnt = e_cnt; v.M = d; v.N = f; v.accumulate = accumulate;
  return launch_gg<WGD>(v, s);
}
