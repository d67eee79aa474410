// bf16 GEMM on the gfx950 matrix cores: C = A*B with fp32 accumulation, LDS-staged 64-deep K tiles,
// v_mfma_f32_32x32x16_bf16, 4 waves per workgroup arranged 2x2, each wave owning a (BM/2)x(BN/2) block of C.
//
// Data path per K tile: global (16-byte loads, coalesced along the contiguous dimension of each operand)
//   -> registers -> LDS [rows][64 + 8 pad] bf16 (reduction index contiguous) -> MFMA operand registers.
// Operands whose reduction index is NOT contiguous in memory (the weight in an activation-gradient GEMM, both
// operands of a weight-gradient GEMM) are transposed in registers in 8x8 blocks between the global load and the
// LDS store, so the MFMA side is identical for all three layouts.  The pad of 8 elements makes the 16 rows read by
// one 16-lane phase of a ds_read_b128 fall into 16 distinct 16-byte bank groups.
// The LDS tile is double buffered: tile k+1 is fetched from HBM while tile k is multiplied, one barrier per tile.
#include "common.hpp"
#include "gemm.hpp"
#include <stdlib.h>

namespace {

constexpr int BK = 64;    // K tile
constexpr int LDK = 72;   // LDS row stride in elements (144 bytes)
constexpr int NTHR = 256;

template <int BX, bool TR>
struct TileLoader {
  static constexpr int NREG = TR ? 8 : (BX / 32);

  // X is [Xdim, Kdim] (row stride ld) when !TR, [Kdim, Xdim] when TR.  Loads the BX x 64 tile at (x0, k0); zero fill.
  static RP_DEV void load(uint4 (&r)[NREG], const bf16* __restrict__ X, long ld, int x0, int Xdim, int k0, int Klim,
                          int tid) {
    if constexpr (!TR) {
#pragma unroll
      for (int it = 0; it < NREG; ++it) {
        const int c = it * NTHR + tid;
        const int gx = x0 + (c >> 3), gk = k0 + (c & 7) * 8;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (gx < Xdim && gk < Klim) v = *reinterpret_cast<const uint4*>(X + (long)gx * ld + gk);
        r[it] = v;
      }
    } else {
      const int rb = (tid >> 1) & 7;
      const int b = (tid & 1) | ((tid >> 4) << 1);
      const int gx = x0 + b * 8;
      const bool ok = (b < BX / 8) && (gx < Xdim);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int gk = k0 + rb * 8 + i;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (ok && gk < Klim) v = *reinterpret_cast<const uint4*>(X + (long)gk * ld + gx);
        r[i] = v;
      }
    }
  }

  static RP_DEV void store(const uint4 (&r)[NREG], bf16* S, int tid) {
    if constexpr (!TR) {
#pragma unroll
      for (int it = 0; it < NREG; ++it) {
        const int c = it * NTHR + tid;
        *reinterpret_cast<uint4*>(S + (c >> 3) * LDK + (c & 7) * 8) = r[it];
      }
    } else {
      const int rb = (tid >> 1) & 7;
      const int b = (tid & 1) | ((tid >> 4) << 1);
      if (b < BX / 8) {
        uint4 t[8];
        transpose8x8_bf16(r, t);
#pragma unroll
        for (int c = 0; c < 8; ++c) *reinterpret_cast<uint4*>(S + (b * 8 + c) * LDK + rb * 8) = t[c];
      }
    }
  }
};

template <int BM, int BN, bool TA, bool TB>
__global__ void __launch_bounds__(NTHR) gemm_kernel(const GemmArgs p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int TM = BM / 64, TN = BN / 64;   // 32x32 MFMA tiles per wave in each direction
  bf16* const sA0 = reinterpret_cast<bf16*>(smem);
  bf16* const sB0 = sA0 + BM * LDK;
  bf16* const sA1 = sB0 + BN * LDK;
  bf16* const sB1 = sA1 + BM * LDK;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int lr = lane & 31, lk = lane >> 5;

  // tile assignment: XCD-aware remap, then groups of 8 tile rows sweep the tile columns
  const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
  const int pid = xcd_remap(blockIdx.x, tiles_m * tiles_n);
  constexpr int GM = 8;
  const int group = pid / (GM * tiles_n);
  const int first_m = group * GM;
  const int gm = (tiles_m - first_m) < GM ? (tiles_m - first_m) : GM;
  const int in_group = pid - group * GM * tiles_n;
  const int tile_m = first_m + in_group % gm, tile_n = in_group / gm;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const bf16* A = reinterpret_cast<const bf16*>(p.A);
  const bf16* B = reinterpret_cast<const bf16*>(p.B);
  const bf16* A2 = reinterpret_cast<const bf16*>(p.A2);
  const bf16* B2 = reinterpret_cast<const bf16*>(p.B2);
  const int nk1 = (p.K + BK - 1) / BK;
  const int nk = nk1 + (p.K2 + BK - 1) / BK;

  using LA = TileLoader<BM, TA>;
  using LB = TileLoader<BN, TB>;
  uint4 ra[LA::NREG], rb[LB::NREG];

  auto fetch = [&](int kt) {
    if (kt < nk1) {
      LA::load(ra, A, p.lda, m0, p.M, kt * BK, p.K, tid);
      LB::load(rb, B, p.ldb, n0, p.N, kt * BK, p.K, tid);
    } else {
      LA::load(ra, A2, p.lda2, m0, p.M, (kt - nk1) * BK, p.K2, tid);
      LB::load(rb, B2, p.ldb2, n0, p.N, (kt - nk1) * BK, p.K2, tid);
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  if (nk > 0) {
    fetch(0);
    LA::store(ra, sA0, tid);
    LB::store(rb, sB0, tid);
  }
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const bool more = (kt + 1) < nk;
    if (more) fetch(kt + 1);
    const bf16* sA = (kt & 1) ? sA1 : sA0;
    const bf16* sB = (kt & 1) ? sB1 : sB0;
    const bf16* pa = sA + (wm * (BM / 2) + lr) * LDK + lk * 8;
    const bf16* pb = sB + (wn * (BN / 2) + lr) * LDK + lk * 8;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      uint4 af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) af[i] = *reinterpret_cast<const uint4*>(pa + i * 32 * LDK + ks * 16);
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[j] = *reinterpret_cast<const uint4*>(pb + j * 32 * LDK + ks * 16);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = mfma32(af[i], bfr[j], acc[i][j]);
    }
    if (more) {
      LA::store(ra, (kt & 1) ? sA0 : sA1, tid);
      LB::store(rb, (kt & 1) ? sB0 : sB1, tid);
    }
    __syncthreads();
  }

  // ------------------------------------------------------------------ epilogue
  // acc[i][j][v] is C[row, col] with row = m0 + wm*BM/2 + i*32 + 8*(v/4) + 4*lk + v%4, col = n0 + wn*BN/2 + j*32 + lr
  const int row_base = m0 + wm * (BM / 2) + 4 * lk;
  const int col_base = n0 + wn * (BN / 2) + lr;
  const float alpha = p.alpha;

  if (p.epi == EPI_BF16) {
    bf16* C = reinterpret_cast<bf16*>(p.C);
    const bf16* R = reinterpret_cast<const bf16*>(p.R);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = col_base + j * 32;
      if (col >= p.N) continue;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = row_base + i * 32 + 8 * (v >> 2) + (v & 3);
          if (row < p.M) {
            float x = alpha * acc[i][j][v];
            if (R) x += (float)R[(long)row * p.ldr + col];
            C[(long)row * p.ldc + col] = (bf16)x;
          }
        }
    }
  } else if (p.epi == EPI_F32 || p.epi == EPI_F32_ATOMIC) {
    float* C = reinterpret_cast<float*>(p.C);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = col_base + j * 32;
      if (col >= p.N) continue;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = row_base + i * 32 + 8 * (v >> 2) + (v & 3);
          if (row < p.M) {
            float* dst = C + (long)row * p.ldc + col;
            const float x = alpha * acc[i][j][v];
            if (p.epi == EPI_F32_ATOMIC) atomicAdd(dst, x);
            else *dst = p.beta ? (*dst + x) : x;
          }
        }
    }
  } else if (p.epi == EPI_CE_STATS) {
    // rows are vocabulary entries, columns are tokens: every lane reduces its own column
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = col_base + j * 32;
      const bool colok = col < p.N;
      const int lab = colok ? p.labels[col] - p.row_offset : -1;
      float mx = -INFINITY;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = row_base + i * 32 + 8 * (v >> 2) + (v & 3);
          if (row < p.M) {
            mx = fmaxf(mx, acc[i][j][v]);
            if (row == lab) p.zlab[col] = acc[i][j][v];
          }
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      float s = 0.f;
      if (mx > -INFINITY) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int row = row_base + i * 32 + 8 * (v >> 2) + (v & 3);
            if (row < p.M) s += __expf(acc[i][j][v] - mx);
          }
      }
      s += __shfl_xor(s, 32, 64);
      if (lk == 0 && colok) p.part[(long)(p.part_row0 + tile_m * 2 + wm) * p.part_ld + col] = make_float2(mx, s);
    }
  } else if (p.epi == EPI_CE_DZ) {
    bf16* C = reinterpret_cast<bf16*>(p.C);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = col_base + j * 32;
      if (col >= p.N) continue;
      const int lab = p.labels[col] - p.row_offset;
      const float lse = p.lse[col], cf = p.coef[col];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = row_base + i * 32 + 8 * (v >> 2) + (v & 3);
          if (row < p.M) {
            float g = __expf(acc[i][j][v] - lse);
            if (row == lab) g -= 1.f;
            C[(long)row * p.ldc + col] = (bf16)(g * cf);
          }
        }
    }
  }
}

template <int BM, int BN, bool TA, bool TB>
hipError_t launch_one(hipStream_t st, const GemmArgs& a) {
  constexpr size_t smem = (size_t)2 * (BM + BN) * LDK * sizeof(bf16);
  static bool attr_done = false;
  auto kern = gemm_kernel<BM, BN, TA, TB>;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)smem);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
  hipLaunchKernelGGL(kern, dim3(tiles), dim3(NTHR), smem, st, a);
  return hipGetLastError();
}

template <bool TA, bool TB>
hipError_t launch_tile(hipStream_t st, const GemmArgs& a, int tile) {
  switch (tile) {
    case 1: return launch_one<256, 256, TA, TB>(st, a);
    case 2: return launch_one<256, 128, TA, TB>(st, a);
    case 3: return launch_one<128, 128, TA, TB>(st, a);
    default: return launch_one<64, 64, TA, TB>(st, a);
  }
}

int env_tile() {
  static int v = -1;
  if (v < 0) {
    const char* s = getenv("RP_GEMM_TILE");
    v = s ? atoi(s) : 0;
  }
  return v;
}

// Picks the tile that minimises (number of 256-CU waves) x (tile area / relative efficiency).
int choose_tile(int M, int N) {
  static const int bm[4] = {256, 256, 128, 64}, bn[4] = {256, 128, 128, 64};
  static const double eff[4] = {1.0, 0.92, 0.8, 0.4};
  int best = 1;
  double best_cost = 1e300;
  for (int t = 0; t < 4; ++t) {
    const long tiles = (long)((M + bm[t] - 1) / bm[t]) * ((N + bn[t] - 1) / bn[t]);
    const long waves = (tiles + 255) / 256;
    const double cost = (double)waves * bm[t] * bn[t] / eff[t];
    if (cost < best_cost) { best_cost = cost; best = t + 1; }
  }
  return best;
}

}  // namespace

void gemm_zero_args(GemmArgs& a) {
  a = GemmArgs{};
  a.alpha = 1.f;
}

int gemm_ce_stats_partials(int M) { return 2 * ((M + 255) / 256); }

int gemm_pick_tile(const GemmArgs& a, int tile_hint) {
  if (a.epi == EPI_CE_STATS) return 1;   // the partial-row numbering assumes 256-row tiles
  if (tile_hint) return tile_hint;
  return env_tile() ? env_tile() : choose_tile(a.M, a.N);
}

hipError_t gemm_launch(hipStream_t st, int layout, const GemmArgs& a, int tile_hint) {
  if (a.M <= 0 || a.N <= 0) return hipSuccess;
  const int tile = gemm_pick_tile(a, tile_hint);
  switch (layout) {
    case GEMM_NT: return launch_tile<false, false>(st, a, tile);
    case GEMM_NN: return launch_tile<false, true>(st, a, tile);
    case GEMM_TN: return launch_tile<true, true>(st, a, tile);
    default: return hipErrorInvalidValue;
  }
}
