// bf16 GEMM on the gfx950 matrix cores: C = A*B with fp32 accumulation, v_mfma_f32_32x32x16_bf16.
//
// Every wave owns a 128x64 block of C (4x2 MFMA tiles, 128 accumulator registers); a workgroup is a WGM x WGN grid of
// such waves:  256x256 = 2x4 waves (K tile 64, one workgroup per CU, two waves per SIMD),
//              256x128 = 2x2 waves (K tile 32, two workgroups per CU), 128x128 = 1x2, 128x64 = one wave.
// Two waves per SIMD is what keeps the matrix pipeline fed: while one wave waits at a barrier, on LDS or on HBM, the
// other one issues MFMAs.
//
// Data path per K tile: HBM -> registers (16-byte buffer loads, coalesced along the contiguous dimension of each
// operand; rows outside the matrix read as zero through the descriptor, so there is no branch in the loop)
//   -> LDS [rows][BK + 8 pad] bf16 with the reduction index contiguous -> MFMA operand registers.
// Operands whose reduction index is NOT contiguous in memory (the weight in an activation-gradient GEMM, both
// operands of a weight-gradient GEMM) are transposed in registers in 8x8 blocks between the load and the LDS store,
// so the MFMA side is the same for all three layouts.  The 8-element pad puts the 16 rows that one 16-lane phase of
// a ds_read_b128 touches into 16 distinct bank groups.  LDS is double buffered (one barrier per K tile); inside a
// tile the operand fragments of step k+1 are read while the MFMAs of step k run, the next tile's global loads are
// issued during the first step and its LDS stores during the last (pinned with sched_group_barrier).
//
// The epilogue stages each wave's block through LDS so that global stores (and the reads of a residual or of the
// fp32 accumulation target) are 16 bytes per lane and cover whole 128-byte lines.
#include "common.hpp"
#include "gemm.hpp"
#include <stdlib.h>
#include <type_traits>

namespace {

constexpr int TM = 4, TN = 2;            // 32x32 MFMA tiles per wave: 128 x 64
constexpr int WAVE_M = 128, WAVE_N = 64;
constexpr int STG_LD = 72;               // epilogue staging row stride in bf16 elements (144 bytes)
constexpr int STG_BYTES = WAVE_M * STG_LD * 2;

typedef __amdgpu_buffer_rsrc_t rsrc_t;
constexpr uint32_t OOB = 0x80000000u;    // byte offset outside every descriptor (operands are smaller than 2 GiB)

RP_DEV rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
RP_DEV uint4 buf_load16(rsrc_t r, uint32_t voff, uint32_t soff) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, (int)soff, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}

// Copies a tile of one operand from HBM to LDS in 16-byte chunks, keeping the memory layout of the operand:
//   !TR: the operand is [Xdim, Kdim] (reduction index contiguous): LDS tile [BX][BK + 8], MFMA fragments are plain
//        16-byte LDS reads;
//    TR: the operand is [Kdim, Xdim] (reduction index strided):    LDS tile [BK][BX + 32], MFMA fragments are read
//        with the transposing LDS load (ds_read_b64_tr_b16), which hands every lane four consecutive reduction
//        indices of its own column -- no register transposes, no extra ALU work.
// The pads (8 resp. 32 elements) keep both kinds of fragment reads free of bank conflicts.
template <int BX, int BK, int NTHR, bool TR>
struct TileLoader {
  static constexpr int ROWS = TR ? BK : BX;
  static constexpr int CH = (TR ? BX : BK) / 8;            // 16-byte chunks per tile row
  static constexpr int LDROW = TR ? BX + 32 : BK + 8;      // LDS row stride in elements
  static constexpr int ELEMS = ROWS * LDROW;
  static constexpr int NREG = ROWS * CH / NTHR;
  static constexpr int RSTEP = NTHR / CH;                  // tile rows between a thread's consecutive chunks
  static_assert((ROWS * CH) % NTHR == 0 && NTHR % CH == 0, "tile does not divide over the threads");
  uint32_t voff[NREG];
  uint32_t kstep;
  int row0, ch;

  RP_DEV void init(long ld, int x0, int Xdim, int tid) {
    row0 = tid / CH;
    ch = tid % CH;
    kstep = TR ? (uint32_t)ld * 2u : 2u;
#pragma unroll
    for (int it = 0; it < NREG; ++it) {
      const int row = row0 + it * RSTEP;
      if constexpr (!TR) {
        const int gx = x0 + row;
        voff[it] = gx < Xdim ? (uint32_t)((long)gx * ld + ch * 8) * 2u : OOB;
      } else {
        const int gx = x0 + ch * 8;
        voff[it] = gx < Xdim ? (uint32_t)((long)row * ld + gx) * 2u : OOB;
      }
    }
  }

  // Loads the tile whose reduction range starts at k0; chunks past Klim read as zero.
  RP_DEV void load(uint4 (&r)[NREG], rsrc_t rs, int k0, int Klim) const {
    const uint32_t soff = (uint32_t)k0 * kstep;
#pragma unroll
    for (int it = 0; it < NREG; ++it) {
      const bool kok = TR ? (k0 + row0 + it * RSTEP) < Klim : (k0 + ch * 8) < Klim;
      r[it] = buf_load16(rs, kok ? voff[it] : OOB, soff);
    }
  }

  RP_DEV void store(const uint4 (&r)[NREG], bf16* S) const {
#pragma unroll
    for (int it = 0; it < NREG; ++it) *reinterpret_cast<uint4*>(S + (row0 + it * RSTEP) * LDROW + ch * 8) = r[it];
  }
};

// MFMA operand fragment (8 consecutive reduction indices of the lane's row/column) of 16-deep step ks.
//   !TR: base points at S[x_lane][8*lk];  TR: base points at S[8*lk + (l%16)/4][x_group + 4*(l%4)], see above.
template <int LDROW, bool TR>
RP_DEV uint4 read_frag(const bf16* base, int x_tile_off, int ks) {
  if constexpr (!TR) {
    return *reinterpret_cast<const uint4*>(base + x_tile_off * LDROW + ks * 16);
  } else {
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4* lds_ptr;
    const bf16* q = base + ks * 16 * LDROW + x_tile_off;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(q));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(q + 4 * LDROW));
    const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
    return make_uint4(l2.x, l2.y, h2.x, h2.y);
  }
}

// Scheduling hints for one 16-deep step of the K loop: after each of the NM MFMAs, its share of the step's NDS LDS
// reads, NVM global loads and NDW LDS writes is pinned, so that memory instructions issue under the MFMA pipeline.
template <int I, int NM, int NDS, int NVM, int NDW>
struct StepHint {
  static RP_DEV void go() {
    if constexpr (I < NM) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      constexpr int ds = ((I + 1) * NDS) / NM - (I * NDS) / NM;
      constexpr int vm = ((I + 1) * NVM) / NM - (I * NVM) / NM;
      constexpr int dw = ((I + 1) * NDW) / NM - (I * NDW) / NM;
      if constexpr (ds > 0) __builtin_amdgcn_sched_group_barrier(0x100, ds, 0);
      if constexpr (vm > 0) __builtin_amdgcn_sched_group_barrier(0x020, vm, 0);
      if constexpr (dw > 0) __builtin_amdgcn_sched_group_barrier(0x200, dw, 0);
      StepHint<I + 1, NM, NDS, NVM, NDW>::go();
    }
  }
};

template <int WGM, int WGN, int BK, bool TA, bool TB>
struct Cfg {
  static constexpr int BM = WGM * WAVE_M, BN = WGN * WAVE_N, NW = WGM * WGN, NTHR = NW * 64;
  using LA = TileLoader<BM, BK, NTHR, TA>;
  using LB = TileLoader<BN, BK, NTHR, TB>;
  static constexpr int MAIN_BYTES = 2 * (LA::ELEMS + LB::ELEMS) * 2;
  static constexpr int SMEM = MAIN_BYTES > NW * STG_BYTES ? MAIN_BYTES : NW * STG_BYTES;
  // waves per SIMD the register budget is set for
  static constexpr int WPS = (NW == 8) ? 2 : (SMEM * 2 <= 160 * 1024 ? 2 : 1);
};

template <int WGM, int WGN, int BK, bool TA, bool TB>
__global__ void __launch_bounds__(WGM* WGN * 64)
    __attribute__((amdgpu_waves_per_eu(Cfg<WGM, WGN, BK, TA, TB>::WPS, Cfg<WGM, WGN, BK, TA, TB>::WPS)))
    gemm_kernel(const GemmArgs p) {
  using C = Cfg<WGM, WGN, BK, TA, TB>;
  using LA = typename C::LA;
  using LB = typename C::LB;
  constexpr int BM = C::BM, BN = C::BN, KS = BK / 16;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* const sA0 = reinterpret_cast<bf16*>(smem);
  bf16* const sB0 = sA0 + LA::ELEMS;
  bf16* const sA1 = sB0 + LB::ELEMS;
  bf16* const sB1 = sA1 + LA::ELEMS;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
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

  const int nk1 = (p.K + BK - 1) / BK;
  const int nk = nk1 + (p.K2 + BK - 1) / BK;

  LA la, la2;
  LB lb, lb2;
  la.init(p.lda, m0, p.M, tid);
  lb.init(p.ldb, n0, p.N, tid);
  const rsrc_t rsA = make_rsrc(p.A, p.bytesA), rsB = make_rsrc(p.B, p.bytesB);
  rsrc_t rsA2 = rsA, rsB2 = rsB;
  if (p.K2 > 0) {
    la2.init(p.lda2, m0, p.M, tid);
    lb2.init(p.ldb2, n0, p.N, tid);
    rsA2 = make_rsrc(p.A2, p.bytesA2);
    rsB2 = make_rsrc(p.B2, p.bytesB2);
  }
  uint4 ra[LA::NREG], rb[LB::NREG];

  auto fetch = [&](int kt) {
    if (kt < nk1) {
      la.load(ra, rsA, kt * BK, p.K);
      lb.load(rb, rsB, kt * BK, p.K);
    } else {
      la2.load(ra, rsA2, (kt - nk1) * BK, p.K2);
      lb2.load(rb, rsB2, (kt - nk1) * BK, p.K2);
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
    la.store(ra, sA0);
    lb.store(rb, sB0);
  }
  __syncthreads();

  // per-lane fragment base offsets inside an operand tile (elements)
  const int l16 = lane & 15, g16 = lane >> 4;
  const int offA = TA ? (8 * lk + (l16 >> 2)) * LA::LDROW + wm * WAVE_M + 16 * (g16 & 1) + 4 * (l16 & 3)
                      : (wm * WAVE_M + lr) * LA::LDROW + lk * 8;
  const int offB = TB ? (8 * lk + (l16 >> 2)) * LB::LDROW + wn * WAVE_N + 16 * (g16 & 1) + 4 * (l16 & 3)
                      : (wn * WAVE_N + lr) * LB::LDROW + lk * 8;
  uint4 af[2][TM], bfr[2][TN];
  auto load_frags = [&](int buf, const bf16* pa, const bf16* pb, int ks) {
#pragma unroll
    for (int i = 0; i < TM; ++i) af[buf][i] = read_frag<LA::LDROW, TA>(pa, i * 32, ks);
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[buf][j] = read_frag<LB::LDROW, TB>(pb, j * 32, ks);
  };
  auto mfma_step = [&](int buf) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[i][j] = mfma32(af[buf][i], bfr[buf][j], acc[i][j]);
  };

  auto tile = [&](int kt, auto more_tag) {
    constexpr bool MORE = decltype(more_tag)::value;
    const bf16* pa = ((kt & 1) ? sA1 : sA0) + offA;
    const bf16* pb = ((kt & 1) ? sB1 : sB0) + offB;
#ifndef RP_DBG_NO_LDSREAD
    load_frags(0, pa, pb, 0);
#endif
#ifndef RP_DBG_NO_GLOBAL
    if constexpr (MORE) fetch(kt + 1);
#endif
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#ifndef RP_DBG_NO_LDSREAD
      if (ks + 1 < KS) load_frags((ks + 1) & 1, pa, pb, ks + 1);
#endif
#ifndef RP_DBG_NO_GLOBAL
      if constexpr (MORE) {
        if (ks == KS - 1) {
          la.store(ra, (kt & 1) ? sA0 : sA1);
          lb.store(rb, (kt & 1) ? sB0 : sB1);
        }
      }
#endif
      mfma_step(ks & 1);
      constexpr int NLD = LA::NREG + LB::NREG;
      constexpr int NDS = TM * (TA ? 2 : 1) + TN * (TB ? 2 : 1);
      if (ks == 0) StepHint<0, TM * TN, (KS > 1) ? NDS : 0, MORE ? NLD : 0, (MORE && KS == 1) ? NLD : 0>::go();
      else if (ks + 1 < KS) StepHint<0, TM * TN, NDS, 0, 0>::go();
      else StepHint<0, TM * TN, 0, 0, MORE ? NLD : 0>::go();
    }
#ifndef RP_DBG_NO_BARRIER
    __syncthreads();
#endif
  };
#ifdef RP_DBG_NO_LDSREAD
  load_frags(0, sA0 + offA, sB0 + offB, 0);
  load_frags(1, sA0 + offA, sB0 + offB, 1);
#endif
  for (int kt = 0; kt + 1 < nk; ++kt) tile(kt, std::true_type{});
  if (nk > 0) tile(nk - 1, std::false_type{});

  // ------------------------------------------------------------------ epilogue
  // acc[i][j][v] is element (i*32 + 8*(v/4) + 4*lk + v%4, j*32 + lr) of the wave's 128x64 block.
  const int wrow0 = m0 + wm * WAVE_M, wcol0 = n0 + wn * WAVE_N;
  unsigned char* const stg = smem + wave * STG_BYTES;
  const int rr = lane >> 3, cc = lane & 7;   // read-back: 8 rows per pass, 8 chunks of 16 bytes per row

  if (p.epi == EPI_BF16 && !p.R) {
    bf16* s16 = reinterpret_cast<bf16*>(stg);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          s16[(i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3)) * STG_LD + j * 32 + lr] = (bf16)(p.alpha * acc[i][j][v]);
    __syncthreads();
    bf16* Cp = reinterpret_cast<bf16*>(p.C);
    const int gcol = wcol0 + cc * 8;
#pragma unroll
    for (int t = 0; t < WAVE_M / 8; ++t) {
      const int row = t * 8 + rr, grow = wrow0 + row;
      if (grow < p.M && gcol < p.N)
        *reinterpret_cast<uint4*>(Cp + (long)grow * p.ldc + gcol) = *reinterpret_cast<const uint4*>(s16 + row * STG_LD + cc * 8);
    }
  } else if (p.epi == EPI_CE_DZ) {
    bf16* s16 = reinterpret_cast<bf16*>(stg);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = wcol0 + j * 32 + lr;
      const bool colok = col < p.N;
      const int lab = colok ? p.labels[col] - p.row_offset : -1;
      const float lse = colok ? p.lse[col] : 0.f, cf = colok ? p.coef[col] : 0.f;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
          float g = __expf(acc[i][j][v] - lse);
          if (wrow0 + row == lab) g -= 1.f;
          s16[row * STG_LD + j * 32 + lr] = (bf16)(g * cf);
        }
    }
    __syncthreads();
    bf16* Cp = reinterpret_cast<bf16*>(p.C);
    const int gcol = wcol0 + cc * 8;
#pragma unroll
    for (int t = 0; t < WAVE_M / 8; ++t) {
      const int row = t * 8 + rr, grow = wrow0 + row;
      if (grow < p.M && gcol < p.N)
        *reinterpret_cast<uint4*>(Cp + (long)grow * p.ldc + gcol) = *reinterpret_cast<const uint4*>(s16 + row * STG_LD + cc * 8);
    }
  } else if (p.epi == EPI_BF16 || p.epi == EPI_F32) {
    // fp32 staging, one 32-column half at a time: [128][36] floats (144-byte rows)
    float* s32 = reinterpret_cast<float*>(stg);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      if (j) __syncthreads();
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s32[(i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3)) * (STG_LD / 2) + lr] = p.alpha * acc[i][j][v];
      __syncthreads();
      const int gcol = wcol0 + j * 32 + cc * 4;
#pragma unroll
      for (int t = 0; t < WAVE_M / 8; ++t) {
        const int row = t * 8 + rr, grow = wrow0 + row;
        if (grow < p.M && gcol < p.N) {
          float4 x = *reinterpret_cast<const float4*>(s32 + row * (STG_LD / 2) + cc * 4);
          if (p.epi == EPI_F32) {
            float4* dst = reinterpret_cast<float4*>(reinterpret_cast<float*>(p.C) + (long)grow * p.ldc + gcol);
            if (p.beta) { const float4 o = *dst; x.x += o.x; x.y += o.y; x.z += o.z; x.w += o.w; }
            *dst = x;
          } else {
            const uint2 r2 = *reinterpret_cast<const uint2*>(reinterpret_cast<const bf16*>(p.R) + (long)grow * p.ldr + gcol);
            x.x += bf16_lo(r2.x); x.y += bf16_hi(r2.x); x.z += bf16_lo(r2.y); x.w += bf16_hi(r2.y);
            *reinterpret_cast<uint2*>(reinterpret_cast<bf16*>(p.C) + (long)grow * p.ldc + gcol) =
                make_uint2(pack_bf16x2(x.x, x.y), pack_bf16x2(x.z, x.w));
          }
        }
      }
    }
  } else if (p.epi == EPI_F32_ATOMIC) {
    float* Cp = reinterpret_cast<float*>(p.C);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = wcol0 + j * 32 + lr;
      if (col >= p.N) continue;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = wrow0 + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
          if (row < p.M) atomicAdd(Cp + (long)row * p.ldc + col, p.alpha * acc[i][j][v]);
        }
    }
  } else if (p.epi == EPI_CE_STATS) {
    // rows are vocabulary entries, columns are tokens: every lane reduces its own column over the wave's 128 rows
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = wcol0 + j * 32 + lr;
      const bool colok = col < p.N;
      const int lab = colok ? p.labels[col] - p.row_offset : -1;
      float mx = -INFINITY;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = wrow0 + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
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
            const int row = wrow0 + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
            if (row < p.M) s += __expf(acc[i][j][v] - mx);
          }
      }
      s += __shfl_xor(s, 32, 64);
      if (lk == 0 && colok) p.part[(long)(p.part_row0 + tile_m * WGM + wm) * p.part_ld + col] = make_float2(mx, s);
    }
  }
}

template <int WGM, int WGN, int BK, bool TA, bool TB>
hipError_t launch_one(hipStream_t st, const GemmArgs& a) {
  using C = Cfg<WGM, WGN, BK, TA, TB>;
  static bool attr_done = false;
  auto kern = gemm_kernel<WGM, WGN, BK, TA, TB>;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, C::SMEM);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int tiles = ((a.M + C::BM - 1) / C::BM) * ((a.N + C::BN - 1) / C::BN);
  RP_LAUNCH(kern, dim3(tiles), dim3(C::NTHR), C::SMEM, st, a);
  return hipGetLastError();
}

template <bool TA, bool TB>
hipError_t launch_tile(hipStream_t st, const GemmArgs& a, int tile) {
  switch (tile) {
    case 1: return launch_one<2, 4, 64, TA, TB>(st, a);
    case 2: return launch_one<2, 2, 32, TA, TB>(st, a);
    case 3: return launch_one<1, 2, 32, TA, TB>(st, a);
    default: return launch_one<1, 1, 32, TA, TB>(st, a);
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

// Picks the tile with the smallest modelled time: n = workgroups on the busiest CU, each costing its area divided by
// a relative efficiency that was measured with one workgroup per CU and with the CU fully occupied.
int choose_tile(int M, int N) {
  static const int bm[4] = {256, 256, 128, 128}, bn[4] = {256, 128, 128, 64};
  static const int per_cu[4] = {1, 2, 3, 5};
  static const double eff_full[4] = {1.0, 0.83, 0.7, 0.4}, eff_single[4] = {1.0, 0.375, 0.25, 0.15};
  int best = 1;
  double best_cost = 1e300;
  for (int t = 0; t < 4; ++t) {
    const long tiles = (long)((M + bm[t] - 1) / bm[t]) * ((N + bn[t] - 1) / bn[t]);
    const long n = (tiles + 255) / 256;
    double e = eff_full[t];
    if (n < per_cu[t]) e = eff_single[t] + (eff_full[t] - eff_single[t]) * (double)(n - 1) / (per_cu[t] - 1);
    const double cost = (double)n * bm[t] * bn[t] / e;
    if (cost < best_cost) { best_cost = cost; best = t + 1; }
  }
  return best;
}

// Bytes spanned by a [rows, cols] bf16 view with row stride ld; 0 for an empty view, ~0 when it does not fit 31 bits.
unsigned extent_bytes(long rows, long cols, long ld) {
  if (rows <= 0 || cols <= 0) return 0;
  const long b = ((rows - 1) * ld + cols) * 2;
  return b < (1L << 31) ? (unsigned)b : ~0u;
}

}  // namespace

void gemm_zero_args(GemmArgs& a) {
  a = GemmArgs{};
  a.alpha = 1.f;
}

int gemm_ce_stats_partials(int M) { return 2 * ((M + 255) / 256); }

int gemm_pick_tile(const GemmArgs& a, int tile_hint) {
  if (a.epi == EPI_CE_STATS) return 1;   // the partial-row numbering assumes 256-row tiles of two wave rows
  if (tile_hint) return tile_hint;
  return env_tile() ? env_tile() : choose_tile(a.M, a.N);
}

hipError_t gemm_launch(hipStream_t st, int layout, const GemmArgs& a_in, int tile_hint) {
  if (a_in.M <= 0 || a_in.N <= 0) return hipSuccess;
  if (layout < GEMM_NT || layout > GEMM_TN) return hipErrorInvalidValue;
  GemmArgs a = a_in;
  // 16-byte accesses everywhere: the output width and every leading dimension must keep rows aligned
  const bool out_f32 = a.epi == EPI_F32 || a.epi == EPI_F32_ATOMIC;
  if (a.N % 8 || a.K % 8 || a.lda % 8 || a.ldb % 8) return hipErrorInvalidValue;
  if (a.epi != EPI_CE_STATS && a.ldc % (out_f32 ? 4 : 8)) return hipErrorInvalidValue;
  if (a.R && a.ldr % 4) return hipErrorInvalidValue;
  const bool ta = layout == GEMM_TN, tb = layout != GEMM_NT;
  if (ta && a.M % 8) return hipErrorInvalidValue;
  if (!a.A2 || !a.B2) a.K2 = 0;
  if (a.K2 && (a.K2 % 8 || a.lda2 % 8 || a.ldb2 % 8)) return hipErrorInvalidValue;
  a.bytesA = ta ? extent_bytes(a.K, a.M, a.lda) : extent_bytes(a.M, a.K, a.lda);
  a.bytesB = tb ? extent_bytes(a.K, a.N, a.ldb) : extent_bytes(a.N, a.K, a.ldb);
  a.bytesA2 = ta ? extent_bytes(a.K2, a.M, a.lda2) : extent_bytes(a.M, a.K2, a.lda2);
  a.bytesB2 = tb ? extent_bytes(a.K2, a.N, a.ldb2) : extent_bytes(a.N, a.K2, a.ldb2);
  // operands are addressed with 32-bit byte offsets
  if (a.bytesA == ~0u || a.bytesB == ~0u || a.bytesA2 == ~0u || a.bytesB2 == ~0u) return hipErrorInvalidValue;
  const int tile = gemm_pick_tile(a, tile_hint);
  switch (layout) {
    case GEMM_NT: return launch_tile<false, false>(st, a, tile);
    case GEMM_NN: return launch_tile<false, true>(st, a, tile);
    default: return launch_tile<true, true>(st, a, tile);
  }
}
