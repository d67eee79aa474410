// bf16 GEMM on the gfx950 matrix cores: C = A*B with fp32 accumulation, v_mfma_f32_32x32x16_bf16.
//
// Every wave owns a 128x64 block of C (4x2 MFMA tiles, 128 accumulator registers); a workgroup is a WGM x WGN grid of
// such waves.  Two waves per SIMD keep the matrix pipeline fed: while one wave waits at a barrier, on LDS or on HBM,
// the other one issues MFMAs.
//
//   256x256 (2x4 waves, K tile 64, the whole LDS of a CU), 256x128 (2x2), 128x128 (1x2), 128x64 (one wave; K tile 32),
//   256x128 with two groups of 2x2 waves (K tile 64)
//
// Operands are staged through registers (16-byte buffer loads; rows outside the matrix read as zero through the
// descriptor, so the loop has no branch) and LDS is double buffered.  The K loop is written slot by slot -- one MFMA
// followed by that slot's share of memory instructions, pinned with scheduling barriers: the fragments of the next
// 16-deep step are read at the start of a step; every 16-byte staging chunk rotates on its own (stored to LDS, then
// reloaded with the tile after next), so that global loads and LDS stores arrive evenly instead of in bursts that
// stall MFMA issue behind a full memory queue, and every load has a whole tile of time to return; the workgroup
// barrier sits before the last four MFMAs of a tile and the first fragments of the next tile are read under them.
// Measured on MI355X the 256x256 tile asks L2 for one byte per 128 FLOP; the matrix pipe is busy 75-79 % of the kernel's
// cycles and the chip runs power-limited near 1.65 GHz under it.  Tried and dropped here: touching lines two tiles
// ahead to pull them into L2, touching the first lines of the workgroup's successor tile before the epilogue,
// staggered K-loop starts, a reduction split merged by the last workgroup to arrive.  The NT product on 256x256 tiles
// has a faster kernel of its own (gemm_dtl.hip: four waves of 128x128, one per SIMD, operands loaded straight into
// LDS); this file keeps every other tile and layout, and the eight-wave 256x256 NT instance as the reference it is
// tested against bit for bit.
// Outputs too small to fill the chip with 256x256 tiles use a 256x128 tile worked
// on by two wave groups that split every K tile (merged through LDS); GEMMs that accumulate into an fp32 output and
// would still leave CUs idle are split along the reduction: the slices write partial products to scratch memory and a
// second kernel adds them in slice order (reproducible run to run).  A variant keeps the B operand out of LDS (BD).
//
// Operands whose reduction index is not contiguous in memory (the weight in an activation-gradient GEMM, both operands
// of a weight-gradient GEMM) keep their memory layout in LDS and are read with the transposing LDS load, so all
// three layouts run the same code.  The epilogue stages each wave's block through LDS (16-byte global accesses).
#include "gemm_device.hpp"
#include <stdlib.h>
#include <type_traits>

using namespace gemm_dev;

namespace {

// Copies a tile of one operand from HBM to LDS through registers, NREG 16-byte chunks per thread.
template <int BX, int BK, int NTHR, bool TR>
struct TileLoader {
  using S = TileShape<BX, BK, TR>;
  static constexpr int NREG = S::ROWS * S::CH / NTHR;
  static constexpr int RSTEP = NTHR / S::CH;               // tile rows between a thread's consecutive chunks
  static_assert((S::ROWS * S::CH) % NTHR == 0 && NTHR % S::CH == 0, "tile does not divide over the threads");
  uint32_t voff[NREG];
  uint32_t kstep;
  int row0, ch;

  // row_map (only for operands whose rows are the tile rows): row gx is read from row row_map[gx] of the buffer.
  // fold_half (only !TR): the tile's rows are the two halves of a folded index range -- rows [0, BX/2) are x0/2 + row,
  // rows [BX/2, BX) are fold_half + x0/2 + row - BX/2 (the gate and up rows of one SwiGLU column block).
  RP_DEV void init(long ld, int x0, int Xdim, int tid, const int* row_map = nullptr, int fold_half = 0) {
    row0 = tid / S::CH;
    ch = tid % S::CH;
    kstep = TR ? (uint32_t)ld * 2u : 2u;
#pragma unroll
    for (int it = 0; it < NREG; ++it) {
      const int row = row0 + it * RSTEP;
      if constexpr (!TR) {
        const int gx = fold_half ? (x0 >> 1) + (row < BX / 2 ? row : fold_half + row - BX / 2) : x0 + row;
        const long src = (row_map && gx < Xdim) ? row_map[gx] : gx;
        voff[it] = gx < Xdim ? (uint32_t)(src * ld + ch * 8) * 2u : OOB;
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

  RP_DEV void store(const uint4 (&r)[NREG], bf16* Sm) const {
#pragma unroll
    for (int it = 0; it < NREG; ++it) *reinterpret_cast<uint4*>(Sm + (row0 + it * RSTEP) * S::LDROW + ch * 8) = r[it];
  }

  // One chunk at a time, for the steady state of the K loop; `other` is the loader of the second operand pair (same
  // thread -> chunk mapping), selected without a branch when second is set.
  RP_DEV uint4 load_one(int it, const TileLoader& other, bool second, rsrc_t rs, int k0, int Klim) const {
    const uint32_t vo = second ? other.voff[it] : voff[it];
    const uint32_t kst = second ? other.kstep : kstep;
    const bool kok = TR ? (k0 + row0 + it * RSTEP) < Klim : (k0 + ch * 8) < Klim;
    return buf_load16(rs, kok ? vo : OOB, (uint32_t)k0 * kst);
  }
  RP_DEV void store_one(int it, const uint4& r, bf16* Sm) const {
    *reinterpret_cast<uint4*>(Sm + (row0 + it * RSTEP) * S::LDROW + ch * 8) = r;
  }
};

// KG wave groups share one output tile: group g runs the 16-deep steps [g*KS/KG, (g+1)*KS/KG) of every K tile, and the
// groups' accumulators are added through LDS before the epilogue.  With KG = 2 a 256x128 tile is worked on by eight
// waves of 128x64 each, which fills the chip with half as many output elements as the 256x256 tile needs.
template <int WGM, int WGN, int BK, bool TA, bool TB, int KG = 1>
struct Cfg {
  static constexpr int BM = WGM * WAVE_M, BN = WGN * WAVE_N, NWT = WGM * WGN, NW = NWT * KG, NTHR = NW * 64;
  static_assert((BK / 16) % KG == 0, "the K tile does not divide over the wave groups");
  static_assert(KG == 1 || NW * (TM * 16 * 64 * 4) <= 160 * 1024, "accumulator exchange does not fit in LDS");
  using LA = TileLoader<BM, BK, NTHR, TA>;
  using LB = TileLoader<BN, BK, NTHR, TB>;
  static constexpr int MAIN_BYTES = 2 * (LA::S::ELEMS + LB::S::ELEMS) * 2;
  static constexpr int XCH_BYTES = KG > 1 ? NW * (TM * 16 * 64 * 4) : 0;   // every wave hands over one column of MFMA tiles
  static constexpr int SMEM0 = MAIN_BYTES > NW * STG_BYTES ? MAIN_BYTES : NW * STG_BYTES;   // every wave stages
  static constexpr int SMEM = SMEM0 > XCH_BYTES ? SMEM0 : XCH_BYTES;
  // waves per SIMD the register budget is set for
  static constexpr int WPS = (NW == 8) ? 2 : (SMEM * 2 <= 160 * 1024 ? 2 : 1);
};

// GATED: the conditional instance (a name of its own in profiles): returns at once unless *p.run_flag is set.
// BD: the B operand does not pass through LDS.  p.B (and p.B2) point at copies in MFMA fragment order (gemm_arrange):
// every wave streams the fragments of its 64 columns straight into registers, 1 KB per load instruction, through a ring
// that holds one K tile and is refilled fragment by fragment right after a fragment's last MFMA -- a whole K tile of
// latency per load.  Half of the LDS stores and a third of the LDS reads of the staged kernel go away.
template <int WGM, int WGN, int BK, bool TA, bool TB, int KG, bool GATED, bool BD>
__global__ void __launch_bounds__(WGM* WGN* KG * 64)
    __attribute__((amdgpu_waves_per_eu(Cfg<WGM, WGN, BK, TA, TB, KG>::WPS, Cfg<WGM, WGN, BK, TA, TB, KG>::WPS)))
    gemm_kernel(const GemmArgs p) {
  using C = Cfg<WGM, WGN, BK, TA, TB, KG>;
  using LA = typename C::LA;
  using LB = typename C::LB;
  constexpr int BM = C::BM, BN = C::BN, KS = BK / 16, KSL = KS / KG;
  constexpr int LDA = LA::S::LDROW, LDB = LB::S::LDROW;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* const sA0 = reinterpret_cast<bf16*>(smem);
  bf16* const sB0 = sA0 + LA::S::ELEMS;
  bf16* const sA1 = sB0 + LB::S::ELEMS;
  bf16* const sB1 = sA1 + LA::S::ELEMS;

  if constexpr (GATED) {
    if (*p.run_flag == 0) return;                      // uniform over the grid
  }
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int kg = wave / C::NWT, wmn = wave % C::NWT;   // wave group, wave within the output tile
  const int wm = wmn / WGN, wn = wmn % WGN;
  const int ks0 = kg * KSL;

  int tile_m, tile_n, m0, Mlim = p.M;
  const bf16* Bbase = static_cast<const bf16*>(p.B);
  if (p.grp_tab) {   // uniform over the grid
    const int tiles_n = (p.N + BN - 1) / BN;
    tile_m = (int)blockIdx.x / tiles_n;
    tile_n = (int)blockIdx.x % tiles_n;
    if (tile_m >= *p.grp_ntiles) return;
    const int4 g = p.grp_tab[tile_m];
    m0 = g.y;
    Mlim = g.y + g.z;
    Bbase += (long)g.x * p.grp_strideB;
  } else {
    tile_of_block(p.M, p.N, BM, BN, tile_m, tile_n);
    m0 = tile_m * BM;
  }
  const int n0 = tile_n * BN;
  const int nk1 = (p.K + BK - 1) / BK;
  const int nk_all = nk1 + (p.K2 + BK - 1) / BK;
  // split along the reduction: slice blockIdx.y takes K tiles [kt0, kt0 + nk)
  const int per_split = (nk_all + (int)gridDim.y - 1) / (int)gridDim.y;
  const int kt0 = (int)blockIdx.y * per_split;
  const int nk = (nk_all - kt0) < per_split ? (nk_all - kt0 > 0 ? nk_all - kt0 : 0) : per_split;

  LA la, la2;
  LB lb, lb2;
  la.init(p.lda, m0, Mlim, tid, TA ? nullptr : p.row_map);
  const int fold = (!TB && p.epi == EPI_SWIGLU_FWD) ? p.N >> 1 : 0;   // uniform
  lb.init(p.ldb, n0, p.N, tid, nullptr, fold);
  const rsrc_t rsA = make_rsrc(p.A, p.bytesA), rsB = make_rsrc(Bbase, p.bytesB);
  rsrc_t rsA2 = rsA, rsB2 = rsB;
  la2 = la;
  lb2 = lb;
  if (p.K2 > 0) {
    la2.init(p.lda2, m0, p.M, tid);
    lb2.init(p.ldb2, n0, p.N, tid, nullptr, fold);
    rsA2 = make_rsrc(p.A2, p.bytesA2);
    rsB2 = make_rsrc(p.B2, p.bytesB2);
  }
  // Staging registers: chunk r < LA::NREG belongs to the A tile, the others to the B tile.  In the steady state
  // every chunk rotates on its own: at its slot of K tile kt it is stored to LDS (it holds tile kt+1, loaded one
  // tile earlier) and immediately reloaded with tile kt+2, so global loads and LDS stores are spread evenly over
  // the MFMAs of a tile instead of arriving in bursts, and every load has a full tile of time to return.
  static_assert(!BD || (KG == 1 && BK == 64), "the direct B path is built for one wave group and K tiles of 64");
  constexpr int NLD = LA::NREG + (BD ? 0 : LB::NREG);
  static_assert(NLD % KSL == 0, "staging chunks do not divide over the steps of a K tile");
  uint4 rg[NLD];
  struct Seg { bool second; int k0, Klim; };
  auto seg_of = [&](int kt_local) {
    const int kt = kt0 + kt_local;
    const bool second = kt >= nk1;
    return Seg{second, (second ? kt - nk1 : kt) * BK, second ? p.K2 : p.K};
  };
  auto load_chunk = [&](int r, const Seg& sg) {
    if (r < LA::NREG) rg[r] = la.load_one(r, la2, sg.second, sg.second ? rsA2 : rsA, sg.k0, sg.Klim);
    else rg[r] = lb.load_one(r - LA::NREG, lb2, sg.second, sg.second ? rsB2 : rsB, sg.k0, sg.Klim);
  };
  auto store_chunk = [&](int r, bf16* sa, bf16* sb) {
    if (r < LA::NREG) la.store_one(r, rg[r], sa);
    else lb.store_one(r - LA::NREG, rg[r], sb);
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // direct B path: fragment (ks, j) of K tile t of the wave's 64-column block blk lies at
  // (((blk * tiles_in_segment + t) * KS + ks) * TN + j) KB of the arranged copy, 16 bytes per lane
  [[maybe_unused]] uint4 bq[KS][TN];
  [[maybe_unused]] const uint32_t bd_blk = (uint32_t)(n0 / WAVE_N + wn);
  [[maybe_unused]] const uint32_t bd_nk2 = (uint32_t)((p.K2 + BK - 1) / BK);
  [[maybe_unused]] auto bd_load = [&](int ks, int j, const Seg& sg) {
    const uint32_t t = bd_blk * (sg.second ? bd_nk2 : (uint32_t)nk1) + (uint32_t)(sg.k0 / BK);
    return buf_load16(sg.second ? rsB2 : rsB, ((t * KS + ks) * TN + j) * 1024u + (uint32_t)lane * 16u, 0u);
  };

  if (nk > 0) {
    const Seg s0 = seg_of(0);
    if constexpr (BD) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int j = 0; j < TN; ++j) bq[ks][j] = bd_load(ks, j, s0);
    }
#pragma unroll
    for (int r = 0; r < NLD; ++r) load_chunk(r, s0);
#pragma unroll
    for (int r = 0; r < NLD; ++r) store_chunk(r, sA0, sB0);
    if (nk > 1) {
      const Seg s1 = seg_of(1);
#pragma unroll
      for (int r = 0; r < NLD; ++r) load_chunk(r, s1);
    }
  }
  __syncthreads();

  const int offA = frag_base<LDA, TA>(lane, wm * WAVE_M);
  const int offB = frag_base<LDB, TB>(lane, wn * WAVE_N);
  uint4 af[2][TM], bfr[2][TN];
  auto load_frags = [&](int buf, const bf16* pa, const bf16* pb, int ks) {
#pragma unroll
    for (int i = 0; i < TM; ++i) af[buf][i] = read_frag<LDA, TA>(pa, i * 32, ks);
    if constexpr (!BD) {
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[buf][j] = read_frag<LDB, TB>(pb, j * 32, ks);
    }
  };
  // One K tile.  STORE: tile kt+1 exists (its chunks are in the staging registers); LOAD: tile kt+2 exists.
  // The tile is a flat sequence of S = KSL * NM slots, one MFMA each, followed by that slot's share of the memory
  // instructions, with a scheduling barrier so that the compiler keeps the order:
  //   - the fragments of the next 16-deep step, one read per slot at the start of a step;
  //   - the chunk rotations, spread evenly over slots 0 .. S-5;
  //   - before slot S-4 the workgroup barrier: by then every wave has stored its chunks of tile kt+1 and has all its
  //     fragments of tile kt in registers, so the first fragments of tile kt+1 are read under the last four MFMAs
  //     and the next tile may overwrite this tile's buffer.
  constexpr int NM = TM * TN, NF = TM + (BD ? 0 : TN), S = KSL * NM, TAIL = 4;
  static_assert(NF <= NM && KSL % 2 == 0 && NLD <= S - TAIL, "slot plan does not fit");
  load_frags(0, sA0 + offA, sB0 + offB, ks0);
  auto tile = [&](int kt, auto store_tag, auto load_tag) {
    constexpr bool STORE = decltype(store_tag)::value, LOAD = decltype(load_tag)::value;
    const bf16* pa = ((kt & 1) ? sA1 : sA0) + offA;
    const bf16* pb = ((kt & 1) ? sB1 : sB0) + offB;
    bf16* const na = (kt & 1) ? sA0 : sA1;
    bf16* const nb = (kt & 1) ? sB0 : sB1;
    const Seg sg = seg_of(kt + 2);
    [[maybe_unused]] const Seg sg1 = seg_of(kt + 1);
#pragma unroll
    for (int sl = 0; sl < S; ++sl) {
      const int ks = sl / NM, I = sl % NM, cur = ks & 1;
      if (STORE && sl == S - TAIL) __syncthreads();
      if constexpr (BD) acc[I / TN][I % TN] = mfma32(af[cur][I / TN], bq[ks][I % TN], acc[I / TN][I % TN]);
      else acc[I / TN][I % TN] = mfma32(af[cur][I / TN], bfr[cur][I % TN], acc[I / TN][I % TN]);
      if (ks + 1 < KSL && I < NF) {
        if (I < TM) af[cur ^ 1][I] = read_frag<LDA, TA>(pa, I * 32, ks0 + ks + 1);
        else if constexpr (!BD) bfr[cur ^ 1][I - TM] = read_frag<LDB, TB>(pb, (I - TM) * 32, ks0 + ks + 1);
      }
      if (STORE && sl >= S - TAIL) {   // first step of tile kt+1, from the other buffer, into the idle fragment set
#pragma unroll
        for (int f = ((sl - (S - TAIL)) * NF) / TAIL; f < ((sl - (S - TAIL) + 1) * NF) / TAIL; ++f) {
          if (f < TM) af[0][f] = read_frag<LDA, TA>(na + offA, f * 32, ks0);
          else if constexpr (!BD) bfr[0][f - TM] = read_frag<LDB, TB>(nb + offB, (f - TM) * 32, ks0);
        }
      }
      if constexpr (BD && STORE) {   // this was the last MFMA of the tile that reads fragment (ks, j): refill it for tile kt+1
        if (I >= NM - TN) bq[ks][I - (NM - TN)] = bd_load(ks, I - (NM - TN), sg1);
      }
#pragma unroll
      for (int q = 0; q < NLD; ++q)
        if (((q + 1) * (S - TAIL)) / NLD - 1 == sl) {
          if constexpr (STORE) store_chunk(q, na, nb);
          if constexpr (LOAD) load_chunk(q, sg);
        }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  for (int kt = 0; kt + 2 < nk; ++kt) tile(kt, std::true_type{}, std::true_type{});
  if (nk > 1) tile(nk - 2, std::true_type{}, std::false_type{});
  if (nk > 0) tile(nk - 1, std::false_type{}, std::false_type{});
  __syncthreads();   // every wave is done with the operand tiles: the epilogue reuses the LDS

  if constexpr (KG > 1) {
    static_assert(KG == 2 && TN == 2, "the exchange pairs two wave groups with the two column halves of a block");
    // The K loop ended with a barrier, so the operand tiles are dead.  The two groups hold partial sums of the same
    // blocks: group 1 hands its left half (tile column 0) to group 0 and takes group 0's right half, in one exchange
    // ([group][wave][register][lane], conflict-free), and each group finishes and writes its own half.
    float* const mine = reinterpret_cast<float*>(smem) + (kg * C::NWT + wmn) * (TM * 16 * 64) + lane;
    float* const theirs = reinterpret_cast<float*>(smem) + ((kg ^ 1) * C::NWT + wmn) * (TM * 16 * 64) + lane;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      if (j == kg) continue;   // wave-uniform: the half this wave gives away is j = 1 - kg
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) mine[(i * 16 + v) * 64] = acc[i][j][v];
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      if (j != kg) continue;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] += theirs[(i * 16 + v) * 64];
    }
    __syncthreads();   // the staging of the epilogue overwrites the exchange area
    epilogue(p, Mlim, acc, smem, wave, lane, m0 + wm * WAVE_M, n0 + wn * WAVE_N, p.part_row0 + tile_m * WGM + wm, kg, kg + 1);
    return;
  }
  // a folded tile's wave columns: waves 0, 1 of a row hold gate columns, waves 2, 3 the up columns that go with them
  const int wcol = fold ? (n0 >> 1) + (wn & 1) * WAVE_N + (wn >> 1) * fold : n0 + wn * WAVE_N;
  epilogue(p, Mlim, acc, smem, wmn, lane, m0 + wm * WAVE_M, wcol, p.part_row0 + tile_m * WGM + wm);
}

template <int WGM, int WGN, int BK, bool TA, bool TB, int KG = 1, bool GATED = false, bool BD = false>
hipError_t launch_one(hipStream_t st, const GemmArgs& a) {
  using C = Cfg<WGM, WGN, BK, TA, TB, KG>;
  static bool attr_done = false;
  auto kern = gemm_kernel<WGM, WGN, BK, TA, TB, KG, GATED, BD>;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, C::SMEM);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  int tiles = ((a.M + C::BM - 1) / C::BM) * ((a.N + C::BN - 1) / C::BN);
  if (a.grp_tab) tiles = a.grp_max_tiles * ((a.N + C::BN - 1) / C::BN);
  RP_LAUNCH(kern, dim3(tiles, a.splits > 0 ? a.splits : 1), dim3(C::NTHR), C::SMEM, st, a);
  return hipGetLastError();
}

template <bool TA, bool TB>
hipError_t launch_tile(hipStream_t st, const GemmArgs& a, int tile) {
  if (a.run_flag) {   // only the frozen head's conditional logits product: NT, 256x256 (checked by gemm_launch)
    if constexpr (!TA && !TB) return launch_one<2, 4, 64, false, false, 1, true>(st, a);
    return hipErrorInvalidValue;
  }
  if (a.b_direct) {   // B in fragment order: its memory layout no longer matters, one instance serves NT and NN
    if constexpr (!TA) return launch_one<2, 4, 64, false, false, 1, false, true>(st, a);
    return hipErrorInvalidValue;
  }
  switch (tile) {
    case 1: return launch_one<2, 4, 64, TA, TB>(st, a);
    case 2: return launch_one<2, 2, 32, TA, TB>(st, a);
    case 3: return launch_one<1, 2, 32, TA, TB>(st, a);
    case 5: return launch_one<2, 2, 64, TA, TB, 2>(st, a);
    default: return launch_one<1, 1, 32, TA, TB>(st, a);
  }
}

// Merge of a reduction split: C (+)= sum over the slices, added in slice order (one thread per four columns).
template <bool OUT_BF16>
__global__ void __launch_bounds__(256) splitk_merge_kernel(const float* __restrict__ ws, int splits, long slice_stride,
                                                           void* __restrict__ Cout, long ldc, int M, int N, int beta) {
  const int n4 = N >> 2;
  const long total = (long)M * n4;
  for (long idx = (long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long)gridDim.x * 256) {
    const long row = idx / n4;
    const int c = (int)(idx - row * n4) * 4;
    const float* src = ws + row * N + c;
    float4 acc = *reinterpret_cast<const float4*>(src);
    for (int s = 1; s < splits; ++s) {
      const float4 v = *reinterpret_cast<const float4*>(src + (long)s * slice_stride);
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    if constexpr (OUT_BF16) {
      *reinterpret_cast<uint2*>(reinterpret_cast<bf16*>(Cout) + row * ldc + c) = make_uint2(pack_bf16x2(acc.x, acc.y), pack_bf16x2(acc.z, acc.w));
    } else {
      float4* dst = reinterpret_cast<float4*>(reinterpret_cast<float*>(Cout) + row * ldc + c);
      if (beta) { const float4 o = *dst; acc.x += o.x; acc.y += o.y; acc.z += o.z; acc.w += o.w; }
      *dst = acc;
    }
  }
}

// One 16-byte chunk of the fragment order per thread (see gemm_arranged_bytes).
__global__ void __launch_bounds__(256) gemm_arrange_kernel(const bf16* __restrict__ B, long ldb, int N, int K, int transposed,
                                                           uint4* __restrict__ out, long chunks, int nkt) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= chunks) return;
  const int lane = (int)(idx & 63);
  const long f = idx >> 6;
  const int j = (int)(f & 1), ks = (int)((f >> 1) & 3);
  const long t = f >> 3;
  const int kt = (int)(t % nkt);
  const int blk = (int)(t / nkt);
  const int n = blk * 64 + j * 32 + (lane & 31), k = kt * 64 + ks * 16 + (lane >> 5) * 8;
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  if (n < N && k < K) {   // K is a multiple of 8: the eight indices are in range together
    if (!transposed) {
      v = *reinterpret_cast<const uint4*>(B + (long)n * ldb + k);
    } else {
      const unsigned short* src = reinterpret_cast<const unsigned short*>(B) + (long)k * ldb + n;
      unsigned short e[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) e[i] = src[(long)i * ldb];
      v = make_uint4(e[0] | ((uint32_t)e[1] << 16), e[2] | ((uint32_t)e[3] << 16), e[4] | ((uint32_t)e[5] << 16), e[6] | ((uint32_t)e[7] << 16));
    }
  }
  out[idx] = v;
}

// Picks the tile with the smallest modelled time: n = workgroups on the busiest CU, each costing its area divided by
// a relative efficiency that was measured with one workgroup per CU and with the CU fully occupied.
// atomic_nk: K tiles of 64 when the output accumulates in fp32, so that an under-filled 256x256 launch can be split
// along the reduction (merged by atomic adds, which only pays off for long reductions); else 0.
// k_tiles: K tiles of 64 in the reduction.  The two-group tile pays a fixed accumulator exchange per output tile, so its
// efficiency against the 256x256 tile grows with the length of the reduction: measured 0.75-0.84 at K = 2048, 0.94 at
// K = 4096, 1.0 at K = 12288 -- modelled as 0.75 at 32 K tiles rising to 0.85 at 96.
int choose_tile(int M, int N, bool plain_epilogue, int atomic_nk, int k_tiles) {
  static const int bm[5] = {256, 256, 128, 128, 256}, bn[5] = {256, 128, 128, 64, 128};
  static const int per_cu[5] = {1, 2, 3, 5, 1};
  const double k2 = 0.75 + 0.1 * (k_tiles <= 32 ? 0.0 : k_tiles >= 96 ? 1.0 : (k_tiles - 32) / 64.0);
  const double eff_full[5] = {1.0, 0.7, 0.6, 0.4, k2}, eff_single[5] = {1.0, 0.375, 0.25, 0.15, k2};
  int best = 1;
  double best_cost = 1e300;
  for (int t = 0; t < (plain_epilogue ? 5 : 4); ++t) {
    const long tiles = (long)((M + bm[t] - 1) / bm[t]) * ((N + bn[t] - 1) / bn[t]);
    const long n = (tiles + 255) / 256;
    double e = eff_full[t];
    if (n < per_cu[t]) e = eff_single[t] + (eff_full[t] - eff_single[t]) * (double)(n - 1) / (per_cu[t] - 1);
    double rounds = (double)n;
    if (t == 0 && atomic_nk >= 128 && tiles <= 128) rounds = 0.55;
    const double cost = rounds * bm[t] * bn[t] / e;
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

size_t gemm_arranged_bytes(int N, int K) { return (size_t)((N + 63) / 64) * (size_t)((K + 63) / 64) * 8192; }

hipError_t gemm_arrange(hipStream_t st, const void* B, long ldb, int N, int K, int transposed, void* out) {
  if (N <= 0 || K <= 0) return hipSuccess;
  if (!B || !out || K % 8 || ldb % 8 || (transposed && N % 8)) return hipErrorInvalidValue;
  const long chunks = (long)(gemm_arranged_bytes(N, K) / 16);
  RP_LAUNCH(gemm_arrange_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, st, (const bf16*)B, ldb, N, K, transposed,
            (uint4*)out, chunks, (K + 63) / 64);
  return hipGetLastError();
}

int gemm_pick_tile(const GemmArgs& a, int tile_hint) {
  if (a.b_direct) return 1;
  if (a.epi == EPI_CE_STATS || a.epi == EPI_F32_COLMAX || a.epi == EPI_CE_P || a.epi == EPI_SWIGLU_FWD) return 1;   // the partial-row numbering assumes 256-row tiles of two wave rows
  if (tile_hint) return tile_hint;
  // the eight-wave 256x128 tile is used for the plain epilogues
  const bool plain = a.epi == EPI_BF16 || a.epi == EPI_F32 || a.epi == EPI_F32_ATOMIC;
  const bool can_split = a.epi == EPI_F32 && (a.beta || a.split_out_bf16) && a.split_ws;
  const int atomic_nk = can_split ? (a.K + 63) / 64 + (a.K2 + 63) / 64 : 0;
  return choose_tile(a.M, a.N, plain, atomic_nk, (a.K + 63) / 64 + (a.K2 + 63) / 64);
}

hipError_t gemm_launch(hipStream_t st, int layout, const GemmArgs& a_in, int tile_hint) {
  if (a_in.M <= 0 || a_in.N <= 0) return hipSuccess;
  if (layout < GEMM_NT || layout > GEMM_TN) return hipErrorInvalidValue;
  GemmArgs a = a_in;
  // 16-byte accesses everywhere: the output width and every leading dimension must keep rows aligned
  const bool out_f32 = a.epi == EPI_F32 || a.epi == EPI_F32_ATOMIC || a.epi == EPI_F32_COLMAX;
  if (a.epi == EPI_F32_COLMAX && (a.beta || !a.part || !a.labels || !a.zlab)) return hipErrorInvalidValue;
  if (a.run_flag && (a.epi != EPI_F32_COLMAX || layout != GEMM_NT)) return hipErrorInvalidValue;
  if (a.epi == EPI_CE_P && (!a.part || !a.labels || !a.zlab || !a.lse)) return hipErrorInvalidValue;
  if (a.N % 8 || a.K % 8 || a.lda % 8 || (!a.b_direct && a.ldb % 8)) return hipErrorInvalidValue;
  if (a.epi != EPI_CE_STATS && a.ldc % (out_f32 ? 4 : 8)) return hipErrorInvalidValue;
  if (a.R && a.ldr % 4) return hipErrorInvalidValue;
  if (a.epi == EPI_SWIGLU_FWD && (layout != GEMM_NT || !a.C2 || a.R || a.b_direct || a.N % 256 || a.ldc2 % 8 || a.alpha != 1.f))
    return hipErrorInvalidValue;
  if (a.epi == EPI_SWIGLU_BWD && (!a.R || a.ldr % 8 || a.ldc % 8 || a.grp_tab)) return hipErrorInvalidValue;
  const bool ta = layout == GEMM_TN, tb = layout != GEMM_NT;
  if (ta && a.M % 8) return hipErrorInvalidValue;
  if (!a.A2 || !a.B2) a.K2 = 0;
  if (a.K2 && (a.K2 % 8 || a.lda2 % 8 || (!a.b_direct && a.ldb2 % 8))) return hipErrorInvalidValue;
  a.bytesA = ta ? extent_bytes(a.K, a.M, a.lda) : extent_bytes(a.M, a.K, a.lda);
  a.bytesB = tb ? extent_bytes(a.K, a.N, a.ldb) : extent_bytes(a.N, a.K, a.ldb);
  a.bytesA2 = ta ? extent_bytes(a.K2, a.M, a.lda2) : extent_bytes(a.M, a.K2, a.lda2);
  a.bytesB2 = tb ? extent_bytes(a.K2, a.N, a.ldb2) : extent_bytes(a.N, a.K2, a.ldb2);
  if (a.b_direct) {
    if (ta || a.grp_tab || a.run_flag) return hipErrorInvalidValue;
    const size_t b1 = gemm_arranged_bytes(a.N, a.K), b2 = a.K2 ? gemm_arranged_bytes(a.N, a.K2) : 0;
    if (b1 >= ((size_t)1 << 31) || b2 >= ((size_t)1 << 31)) return hipErrorInvalidValue;
    a.bytesB = (unsigned)b1;
    a.bytesB2 = (unsigned)b2;
  }
  // operands are addressed with 32-bit byte offsets
  if (a.bytesA == ~0u || a.bytesB == ~0u || a.bytesA2 == ~0u || a.bytesB2 == ~0u) return hipErrorInvalidValue;
  int tile = gemm_pick_tile(a, tile_hint == 7 ? 1 : tile_hint);
  if (a.grp_tab) {   // grouped: 256-row tiles as in the table, rows of A are tile rows, one operand pair
    if (ta || a.K2 || !a.grp_ntiles || a.grp_max_tiles <= 0 || (a.epi != EPI_BF16 && a.epi != EPI_F32 && a.epi != EPI_SWIGLU_FWD)) return hipErrorInvalidValue;
    tile = 1;
    if (a.row_map) {
      a.bytesA = extent_bytes(a.row_map_rows, a.K, a.lda);
      if (a.bytesA == ~0u || a.row_map_rows <= 0) return hipErrorInvalidValue;
    }
  }
  // Reduction split: only for outputs that accumulate in fp32 (or skinny products merged into bf16) and only when the
  // caller gave scratch memory for the slices' partial products, when the 256x256 tiling would leave at least half of
  // the CUs without work and every slice still gets a long K loop.  The slices are added in a fixed order by a second
  // kernel: results are reproducible run to run.
  a.splits = 1;
  a.c_slice_stride = 0;
  if (a.split_out_bf16 && (a.epi != EPI_F32 || !a.split_ws || a.ldc % 4 || (size_t)a.M * a.N * 4 > a.split_ws_bytes)) return hipErrorInvalidValue;
  if ((tile == 1 || tile == 5) && a.epi == EPI_F32 && (a.beta || a.split_out_bf16) && a.split_ws) {
    const int bn = tile == 1 ? 256 : 128;
    const long tiles = (long)((a.M + 255) / 256) * ((a.N + bn - 1) / bn);
    const int nk = (a.K + 63) / 64 + (a.K2 + 63) / 64;
    int sp = (int)(256 / tiles);
    // a skinny output (few rows or few columns) is bound by reading the other operand once: short slices are fine,
    // idle CUs are not
    const bool skinny = a.N <= 64 || a.M <= 64;
    const int min_slice = skinny ? 4 : 16;
    while (sp > 1 && nk / sp < min_slice) --sp;
    if (sp > (skinny ? 16 : 8)) sp = skinny ? 16 : 8;
    while (sp > 1 && (size_t)sp * a.M * a.N * 4 > a.split_ws_bytes) --sp;
    a.splits = sp;
  }
  if (a.split_out_bf16 && a.splits == 1) { a.epi = EPI_BF16; a.split_out_bf16 = 0; }   // nothing to merge: one direct pass
  void* const C_final = a.C;
  const long ldc_final = a.ldc;
  const int beta_final = a.beta;
  const bool merged = a.splits > 1;
  if (merged) {   // the slices write fp32 partials [slice][M][N]
    a.C = a.split_ws; a.ldc = a.N; a.beta = 0; a.c_slice_stride = (long)a.M * a.N;
  }
  hipError_t e;
  // Products on 256x256 tiles run the four-wave kernel that loads its operands straight into LDS (gemm_dtl.hip) when
  // the reduction is at least 40 K tiles long -- its per-tile fixed cost (four waves doing the epilogue in two halves, a
  // deeper prologue) is higher, and at K = 2048 with a cross-entropy or SwiGLU epilogue the eight-wave kernel is 9 %
  // faster -- unless a kernel is asked for by name (hint 1: eight waves, hint 7: four) or the variant has no
  // counterpart there.
  // Skinny outputs (the LoRA products, bound by reading the other operand once) stay on the eight-wave kernel too: +14 %.
  const bool dtl = tile == 1 && tile_hint != 1 && !a.run_flag && !a.b_direct && (tile_hint == 7 || (a.K + a.K2 >= 2560 && a.M > 64 && a.N > 64));
  if (dtl) {
    e = gemm_dtl_launch(st, a, layout);
  } else {
    switch (layout) {
      case GEMM_NT: e = launch_tile<false, false>(st, a, tile); break;
      case GEMM_NN: e = launch_tile<false, true>(st, a, tile); break;
      default: e = launch_tile<true, true>(st, a, tile); break;
    }
  }
  if (e != hipSuccess || !merged) return e;
  const long quads = (long)a.M * (a.N / 4);
  const int grid = (int)((quads + 255) / 256 < 4096 ? (quads + 255) / 256 : 4096);
  if (a.split_out_bf16)
    RP_LAUNCH(splitk_merge_kernel<true>, dim3(grid), dim3(256), 0, st, a.split_ws, a.splits, a.c_slice_stride, C_final, ldc_final, a.M, a.N, 0);
  else
    RP_LAUNCH(splitk_merge_kernel<false>, dim3(grid), dim3(256), 0, st, a.split_ws, a.splits, a.c_slice_stride, C_final, ldc_final, a.M, a.N, beta_final);
  return hipGetLastError();
}
