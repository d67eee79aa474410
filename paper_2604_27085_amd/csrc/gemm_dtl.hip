// bf16 GEMM C = A * B^T (NT: both operands reduction-contiguous), C = A * B (NN: B is [K, N]) or C = A^T * B (TN: A is
// [K, M] as well), 256x256 output tile, operands loaded from HBM straight into LDS (no staging registers, no LDS store instructions) and four waves of 128x128
// each -- one wave per SIMD, 256 accumulator registers per lane (the AGPR half of the register file).
//
// Against the eight-wave kernel of gemm.hip a K tile of the same output tile costs a third fewer fragment reads (every
// fragment feeds four MFMAs), no LDS stores and hardly any vector or scalar arithmetic: the loop is 64 MFMAs, 32
// fragment reads, 16 loads and a barrier.  What pays for it is that nothing covers a stall -- there is no second wave on
// the SIMD -- so the loop is laid out slot by slot (one MFMA plus at most one memory instruction, which has to issue
// within the 32 cycles the MFMA runs), every fragment is read a 16-deep step ahead and every load one to two K tiles
// ahead.  Measured on MI355X (8192^3, same box): 1.38-1.42 PFLOP/s against 1.29-1.31 for the eight-wave kernel as NT,
// 1.43 against 1.31 as NN, 1.30 against 1.20 as TN; matrix pipe busy 85 % of the kernel's cycles against 77-78 %.
//
//   LDS       a ring of five 32 KB units; a unit is one operand of one K tile of 64: 256 rows of 128 bytes -- a load
//             fetches whole 128-byte lines (rows of 64 bytes, as a K tile of 32 would have, double the requests to L2:
//             measured, and slower than the staged kernel).  The 16-byte chunk c of row r sits at chunk position
//             c ^ ((r >> 1) & 7): fragment reads meet no bank conflict, and since a load instruction fills 1 KB of LDS
//             with consecutive lanes while the 16 bytes a lane fetches are free to choose, the swizzle costs nothing.
//             Units are used in the order B(0), A(0), B(1), A(1), ...: unit u lives in ring slot u mod 5.
//   loads     eight per wave and unit, one every other slot where no fragment is read.  B(t+2) is issued in the
//             first half of tile t (into the slot of A(t-1), free since the barrier of tile t-1), A(t+2) behind the
//             barrier of tile t (into the slot of B(t)).
//   barrier   one per K tile, at slot 44 of 64: by then the wave has all its fragments of tile t.  Before it the wave
//             waits for its own loads of tile t+1 (s_waitcnt vmcnt(8): B(t+2) may be in flight); after it tile t+1 is
//             complete in LDS and its first fragments are read under the last step of tile t.
//   tail      tiles past the end are "loaded" with an offset outside the descriptor (no memory traffic), which keeps
//             the number of loads in flight -- and with it the s_waitcnt immediates -- the same to the end.
//
// The loads are inline assembly: the compiler orders a buffer-load-to-LDS builtin against every later LDS read with
// s_waitcnt vmcnt(0), which would serialise the pipeline; here the counts are kept by hand, and no compiler-visible
// memory instruction may be pending when the loop is entered (see the rare paths of the load state).
//   NN        B's units keep the operand's [K, N] layout (64 rows of 512 bytes; the 64-byte segment of MFMA tile column
//             s of row k at segment s ^ (k & 3)), its fragments are two transposing reads (ds_read_b64_tr_b16) each:
//             twelve read instructions and four loads per 16-slot step, a slot plan of its own.
//   TN        the same for A: sixteen reads per step, one per slot, the loads on top of them.
// Second operand pair, row map, grouped mode, reduction slices and every epilogue of gemm_device.hpp (applied to the
// two 128x64 halves of a wave's block in turn) as in gemm.hip; results are bit-identical to its 256x256 tile (same
// MFMA, same order of the reduction).  gemm_launch picks this kernel for reductions of 40 K tiles or more and outputs
// that are not skinny: its fixed cost per output tile is higher than the eight-wave kernel's.
#include "gemm_device.hpp"
#include <type_traits>
#include <utility>

using namespace gemm_dev;

namespace {

typedef int i32x4 __attribute__((ext_vector_type(4)));
template <int V>
using IC = std::integral_constant<int, V>;
// f(IC<0>), f(IC<1>), ... in order: a loop whose index is a constant expression in its body
template <class F, int... S>
RP_DEV void for_seq(F&& f, std::integer_sequence<int, S...>) {
  (f(IC<S>{}), ...);
}

constexpr int BK = 64;                            // reduction indices per K tile: a row of a tile is one 128-byte line
constexpr int UNIT_BYTES = 256 * BK * 2;          // one operand of one K tile: 256 rows of 128 bytes, 32 KB
constexpr int NUNIT = 5;
constexpr int DTL_SMEM = NUNIT * UNIT_BYTES;      // 160 KB: the whole LDS of a CU; the epilogue's four staging areas (72 KB) reuse it
static_assert(DTL_SMEM >= 4 * STG_BYTES, "epilogue staging does not fit");

// 64 lanes x 16 bytes from the buffer (per-lane byte offset voff, wave-uniform soff) to LDS bytes [lds + IMM,
// lds + IMM + 1024) of the workgroup, lane l at + 16 l.  Lanes whose offset lies outside the descriptor deliver zeros.
// The LDS address travels in M0.
template <int IMM>
RP_DEV void load_to_lds(uint32_t lds, uint32_t voff, i32x4 rs, uint32_t soff) {
  asm volatile("s_add_u32 m0, %0, %3\n\tbuffer_load_dwordx4 %1, %2, %4 offen lds"
               :
               : "s"(lds), "v"(voff), "s"(rs), "n"(IMM), "s"(soff)
               : "memory", "scc");
}

RP_DEV i32x4 raw_rsrc(const void* base, uint32_t bytes) {
  const uint64_t b = reinterpret_cast<uint64_t>(base);
  i32x4 r;
  r.x = (int)(uint32_t)b;
  r.y = (int)((uint32_t)(b >> 32) & 0xffffu);
  r.z = (int)bytes;
  r.w = 0x00020000;
  return r;
}

// TB: the B operand is [K, N] (reduction index strided, the NN product); its units keep that layout and its fragments
// are read with the transposing LDS load.  TA (with TB: the TN product): the same for A, which is [K, M].
template <bool TA, bool TB>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) gemm_dtl_kernel(const GemmArgs p) {
  static_assert(!TA || TB, "A transposed alone is not a layout of this library");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int lr = lane & 31, lk = lane >> 5;

  int tile_m, tile_n, m0, Mlim = p.M;
  const bf16* Bbase = static_cast<const bf16*>(p.B);
  if (p.grp_tab) {   // uniform over the grid
    const int tiles_n = (p.N + 255) / 256;
    tile_m = (int)blockIdx.x / tiles_n;
    tile_n = (int)blockIdx.x % tiles_n;
    if (tile_m >= *p.grp_ntiles) return;
    const int4 g = p.grp_tab[tile_m];
    m0 = g.y;
    Mlim = g.y + g.z;
    Bbase += (long)g.x * p.grp_strideB;
  } else {
    // narrow outputs (up to 24 tile columns) sweep their columns in groups of 4 tile rows, wide ones of 8: measured
    // +2-3 % at N = 5120, -1.5-2 % at N >= 10240 for groups of 4
    tile_of_block(p.M, p.N, 256, 256, tile_m, tile_n, (p.N + 255) / 256 <= 24 ? 4 : 8);
    m0 = tile_m * 256;
  }
  const int n0 = tile_n * 256;
  const int nk1 = (p.K + BK - 1) / BK;
  const int nk_all = nk1 + (p.K2 + BK - 1) / BK;
  const int per_split = (nk_all + (int)gridDim.y - 1) / (int)gridDim.y;
  const int kt0 = (int)blockIdx.y * per_split;
  const int nk = (nk_all - kt0) < per_split ? (nk_all - kt0 > 0 ? nk_all - kt0 : 0) : per_split;

  // a folded tile (SwiGLU forward): every wave's block is 64 gate columns and the 64 up columns that go with them
  const int fold = (!TB && p.epi == EPI_SWIGLU_FWD) ? p.N >> 1 : 0;   // uniform

  // Load instruction i (0..7 per operand) of this wave fills the 1 KB block 8*wave + i of a unit.
  //   reduction-contiguous operand: operand rows 8*(8*wave + i) .. + 7, lane l -> row + (l >> 3), chunk position l & 7,
  //     i.e. data chunk (l & 7) ^ ((row >> 1) & 7);
  //   TB: the unit is [64 reduction rows][256 columns] (512-byte rows, eight 64-byte segments = MFMA tile columns each);
  //     reduction rows 2*(8*wave + i), + 1, lane l -> row + (l >> 5), chunk position l & 31, whose segment (l & 31) >> 2
  //     holds data segment ((l & 31) >> 2) ^ (row & 3): the four reduction rows a transposing read touches at once
  //     lie in four different quarters of the banks.
  uint32_t voA[8], voB[8];
  int lch[2];     // the lane's data chunk in even / odd instructions (rows 8 apart flip bit 2 of the swizzle)
  auto b_offset = [&](int i, long ldb) -> uint32_t {   // byte offset of the lane's chunk of load i of a B unit at reduction offset 0
    if constexpr (!TB) {
      const int r = 8 * (8 * wave + i) + (lane >> 3);
      const int ch = (lane & 7) ^ ((r >> 1) & 7);
      const int gn = fold ? (n0 >> 1) + (r >> 7) * 64 + (r & 63) + ((r >> 6) & 1) * fold : n0 + r;
      return gn < p.N ? (uint32_t)((long)gn * ldb + ch * 8) * 2u : OOB;
    } else {
      const int kr = 2 * (8 * wave + i) + (lane >> 5);
      const int pos = lane & 31;
      const int gn = n0 + (((pos >> 2) ^ (kr & 3)) * 32) + (pos & 3) * 8;
      return gn < p.N ? (uint32_t)((long)kr * ldb + gn) * 2u : OOB;
    }
  };
  auto a_offset = [&](int i, long lda, bool first) -> uint32_t {   // the same for A (rows of a transposed A are not mapped)
    if constexpr (!TA) {
      const int r = 8 * (8 * wave + i) + (lane >> 3);
      const int ch = (lane & 7) ^ ((r >> 1) & 7);
      const int gm = m0 + r;
      if (!first) return gm < p.M ? (uint32_t)((long)gm * lda + ch * 8) * 2u : OOB;
      const long srcm = (p.row_map && gm < Mlim) ? p.row_map[gm] : gm;
      return gm < Mlim ? (uint32_t)(srcm * lda + ch * 8) * 2u : OOB;
    } else {
      const int kr = 2 * (8 * wave + i) + (lane >> 5);
      const int pos = lane & 31;
      const int gm = m0 + (((pos >> 2) ^ (kr & 3)) * 32) + (pos & 3) * 8;
      return gm < (first ? Mlim : p.M) ? (uint32_t)((long)kr * lda + gm) * 2u : OOB;
    }
  };
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = 8 * (8 * wave + i) + (lane >> 3);
    const int ch = (lane & 7) ^ ((r >> 1) & 7);
    lch[i & 1] = ch;
    voA[i] = a_offset(i, p.lda, true);
    voB[i] = b_offset(i, p.ldb);
  }
  const i32x4 rsA = raw_rsrc(p.A, p.bytesA), rsB = raw_rsrc(Bbase, p.bytesB);
  i32x4 rsA2 = rsA, rsB2 = rsB;
  if (p.K2 > 0) {
    rsA2 = raw_rsrc(p.A2, p.bytesA2);
    rsB2 = raw_rsrc(p.B2, p.bytesB2);
  }
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const uint32_t lds_wave = lds0 + (uint32_t)wave * 8192u;

  // Loads are issued tile by tile in order (B of a tile, then A); the state of the tile being loaded: its offsets and
  // descriptors (first or second operand pair), its reduction offset, the masks that send the chunks past the end of the
  // reduction outside the descriptor (all zero except in the last tile of an operand pair), and its two ring slots.
  uint32_t vcA[8], vcB[8];
  i32x4 rcA = rsA, rcB = rsB;
#pragma unroll
  for (int i = 0; i < 8; ++i) { vcA[i] = voA[i]; vcB[i] = voB[i]; }
  int ld_kt = kt0, ld_k0 = kt0 * BK, ld_Klim = p.K;
  bool ld_second = false, ld_live = true;
  uint32_t ld_soff = 0, ld_soffB = 0;
  uint32_t ld_kstepA = TA ? (uint32_t)p.lda * 2u : 2u;
  uint32_t ld_kstepB = TB ? (uint32_t)p.ldb * 2u : 2u;   // bytes per reduction index in the B operand
  uint32_t ld_ring = 0;          // byte offset of the ring slot of the tile's B unit; its A unit is the next slot
  uint32_t ld_ldsB = 0, ld_ldsA = 0;
  // before the loads of local tile s = 0, 1, 2, ..., in three parts (for slots of their own in the K loop); tiles past
  // the end take neither of the two rare paths, which drain the loads in flight
  auto setup_pair = [&](int s) {
    ld_live = s < nk;
    if (ld_live && !ld_second && ld_kt >= nk1) {   // uniform, at most once per kernel: on to the second operand pair
      asm volatile("" ::: "memory");    // (keeps this a branch: as selects it would cost dozens of instructions per tile)
      ld_second = true;
      ld_k0 = (ld_kt - nk1) * BK;
      ld_Klim = p.K2;
      rcA = rsA2;
      rcB = rsB2;
      if (p.K2 > 0) {   // the offsets of the second pair are worked out here rather than kept in registers through the loop
        if constexpr (TB) ld_kstepB = (uint32_t)p.ldb2 * 2u;
        if constexpr (TA) ld_kstepA = (uint32_t)p.lda2 * 2u;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          vcA[i] = a_offset(i, p.lda2, false);
          vcB[i] = b_offset(i, p.ldb2);
        }
      }
      // Whatever the compiler reloads from scratch memory on this path counts in vmcnt like the loads above; left
      // pending, its own s_waitcnt before the first use of such a register would sit in the K loop and drain the
      // pipeline every tile.
      __builtin_amdgcn_s_waitcnt(0x0f70);
    }
    ld_soff = s < nk ? (uint32_t)ld_k0 * ld_kstepA : OOB;   // (from s, not from the flag: the scalar offset has to stay provably wave-uniform)
    ld_soffB = s < nk ? (uint32_t)ld_k0 * ld_kstepB : OOB;
    ++ld_kt;
  };
  auto setup_mask = [&]() {
    if (ld_live && ld_k0 + BK > ld_Klim) {   // uniform: the last tile of an operand pair that is not a multiple of 64 deep
      asm volatile("" ::: "memory");
      // chunks past the end of the reduction move outside the descriptor; the offsets are not needed unmasked again
      // (the next tile belongs to the other pair, whose offsets are worked out afresh, or lies past the end)
      const uint32_t mk0 = (ld_k0 + lch[0] * 8 < ld_Klim) ? 0u : OOB, mk1 = (ld_k0 + lch[1] * 8 < ld_Klim) ? 0u : OOB;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint32_t mkr = (ld_k0 + 2 * (8 * wave + i) + (lane >> 5) < ld_Klim) ? 0u : OOB;   // row-wise, for [K, X] units
        vcA[i] |= TA ? mkr : ((i & 1) ? mk1 : mk0);
        vcB[i] |= TB ? mkr : ((i & 1) ? mk1 : mk0);
      }
      __builtin_amdgcn_s_waitcnt(0x0f70);   // as at the end of the pair switch
    }
    ld_k0 += BK;
  };
  auto setup_lds = [&]() {
    ld_ldsB = lds_wave + ld_ring;
    ld_ring = ld_ring + UNIT_BYTES == (uint32_t)DTL_SMEM ? 0u : ld_ring + UNIT_BYTES;
    ld_ldsA = lds_wave + ld_ring;
    ld_ring = ld_ring + UNIT_BYTES == (uint32_t)DTL_SMEM ? 0u : ld_ring + UNIT_BYTES;
  };
  auto tile_setup = [&](int s) { setup_pair(s); setup_mask(); setup_lds(); };
  auto issue_b = [&](auto itag) __attribute__((always_inline)) {
    constexpr int i = decltype(itag)::value;
    load_to_lds<i * 1024>(ld_ldsB, vcB[i], rcB, ld_soffB);
  };
  auto issue_a = [&](auto itag) __attribute__((always_inline)) {
    constexpr int i = decltype(itag)::value;
    load_to_lds<i * 1024>(ld_ldsA, vcA[i], rcA, ld_soff);
  };

  f32x16 acc[2][TM][TN];
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[h][i][j][v] = 0.f;

  // fragment reads: lane -> row lr of a 32-row MFMA tile, data chunk 2*ks + lk, at chunk position chunk ^ ((lr >> 1) & 7).
  // fkA[ks] / fkB[ks]: byte offset of the lane's chunk of step ks in the wave's first MFMA tile of a unit; MFMA tile i
  // (j) lies another 4 KB further each.
  const int s7 = (lr >> 1) & 7;
  uint32_t fkA[4], fkB[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    fkA[ks] = (uint32_t)((wm * 128 + lr) * 128 + ((2 * ks + lk) ^ s7) * 16);
    fkB[ks] = (uint32_t)((wn * 128 + lr) * 128 + ((2 * ks + lk) ^ s7) * 16);
  }
  uint4 af[2][4], bfr[2][4];
  auto read_a = [&](int set, uint32_t off, int i) { af[set][i] = *reinterpret_cast<const uint4*>(smem + off + i * 4096); };
  auto read_b = [&](int set, uint32_t off, int j) { bfr[set][j] = *reinterpret_cast<const uint4*>(smem + off + j * 4096); };
  // TB: a fragment of B is two transposing reads (reduction rows +0..3 and +4..7 of the lane's half of the 16-deep step).
  // fkBt[j]: byte offset of the lane's first read of step 0 for MFMA tile column j of the wave: reduction row
  // 8*lk + (l%16)/4, the tile column's segment moved by the row's swizzle, columns 16*((l/16)%2) + 4*(l%4) of the tile.
  [[maybe_unused]] uint32_t fkBt[4];
  if constexpr (TB) {
    const int l16 = lane & 15, g16 = lane >> 4, c2 = l16 >> 2;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      fkBt[j] = (uint32_t)((8 * lk + c2) * 512 + (((wn * 4 + j) ^ c2) * 64) + 32 * (g16 & 1) + 8 * (l16 & 3));
  }
  [[maybe_unused]] uint32_t fkAt[4];
  if constexpr (TA) {
    const int l16 = lane & 15, g16 = lane >> 4, c2 = l16 >> 2;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      fkAt[i] = (uint32_t)((8 * lk + c2) * 512 + (((wm * 4 + i) ^ c2) * 64) + 32 * (g16 & 1) + 8 * (l16 & 3));
  }
  [[maybe_unused]] auto read_at = [&](int set, uint32_t off, int i, int half) {
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4* lds_ptr;
    const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(smem + off + half * 2048));
    const uint2 u = __builtin_bit_cast(uint2, v);
    if (half == 0) { af[set][i].x = u.x; af[set][i].y = u.y; }
    else { af[set][i].z = u.x; af[set][i].w = u.y; }
  };
  [[maybe_unused]] auto read_bt = [&](int set, uint32_t off, int j, int half) {   // off includes the step: + ks * 8192
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4* lds_ptr;
    const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(smem + off + half * 2048));
    const uint2 u = __builtin_bit_cast(uint2, v);
    if (half == 0) { bfr[set][j].x = u.x; bfr[set][j].y = u.y; }
    else { bfr[set][j].z = u.x; bfr[set][j].w = u.y; }
  };

  // prologue: tiles 0 and 1 set out (in the order of the K loop: B, then A); tile 0 has landed everywhere after the barrier
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    tile_setup(s);
    issue_b(IC<0>{}); issue_b(IC<1>{}); issue_b(IC<2>{}); issue_b(IC<3>{}); issue_b(IC<4>{}); issue_b(IC<5>{}); issue_b(IC<6>{}); issue_b(IC<7>{});
    issue_a(IC<0>{}); issue_a(IC<1>{}); issue_a(IC<2>{}); issue_a(IC<3>{}); issue_a(IC<4>{}); issue_a(IC<5>{}); issue_a(IC<6>{}); issue_a(IC<7>{});
  }
  if constexpr (!TB) tile_setup(2);   // (the loops for transposed operands set the state of tile t+2 up in their first slots)
  __builtin_amdgcn_s_waitcnt(0x0f70 | (16 & 15) | ((16 >> 4) << 14));   // vmcnt(16)
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if constexpr (!TA) read_a(0, UNIT_BYTES + fkA[0], i);
    else { read_at(0, UNIT_BYTES + fkAt[i], i, 0); read_at(0, UNIT_BYTES + fkAt[i], i, 1); }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if constexpr (!TB) read_b(0, fkB[0], j);
    else { read_bt(0, fkBt[j], j, 0); read_bt(0, fkBt[j], j, 1); }
  }

  // Slot plan of tile t (64 slots of one MFMA; 16-deep step ks = slots 16 ks .. 16 ks + 15, fragment set ks & 1).  A slot
  // holds at most one memory instruction: with one wave per SIMD whatever a slot issues beside its MFMA has to fit into
  // the 32 cycles the MFMA runs, and a load or a fragment read that meets a busy texture unit or LDS queue already
  // takes most of them.
  //   slots 16 ks + 0..7   the fragment reads of step ks + 1 (of step 0 of tile t+1 for ks = 3), one per slot
  //   slots 8..15, 24..31  every other one: the loads of B of tile t+2; its ring slot (A of tile t-1) is free since
  //                        the barrier of tile t-1
  //   slot  BAR = 44       every read of this tile has returned.  vmcnt(8): the wave's loads of tile t+1 have landed
  //                        (those of B of tile t+2 may be in flight); barrier: tile t+1 is complete in LDS, this
  //                        tile's two ring slots are free
  //   slots 45..47, 56..60 the loads of A of tile t+2, into the slot of B of this tile
  //   slots 61, 62         the state of the loads of tile t+3
  constexpr int BAR = 44;
  auto main_loop = [&](auto wtag) __attribute__((always_inline)) {
    constexpr int W = decltype(wtag)::value;
    uint32_t ring = 0;                 // ring slot of B of the current tile; A follows
    uint32_t curA = UNIT_BYTES, curB = 0, nA = 0;
    uint32_t fa = curA + fkA[1], fb = curB + fkB[1];   // offsets of the reads of the coming step
    for (int t = 0; t < nk; ++t) {
      auto slot = [&](auto sltag) __attribute__((always_inline)) {
        constexpr int sl = decltype(sltag)::value;
        constexpr int ks = sl >> 4, I = sl & 15, i = I >> 2, jj = I & 3, set = ks & 1;
        if constexpr (sl == BAR) {
          __builtin_amdgcn_s_waitcnt(0x0f70 | 8);
          __syncthreads();
        }
        // one wait per step for all of its fragments (read eight slots or more ago) instead of one per fragment
        if constexpr (I == 0 && ks < 3) __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
        acc[jj >> 1][i][jj & 1] = mfma32(af[set][i], bfr[set][jj], acc[jj >> 1][i][jj & 1]);
        if constexpr (I < 4) read_a(set ^ 1, fa, I);
        if constexpr (I >= 4 && I < 8) read_b(set ^ 1, fb, I - 4);
        // address arithmetic for the reads of the coming step, in slots without a memory instruction
        if constexpr (sl == 8 + (W & 1)) fa = curA + fkA[2];
        if constexpr (sl == 10 + (W & 1)) fb = curB + fkB[2];
        if constexpr (sl == 24 + (W & 1)) fa = curA + fkA[3];
        if constexpr (sl == 26 + (W & 1)) fb = curB + fkB[3];
        if constexpr (sl == 28 + (W & 1)) ring = ring + 2 * UNIT_BYTES >= (uint32_t)DTL_SMEM ? ring + 2 * UNIT_BYTES - DTL_SMEM : ring + 2 * UNIT_BYTES;
        if constexpr (sl == 30 + (W & 1)) nA = ring + UNIT_BYTES == (uint32_t)DTL_SMEM ? 0u : ring + UNIT_BYTES;
        if constexpr (sl == 40) fa = nA + fkA[0];
        if constexpr (sl == 41) fb = ring + fkB[0];
        if constexpr (sl == 63) { fa = nA + fkA[1]; fb = ring + fkB[1]; }
        if constexpr ((sl < 32) && (I >= 8) && ((I & 1) != (W & 1))) issue_b(IC<((ks * 8 + I - 8) >> 1)>{});
        if constexpr (sl >= 45 && sl < 48) issue_a(IC<(sl - 45)>{});
        if constexpr (sl >= 56 && sl < 61) issue_a(IC<(sl - 56 + 3)>{});
        if constexpr (sl == 61) setup_pair(t + 3);
        if constexpr (sl == 62) { setup_mask(); setup_lds(); }
        __builtin_amdgcn_sched_barrier(0);
      };
      for_seq(slot, std::make_integer_sequence<int, 64>{});
      curB = ring;
      curA = nA;
    }
  };
  // The same for TB.  A step reads twelve fragments' worth of instructions (four for A, two each for the four of B), so
  // only four slots of a step are left for loads and none are empty:
  //   slots 16 ks + 0..3, 4..11  the fragment reads of A and B of step ks + 1 (of step 0 of tile t+1 for ks = 3)
  //   slots 1, 2                 the state of the loads of tile t+2
  //   slots 12..15, 28..31       the loads of B of tile t+2
  //   slot  46                   vmcnt(8); barrier
  //   slots 47, 53, 55, 57, 60..63  the loads of A of tile t+2
  [[maybe_unused]] auto main_loop_tb = [&]() __attribute__((always_inline)) {
    constexpr int BARB = 46;
    uint32_t ring = 0;
    uint32_t curA = UNIT_BYTES, nA = 0;
    uint32_t fa = curA + fkA[1];
    uint32_t fbj[4], nfbj[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) { fbj[j] = fkBt[j]; nfbj[j] = 0; }
    for (int t = 0; t < nk; ++t) {
      auto slot = [&](auto sltag) __attribute__((always_inline)) {
        constexpr int sl = decltype(sltag)::value;
        constexpr int ks = sl >> 4, I = sl & 15, i = I >> 2, jj = I & 3, set = ks & 1;
        if constexpr (sl == BARB) {
          __builtin_amdgcn_s_waitcnt(0x0f70 | 8);
          __syncthreads();
        }
        if constexpr (I == 0 && ks < 3) __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
        acc[jj >> 1][i][jj & 1] = mfma32(af[set][i], bfr[set][jj], acc[jj >> 1][i][jj & 1]);
        if constexpr (I < 4) read_a(set ^ 1, fa, I);
        if constexpr (I >= 4 && I < 12) {
          constexpr int j = (I - 4) >> 1, half = (I - 4) & 1;
          if constexpr (ks < 3) read_bt(set ^ 1, fbj[j] + (ks + 1) * 8192, j, half);
          else read_bt(0, nfbj[j], j, half);
        }
        if constexpr (sl == 1) setup_pair(t + 2);
        if constexpr (sl == 2) { setup_mask(); setup_lds(); }
        if constexpr (sl == 13) fa = curA + fkA[2];
        if constexpr (sl == 14) ring = ring + 2 * UNIT_BYTES >= (uint32_t)DTL_SMEM ? ring + 2 * UNIT_BYTES - DTL_SMEM : ring + 2 * UNIT_BYTES;
        if constexpr (sl == 15) nA = ring + UNIT_BYTES == (uint32_t)DTL_SMEM ? 0u : ring + UNIT_BYTES;
        if constexpr (sl == 29) fa = curA + fkA[3];
        if constexpr (sl == 44) { nfbj[0] = ring + fkBt[0]; nfbj[1] = ring + fkBt[1]; }
        if constexpr (sl == 45) { nfbj[2] = ring + fkBt[2]; nfbj[3] = ring + fkBt[3]; fa = nA + fkA[0]; }
        if constexpr (sl == 59) fa = nA + fkA[1];
        if constexpr (sl >= 12 && sl < 16) issue_b(IC<(sl - 12)>{});
        if constexpr (sl >= 28 && sl < 32) issue_b(IC<(sl - 28 + 4)>{});
        if constexpr (sl == 47) issue_a(IC<0>{});
        if constexpr (sl == 53) issue_a(IC<1>{});
        if constexpr (sl == 55) issue_a(IC<2>{});
        if constexpr (sl == 57) issue_a(IC<3>{});
        if constexpr (sl >= 60) issue_a(IC<(sl >= 60 ? sl - 60 + 4 : 0)>{});
        __builtin_amdgcn_sched_barrier(0);
      };
      for_seq(slot, std::make_integer_sequence<int, 64>{});
      curA = nA;
#pragma unroll
      for (int j = 0; j < 4; ++j) fbj[j] = nfbj[j];
    }
  };
  // TN: sixteen transposing reads per step, one per slot (two per slot in step 2, so that the tile's last read is
  // five slots old at the barrier), the loads on top of them:
  //   slots 1, 2                    the state of the loads of tile t+2
  //   slots 3, 7, .., 31            the loads of B of tile t+2
  //   slots 32..39                  the reads of step 3, two per slot;  40..43 the read offsets of tile t+1
  //   slot  44                      vmcnt(8); barrier
  //   slots 45, 46, 47, 51, 55, 59, 62, 63   the loads of A of tile t+2
  //   slots 48..63                  the reads of step 0 of tile t+1
  [[maybe_unused]] auto main_loop_tn = [&]() __attribute__((always_inline)) {
    constexpr int BARB = 44;
    uint32_t ring = 0, nA = 0;
    uint32_t faj[4], fbj[4], nfaj[4], nfbj[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) { faj[j] = UNIT_BYTES + fkAt[j]; fbj[j] = fkBt[j]; nfaj[j] = 0; nfbj[j] = 0; }
    for (int t = 0; t < nk; ++t) {
      auto slot = [&](auto sltag) __attribute__((always_inline)) {
        constexpr int sl = decltype(sltag)::value;
        constexpr int ks = sl >> 4, I = sl & 15, i = I >> 2, jj = I & 3, set = ks & 1;
        if constexpr (sl == BARB) {
          __builtin_amdgcn_s_waitcnt(0x0f70 | 8);
          __syncthreads();
        }
        if constexpr (I == 0 && ks < 3) __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
        acc[jj >> 1][i][jj & 1] = mfma32(af[set][i], bfr[set][jj], acc[jj >> 1][i][jj & 1]);
        if constexpr (ks < 2 || ks == 3) {   // one read per slot: A fragments in slots 0..7, B in 8..15
          constexpr int f = (I & 7) >> 1, half = I & 1;
          if constexpr (ks < 2) {
            if constexpr (I < 8) read_at(set ^ 1, faj[f] + (ks + 1) * 8192, f, half);
            else read_bt(set ^ 1, fbj[f] + (ks + 1) * 8192, f, half);
          } else {
            if constexpr (I < 8) read_at(0, nfaj[f], f, half);
            else read_bt(0, nfbj[f], f, half);
          }
        } else if constexpr (I < 8) {        // step 2: the reads of step 3, two per slot
          constexpr int f = I >> 1, half = I & 1;
          read_at(set ^ 1, faj[f] + 3 * 8192, f, half);
          read_bt(set ^ 1, fbj[f] + 3 * 8192, f, half);
        }
        if constexpr (sl == 1) setup_pair(t + 2);
        if constexpr (sl == 2) { setup_mask(); setup_lds(); }
        if constexpr (sl == 13) ring = ring + 2 * UNIT_BYTES >= (uint32_t)DTL_SMEM ? ring + 2 * UNIT_BYTES - DTL_SMEM : ring + 2 * UNIT_BYTES;
        if constexpr (sl == 14) nA = ring + UNIT_BYTES == (uint32_t)DTL_SMEM ? 0u : ring + UNIT_BYTES;
        if constexpr (sl >= 40 && sl < 44) { nfaj[sl - 40] = nA + fkAt[sl - 40]; nfbj[sl - 40] = ring + fkBt[sl - 40]; }
        if constexpr (sl < 32 && (sl & 3) == 3) issue_b(IC<(sl >> 2)>{});
        if constexpr (sl >= 45 && sl < 48) issue_a(IC<(sl - 45)>{});
        if constexpr (sl == 51) issue_a(IC<3>{});
        if constexpr (sl == 55) issue_a(IC<4>{});
        if constexpr (sl == 59) issue_a(IC<5>{});
        if constexpr (sl == 62) issue_a(IC<6>{});
        if constexpr (sl == 63) issue_a(IC<7>{});
        __builtin_amdgcn_sched_barrier(0);
      };
      for_seq(slot, std::make_integer_sequence<int, 64>{});
#pragma unroll
      for (int j = 0; j < 4; ++j) { faj[j] = nfaj[j]; fbj[j] = nfbj[j]; }
    }
  };
  if constexpr (TA) {
    main_loop_tn();
  } else if constexpr (TB) {
    main_loop_tb();
  } else {
  // (one plan for all four waves: staggering the waves' load slots against each other measured 0.5-1.5 % slower)
  main_loop(std::integral_constant<int, 1>{});
  }
  __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0): the empty loads past the end write LDS too
  __syncthreads();                      // every wave is done with the operand stages: the epilogue reuses the LDS

  // The accumulators live in the AGPR half of the register file, which only MFMAs and copies can address.  Left to the
  // compiler all 256 are copied out at once behind the loop and half of them spilled; here each 128x64 half is copied
  // out right before its epilogue.
  f32x16 half[TM][TN];
  auto fetch = [&](int h) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(half[i][j][v]) : "a"(acc[h][i][j][v]));
  };
  asm volatile("s_nop 7\n\ts_nop 7");   // the last MFMA has long retired (a barrier ago); the copies are invisible to the hazard checks
  const int wrow = m0 + wm * 128;
  const int part_row = p.part_row0 + tile_m * 2 + wm;
  if (fold) {
    // gate | up as by EPI_BF16, then silu(gate) * up from the rounded values (what the SwiGLU kernel would read back)
    GemmArgs q = p;
    q.epi = EPI_BF16;
    const int gcol = (n0 >> 1) + wn * 64;
    fetch(1);
    epilogue(q, Mlim, half, smem, wave, lane, wrow, gcol + fold, part_row);
    fetch(0);
    epilogue(q, Mlim, half, smem, wave, lane, wrow, gcol, part_row);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float up;
          asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(up) : "a"(acc[1][i][j][v]));
          const float g = bf16_bits_to_f32(f32_to_bf16_bits(half[i][j][v])), u = bf16_bits_to_f32(f32_to_bf16_bits(up));
          half[i][j][v] = g / (1.f + __expf(-g)) * u;
        }
    q.C = p.C2;
    q.ldc = p.ldc2;
    q.N = fold;
    epilogue(q, Mlim, half, smem, wave, lane, wrow, gcol, part_row);
    return;
  }
  fetch(0);
  epilogue(p, Mlim, half, smem, wave, lane, wrow, n0 + wn * 128, part_row);
  fetch(1);
  epilogue(p, Mlim, half, smem, wave, lane, wrow, n0 + wn * 128 + 64, part_row);
}

}  // namespace

template <bool TA, bool TB>
static hipError_t dtl_launch_one(hipStream_t st, const GemmArgs& a) {
  static bool attr_done = false;
  auto kern = gemm_dtl_kernel<TA, TB>;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, DTL_SMEM);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  int tiles = ((a.M + 255) / 256) * ((a.N + 255) / 256);
  if (a.grp_tab) tiles = a.grp_max_tiles * ((a.N + 255) / 256);
  RP_LAUNCH(kern, dim3(tiles, a.splits > 0 ? a.splits : 1), dim3(256), DTL_SMEM, st, a);
  return hipGetLastError();
}

hipError_t gemm_dtl_launch(hipStream_t st, const GemmArgs& a, int layout) {
  switch (layout) {
    case GEMM_NT: return dtl_launch_one<false, false>(st, a);
    case GEMM_NN: return dtl_launch_one<false, true>(st, a);
    default: return dtl_launch_one<true, true>(st, a);
  }
}
