// Device-side building blocks shared by the GEMM kernels: buffer loads, operand tile layouts in LDS, MFMA fragment
// reads (plain and hardware-transposed), the workgroup -> tile mapping and the LDS-staged epilogue.
#pragma once
#include "common.hpp"
#include "gemm.hpp"

namespace gemm_dev {

constexpr int TM = 4, TN = 2;            // 32x32 MFMA tiles per wave: every wave owns a 128 x 64 block of C
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

// LDS layout of one operand tile.
//   !TR: the operand is [Xdim, Kdim] in memory (reduction index contiguous): tile [BX][BK + 8]; MFMA fragments are
//        plain 16-byte LDS reads.
//    TR: the operand is [Kdim, Xdim] (reduction index strided): tile [BK][BX + 32] -- the memory layout is kept, and
//        fragments are read with the transposing LDS load (ds_read_b64_tr_b16), which hands every lane four
//        consecutive reduction indices of its own column.  No register transposes anywhere.
// The pads (8 resp. 32 elements) keep both kinds of fragment reads free of bank conflicts.
template <int BX, int BK, bool TR>
struct TileShape {
  static constexpr int ROWS = TR ? BK : BX;
  static constexpr int CH = (TR ? BX : BK) / 8;            // 16-byte data chunks per tile row
  static constexpr int PADCH = TR ? 4 : 1;                 // 16-byte pad chunks per tile row
  static constexpr int LDROW = (CH + PADCH) * 8;           // row stride in elements
  static constexpr int ELEMS = ROWS * LDROW;
};

// MFMA operand fragment (8 consecutive reduction indices of the lane's row/column) of 16-deep step ks.
//   !TR: base points at S[x_lane][8*lk];  TR: base points at S[8*lk + (l%16)/4][x_group + 4*(l%4)].
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

// Per-lane offset (elements) of the fragment base inside an operand tile, for the wave whose block starts at x_wave.
template <int LDROW, bool TR>
RP_DEV int frag_base(int lane, int x_wave) {
  const int lr = lane & 31, lk = lane >> 5, l16 = lane & 15, g16 = lane >> 4;
  return TR ? (8 * lk + (l16 >> 2)) * LDROW + x_wave + 16 * (g16 & 1) + 4 * (l16 & 3) : (x_wave + lr) * LDROW + lk * 8;
}

// Workgroup -> output tile: XCD-aware remap (consecutive logical ids share an XCD's L2), then groups of GM tile rows
// sweep the tile columns.
RP_DEV void tile_of_block(int M, int N, int BM, int BN, int& tile_m, int& tile_n, int GM = 8) {
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  const int pid = xcd_remap(blockIdx.x, tiles_m * tiles_n);
  const int group = pid / (GM * tiles_n);
  const int first_m = group * GM;
  const int gm = (tiles_m - first_m) < GM ? (tiles_m - first_m) : GM;
  const int in_group = pid - group * GM * tiles_n;
  tile_m = first_m + in_group % gm;
  tile_n = in_group / gm;
}

// A wave stages its block through LDS that no other wave touches: the LDS executes one wave's accesses in order, so
// the read-back only has to stay behind the writes in the instruction stream.
RP_DEV void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Local row (relative to the wave's block, minus the lane's 4*lk) of accumulator register v of MFMA tile row i.
RP_DEV constexpr int acc_row(int i, int v) { return i * 32 + 8 * (v >> 2) + (v & 3); }

// max(a, b, c) as one instruction (the accumulators need no NaN canonicalisation)
RP_DEV float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// Maximum of a lane's 64 accumulators of tile column j (all of the wave's 128 rows after the exchange between the
// half-waves).
RP_DEV float column_max(const f32x16 (&acc)[TM][TN], int j) {
  float mx = acc[0][j][0];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int v = (i == 0 ? 1 : 0); v + 1 < 16; v += 2) mx = max3(mx, acc[i][j][v], acc[i][j][v + 1]);
  mx = fmaxf(mx, acc[0][j][15]);
  return fmaxf(mx, __shfl_xor(mx, 32, 64));
}

// The accumulator of tile column j whose local row is lab_local (= label row - first row of the wave's block - 4*lk),
// if this lane holds it.  Called only when some lane of the wave has its label inside the block.
RP_DEV bool label_logit(const f32x16 (&acc)[TM][TN], int j, int lab_local, float& z) {
  bool found = false;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const bool hit = lab_local == acc_row(i, v);
      z = hit ? acc[i][j][v] : z;
      found |= hit;
    }
  return found;
}

// Epilogue.  acc[i][j][v] is element (i*32 + 8*(v/4) + 4*lk + v%4, j*32 + lr) of the wave's 128x64 block whose top
// left corner is (wrow0, wcol0).  Every wave stages its block through its own 18 KB of LDS (all waves must have
// finished the K loop) so that global accesses are 16 bytes per lane and cover whole 128-byte lines; no workgroup
// barrier inside.
// part_row: row of the cross-entropy partial array this wave writes (EPI_CE_STATS).
// M: rows of C that exist (the end of the group's rows in grouped mode).
// j0, j1 (wave-uniform): the 32-column halves [j0, j1) of the block this wave writes -- both, except in the plain
// epilogues of the two-group tile, where the groups take one half each.
RP_DEV void epilogue(const GemmArgs& p, int M, const f32x16 (&acc)[TM][TN], unsigned char* smem, int wave, int lane,
                     int wrow0, int wcol0, int part_row, int j0 = 0, int j1 = TN) {
  const int lr = lane & 31, lk = lane >> 5;
  unsigned char* const stg = smem + wave * STG_BYTES;
  const int rr = lane >> 3, cc = lane & 7;   // read-back: 8 rows per pass, 8 chunks of 16 bytes per row

  if ((p.epi == EPI_BF16 && !p.R) || p.epi == EPI_CE_DZ || p.epi == EPI_SWIGLU_BWD || p.epi == EPI_CE_P || p.epi == EPI_SWIGLU_FWD) {
    bf16* s16 = reinterpret_cast<bf16*>(stg);
    unsigned short* const h16 = reinterpret_cast<unsigned short*>(stg);
    // two rows of a column are converted by one instruction and go out as the halves of its result
    auto stage2 = [&](int i, int j, int v, float x0, float x1) {
      const uint32_t pk = pack_bf16x2(x0, x1);
      unsigned short* const d = h16 + (acc_row(i, v) + 4 * lk) * STG_LD + j * 32 + lr;
      d[0] = (unsigned short)pk;
      d[STG_LD] = (unsigned short)(pk >> 16);
    };
    if (p.epi == EPI_CE_P) {
      // p = exp(z - ref) for a frozen head's later vocabulary chunks: every lane owns token columns, so the chunk's
      // per-token maximum and sum of exponentials over the wave's 128 rows come from the registers; rows past the end of
      // the vocabulary are excluded from both (their staged values are never stored)
      constexpr float LOG2E = 1.4426950408889634f;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = wcol0 + j * 32 + lr;
        const bool colok = col < p.N;
        const int lab = colok ? p.labels[col] - p.row_offset : -1;
        const float nr = colok ? -LOG2E * p.lse[col] : 0.f;
        const float cap = RP_CE_P_CLAMP * LOG2E;
        float mx, sum = 0.f, sum2 = 0.f;
        if (wrow0 + WAVE_M <= M) {   // wave-uniform: no row of the block is past the end
          mx = column_max(acc, j);
          if (__ballot(lab >= wrow0 && lab < wrow0 + WAVE_M)) {
            float z = 0.f;
            if (label_logit(acc, j, lab - wrow0 - 4 * lk, z)) p.zlab[col] = z;
          }
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; v += 2) {
              const float e0 = __builtin_amdgcn_exp2f(fminf(fmaf(acc[i][j][v], LOG2E, nr), cap));
              const float e1 = __builtin_amdgcn_exp2f(fminf(fmaf(acc[i][j][v + 1], LOG2E, nr), cap));
              sum += e0; sum2 += e1;
              stage2(i, j, v, e0, e1);
            }
        } else {
          mx = -INFINITY;
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; v += 2) {
              const int row = wrow0 + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
              float e0 = 0.f, e1 = 0.f;
              if (row < M) {
                mx = fmaxf(mx, acc[i][j][v]);
                if (row == lab) p.zlab[col] = acc[i][j][v];
                e0 = __builtin_amdgcn_exp2f(fminf(fmaf(acc[i][j][v], LOG2E, nr), cap));
              }
              if (row + 1 < M) {
                mx = fmaxf(mx, acc[i][j][v + 1]);
                if (row + 1 == lab) p.zlab[col] = acc[i][j][v + 1];
                e1 = __builtin_amdgcn_exp2f(fminf(fmaf(acc[i][j][v + 1], LOG2E, nr), cap));
              }
              sum += e0; sum2 += e1;
              stage2(i, j, v, e0, e1);
            }
          mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        }
        sum += sum2;
        sum += __shfl_xor(sum, 32, 64);
        if (lk == 0 && colok) p.part[(long)part_row * p.part_ld + col] = make_float2(mx, sum);
      }
    } else if (p.epi != EPI_CE_DZ) {
      if (p.alpha == 1.f) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          if (j < j0 || j >= j1) continue;
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; v += 2) stage2(i, j, v, acc[i][j][v], acc[i][j][v + 1]);
        }
      } else {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          if (j < j0 || j >= j1) continue;
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; v += 2) stage2(i, j, v, p.alpha * acc[i][j][v], p.alpha * acc[i][j][v + 1]);
        }
      }
    } else {
      // dZ^T = (softmax - onehot) * coef: rows are vocabulary entries, columns tokens.  Every element gets
      // exp(z - lse) * coef (rows past the end of the vocabulary are never stored); the one element per column that
      // is the label is fixed up in the staging buffer afterwards.
      constexpr float LOG2E = 1.4426950408889634f;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = wcol0 + j * 32 + lr;
        const bool colok = col < p.N;
        const int lab = colok ? p.labels[col] - p.row_offset - wrow0 : -1;
        const float nl = colok ? -LOG2E * p.lse[col] : 0.f, cf = colok ? p.coef[col] : 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int v = 0; v < 16; v += 2)
            stage2(i, j, v, __builtin_amdgcn_exp2f(fmaf(acc[i][j][v], LOG2E, nl)) * cf,
                   __builtin_amdgcn_exp2f(fmaf(acc[i][j][v + 1], LOG2E, nl)) * cf);
        if (__ballot(lab >= 0 && lab < WAVE_M)) {   // wave-uniform, rare
          float z = 0.f;
          if (label_logit(acc, j, lab - 4 * lk, z))
            s16[lab * STG_LD + j * 32 + lr] = (bf16)((__builtin_amdgcn_exp2f(fmaf(z, LOG2E, nl)) - 1.f) * cf);
        }
      }
    }
    wave_lds_fence();
    bf16* Cp = reinterpret_cast<bf16*>(p.C);
    if (p.epi == EPI_SWIGLU_BWD) {
      // a lane takes 8 columns of a row of the staged product d (the gradient of silu(gate) * up), reads gate and up
      // there and writes  d_gate = d * up * s * (1 + gate * (1 - s)),  d_up = d * gate * s,  s = sigmoid(gate);
      // the loads of four row groups are in flight before anything is stored
      const bf16* Rp = reinterpret_cast<const bf16*>(p.R);
      const int gcol = wcol0 + cc * 8;
      constexpr int NB = 4;
#pragma unroll
      for (int t0 = 0; t0 < WAVE_M / 8; t0 += NB) {
        uint4 gv[NB], uv[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) {
          const int grow = wrow0 + (t0 + u) * 8 + rr;
          gv[u] = make_uint4(0u, 0u, 0u, 0u);
          uv[u] = gv[u];
          if (grow < M && gcol < p.N) {
            gv[u] = *reinterpret_cast<const uint4*>(Rp + (long)grow * p.ldr + gcol);
            uv[u] = *reinterpret_cast<const uint4*>(Rp + (long)grow * p.ldr + p.N + gcol);
          }
        }
#pragma unroll
        for (int u = 0; u < NB; ++u) {
          const int row = (t0 + u) * 8 + rr, grow = wrow0 + row;
          const uint4 dv = *reinterpret_cast<const uint4*>(s16 + row * STG_LD + cc * 8);
          const uint32_t dw[4] = {dv.x, dv.y, dv.z, dv.w}, gw[4] = {gv[u].x, gv[u].y, gv[u].z, gv[u].w},
                         uw[4] = {uv[u].x, uv[u].y, uv[u].z, uv[u].w};
          uint32_t og[4], ou[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            float dg2[2], du2[2];
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
              const float d = hh ? bf16_hi(dw[e]) : bf16_lo(dw[e]), g = hh ? bf16_hi(gw[e]) : bf16_lo(gw[e]),
                          up = hh ? bf16_hi(uw[e]) : bf16_lo(uw[e]);
              const float sg = 1.f / (1.f + __expf(-g));
              dg2[hh] = d * up * sg * (1.f + g * (1.f - sg));
              du2[hh] = d * g * sg;
            }
            og[e] = pack_bf16x2(dg2[0], dg2[1]);
            ou[e] = pack_bf16x2(du2[0], du2[1]);
          }
          if (grow < M && gcol < p.N) {
            *reinterpret_cast<uint4*>(Cp + (long)grow * p.ldc + gcol) = make_uint4(og[0], og[1], og[2], og[3]);
            *reinterpret_cast<uint4*>(Cp + (long)grow * p.ldc + p.N + gcol) = make_uint4(ou[0], ou[1], ou[2], ou[3]);
          }
        }
      }
    } else if (j1 - j0 == TN) {
      const int gcol = wcol0 + cc * 8;
#pragma unroll
      for (int t = 0; t < WAVE_M / 8; ++t) {
        const int row = t * 8 + rr, grow = wrow0 + row;
        if (grow < M && gcol < p.N)
          *reinterpret_cast<uint4*>(Cp + (long)grow * p.ldc + gcol) = *reinterpret_cast<const uint4*>(s16 + row * STG_LD + cc * 8);
      }
    } else {   // one half: 16 rows per pass, 4 chunks of 16 bytes per row
      const int lcol = j0 * 32 + (lane & 3) * 8, gcol = wcol0 + lcol;
#pragma unroll
      for (int t = 0; t < WAVE_M / 16; ++t) {
        const int row = t * 16 + (lane >> 2), grow = wrow0 + row;
        if (grow < M && gcol < p.N)
          *reinterpret_cast<uint4*>(Cp + (long)grow * p.ldc + gcol) = *reinterpret_cast<const uint4*>(s16 + row * STG_LD + lcol);
      }
    }
    if (p.epi == EPI_SWIGLU_FWD) {
      // silu(gate) * up from the staged (rounded) blocks: wave wn holds gate columns, wave wn + 2 of the same row the up
      // columns that go with them; each of the two takes 64 of the 128 rows.  Same arithmetic as the SwiGLU kernel.
      __syncthreads();
      const int wn = wave & 3;
      const bf16* const gs = reinterpret_cast<const bf16*>(smem + (wave & ~2) * STG_BYTES);
      const bf16* const us = reinterpret_cast<const bf16*>(smem + (wave | 2) * STG_BYTES);
      bf16* const Ap = reinterpret_cast<bf16*>(p.C2);
      const int acol = (wn < 2 ? wcol0 : wcol0 - (p.N >> 1)) + cc * 8;     // gate column = activation column
#pragma unroll
      for (int t = 0; t < WAVE_M / 16; ++t) {
        const int row = (wn >> 1) * (WAVE_M / 2) + t * 8 + rr, grow = wrow0 + row;
        const uint4 gv = *reinterpret_cast<const uint4*>(gs + row * STG_LD + cc * 8);
        const uint4 uv = *reinterpret_cast<const uint4*>(us + row * STG_LD + cc * 8);
        const uint32_t gw[4] = {gv.x, gv.y, gv.z, gv.w}, uw[4] = {uv.x, uv.y, uv.z, uv.w};
        uint32_t o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float g0 = bf16_lo(gw[e]), g1 = bf16_hi(gw[e]);
          o[e] = pack_bf16x2(g0 / (1.f + __expf(-g0)) * bf16_lo(uw[e]), g1 / (1.f + __expf(-g1)) * bf16_hi(uw[e]));
        }
        if (grow < M) *reinterpret_cast<uint4*>(Ap + (long)grow * p.ldc2 + acol) = make_uint4(o[0], o[1], o[2], o[3]);
      }
    }
  } else if (p.epi == EPI_BF16 || p.epi == EPI_F32 || p.epi == EPI_F32_COLMAX) {
    if (p.epi == EPI_F32_COLMAX) {
      // rows are vocabulary entries, columns tokens: the maximum of every column over the wave's 128 rows, from the
      // registers, before the tile goes out
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = wcol0 + j * 32 + lr;
        const bool colok = col < p.N;
        const int lab = colok ? p.labels[col] - p.row_offset : -1;
        float mx;
        if (wrow0 + WAVE_M <= M) {   // wave-uniform: no row of the block is past the end
          mx = column_max(acc, j);
          if (__ballot(lab >= wrow0 && lab < wrow0 + WAVE_M)) {
            float z = 0.f;
            if (label_logit(acc, j, lab - wrow0 - 4 * lk, z)) p.zlab[col] = z;
          }
        } else {
          mx = -INFINITY;
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int row = wrow0 + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
              if (row < M) {
                mx = fmaxf(mx, acc[i][j][v]);
                if (row == lab) p.zlab[col] = acc[i][j][v];
              }
            }
          mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        }
        if (lk == 0 && colok) p.part[(long)part_row * p.part_ld + col] = make_float2(mx, 0.f);
      }
    }
    // fp32 staging, one 32-column half at a time: [128][36] floats (144-byte rows)
    float* s32 = reinterpret_cast<float*>(stg);
    const bool unit = p.alpha == 1.f;   // uniform
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      if (j < j0 || j >= j1) continue;
      if (j > j0) wave_lds_fence();
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        float* const d = s32 + (i * 32 + 4 * lk) * (STG_LD / 2) + lr;
        if (unit) {
#pragma unroll
          for (int v = 0; v < 16; ++v) d[acc_row(0, v) * (STG_LD / 2)] = acc[i][j][v];
        } else {
#pragma unroll
          for (int v = 0; v < 16; ++v) d[acc_row(0, v) * (STG_LD / 2)] = p.alpha * acc[i][j][v];
        }
      }
      wave_lds_fence();
      const int gcol = wcol0 + j * 32 + cc * 4;
      const bool colok = gcol < p.N;
      // What is added from memory (the fp32 output itself when it accumulates, the bf16 residual) is loaded for eight
      // row groups at a time before anything is stored: the compiler cannot tell that the stores leave the later
      // loads alone, and one load-add-store round trip after the other costs 16-20 us per tile.
      constexpr int NB = 8;
#pragma unroll
      for (int t0 = 0; t0 < WAVE_M / 8; t0 += NB) {
        if (p.epi != EPI_BF16) {
          float* const Cf = reinterpret_cast<float*>(p.C) + (long)blockIdx.y * p.c_slice_stride;   // slice of a reduction split
          float4 o[NB];
          if (p.beta) {
#pragma unroll
            for (int u = 0; u < NB; ++u) {
              const int grow = wrow0 + (t0 + u) * 8 + rr;
              o[u] = (grow < M && colok) ? *reinterpret_cast<const float4*>(Cf + (long)grow * p.ldc + gcol) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
          } else {
#pragma unroll
            for (int u = 0; u < NB; ++u) o[u] = make_float4(0.f, 0.f, 0.f, 0.f);
          }
#pragma unroll
          for (int u = 0; u < NB; ++u) {
            const int row = (t0 + u) * 8 + rr, grow = wrow0 + row;
            float4 x = *reinterpret_cast<const float4*>(s32 + row * (STG_LD / 2) + cc * 4);
            x.x += o[u].x; x.y += o[u].y; x.z += o[u].z; x.w += o[u].w;
            if (grow < M && colok) *reinterpret_cast<float4*>(Cf + (long)grow * p.ldc + gcol) = x;
          }
        } else {
          uint2 r2[NB];
#pragma unroll
          for (int u = 0; u < NB; ++u) {
            const int grow = wrow0 + (t0 + u) * 8 + rr;
            r2[u] = (grow < M && colok) ? *reinterpret_cast<const uint2*>(reinterpret_cast<const bf16*>(p.R) + (long)grow * p.ldr + gcol)
                                        : make_uint2(0u, 0u);
          }
#pragma unroll
          for (int u = 0; u < NB; ++u) {
            const int row = (t0 + u) * 8 + rr, grow = wrow0 + row;
            float4 x = *reinterpret_cast<const float4*>(s32 + row * (STG_LD / 2) + cc * 4);
            x.x += bf16_lo(r2[u].x); x.y += bf16_hi(r2[u].x); x.z += bf16_lo(r2[u].y); x.w += bf16_hi(r2[u].y);
            if (grow < M && colok)
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
      if (col >= p.N || j < j0 || j >= j1) continue;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = wrow0 + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
          if (row < M) atomicAdd(Cp + (long)row * p.ldc + col, p.alpha * acc[i][j][v]);
        }
    }
  } else if (p.epi == EPI_CE_STATS) {
    // rows are vocabulary entries, columns are tokens: every lane reduces its own column over the wave's 128 rows
    constexpr float LOG2E = 1.4426950408889634f;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = wcol0 + j * 32 + lr;
      const bool colok = col < p.N;
      const int lab = colok ? p.labels[col] - p.row_offset : -1;
      float mx, s = 0.f;
      if (wrow0 + WAVE_M <= M) {   // wave-uniform: no row of the block is past the end
        mx = column_max(acc, j);
        if (__ballot(lab >= wrow0 && lab < wrow0 + WAVE_M)) {
          float z = 0.f;
          if (label_logit(acc, j, lab - wrow0 - 4 * lk, z)) p.zlab[col] = z;
        }
        const float nm = -LOG2E * mx;
        float s2 = 0.f;   // two chains
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int v = 0; v < 16; v += 2) {
            s += __builtin_amdgcn_exp2f(fmaf(acc[i][j][v], LOG2E, nm));
            s2 += __builtin_amdgcn_exp2f(fmaf(acc[i][j][v + 1], LOG2E, nm));
          }
        s += s2;
      } else {
        mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int row = wrow0 + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
            if (row < M) {
              mx = fmaxf(mx, acc[i][j][v]);
              if (row == lab) p.zlab[col] = acc[i][j][v];
            }
          }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        if (mx > -INFINITY) {
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int row = wrow0 + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
              if (row < M) s += __expf(acc[i][j][v] - mx);
            }
        }
      }
      s += __shfl_xor(s, 32, 64);
      if (lk == 0 && colok) p.part[(long)part_row * p.part_ld + col] = make_float2(mx, s);
    }
  }
}

}  // namespace gemm_dev
