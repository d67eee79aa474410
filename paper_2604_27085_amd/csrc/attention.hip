// Causal grouped-query attention on the gfx950 matrix cores, flash style (no s x s matrix ever leaves the CU).
//
// All three kernels use v_mfma_f32_32x32x16_bf16 with the score tile computed TRANSPOSED relative to the row that is
// being normalised: the 32x32 accumulator layout gives every lane one column and 16 rows, so with queries (forward,
// dQ) as columns the softmax reductions are in-lane plus one exchange with lane^32, and the probabilities already sit
// in the register layout the next MFMA wants as its B operand.  Within a 16-deep step that layout holds, for lane
// half h, the reduction indices {4h..4h+3, 8+4h..8+4h+3}; the A operand of the same MFMA is read from LDS in exactly
// that order.  An operand whose reduction index is contiguous in memory (K for Q.K^T, V for dO.V^T, Q and dO in the
// score products of the dK/dV kernel) is read with plain 16-byte LDS loads from a [rows][D + 8] tile; an operand
// whose reduction index is the row index of the tile (V for P.V, K for dS.K, Q and dO for dK/dV) is read with the
// transposing LDS load from a [rows][D + 32] tile.  A tile needed both ways (K in the dQ kernel, Q and dO in the dK/dV
// kernel at d = 128) has the row stride D + 24, which serves both kinds of reads (the transposing ones with some bank
// conflicts), and is stored once; nothing is transposed in registers.  Global loads are 16-byte buffer loads whose descriptor ends with the
// sequence, so rows past the end read as zero without a branch.
//
//   forward : workgroup = NW waves x 32*QT queries of one head, loop over 64-key tiles up to the diagonal; NW = 8 (one
//             workgroup per CU, two sets of K/V tiles, one barrier per tile) when the grid is large enough, else 4
//   dQ      : same decomposition; recomputes S^T and dP^T, accumulates dQ^T
//   dK, dV  : workgroup = 128 keys against ONE query head, loops over 64-query tiles from the diagonal on and
//             accumulates dK^T, dV^T in registers.  d = 128: eight waves, pairs of waves share 32 keys, split the
//             accumulators over the head dimension and the score recomputation over the queries
//             (attn_bwd_dkv_pair_kernel); d = 64: four waves x 32 keys (attn_bwd_dkv_fused_kernel).  With grouped queries
//             every query head of a group writes an fp32 partial and a small kernel adds the group's partials in head
//             order (no atomics, fixed order); one workgroup per query head rather than per kv head multiplies the
//             workgroup count, which is what lets the triangular work balance over the CUs.
// Launch orders keep an XCD (eight of them, each with its own L2) on few heads: see xcd_head() and the dK/dV kernels.
#include "common.hpp"
#include "kernels.hpp"
#include <stdlib.h>

namespace {

typedef __amdgpu_buffer_rsrc_t rsrc_t;

struct AttnArgs {
  const bf16 *q, *k, *v, *dout;
  bf16 *o, *dq, *dk, *dv;
  float* lse;
  const float* lse_in;
  const float* delta;
  float *dk_part, *dv_part;   // fp32 [T, a*d] partials of the dK/dV kernel when a > kh
  long ldq, ldk, ldv, ldo, lddo, lddq, lddk, lddv;
  int batch, seq, a, kh;
  float scale_log2e, scale;
  int fold;   // see heavy_rank()
  int kblock; // dK/dV kernel: key tiles per run of one head in an XCD's launch order (0: key-tile-major order over all heads)
};

// Launch position -> rank in the order "heaviest workgroup first".  A kernel that keeps two workgroups per CU and whose
// grid fits on the chip at once (at most 2 x 256 workgroups) has all of them resident from the start, CU c holding
// positions c and 256 + c; nothing is rescheduled later, so what counts is that every CU's pair sums to the same
// work: the second half of the grid is handed out lightest first (fold; measured 5 % on the forward kernel at 4096
// tokens, while pairing neighbouring positions instead made it 20 % slower).  Larger grids are handed out as
// workgroups finish, where heaviest-first is the right order.
RP_DEV int heavy_rank(int pos, int n, int fold) { return (fold && pos >= 256) ? n - 1 - (pos - 256) : pos; }

// Consecutive workgroups go to consecutive XCDs (eight, each with an L2 of its own).  The i-th of the nhb workgroups of a
// query tile therefore takes head (i mod 8) * nhb/8 + i/8 instead of head i: an XCD then works on nhb/8 neighbouring query
// heads, i.e. on one or two K/V heads with grouped queries, and its L2 fetches their K/V tiles once for all the workgroups
// that stream them side by side -- instead of every XCD fetching every K/V head.
RP_DEV int xcd_head(int i, int nhb) { return (nhb & 7) ? i : (i & 7) * (nhb >> 3) + (i >> 3); }

RP_DEV rsrc_t seq_rsrc(const bf16* base, long ld, int seq, int D) {
  // covers rows 0..seq-1 of one head: later rows are out of range and read as zero
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16*>(base), 0, (int)(((long)(seq - 1) * ld + D) * 2), 0x00020000);
}
RP_DEV uint4 buf_load16(rsrc_t r, uint32_t voff) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, 0, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}

// ---- 64 x D tile: global -> registers -> LDS -----------------------------------------------------------------
template <int D, int NT>
struct Tile64 {
  static constexpr int CH = D / 8, NREG = 64 * CH / NT;
  static_assert((64 * CH) % NT == 0, "tile does not divide over the threads");
  // rows row0..row0+63 of a [seq, D] view with row stride ld (elements)
  static RP_DEV void load(uint4 (&r)[NREG], rsrc_t rs, long ld, int row0, int tid) {
#pragma unroll
    for (int it = 0; it < NREG; ++it) {
      const int c = it * NT + tid;
      r[it] = buf_load16(rs, (uint32_t)(((long)(row0 + c / CH) * ld + (c % CH) * 8) * 2));
    }
  }
  template <int LDS_LD>
  static RP_DEV void store(const uint4 (&r)[NREG], bf16* S, int tid) {
#pragma unroll
    for (int it = 0; it < NREG; ++it) {
      const int c = it * NT + tid;
      *reinterpret_cast<uint4*>(S + (c / CH) * LDS_LD + (c % CH) * 8) = r[it];
    }
  }
};

// A-operand fragment from a [64][LD] tile whose rows are the reduction index (keys or queries) and whose columns are
// the MFMA rows: the 8 values are tile rows {16g + 4h + e, 16g + 8 + 4h + e}, e = 0..3, at column x -- the order in
// which the 32x32 accumulator of the score tile holds them.  base = S + (4h + (l%16)/4)*LD + 16*((l/16)&1) + 4*(l%4).
template <int LD>
RP_DEV uint4 read_frag_tr(const bf16* base, int g, int x_off) {
  typedef short s16x4 __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) s16x4* lds_ptr;
  const bf16* q = base + 16 * g * LD + x_off;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(q));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(q + 8 * LD));
  const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
  return make_uint4(l2.x, l2.y, h2.x, h2.y);
}
template <int LD>
RP_DEV int tr_base(int lane) {
  const int lk = lane >> 5, l16 = lane & 15, g16 = lane >> 4;
  return (4 * lk + (l16 >> 2)) * LD + 16 * (g16 & 1) + 4 * (l16 & 3);
}

RP_DEV uint4 pack_frag(const f32x16& s, int off) {
  return make_uint4(pack_bf16x2(s[off + 0], s[off + 1]), pack_bf16x2(s[off + 2], s[off + 3]),
                    pack_bf16x2(s[off + 4], s[off + 5]), pack_bf16x2(s[off + 6], s[off + 7]));
}

RP_DEV float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Two waves share a SIMD in the forward kernel.  Left alone they fall into step: both issue their matrix products at
// the same time (each at half rate) and then both do their exponentials, so the matrix pipeline idles while the vector
// pipeline works and the other way round.  A wave raises its issue priority for its runs of MFMAs: whichever wave gets
// there first keeps the matrix pipeline to itself, the other one falls behind by a phase, and from then on one wave's
// exponentials run under the other wave's products (forward kernel +6 % at 8192 to 31744 tokens; the dQ kernel, whose
// vector phase is short against its three products, does not change).
#define MFMA_PHASE_BEGIN() __builtin_amdgcn_s_setprio(1)
#define MFMA_PHASE_END() __builtin_amdgcn_s_setprio(0)

// x as the sum of three bf16 numbers (most significant first) in the first three slots of an MFMA operand chunk, zeros
// in the other five: 24 mantissa bits survive, so an MFMA step against ones adds x to an fp32 accumulator exactly
// enough for a softmax exponent.
RP_DEV uint4 split3(float x) {
  const uint32_t h = f32_to_bf16_bits(x);
  const float r1 = x - bf16_bits_to_f32(h);
  const uint32_t m = f32_to_bf16_bits(r1);
  const uint32_t l = f32_to_bf16_bits(r1 - bf16_bits_to_f32(m));
  return make_uint4(h | (m << 16), l, 0u, 0u);
}
// The other operand of that step: ones in the same three slots for the lanes that hold reduction indices 0..7.
RP_DEV uint4 ones3(int lk) { return lk == 0 ? make_uint4(0x3F803F80u, 0x00003F80u, 0u, 0u) : make_uint4(0u, 0u, 0u, 0u); }

// Writes a wave's 32 x D transposed accumulator (columns = the wave's 32 rows of the output) through LDS to global.
template <int D>
RP_DEV void store_acc_T(const f32x16 (&acc)[D / 32], float mul, bf16* stage /* [32][D+8] */, bf16* __restrict__ out,
                        long ld, int row0, int nrows, int lane) {
  const int lr = lane & 31, lk = lane >> 5;
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int vg = 0; vg < 4; ++vg) {
      const int dd = 32 * dt + 8 * vg + 4 * lk;
      *reinterpret_cast<uint2*>(stage + lr * (D + 8) + dd) =
          make_uint2(pack_bf16x2(acc[dt][4 * vg] * mul, acc[dt][4 * vg + 1] * mul),
                     pack_bf16x2(acc[dt][4 * vg + 2] * mul, acc[dt][4 * vg + 3] * mul));
    }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < (32 * (D / 8)) / 64; ++it) {
    const int idx = it * 64 + lane;
    const int row = idx / (D / 8), ch = idx % (D / 8);
    if (row0 + row < nrows)
      *reinterpret_cast<uint4*>(out + (long)(row0 + row) * ld + ch * 8) =
          *reinterpret_cast<const uint4*>(stage + row * (D + 8) + ch * 8);
  }
  __syncthreads();
}

// Same for an fp32 destination; stage is [32][D + 4] floats per wave.
template <int D>
RP_DEV void store_acc_T_f32(const f32x16 (&acc)[D / 32], float mul, float* stage, float* __restrict__ out, long ld,
                            int row0, int nrows, int lane) {
  const int lr = lane & 31, lk = lane >> 5;
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int vg = 0; vg < 4; ++vg)
      *reinterpret_cast<float4*>(stage + lr * (D + 4) + 32 * dt + 8 * vg + 4 * lk) =
          make_float4(acc[dt][4 * vg] * mul, acc[dt][4 * vg + 1] * mul, acc[dt][4 * vg + 2] * mul, acc[dt][4 * vg + 3] * mul);
  __syncthreads();
#pragma unroll
  for (int it = 0; it < (32 * (D / 4)) / 64; ++it) {
    const int idx = it * 64 + lane;
    const int row = idx / (D / 4), ch = idx % (D / 4);
    if (row0 + row < nrows)
      *reinterpret_cast<float4*>(out + (long)(row0 + row) * ld + ch * 4) =
          *reinterpret_cast<const float4*>(stage + row * (D + 4) + ch * 4);
  }
  __syncthreads();
}

// ================================================================================================ forward
template <int D, int QT, int NW>
__global__ void __launch_bounds__(NW * 64, (QT == 1 && NW <= 4) ? 2 : 1) attn_fwd_kernel(const AttnArgs p) {
  constexpr int LDK = D + 8, LDV = D + 32, KS = D / 16, DT = D / 32, NT = NW * 64, BQ = NW * 32 * QT;
  using T64 = Tile64<D, NT>;
  extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];   // fwd_smem_bytes(D, NW)
  bf16* const smem = reinterpret_cast<bf16*>(dyn_smem);
  // eight-wave workgroups have the CU to themselves: two sets of K/V tiles, one barrier per key tile
  constexpr bool DB = NW >= 8;
  constexpr int SET = 64 * LDK + 64 * LDV;
  bf16* const Ks = smem;
  bf16* const Vs = smem + 64 * LDK;

  const int tid = threadIdx.x, lane = tid & 63, lr = lane & 31, lk = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nQ = (p.seq + BQ - 1) / BQ;
  const int nhb = p.a * p.batch;
  const int rank = heavy_rank((int)blockIdx.x, (int)gridDim.x, p.fold);
  const int qtile = nQ - 1 - rank / nhb;     // the heaviest query tiles of every head go first
  const int hb = xcd_head(rank % nhb, nhb);
  const int hq = hb % p.a, b = hb / p.a;
  const int g = hq / (p.a / p.kh);
  const int q0 = qtile * BQ, qw0 = q0 + w * 32 * QT;
  const long tok0 = (long)b * p.seq;
  const bf16* qb = p.q + tok0 * p.ldq + hq * D;
  const rsrc_t rk = seq_rsrc(p.k + tok0 * p.ldk + g * D, p.ldk, p.seq, D);
  const rsrc_t rv = seq_rsrc(p.v + tok0 * p.ldv + g * D, p.ldv, p.seq, D);

  uint4 qf[QT][KS];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const int qpos = qw0 + 32 * t + lr;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qf[t][ks] = make_uint4(0u, 0u, 0u, 0u);
      if (qpos < p.seq) qf[t][ks] = *reinterpret_cast<const uint4*>(qb + (long)qpos * p.ldq + 16 * ks + 8 * lk);
    }
  }
  const int kv_end = (q0 + BQ < p.seq) ? (q0 + BQ) : p.seq;
  const int nkv = (kv_end + 63) / 64;

  float m_run[QT], l_run[QT];
  f32x16 oacc[QT][DT];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    m_run[t] = -INFINITY;
    l_run[t] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[t][dt][v] = 0.f;
  }

  const bf16* const kfrag0 = Ks + lr * LDK + 8 * lk;
  const bf16* const vfrag0 = Vs + tr_base<LDV>(lane);
  uint4 kreg[T64::NREG], vreg[T64::NREG];
  T64::load(kreg, rk, p.ldk, 0, tid);
  T64::load(vreg, rv, p.ldv, 0, tid);

  if constexpr (DB) {     // tile 0 into set 0, tile 1 on its way
    T64::template store<LDK>(kreg, Ks, tid);
    T64::template store<LDV>(vreg, Vs, tid);
    if (nkv > 1) {
      T64::load(kreg, rk, p.ldk, 64, tid);
      T64::load(vreg, rv, p.ldv, 64, tid);
    }
  }
  for (int j = 0; j < nkv; ++j) {
    __syncthreads();
    if constexpr (DB) {
      // everyone is done with tile j-1: its set takes tile j+1 (in registers since the last trip), tile j+2 sets out
      if (j + 1 < nkv) {
        T64::template store<LDK>(kreg, Ks + ((j + 1) & 1) * SET, tid);
        T64::template store<LDV>(vreg, Vs + ((j + 1) & 1) * SET, tid);
      }
      if (j + 2 < nkv) {
        T64::load(kreg, rk, p.ldk, (j + 2) * 64, tid);
        T64::load(vreg, rv, p.ldv, (j + 2) * 64, tid);
      }
    } else {
      T64::template store<LDK>(kreg, Ks, tid);
      T64::template store<LDV>(vreg, Vs, tid);
      __syncthreads();
      if (j + 1 < nkv) {
        T64::load(kreg, rk, p.ldk, (j + 1) * 64, tid);
        T64::load(vreg, rv, p.ldv, (j + 1) * 64, tid);
      }
    }
    const bf16* const kfrag = kfrag0 + (DB ? (j & 1) * SET : 0);
    const bf16* const vfrag = vfrag0 + (DB ? (j & 1) * SET : 0);
    const int kv0 = j * 64;
    // Waves whose queries all precede this tile's keys (the last tile of the two upper waves) run it fully masked
    // rather than skip it: they would wait at the next barrier anyway, and a skipped update would make the compiler
    // keep a second copy of the accumulator.
    {
      f32x16 sT[QT][2];
      const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      // every LDS fragment is requested AHEAD products before the one that consumes it, so that the MFMAs do not each
      // wait out an LDS round trip
      constexpr int AHEAD = 3;
      {
        constexpr int NS = 2 * KS;
        auto sfrag_at = [&](int n) { return *reinterpret_cast<const uint4*>(kfrag + 32 * (n & 1) * LDK + 16 * (n >> 1)); };
        uint4 ring[AHEAD];
#pragma unroll
        for (int n = 0; n < AHEAD; ++n) ring[n] = sfrag_at(n);
        MFMA_PHASE_BEGIN();
#pragma unroll
        for (int n = 0; n < NS; ++n) {
          const uint4 a = ring[n % AHEAD];
          if (n + AHEAD < NS) ring[n % AHEAD] = sfrag_at(n + AHEAD);
          const int ks = n >> 1, kt = n & 1;
#pragma unroll
          for (int t = 0; t < QT; ++t) sT[t][kt] = mfma32(a, qf[t][ks], ks == 0 ? zero16 : sT[t][kt]);
          __builtin_amdgcn_sched_barrier(0);
        }
        MFMA_PHASE_END();
      }
      // the first V fragments are requested now, under the softmax arithmetic
      constexpr int NU = 4 * DT;
      auto ufrag_at = [&](int n) { return read_frag_tr<LDV>(vfrag, n / DT, 32 * (n % DT)); };
      uint4 uring[AHEAD];
#pragma unroll
      for (int n = 0; n < AHEAD; ++n) uring[n] = ufrag_at(n);
      __builtin_amdgcn_sched_barrier(0);
      const bool need_mask = (kv0 + 63 > qw0) || (kv0 + 64 > p.seq);   // wave-uniform
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        const int qpos = qw0 + 32 * t + lr;
        if (need_mask) {
#pragma unroll
          for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int kpos = kv0 + 32 * kt + 8 * (v >> 2) + 4 * lk + (v & 3);
              sT[t][kt][v] = (kpos > qpos || kpos >= p.seq) ? -INFINITY : sT[t][kt][v];
            }
        }
        float mx = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sT[t][kt][v]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * p.scale_log2e;
        // The accumulator is rescaled on every key tile, without a branch: a conditional rescale (only when the
        // maximum grows) makes the compiler carry a second copy of the accumulator through the loop, which costs more
        // than the multiplies.  The first key tile contains key 0 <= qpos, so m_run is finite from then on.
        {
          // m_run is a reference exponent, not the exact running maximum: it moves only when a row's maximum outgrows
          // it by 2^8 (the probabilities stay below 256, harmless in fp32 sums and bf16 operands), so after the first
          // few key tiles almost every tile skips the rescale of the accumulator.  The skip is a wave-uniform branch,
          // and alpha passes through an empty asm statement so that the multiplies cannot be hoisted out of it.
          const bool grow = mx > m_run[t] + 8.f;
          if (__builtin_amdgcn_ballot_w64(grow) != 0ull) {
            const float m_new = grow ? mx : m_run[t];
            float alpha = fast_exp2(m_run[t] - m_new);
            asm volatile("" : "+v"(alpha));
            l_run[t] *= alpha;
            m_run[t] = m_new;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
              for (int v = 0; v < 16; ++v) oacc[t][dt][v] *= alpha;
          }
        }
        float psum = 0.f;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const float e = fast_exp2(__builtin_fmaf(sT[t][kt][v], p.scale_log2e, -m_run[t]));
            sT[t][kt][v] = e;
            psum += e;
          }
        l_run[t] += psum;
      }
      {
        uint4 pf[4][QT];
#pragma unroll
        for (int gk = 0; gk < 4; ++gk)
#pragma unroll
          for (int t = 0; t < QT; ++t) pf[gk][t] = pack_frag(sT[t][gk >> 1], 8 * (gk & 1));
        MFMA_PHASE_BEGIN();
#pragma unroll
        for (int n = 0; n < NU; ++n) {
          const uint4 a = uring[n % AHEAD];
          if (n + AHEAD < NU) uring[n % AHEAD] = ufrag_at(n + AHEAD);
#pragma unroll
          for (int t = 0; t < QT; ++t) oacc[t][n % DT] = mfma32(a, pf[n / DT][t], oacc[t][n % DT]);
          __builtin_amdgcn_sched_barrier(0);
        }
        MFMA_PHASE_END();
      }
    }
  }

  __syncthreads();
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const int qpos = qw0 + 32 * t + lr;
    const float l_tot = l_run[t] + __shfl_xor(l_run[t], 32, 64);
    if (lk == 0 && qpos < p.seq) p.lse[((long)b * p.a + hq) * p.seq + qpos] = m_run[t] * 0.6931471805599453f + logf(l_tot);
    store_acc_T<D>(oacc[t], 1.f / l_tot, smem + w * 32 * LDK, p.o + tok0 * p.ldo + hq * D, p.ldo, qw0 + 32 * t, p.seq, lane);
  }
}

// ================================================================================================ delta = rowsum(dO * O)
template <int D>
__global__ void __launch_bounds__(256) attn_delta_kernel(const bf16* __restrict__ o, const bf16* __restrict__ dout,
                                                         float* __restrict__ delta, long ldo, long lddo, int batch,
                                                         int seq, int a) {
  constexpr int LPH = D / 8;
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  const long item = idx / LPH;          // (token, head)
  const int sub = (int)(idx % LPH);
  const long total = (long)batch * seq * a;
  float s = 0.f;
  long t = 0;
  int h = 0;
  if (item < total) {
    t = item / a;
    h = (int)(item - t * a);
    const uint4 uo = reinterpret_cast<const uint4*>(o + t * ldo + h * D)[sub];
    const uint4 ud = reinterpret_cast<const uint4*>(dout + t * lddo + h * D)[sub];
    s = bf16_lo(uo.x) * bf16_lo(ud.x) + bf16_hi(uo.x) * bf16_hi(ud.x) + bf16_lo(uo.y) * bf16_lo(ud.y) +
        bf16_hi(uo.y) * bf16_hi(ud.y) + bf16_lo(uo.z) * bf16_lo(ud.z) + bf16_hi(uo.z) * bf16_hi(ud.z) +
        bf16_lo(uo.w) * bf16_lo(ud.w) + bf16_hi(uo.w) * bf16_hi(ud.w);
  }
#pragma unroll
  for (int off = LPH / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
  if (item < total && sub == 0) {
    const long bi = t / seq, pos = t - bi * seq;
    delta[(bi * a + h) * seq + pos] = s;
  }
}

// ================================================================================================ dQ
template <int D, int QT, int NW>
__global__ void __launch_bounds__(NW * 64, (QT == 1 && NW <= 4) ? 2 : 1) attn_bwd_dq_kernel(const AttnArgs p) {
  // K is read both ways (plain for S, transposing for dQ += dS K): its tile has the row stride d + 24 that serves both
  // (see attn_bwd_dkv_pair_kernel) and is stored once
  constexpr int LDK = D + 8, LDU = D + 24, KS = D / 16, DT = D / 32, NT = NW * 64, BQ = NW * 32 * QT;
  using T64 = Tile64<D, NT>;
  extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];   // dq_smem_bytes(D, NW)
  bf16* const smem = reinterpret_cast<bf16*>(dyn_smem);
  bf16* const Ks = smem;
  bf16* const Vs = smem + 64 * LDU;

  const int tid = threadIdx.x, lane = tid & 63, lr = lane & 31, lk = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nQ = (p.seq + BQ - 1) / BQ;
  const int nhb = p.a * p.batch;
  const int rank = heavy_rank((int)blockIdx.x, (int)gridDim.x, p.fold);
  const int qtile = nQ - 1 - rank / nhb;
  const int hb = xcd_head(rank % nhb, nhb);
  const int hq = hb % p.a, b = hb / p.a;
  const int g = hq / (p.a / p.kh);
  const int q0 = qtile * BQ, qw0 = q0 + w * 32 * QT;
  const long tok0 = (long)b * p.seq;
  const bf16* qb = p.q + tok0 * p.ldq + hq * D;
  const bf16* dob = p.dout + tok0 * p.lddo + hq * D;
  const rsrc_t rk = seq_rsrc(p.k + tok0 * p.ldk + g * D, p.ldk, p.seq, D);
  const rsrc_t rv = seq_rsrc(p.v + tok0 * p.ldv + g * D, p.ldv, p.seq, D);

  uint4 qf[QT][KS], dof[QT][KS];
  float lse2[QT], dl[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const int qpos = qw0 + 32 * t + lr;
    const bool qok = qpos < p.seq;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qf[t][ks] = make_uint4(0u, 0u, 0u, 0u);
      dof[t][ks] = make_uint4(0u, 0u, 0u, 0u);
      if (qok) {
        qf[t][ks] = *reinterpret_cast<const uint4*>(qb + (long)qpos * p.ldq + 16 * ks + 8 * lk);
        dof[t][ks] = *reinterpret_cast<const uint4*>(dob + (long)qpos * p.lddo + 16 * ks + 8 * lk);
      }
    }
    const long stat = ((long)b * p.a + hq) * p.seq + qpos;
    lse2[t] = qok ? p.lse_in[stat] * 1.4426950408889634f : INFINITY;   // padded rows get P = 0
    dl[t] = qok ? p.delta[stat] : 0.f;
  }

  const int kv_end = (q0 + BQ < p.seq) ? (q0 + BQ) : p.seq;
  const int nkv = (kv_end + 63) / 64;
  f32x16 dqacc[QT][DT];
#pragma unroll
  for (int t = 0; t < QT; ++t)
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) dqacc[t][dt][v] = 0.f;

  const bf16* const kfrag0 = Ks + lr * LDU + 8 * lk;
  const bf16* const vfrag0 = Vs + lr * LDK + 8 * lk;
  const bf16* const ktfrag0 = Ks + tr_base<LDU>(lane);
  uint4 kreg[T64::NREG], vreg[T64::NREG];
  T64::load(kreg, rk, p.ldk, 0, tid);
  T64::load(vreg, rv, p.ldv, 0, tid);
  // eight-wave workgroups have the CU to themselves: two sets of tiles, one barrier per key tile (see the forward kernel)
  constexpr bool DB = NW >= 8;
  constexpr int SET = 64 * LDU + 64 * LDK;
  auto store_tiles = [&](int set) {
    T64::template store<LDU>(kreg, Ks + set * SET, tid);
    T64::template store<LDK>(vreg, Vs + set * SET, tid);
  };
  auto load_tiles = [&](int jj) {
    T64::load(kreg, rk, p.ldk, jj * 64, tid);
    T64::load(vreg, rv, p.ldv, jj * 64, tid);
  };
  if constexpr (DB) {
    store_tiles(0);
    if (nkv > 1) load_tiles(1);
  }

  for (int j = 0; j < nkv; ++j) {
    __syncthreads();
    if constexpr (DB) {
      if (j + 1 < nkv) store_tiles((j + 1) & 1);
      if (j + 2 < nkv) load_tiles(j + 2);
    } else {
      store_tiles(0);
      __syncthreads();
      if (j + 1 < nkv) load_tiles(j + 1);
    }
    const bf16* const kfrag = kfrag0 + (DB ? (j & 1) * SET : 0);
    const bf16* const vfrag = vfrag0 + (DB ? (j & 1) * SET : 0);
    const bf16* const ktfrag = ktfrag0 + (DB ? (j & 1) * SET : 0);
    const int kv0 = j * 64;
    {   // a wave whose queries all precede this tile's keys runs it fully masked (see the forward kernel)
      const bool need_mask = (kv0 + 63 > qw0) || (kv0 + 64 > p.seq);
      const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      // the two 32-key halves of the tile one after the other: half as many score registers live at a time
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        f32x16 sT[QT], dpT[QT];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const uint4 ak = *reinterpret_cast<const uint4*>(kfrag + 32 * kt * LDU + 16 * ks);
          const uint4 av = *reinterpret_cast<const uint4*>(vfrag + 32 * kt * LDK + 16 * ks);
#pragma unroll
          for (int t = 0; t < QT; ++t) {
            sT[t] = mfma32(ak, qf[t][ks], ks == 0 ? zero16 : sT[t]);
            dpT[t] = mfma32(av, dof[t][ks], ks == 0 ? zero16 : dpT[t]);
          }
        }
        // one wave-uniform branch per half tile around two whole element loops (a test per element would be
        // compiled into a branch per element)
        if (need_mask) {
#pragma unroll
          for (int t = 0; t < QT; ++t) {
            const int qpos = qw0 + 32 * t + lr;
            const int klim = (qpos < p.seq - 1 ? qpos : p.seq - 1) - (kv0 + 32 * kt + 4 * lk);   // local key index <= klim
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              float pr = fast_exp2(__builtin_fmaf(sT[t][v], p.scale_log2e, -lse2[t]));
              pr = (8 * (v >> 2) + (v & 3) > klim) ? 0.f : pr;
              sT[t][v] = pr * (dpT[t][v] - dl[t]);   // dS^T
            }
          }
        } else {
#pragma unroll
          for (int t = 0; t < QT; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v)
              sT[t][v] = fast_exp2(__builtin_fmaf(sT[t][v], p.scale_log2e, -lse2[t])) * (dpT[t][v] - dl[t]);   // dS^T
        }
        {   // the 2*DT accumulator updates as one sequence, K^T fragments requested AHEAD updates early
          constexpr int NU = 2 * DT, AHEAD = 2;
          uint4 df[2][QT];
#pragma unroll
          for (int g2 = 0; g2 < 2; ++g2)
#pragma unroll
            for (int t = 0; t < QT; ++t) df[g2][t] = pack_frag(sT[t], 8 * g2);
          auto ufrag_at = [&](int n) { return read_frag_tr<LDU>(ktfrag, 2 * kt + n / DT, 32 * (n % DT)); };
          uint4 uring[AHEAD];
#pragma unroll
          for (int n = 0; n < AHEAD; ++n) uring[n] = ufrag_at(n);
#pragma unroll
          for (int n = 0; n < NU; ++n) {
            const uint4 a = uring[n % AHEAD];
            if (n + AHEAD < NU) uring[n % AHEAD] = ufrag_at(n + AHEAD);
#pragma unroll
            for (int t = 0; t < QT; ++t) dqacc[t][n % DT] = mfma32(a, df[n / DT][t], dqacc[t][n % DT]);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int t = 0; t < QT; ++t)
    store_acc_T<D>(dqacc[t], p.scale, smem + w * 32 * LDK, p.dq + tok0 * p.lddq + hq * D, p.lddq, qw0 + 32 * t, p.seq, lane);
}

// ================================================================================================ dK, dV in one kernel
// One wave per SIMD at head dimension 128 (the K and V fragments plus both accumulators take more than 256 registers
// per lane), two at 64; four recomputed/updated products per tile.  A version split into a dV and a dK kernel at two
// waves per SIMD each (the scores recomputed in both) was as fast at best once the LDS reads here were issued ahead
// of their MFMAs (sequence 8192 to 31744: 0 to 3 % slower; 16 % slower at head dimension 64) and is gone.  Staggering
// the two 32-query halves so that one half's exponentials sit in the slots of the other half's MFMAs was 12-20 % slower
// (a wave issues in order: the dependent multiply-exp-multiply chains hold back the next MFMA).  Two sets of LDS tiles
// at d = 128 (the next query tile stored during the updates, one barrier per tile instead of two) changed nothing.
template <int D>
__global__ void __launch_bounds__(256) attn_bwd_dkv_fused_kernel(const AttnArgs p) {
  constexpr int LDK = D + 8, LDT = D + 32, KS = D / 16, DT = D / 32;
  using T64 = Tile64<D, 256>;
  extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];
  bf16* const smem = reinterpret_cast<bf16*>(dyn_smem);             // 2*64*LDK + 2*64*LDT elements
  bf16* const Qs = smem;
  bf16* const dOs = smem + 64 * LDK;
  bf16* const Qt = smem + 2 * 64 * LDK;
  bf16* const dOt = Qt + 64 * LDT;

  const int tid = threadIdx.x, lane = tid & 63, lr = lane & 31, lk = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nhb = p.a * p.batch;
  // Workgroups of one query head stream the same Q and dO tiles, a few tiles apart (key tile j starts at query tile 2j
  // and all advance at the same pace).  Consecutive workgroups go to consecutive XCDs, so XCD x (launch positions x,
  // x + 8, ...) takes nhb/8 neighbouring heads and walks them in runs of `kblock` key tiles: its 32 resident workgroups
  // are two such runs, and the XCD's L2 fetches a Q/dO tile once for a whole run.  Key tile 0 sees every query, so the
  // order is still heaviest first at the grain of a run; positions past the last key tile (ragged last run) exit.
  int kvt, hb;
  if (p.kblock) {
    const int hp = nhb >> 3, per = hp * p.kblock;
    const int s = (int)blockIdx.x >> 3, r = s % per;
    hb = ((int)blockIdx.x & 7) * hp + r / p.kblock;
    kvt = (s / per) * p.kblock + r % p.kblock;
    if (kvt * 128 >= p.seq) return;          // uniform over the workgroup, before any barrier
  } else {
    kvt = (int)blockIdx.x / nhb;             // key tile 0 sees every query: heaviest first, for every head
    hb = (int)blockIdx.x % nhb;
  }
  const int hq = hb % p.a, b = hb / p.a;
  const int grp = p.a / p.kh;
  const int g = hq / grp;
  const int kv0 = kvt * 128, kw0 = kv0 + 32 * w;
  const long tok0 = (long)b * p.seq;
  const bf16* kb = p.k + tok0 * p.ldk + g * D;
  const bf16* vb = p.v + tok0 * p.ldv + g * D;
  const int kpos = kw0 + lr;
  const bool kok = kpos < p.seq;

  uint4 kf[KS], vf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    kf[ks] = make_uint4(0u, 0u, 0u, 0u);
    vf[ks] = make_uint4(0u, 0u, 0u, 0u);
    if (kok) {
      kf[ks] = *reinterpret_cast<const uint4*>(kb + (long)kpos * p.ldk + 16 * ks + 8 * lk);
      vf[ks] = *reinterpret_cast<const uint4*>(vb + (long)kpos * p.ldv + 16 * ks + 8 * lk);
    }
  }
  f32x16 dkacc[DT], dvacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) { dkacc[dt][v] = 0.f; dvacc[dt][v] = 0.f; }

  const int nQ = (p.seq + 63) / 64;
  const int qt0 = kv0 / 64;
  const int niter = nQ - qt0;

  const bf16* qfrag = Qs + lr * LDK + 8 * lk;
  const bf16* dofrag = dOs + lr * LDK + 8 * lk;
  const bf16* qtfrag = Qt + tr_base<LDT>(lane);
  const bf16* dotfrag = dOt + tr_base<LDT>(lane);
  // The per-query terms of the softmax recomputation ride along in the products: the pad chunk of a Q row holds
  // -lse/scale split into three bf16 numbers, that of a dO row -delta, and one extra MFMA step against ones3() adds
  // them, so the score tile comes out as q.k - lse/scale and the dP tile as dO.v - delta.  (Rows of the score tile are
  // queries here: without this every lane would need sixteen different lse and delta values per tile.)
  const bf16* qx = Qs + lr * LDK + D;
  const bf16* dox = dOs + lr * LDK + D;
  const uint4 one_f = ones3(lk);

  uint4 qreg[T64::NREG], doreg[T64::NREG];
  float st_reg = 0.f;
  const rsrc_t rq = seq_rsrc(p.q + tok0 * p.ldq + hq * D, p.ldq, p.seq, D);
  const rsrc_t rdo = seq_rsrc(p.dout + tok0 * p.lddo + hq * D, p.lddo, p.seq, D);
  auto prefetch = [&](int it) {
    const int q0 = (qt0 + it) * 64;
    T64::load(qreg, rq, p.ldq, q0, tid);
    T64::load(doreg, rdo, p.lddo, q0, tid);
    if (tid < 128) {
      const int qi = q0 + (tid & 63);
      const long sidx = ((long)b * p.a + hq) * p.seq + (qi < p.seq ? qi : 0);
      const float v = tid < 64 ? -p.lse_in[sidx] / p.scale : -p.delta[sidx];
      st_reg = qi < p.seq ? v : (tid < 64 ? -3.0e4f : 0.f);   // padded query rows get P = exp(-3e4 scale) = 0
    }
  };
  if (niter > 0) prefetch(0);

  for (int it = 0; it < niter; ++it) {
    __syncthreads();
    T64::template store<LDK>(qreg, Qs, tid);
    T64::template store<LDT>(qreg, Qt, tid);
    T64::template store<LDK>(doreg, dOs, tid);
    T64::template store<LDT>(doreg, dOt, tid);
    if (tid < 64) *reinterpret_cast<uint4*>(Qs + tid * LDK + D) = split3(st_reg);
    else if (tid < 128) *reinterpret_cast<uint4*>(dOs + (tid - 64) * LDK + D) = split3(st_reg);
    __syncthreads();
    if (it + 1 < niter) prefetch(it + 1);
    const int q0 = (qt0 + it) * 64;
    {   // a wave whose keys all follow this tile's queries runs it fully masked (see the forward kernel)
      const bool need_mask = (q0 < kw0 + 31) || (kw0 + 32 > p.seq);   // wave-uniform
      const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      // the two 32-query halves of the tile one after the other: half as many score registers live at a time
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        f32x16 s = zero16, dp = zero16;
        // One wave per SIMD: nothing else covers the LDS latency, so every fragment is requested AHEAD MFMAs before
        // the one that consumes it.  Score phase: 2*(KS+1) products, alternately S and dP; the last pair are the
        // extra steps that bring in -lse/scale and -delta.
        constexpr int AHEAD = 4;
        {
          constexpr int NS = 2 * (KS + 1);
          auto sfrag_at = [&](int n) {
            const int ks = n >> 1;
            const bf16* src = ks < KS ? ((n & 1) ? dofrag : qfrag) + 16 * ks : ((n & 1) ? dox : qx);
            return *reinterpret_cast<const uint4*>(src + 32 * t2 * LDK);
          };
          uint4 ring[AHEAD];
#pragma unroll
          for (int n = 0; n < AHEAD; ++n) ring[n] = sfrag_at(n);
#pragma unroll
          for (int n = 0; n < NS; ++n) {
            const uint4 a = ring[n % AHEAD];
            if (n + AHEAD < NS) ring[n % AHEAD] = sfrag_at(n + AHEAD);
            const int ks = n >> 1;
            if (n & 1) dp = mfma32(a, ks < KS ? vf[ks] : one_f, dp);
            else s = mfma32(a, ks < KS ? kf[ks] : one_f, s);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        // the first fragments of the update phase are requested now, under the exponentials
        constexpr int NU = 4 * DT;
        auto ufrag_at = [&](int n) {   // n = (g2 * DT + dt) * 2 + which
          return read_frag_tr<LDT>((n & 1) ? qtfrag : dotfrag, 2 * t2 + n / (2 * DT), 32 * ((n >> 1) % DT));
        };
        uint4 uring[AHEAD];
#pragma unroll
        for (int n = 0; n < AHEAD; ++n) uring[n] = ufrag_at(n);
        __builtin_amdgcn_sched_barrier(0);
        // rows of the score tile are queries: q = q0 + 32*t2 + 8*(v/4) + 4*lk + v%4
        // the branch is taken per tile, not per element: away from the diagonal nothing below compares positions
        if (need_mask) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int qpos = q0 + 32 * t2 + 8 * (v >> 2) + 4 * lk + (v & 3);
            float pr = fast_exp2(s[v] * p.scale_log2e);
            pr = (kpos > qpos || !kok) ? 0.f : pr;
            s[v] = pr;                         // P
            dp[v] = pr * dp[v];                // dS
          }
        } else {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const float pr = fast_exp2(s[v] * p.scale_log2e);
            s[v] = pr;
            dp[v] = pr * dp[v];
          }
        }
        // the 4*DT accumulator updates as one sequence, fragments AHEAD updates early
        {
          const uint4 pfg[2] = {pack_frag(s, 0), pack_frag(s, 8)};
          const uint4 dfg[2] = {pack_frag(dp, 0), pack_frag(dp, 8)};
#pragma unroll
          for (int n = 0; n < NU; ++n) {
            const uint4 a = uring[n % AHEAD];
            if (n + AHEAD < NU) uring[n % AHEAD] = ufrag_at(n + AHEAD);
            const int g2 = n / (2 * DT), dt = (n >> 1) % DT;
            if (n & 1) dkacc[dt] = mfma32(a, dfg[g2], dkacc[dt]);
            else dvacc[dt] = mfma32(a, pfg[g2], dvacc[dt]);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
    }
  }
  __syncthreads();
  if (grp == 1) {
    store_acc_T<D>(dkacc, p.scale, smem + w * 32 * LDK, p.dk + tok0 * p.lddk + g * D, p.lddk, kw0, p.seq, lane);
    store_acc_T<D>(dvacc, 1.f, smem + w * 32 * LDK, p.dv + tok0 * p.lddv + g * D, p.lddv, kw0, p.seq, lane);
  } else {
    float* const stage = reinterpret_cast<float*>(smem) + w * 32 * (D + 4);
    const long ldp = (long)p.a * D;
    store_acc_T_f32<D>(dkacc, p.scale, stage, p.dk_part + tok0 * ldp + hq * D, ldp, kw0, p.seq, lane);
    store_acc_T_f32<D>(dvacc, 1.f, stage, p.dv_part + tok0 * ldp + hq * D, ldp, kw0, p.seq, lane);
  }
}

// The same products with two waves per SIMD.  A workgroup is eight waves: the 32 keys of key group w = wave / 2 are shared
// by a pair of waves, and wave h = wave % 2 of the pair keeps the accumulators of one half of the head dimension only
// (dK^T, dV^T rows [h*D/2, (h+1)*D/2): half the registers).  The scores need the whole head dimension, so the pair splits
// them by queries instead: wave h recomputes S and dP for the 32 queries of half h of the tile, turns them into P and dS, and
// hands both (already in the operand layout of the update products, identical in the two waves since they own the same
// keys) to its partner through LDS.  Every wave then updates its half of the accumulators with its own 32 queries --
// before the workgroup barrier that publishes the exchange -- and with the partner's 32 queries after it.  Same number of
// MFMAs per workgroup as the one-wave-per-SIMD kernel, same LDS fragment traffic per CU, 8 KB of exchange per pair and tile.
template <int D>
__global__ void __launch_bounds__(512) attn_bwd_dkv_pair_kernel(const AttnArgs p) {
  // One LDS layout serves both kinds of fragment reads, so that every Q and dO tile is stored once: a row stride of
  // D + 24 elements is 12 banks past a multiple of 64, which keeps the 16 rows of a plain 16-byte read phase on distinct
  // banks; the transposing 8-byte reads (32 lanes a phase: 4 rows x 64 bytes) overlap on a quarter of their banks
  // (SQ_LDS_BANK_CONFLICT: 22 % of the LDS-active cycles).  Measured cheaper than storing the tiles twice (-3 %); a
  // layout with the transposing stride D + 32 and the 16-byte chunks of a row permuted (c ^ (row / 4 & 3)) removes the
  // conflicts altogether (LDS-active cycles -20 %) and is not faster; neither is a variant with one workgroup barrier
  // per tile and a flag handshake inside the pair.  No unit is more than half busy: the waves wait on their own chain.
  constexpr int LDU = D + 24, KS = D / 16, DT = D / 32, DH = DT / 2;
  static_assert(DT % 2 == 0, "the head dimension is split over two waves");
  using T64 = Tile64<D, 512>;
  extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];
  bf16* const smem = reinterpret_cast<bf16*>(dyn_smem);             // two sets (tile parity) of Q | dO, then the exchange
  constexpr int TSET = 2 * 64 * LDU;
  uint4* const exch = reinterpret_cast<uint4*>(smem + 2 * TSET);    // [8 waves][4 fragments][64 lanes]

  const int tid = threadIdx.x, lane = tid & 63, lr = lane & 31, lk = lane >> 5;
  const int w8 = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int w = w8 >> 1, h = w8 & 1;
  const int nhb = p.a * p.batch;
  int kvt, hb;                                 // launch order: see attn_bwd_dkv_fused_kernel
  if (p.kblock) {
    const int hp = nhb >> 3, per = hp * p.kblock;
    const int s = (int)blockIdx.x >> 3, r = s % per;
    hb = ((int)blockIdx.x & 7) * hp + r / p.kblock;
    kvt = (s / per) * p.kblock + r % p.kblock;
    if (kvt * 128 >= p.seq) return;
  } else {
    kvt = (int)blockIdx.x / nhb;
    hb = (int)blockIdx.x % nhb;
  }
  const int hq = hb % p.a, b = hb / p.a;
  const int grp = p.a / p.kh;
  const int g = hq / grp;
  const int kv0 = kvt * 128, kw0 = kv0 + 32 * w;
  const long tok0 = (long)b * p.seq;
  const bf16* kb = p.k + tok0 * p.ldk + g * D;
  const bf16* vb = p.v + tok0 * p.ldv + g * D;
  const int kpos = kw0 + lr;
  const bool kok = kpos < p.seq;

  uint4 kf[KS], vf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    kf[ks] = make_uint4(0u, 0u, 0u, 0u);
    vf[ks] = make_uint4(0u, 0u, 0u, 0u);
    if (kok) {
      kf[ks] = *reinterpret_cast<const uint4*>(kb + (long)kpos * p.ldk + 16 * ks + 8 * lk);
      vf[ks] = *reinterpret_cast<const uint4*>(vb + (long)kpos * p.ldv + 16 * ks + 8 * lk);
    }
  }
  f32x16 dkacc[DH], dvacc[DH];
#pragma unroll
  for (int dt = 0; dt < DH; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) { dkacc[dt][v] = 0.f; dvacc[dt][v] = 0.f; }

  const int nQ = (p.seq + 63) / 64;
  const int qt0 = kv0 / 64;
  const int niter = nQ - qt0;

  // this wave's 32 queries of a tile: rows 32*h .. 32*h + 31
  const bf16* qfrag = smem + (32 * h + lr) * LDU + 8 * lk;
  const bf16* dofrag = qfrag + 64 * LDU;
  const bf16* qx = smem + (32 * h + lr) * LDU + D;
  const bf16* dox = qx + 64 * LDU;
  // this wave's half of the head dimension: columns 32*DH*h .. of the transposed tiles
  const bf16* qtfrag = smem + tr_base<LDU>(lane) + 32 * DH * h;
  const bf16* dotfrag = qtfrag + 64 * LDU;
  const uint4 one_f = ones3(lk);
  uint4* const ex_mine = exch + (w8 * 4) * 64 + lane;
  const uint4* const ex_theirs = exch + ((w8 ^ 1) * 4) * 64 + lane;

  uint4 qreg[T64::NREG], doreg[T64::NREG];
  float st_reg = 0.f;
  const rsrc_t rq = seq_rsrc(p.q + tok0 * p.ldq + hq * D, p.ldq, p.seq, D);
  const rsrc_t rdo = seq_rsrc(p.dout + tok0 * p.lddo + hq * D, p.lddo, p.seq, D);
  auto prefetch = [&](int it) {
    const int q0 = (qt0 + it) * 64;
    T64::load(qreg, rq, p.ldq, q0, tid);
    T64::load(doreg, rdo, p.lddo, q0, tid);
    if (tid < 128) {
      const int qi = q0 + (tid & 63);
      const long sidx = ((long)b * p.a + hq) * p.seq + (qi < p.seq ? qi : 0);
      const float v = tid < 64 ? -p.lse_in[sidx] / p.scale : -p.delta[sidx];
      st_reg = qi < p.seq ? v : (tid < 64 ? -3.0e4f : 0.f);
    }
  };
  if (niter > 0) prefetch(0);

  constexpr int AHEAD = 2;     // two waves per SIMD cover each other's LDS latency: a short ring is enough
  // the update products of one 32-query half t2 with the fragments pf (P) and df (dS): 4 * DH MFMAs
  auto update_half = [&](int set, int t2, const uint4 (&pf)[2], const uint4 (&df)[2]) {
    constexpr int NU = 4 * DH;
    auto ufrag_at = [&](int n) {   // n = (g2 * DH + dt) * 2 + which
      return read_frag_tr<LDU>(((n & 1) ? qtfrag : dotfrag) + set * TSET, 2 * t2 + n / (2 * DH), 32 * ((n >> 1) % DH));
    };
    uint4 uring[AHEAD];
#pragma unroll
    for (int n = 0; n < AHEAD; ++n) uring[n] = ufrag_at(n);
    MFMA_PHASE_BEGIN();
#pragma unroll
    for (int n = 0; n < NU; ++n) {
      const uint4 a = uring[n % AHEAD];
      if (n + AHEAD < NU) uring[n % AHEAD] = ufrag_at(n + AHEAD);
      const int g2 = n / (2 * DH), dt = (n >> 1) % DH;
      if (n & 1) dkacc[dt] = mfma32(a, df[g2], dkacc[dt]);
      else dvacc[dt] = mfma32(a, pf[g2], dvacc[dt]);
      __builtin_amdgcn_sched_barrier(0);
    }
    MFMA_PHASE_END();
  };

  // Two barriers per tile.  After the first one every wave is done with the previous tile's score phase and has
  // published its fragments: the new tile is stored (into the other set) and, meanwhile, the
  // accumulators are updated with the partner's half of the PREVIOUS tile, whose set is still in place.
  auto partner_update = [&](int it_prev) {
    const uint4 ppf[2] = {ex_theirs[0], ex_theirs[64]};
    const uint4 pdf[2] = {ex_theirs[128], ex_theirs[192]};
    update_half(it_prev & 1, h ^ 1, ppf, pdf);
  };
  for (int it = 0; it < niter; ++it) {
    __syncthreads();
    bf16* const q_set = smem + (it & 1) * TSET;
    T64::template store<LDU>(qreg, q_set, tid);
    T64::template store<LDU>(doreg, q_set + 64 * LDU, tid);
    if (tid < 64) *reinterpret_cast<uint4*>(q_set + tid * LDU + D) = split3(st_reg);
    else if (tid < 128) *reinterpret_cast<uint4*>(q_set + 64 * LDU + (tid - 64) * LDU + D) = split3(st_reg);
    if (it > 0) partner_update(it - 1);
    __syncthreads();
    if (it + 1 < niter) prefetch(it + 1);
    const int q0 = (qt0 + it) * 64;
    const int qh0 = q0 + 32 * h;                                            // first query of this wave's half
    const bool need_mask = (qh0 < kw0 + 31) || (kw0 + 32 > p.seq);          // wave-uniform
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 s = zero16, dp = zero16;
    {
      constexpr int NS = 2 * (KS + 1);
      auto sfrag_at = [&](int n) {
        const int ks = n >> 1;
        const bf16* src = ks < KS ? ((n & 1) ? dofrag : qfrag) + 16 * ks : ((n & 1) ? dox : qx);
        return *reinterpret_cast<const uint4*>(src + (it & 1) * TSET);
      };
      uint4 ring[AHEAD];
#pragma unroll
      for (int n = 0; n < AHEAD; ++n) ring[n] = sfrag_at(n);
      MFMA_PHASE_BEGIN();
#pragma unroll
      for (int n = 0; n < NS; ++n) {
        const uint4 a = ring[n % AHEAD];
        if (n + AHEAD < NS) ring[n % AHEAD] = sfrag_at(n + AHEAD);
        const int ks = n >> 1;
        if (n & 1) dp = mfma32(a, ks < KS ? vf[ks] : one_f, dp);
        else s = mfma32(a, ks < KS ? kf[ks] : one_f, s);
        __builtin_amdgcn_sched_barrier(0);
      }
      MFMA_PHASE_END();
    }
    // rows of the score tile are queries: q = qh0 + 8*(v/4) + 4*lk + v%4
    if (need_mask) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int qpos = qh0 + 8 * (v >> 2) + 4 * lk + (v & 3);
        float pr = fast_exp2(s[v] * p.scale_log2e);
        pr = (kpos > qpos || !kok) ? 0.f : pr;
        s[v] = pr;                         // P
        dp[v] = pr * dp[v];                // dS
      }
    } else {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float pr = fast_exp2(s[v] * p.scale_log2e);
        s[v] = pr;
        dp[v] = pr * dp[v];
      }
    }
    const uint4 pfg[2] = {pack_frag(s, 0), pack_frag(s, 8)};
    const uint4 dfg[2] = {pack_frag(dp, 0), pack_frag(dp, 8)};
    // the partner read last tile's fragments before the barrier above: the slots are free
    ex_mine[0] = pfg[0]; ex_mine[64] = pfg[1]; ex_mine[128] = dfg[0]; ex_mine[192] = dfg[1];
    update_half(it & 1, h, pfg, dfg);
  }
  __syncthreads();
  if (niter > 0) partner_update(niter - 1);
  __syncthreads();
  if (grp == 1) {
    bf16* const stage = smem + w8 * 32 * (D / 2 + 8);
    store_acc_T<D / 2>(dkacc, p.scale, stage, p.dk + tok0 * p.lddk + g * D + h * (D / 2), p.lddk, kw0, p.seq, lane);
    store_acc_T<D / 2>(dvacc, 1.f, stage, p.dv + tok0 * p.lddv + g * D + h * (D / 2), p.lddv, kw0, p.seq, lane);
  } else {
    float* const stage = reinterpret_cast<float*>(smem) + w8 * 32 * (D / 2 + 4);
    const long ldp = (long)p.a * D;
    store_acc_T_f32<D / 2>(dkacc, p.scale, stage, p.dk_part + tok0 * ldp + hq * D + h * (D / 2), ldp, kw0, p.seq, lane);
    store_acc_T_f32<D / 2>(dvacc, 1.f, stage, p.dv_part + tok0 * ldp + hq * D + h * (D / 2), ldp, kw0, p.seq, lane);
  }
}

// dk[t, g, :] = sum over the query heads of group g of the fp32 partials, in head order; same for dv.
template <int D>
__global__ void __launch_bounds__(256) attn_dkv_reduce_kernel(const float* __restrict__ dk_part, const float* __restrict__ dv_part,
                                                              bf16* __restrict__ dk, bf16* __restrict__ dv, long lddk,
                                                              long lddv, long T, int a, int kh) {
  constexpr int CH = D / 8;
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  const long per = T * kh * CH;
  if (idx >= 2 * per) return;
  const bool is_v = idx >= per;
  const long i = is_v ? idx - per : idx;
  const int ch = (int)(i % CH);
  const int g = (int)((i / CH) % kh);
  const long t = i / ((long)CH * kh);
  const int grp = a / kh;
  const float* src = (is_v ? dv_part : dk_part) + t * (long)a * D + (long)g * grp * D + ch * 8;
  float4 s0 = make_float4(0.f, 0.f, 0.f, 0.f), s1 = s0;
  for (int j = 0; j < grp; ++j) {
    const float4 x0 = *reinterpret_cast<const float4*>(src + (long)j * D);
    const float4 x1 = *reinterpret_cast<const float4*>(src + (long)j * D + 4);
    s0.x += x0.x; s0.y += x0.y; s0.z += x0.z; s0.w += x0.w;
    s1.x += x1.x; s1.y += x1.y; s1.z += x1.z; s1.w += x1.w;
  }
  bf16* dst = is_v ? dv + t * lddv + g * D + ch * 8 : dk + t * lddk + g * D + ch * 8;
  *reinterpret_cast<uint4*>(dst) = make_uint4(pack_bf16x2(s0.x, s0.y), pack_bf16x2(s0.z, s0.w), pack_bf16x2(s1.x, s1.y),
                                              pack_bf16x2(s1.z, s1.w));
}

// operand tiles, or the epilogue's staging of every wave's 32 x d block, whichever is larger
constexpr int max_i(int a, int b) { return a > b ? a : b; }
constexpr int fwd_smem_bytes(int d, int nw) { return max_i((nw >= 8 ? 2 : 1) * (64 * (d + 8) + 64 * (d + 32)), nw * 32 * (d + 8)) * 2; }
constexpr int dq_smem_bytes(int d, int nw) { return max_i((nw >= 8 ? 2 : 1) * (64 * (d + 24) + 64 * (d + 8)), nw * 32 * (d + 8)) * 2; }
constexpr int dkv_fused_smem_bytes(int d) { return (2 * 64 * (d + 8) + 2 * 64 * (d + 32)) * 2; }
constexpr int dkv_pair_smem_bytes(int d) { return 2 * (2 * 64 * (d + 24)) * 2 + 8 * 4 * 64 * 16; }
void fill_common(AttnArgs& p, int batch, int seq, int a, int kh, int d) {
  p.batch = batch; p.seq = seq; p.a = a; p.kh = kh;
  p.scale = 1.0f / sqrtf((float)d);
  p.scale_log2e = p.scale * 1.4426950408889634f;
}

template <typename K>
hipError_t set_smem(K kern, int bytes, bool& done) {
  if (done) return hipSuccess;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) done = true;
  return e;
}

template <int D, int QT, int NW>
hipError_t launch_fwd(hipStream_t st, const AttnArgs& p) {
  constexpr int BQ = NW * 32 * QT;
  static bool done = false;
  hipError_t e = set_smem(attn_fwd_kernel<D, QT, NW>, fwd_smem_bytes(D, NW), done);
  if (e != hipSuccess) return e;
  const int grid = ((p.seq + BQ - 1) / BQ) * p.a * p.batch;
  AttnArgs pf = p;
  pf.fold = NW <= 4 && grid > 256 && grid <= 512;
  RP_LAUNCH((attn_fwd_kernel<D, QT, NW>), dim3(grid), dim3(NW * 64), fwd_smem_bytes(D, NW), st, pf);
  return hipGetLastError();
}

template <int D>
hipError_t launch_dkv_fused(hipStream_t st, const AttnArgs& p, int grid) {
  static bool done = false;
  hipError_t e = set_smem(attn_bwd_dkv_fused_kernel<D>, dkv_fused_smem_bytes(D), done);
  if (e != hipSuccess) return e;
  RP_LAUNCH((attn_bwd_dkv_fused_kernel<D>), dim3(grid), dim3(256), dkv_fused_smem_bytes(D), st, p);
  return hipGetLastError();
}

template <int D>
hipError_t launch_dkv_pair(hipStream_t st, const AttnArgs& p, int grid) {
  static bool done = false;
  hipError_t e = set_smem(attn_bwd_dkv_pair_kernel<D>, dkv_pair_smem_bytes(D), done);
  if (e != hipSuccess) return e;
  RP_LAUNCH((attn_bwd_dkv_pair_kernel<D>), dim3(grid), dim3(512), dkv_pair_smem_bytes(D), st, p);
  return hipGetLastError();
}

template <int D, int QT, int NW>
hipError_t launch_dq(hipStream_t st, const AttnArgs& p) {
  constexpr int BQ = NW * 32 * QT;
  static bool done = false;
  hipError_t e = set_smem(attn_bwd_dq_kernel<D, QT, NW>, dq_smem_bytes(D, NW), done);
  if (e != hipSuccess) return e;
  const int grid = ((p.seq + BQ - 1) / BQ) * p.a * p.batch;
  AttnArgs pf = p;
  pf.fold = NW <= 4 && grid > 256 && grid <= 512;
  RP_LAUNCH((attn_bwd_dq_kernel<D, QT, NW>), dim3(grid), dim3(NW * 64), dq_smem_bytes(D, NW), st, pf);
  return hipGetLastError();
}

}  // namespace

// ------------------------------------------------------------------------------------------------ launchers
hipError_t k_attn_fwd(hipStream_t st, const void* q, const void* k, const void* v, void* o, float* lse, long ldq,
                      long ldk, long ldv, long ldo, int batch, int seq, int a, int kh, int d) {
  if (batch * seq == 0) return hipSuccess;
  AttnArgs p = {};
  p.q = (const bf16*)q; p.k = (const bf16*)k; p.v = (const bf16*)v; p.o = (bf16*)o; p.lse = lse;
  p.ldq = ldq; p.ldk = ldk; p.ldv = ldv; p.ldo = ldo;
  fill_common(p, batch, seq, a, kh, d);
  // workgroup = 4 waves x 32 queries; 64 queries per wave halve the LDS reads per MFMA but spill at d = 128
  // eight waves per workgroup (256 queries) store every K/V tile once for twice the products; enough workgroups needed
  // (d = 128 only: at d = 64 the four-wave kernel fits three waves per SIMD and is 20 % faster than the eight-wave one)
  const bool big = (long)((seq + 255) / 256) * a * batch >= 1024;
  if (d == 128 && big) return launch_fwd<128, 1, 8>(st, p);
  if (d == 128) return launch_fwd<128, 1, 4>(st, p);
  if (d == 64) return launch_fwd<64, 1, 4>(st, p);
  return hipErrorInvalidValue;
}

hipError_t k_attn_delta(hipStream_t st, const void* o, const void* dout, float* delta, long ldo, long lddo, int batch,
                        int seq, int a, int d) {
  const long items = (long)batch * seq * a * (d / 8);
  if (items == 0) return hipSuccess;
  const int grid = (int)((items + 255) / 256);
  if (d == 128) RP_LAUNCH(attn_delta_kernel<128>, dim3(grid), dim3(256), 0, st, (const bf16*)o, (const bf16*)dout, delta, ldo, lddo, batch, seq, a);
  else if (d == 64) RP_LAUNCH(attn_delta_kernel<64>, dim3(grid), dim3(256), 0, st, (const bf16*)o, (const bf16*)dout, delta, ldo, lddo, batch, seq, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t k_attn_bwd(hipStream_t st, int part, const void* q, const void* k, const void* v, const void* dout,
                      const float* lse, const float* delta, void* dq, void* dk, void* dv, float* scratch, long ldq,
                      long ldk, long ldv, long lddo, long lddq, long lddk, long lddv, int batch, int seq, int a, int kh,
                      int d) {
  if (batch * seq == 0) return hipSuccess;
  AttnArgs p = {};
  p.q = (const bf16*)q; p.k = (const bf16*)k; p.v = (const bf16*)v; p.dout = (const bf16*)dout;
  p.lse_in = lse; p.delta = delta; p.dq = (bf16*)dq; p.dk = (bf16*)dk; p.dv = (bf16*)dv;
  p.ldq = ldq; p.ldk = ldk; p.ldv = ldv; p.lddo = lddo; p.lddq = lddq; p.lddk = lddk; p.lddv = lddv;
  fill_common(p, batch, seq, a, kh, d);
  if (d != 128 && d != 64) return hipErrorInvalidValue;
  if (a != kh && !scratch) return hipErrorInvalidValue;
  const long T = (long)batch * seq;
  p.dk_part = scratch;
  p.dv_part = scratch ? scratch + T * a * d : nullptr;
  hipError_t e = hipSuccess;
  if (part == 2) {   // sum of the group's partials
    if (a == kh) return hipSuccess;
    const long items = 2 * T * kh * (d / 8);
    const int grid = (int)((items + 255) / 256);
    if (d == 128) RP_LAUNCH(attn_dkv_reduce_kernel<128>, dim3(grid), dim3(256), 0, st, p.dk_part, p.dv_part, p.dk, p.dv, lddk, lddv, T, a, kh);
    else RP_LAUNCH(attn_dkv_reduce_kernel<64>, dim3(grid), dim3(256), 0, st, p.dk_part, p.dv_part, p.dk, p.dv, lddk, lddv, T, a, kh);
    return hipGetLastError();
  }
  if (part == 0) {
    const int nkv = (seq + 127) / 128, nhb = a * batch;
    int nk = nkv * nhb;                               // one workgroup per 128 keys and query head
    // XCD-aware order (see the kernel) from 96 key tiles on: 5-7 % at 16-32 k tokens; below that the re-fetches it saves
    // do not matter and the plain order balances the few rounds of workgroups better (4096 tokens: 10 % slower with it)
    if (nhb % 8 == 0 && nkv >= 96) {
      p.kblock = nkv >= 192 ? 32 : 16;
      nk = ((nkv + p.kblock - 1) / p.kblock) * p.kblock * nhb;
    }
    if (d == 128) return launch_dkv_pair<128>(st, p, nk);
    return launch_dkv_fused<64>(st, p, nk);   // d = 64: its registers already allow two waves per SIMD
  } else {
    const bool big = (long)((seq + 255) / 256) * a * batch >= 1024;
    if (d == 128 && big) return launch_dq<128, 1, 8>(st, p);
    return d == 128 ? launch_dq<128, 1, 4>(st, p) : launch_dq<64, 1, 4>(st, p);
  }
  return hipGetLastError();
}
