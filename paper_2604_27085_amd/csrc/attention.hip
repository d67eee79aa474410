// Causal grouped-query attention on the gfx950 matrix cores, flash style (no s x s matrix ever leaves the CU).
//
// All three kernels use v_mfma_f32_32x32x16_bf16 with the score tile computed TRANSPOSED relative to the row that is
// being normalised: the 32x32 accumulator layout gives every lane one column and 16 rows, so with queries (forward,
// dQ) as columns the softmax reductions are in-lane plus one exchange with lane^32, and the probabilities already sit
// in the register layout the next MFMA wants as its B operand.  The operand whose reduction index is not contiguous in
// memory (V for P.V, K for dS.K, Q and dO for the dK/dV products) is transposed in registers (8x8 blocks) on its way
// into LDS, with the reduction index permuted to match the accumulator layout of the score tile.
//
//   forward : block = 128 queries of one head (4 waves x 32), loop over 64-key tiles up to the diagonal
//   dQ      : same decomposition; recomputes S^T and dP^T, accumulates dQ^T
//   dK, dV  : block = 128 keys of one kv head (4 waves x 32), loops over the query heads of the group and over 64-query
//             tiles from the diagonal on; accumulates dK^T, dV^T in registers, so no atomics and a fixed summation order
#include "common.hpp"
#include "kernels.hpp"

namespace {

constexpr int LDT = 72;   // row stride of transposed [D][64 + 8] LDS tiles

struct AttnArgs {
  const bf16 *q, *k, *v, *dout;
  bf16 *o, *dq, *dk, *dv;
  float* lse;
  const float* lse_in;
  const float* delta;
  long ldq, ldk, ldv, ldo, lddo, lddq, lddk, lddv;
  int batch, seq, a, kh;
  float scale_log2e, scale;
};

// ---- 64 x D tile loaders --------------------------------------------------------------------------------------
template <int D>
RP_DEV void load_direct64(uint4 (&r)[D / 32], const bf16* __restrict__ base, long ld, int row0, int nrows, int tid) {
#pragma unroll
  for (int it = 0; it < D / 32; ++it) {
    const int c = it * 256 + tid;
    const int row = row0 + c / (D / 8), ch = c % (D / 8);
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (row < nrows) v = *reinterpret_cast<const uint4*>(base + (long)row * ld + ch * 8);
    r[it] = v;
  }
}
template <int D>
RP_DEV void store_direct64(const uint4 (&r)[D / 32], bf16* S, int tid) {
#pragma unroll
  for (int it = 0; it < D / 32; ++it) {
    const int c = it * 256 + tid;
    *reinterpret_cast<uint4*>(S + (c / (D / 8)) * (D + 8) + (c % (D / 8)) * 8) = r[it];
  }
}
// 8x8 blocks: thread -> (row block rb of 8 tile rows, column block b of 8 features)
template <int D>
RP_DEV void load_trans64(uint4 (&r)[8], const bf16* __restrict__ base, long ld, int row0, int nrows, int tid) {
  const int rb = (tid >> 1) & 7;
  const int b = (tid & 1) | ((tid >> 4) << 1);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = row0 + rb * 8 + i;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (b < D / 8 && row < nrows) v = *reinterpret_cast<const uint4*>(base + (long)row * ld + b * 8);
    r[i] = v;
  }
}
// Writes the transposed tile St[feature][64 tile rows] with the tile-row index permuted inside every group of 16:
// tile row 16g + 8p + 4h + e is stored at column 16g + 8h + 4p + e, which is the order in which a lane of the 32x32
// accumulator (half h) holds its 8 values of that group.
template <int D>
RP_DEV void store_trans64_perm(const uint4 (&r)[8], bf16* St, int tid) {
  const int rb = (tid >> 1) & 7;
  const int b = (tid & 1) | ((tid >> 4) << 1);
  if (b < D / 8) {
    uint4 t[8];
    transpose8x8_bf16(r, t);
    const int g = rb >> 1, pp = rb & 1;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      bf16* row = St + (b * 8 + c) * LDT + 16 * g + 4 * pp;
      *reinterpret_cast<uint2*>(row) = make_uint2(t[c].x, t[c].y);
      *reinterpret_cast<uint2*>(row + 8) = make_uint2(t[c].z, t[c].w);
    }
  }
}

RP_DEV uint4 pack_frag(const f32x16& s, int off) {
  return make_uint4(pack_bf16x2(s[off + 0], s[off + 1]), pack_bf16x2(s[off + 2], s[off + 3]),
                    pack_bf16x2(s[off + 4], s[off + 5]), pack_bf16x2(s[off + 6], s[off + 7]));
}

RP_DEV float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

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
}

// ================================================================================================ forward
template <int D>
__global__ void __launch_bounds__(256) attn_fwd_kernel(const AttnArgs p) {
  constexpr int LDKD = D + 8, KS = D / 16, DT = D / 32;
  __shared__ __attribute__((aligned(16))) bf16 smem[64 * LDKD + D * LDT];
  bf16* const Ks = smem;
  bf16* const Vt = smem + 64 * LDKD;

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, lr = lane & 31, lk = lane >> 5;
  const int nQ = (p.seq + 127) / 128;
  int bid = blockIdx.x;
  const int qt = nQ - 1 - (bid % nQ);
  bid /= nQ;
  const int hq = bid % p.a, b = bid / p.a;
  const int g = hq / (p.a / p.kh);
  const int q0 = qt * 128;
  const long tok0 = (long)b * p.seq;
  const bf16* qb = p.q + tok0 * p.ldq + hq * D;
  const bf16* kb = p.k + tok0 * p.ldk + g * D;
  const bf16* vb = p.v + tok0 * p.ldv + g * D;
  const int qpos = q0 + 32 * w + lr;

  uint4 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    qf[ks] = make_uint4(0u, 0u, 0u, 0u);
    if (qpos < p.seq) qf[ks] = *reinterpret_cast<const uint4*>(qb + (long)qpos * p.ldq + 16 * ks + 8 * lk);
  }
  const int kv_end = (q0 + 128 < p.seq) ? (q0 + 128) : p.seq;
  const int nkv = (kv_end + 63) / 64;

  float m_run = -INFINITY, l_run = 0.f;
  f32x16 oacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[dt][v] = 0.f;

  uint4 kreg[D / 32], vreg[8];
  load_direct64<D>(kreg, kb, p.ldk, 0, p.seq, tid);
  load_trans64<D>(vreg, vb, p.ldv, 0, p.seq, tid);

  for (int j = 0; j < nkv; ++j) {
    __syncthreads();
    store_direct64<D>(kreg, Ks, tid);
    store_trans64_perm<D>(vreg, Vt, tid);
    __syncthreads();
    if (j + 1 < nkv) {
      load_direct64<D>(kreg, kb, p.ldk, (j + 1) * 64, p.seq, tid);
      load_trans64<D>(vreg, vb, p.ldv, (j + 1) * 64, p.seq, tid);
    }
    const int kv0 = j * 64;
    if (kv0 <= q0 + 32 * w + 31) {
      f32x16 sT[2];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int v = 0; v < 16; ++v) sT[kt][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
          const uint4 a = *reinterpret_cast<const uint4*>(Ks + (32 * kt + lr) * LDKD + 16 * ks + 8 * lk);
          sT[kt] = mfma32(a, qf[ks], sT[kt]);
        }
      const bool need_mask = (kv0 + 63 > q0 + 32 * w) || (kv0 + 64 > p.seq);
      float mx = -INFINITY;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float s = sT[kt][v] * p.scale_log2e;
          if (need_mask) {
            const int kpos = kv0 + 32 * kt + 8 * (v >> 2) + 4 * lk + (v & 3);
            if (kpos > qpos || kpos >= p.seq) s = -INFINITY;
          }
          sT[kt][v] = s;
          mx = fmaxf(mx, s);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run, mx);
      const float alpha = fast_exp2(m_run - m_new);
      float psum = 0.f;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float e = fast_exp2(sT[kt][v] - m_new);
          sT[kt][v] = e;
          psum += e;
        }
      l_run = l_run * alpha + psum;
      m_run = m_new;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[dt][v] *= alpha;
#pragma unroll
      for (int gk = 0; gk < 4; ++gk) {
        const uint4 pf = pack_frag(sT[gk >> 1], 8 * (gk & 1));
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const uint4 a = *reinterpret_cast<const uint4*>(Vt + (32 * dt + lr) * LDT + 16 * gk + 8 * lk);
          oacc[dt] = mfma32(a, pf, oacc[dt]);
        }
      }
    }
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.f / l_tot;
  if (lk == 0 && qpos < p.seq)
    p.lse[((long)b * p.a + hq) * p.seq + qpos] = m_run * 0.6931471805599453f + logf(l_tot);
  __syncthreads();
  store_acc_T<D>(oacc, inv, smem + w * 32 * LDKD, p.o + tok0 * p.ldo + hq * D, p.ldo, q0 + 32 * w, p.seq, lane);
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
template <int D>
__global__ void __launch_bounds__(256) attn_bwd_dq_kernel(const AttnArgs p) {
  constexpr int LDKD = D + 8, KS = D / 16, DT = D / 32;
  __shared__ __attribute__((aligned(16))) bf16 smem[2 * 64 * LDKD + D * LDT];
  bf16* const Ks = smem;
  bf16* const Vs = smem + 64 * LDKD;
  bf16* const Kt = smem + 2 * 64 * LDKD;

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, lr = lane & 31, lk = lane >> 5;
  const int nQ = (p.seq + 127) / 128;
  int bid = blockIdx.x;
  const int qt = nQ - 1 - (bid % nQ);
  bid /= nQ;
  const int hq = bid % p.a, b = bid / p.a;
  const int g = hq / (p.a / p.kh);
  const int q0 = qt * 128;
  const long tok0 = (long)b * p.seq;
  const bf16* qb = p.q + tok0 * p.ldq + hq * D;
  const bf16* dob = p.dout + tok0 * p.lddo + hq * D;
  const bf16* kb = p.k + tok0 * p.ldk + g * D;
  const bf16* vb = p.v + tok0 * p.ldv + g * D;
  const int qpos = q0 + 32 * w + lr;
  const bool qok = qpos < p.seq;

  uint4 qf[KS], dof[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    qf[ks] = make_uint4(0u, 0u, 0u, 0u);
    dof[ks] = make_uint4(0u, 0u, 0u, 0u);
    if (qok) {
      qf[ks] = *reinterpret_cast<const uint4*>(qb + (long)qpos * p.ldq + 16 * ks + 8 * lk);
      dof[ks] = *reinterpret_cast<const uint4*>(dob + (long)qpos * p.lddo + 16 * ks + 8 * lk);
    }
  }
  const long stat = ((long)b * p.a + hq) * p.seq + qpos;
  const float lse2 = qok ? p.lse_in[stat] * 1.4426950408889634f : INFINITY;   // padded rows get P = 0
  const float dl = qok ? p.delta[stat] : 0.f;

  const int kv_end = (q0 + 128 < p.seq) ? (q0 + 128) : p.seq;
  const int nkv = (kv_end + 63) / 64;
  f32x16 dqacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) dqacc[dt][v] = 0.f;

  uint4 kreg[D / 32], vreg[D / 32], ktreg[8];
  load_direct64<D>(kreg, kb, p.ldk, 0, p.seq, tid);
  load_direct64<D>(vreg, vb, p.ldv, 0, p.seq, tid);
  load_trans64<D>(ktreg, kb, p.ldk, 0, p.seq, tid);

  for (int j = 0; j < nkv; ++j) {
    __syncthreads();
    store_direct64<D>(kreg, Ks, tid);
    store_direct64<D>(vreg, Vs, tid);
    store_trans64_perm<D>(ktreg, Kt, tid);
    __syncthreads();
    if (j + 1 < nkv) {
      load_direct64<D>(kreg, kb, p.ldk, (j + 1) * 64, p.seq, tid);
      load_direct64<D>(vreg, vb, p.ldv, (j + 1) * 64, p.seq, tid);
      load_trans64<D>(ktreg, kb, p.ldk, (j + 1) * 64, p.seq, tid);
    }
    const int kv0 = j * 64;
    if (kv0 <= q0 + 32 * w + 31) {
      f32x16 sT[2], dpT[2];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int v = 0; v < 16; ++v) { sT[kt][v] = 0.f; dpT[kt][v] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
          const uint4 ak = *reinterpret_cast<const uint4*>(Ks + (32 * kt + lr) * LDKD + 16 * ks + 8 * lk);
          sT[kt] = mfma32(ak, qf[ks], sT[kt]);
          const uint4 av = *reinterpret_cast<const uint4*>(Vs + (32 * kt + lr) * LDKD + 16 * ks + 8 * lk);
          dpT[kt] = mfma32(av, dof[ks], dpT[kt]);
        }
      const bool need_mask = (kv0 + 63 > q0 + 32 * w) || (kv0 + 64 > p.seq);
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float pr = fast_exp2(sT[kt][v] * p.scale_log2e - lse2);
          if (need_mask) {
            const int kpos = kv0 + 32 * kt + 8 * (v >> 2) + 4 * lk + (v & 3);
            if (kpos > qpos || kpos >= p.seq) pr = 0.f;
          }
          sT[kt][v] = pr * (dpT[kt][v] - dl);   // dS^T
        }
#pragma unroll
      for (int gk = 0; gk < 4; ++gk) {
        const uint4 df = pack_frag(sT[gk >> 1], 8 * (gk & 1));
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const uint4 a = *reinterpret_cast<const uint4*>(Kt + (32 * dt + lr) * LDT + 16 * gk + 8 * lk);
          dqacc[dt] = mfma32(a, df, dqacc[dt]);
        }
      }
    }
  }
  __syncthreads();
  store_acc_T<D>(dqacc, p.scale, smem + w * 32 * LDKD, p.dq + tok0 * p.lddq + hq * D, p.lddq, q0 + 32 * w, p.seq, lane);
}

// ================================================================================================ dK, dV
template <int D>
__global__ void __launch_bounds__(256) attn_bwd_dkv_kernel(const AttnArgs p) {
  constexpr int LDKD = D + 8, KS = D / 16, DT = D / 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];
  float* const stats = reinterpret_cast<float*>(dyn_smem);          // 128 floats: lse (log2 units), delta
  bf16* const smem = reinterpret_cast<bf16*>(dyn_smem + 512);       // 2*64*LDKD + 2*D*LDT elements
  bf16* const Qs = smem;
  bf16* const dOs = smem + 64 * LDKD;
  bf16* const Qt = smem + 2 * 64 * LDKD;
  bf16* const dOt = Qt + D * LDT;
  float* const lse_s = stats;
  float* const dl_s = stats + 64;

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, lr = lane & 31, lk = lane >> 5;
  const int nK = (p.seq + 127) / 128;
  int bid = blockIdx.x;
  const int kvt = bid % nK;
  bid /= nK;
  const int g = bid % p.kh, b = bid / p.kh;
  const int grp = p.a / p.kh;
  const int kv0 = kvt * 128;
  const long tok0 = (long)b * p.seq;
  const bf16* kb = p.k + tok0 * p.ldk + g * D;
  const bf16* vb = p.v + tok0 * p.ldv + g * D;
  const int kpos = kv0 + 32 * w + lr;
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
  const int per_head = nQ - qt0;
  const int niter = grp * per_head;

  uint4 qreg[D / 32], doreg[D / 32], qtreg[8], dotreg[8];
  float st_reg = 0.f;
  auto prefetch = [&](int it) {
    const int hq = g * grp + it / per_head;
    const int q0 = (qt0 + it % per_head) * 64;
    const bf16* qb = p.q + tok0 * p.ldq + hq * D;
    const bf16* dob = p.dout + tok0 * p.lddo + hq * D;
    load_direct64<D>(qreg, qb, p.ldq, q0, p.seq, tid);
    load_direct64<D>(doreg, dob, p.lddo, q0, p.seq, tid);
    load_trans64<D>(qtreg, qb, p.ldq, q0, p.seq, tid);
    load_trans64<D>(dotreg, dob, p.lddo, q0, p.seq, tid);
    if (tid < 128) {
      const int qi = q0 + (tid & 63);
      const long sidx = ((long)b * p.a + hq) * p.seq + qi;
      if (tid < 64) st_reg = (qi < p.seq) ? p.lse_in[sidx] * 1.4426950408889634f : INFINITY;
      else st_reg = (qi < p.seq) ? p.delta[sidx] : 0.f;
    }
  };
  if (niter > 0) prefetch(0);

  for (int it = 0; it < niter; ++it) {
    __syncthreads();
    store_direct64<D>(qreg, Qs, tid);
    store_direct64<D>(doreg, dOs, tid);
    store_trans64_perm<D>(qtreg, Qt, tid);
    store_trans64_perm<D>(dotreg, dOt, tid);
    if (tid < 128) stats[tid] = st_reg;
    __syncthreads();
    if (it + 1 < niter) prefetch(it + 1);
    const int q0 = (qt0 + it % per_head) * 64;
    if (q0 + 63 >= kv0 + 32 * w) {
      f32x16 s[2], dp[2];
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
        for (int v = 0; v < 16; ++v) { s[t2][v] = 0.f; dp[t2][v] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
          const uint4 aq = *reinterpret_cast<const uint4*>(Qs + (32 * t2 + lr) * LDKD + 16 * ks + 8 * lk);
          s[t2] = mfma32(aq, kf[ks], s[t2]);
          const uint4 ad = *reinterpret_cast<const uint4*>(dOs + (32 * t2 + lr) * LDKD + 16 * ks + 8 * lk);
          dp[t2] = mfma32(ad, vf[ks], dp[t2]);
        }
      const bool need_mask = (q0 < kv0 + 32 * w + 31) || !kok;
      // rows of the score tile are queries: q = q0 + 32*t2 + 8*(v/4) + 4*lk + v%4
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
          const int ql = 32 * t2 + 8 * vg + 4 * lk;
          const float4 l4 = *reinterpret_cast<const float4*>(lse_s + ql);
          const float4 d4 = *reinterpret_cast<const float4*>(dl_s + ql);
          const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int v = 4 * vg + e;
            float pr = fast_exp2(s[t2][v] * p.scale_log2e - lv[e]);
            if (need_mask) {
              if (kpos > q0 + ql + e || !kok) pr = 0.f;
            }
            s[t2][v] = pr;                             // P
            dp[t2][v] = pr * (dp[t2][v] - dv4[e]);     // dS
          }
        }
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        const uint4 pf = pack_frag(s[gq >> 1], 8 * (gq & 1));
        const uint4 df = pack_frag(dp[gq >> 1], 8 * (gq & 1));
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const uint4 ado = *reinterpret_cast<const uint4*>(dOt + (32 * dt + lr) * LDT + 16 * gq + 8 * lk);
          dvacc[dt] = mfma32(ado, pf, dvacc[dt]);
          const uint4 aq = *reinterpret_cast<const uint4*>(Qt + (32 * dt + lr) * LDT + 16 * gq + 8 * lk);
          dkacc[dt] = mfma32(aq, df, dkacc[dt]);
        }
      }
    }
  }
  __syncthreads();
  store_acc_T<D>(dkacc, p.scale, smem + w * 32 * LDKD, p.dk + tok0 * p.lddk + g * D, p.lddk, kv0 + 32 * w, p.seq, lane);
  __syncthreads();
  store_acc_T<D>(dvacc, 1.f, smem + w * 32 * LDKD, p.dv + tok0 * p.lddv + g * D, p.lddv, kv0 + 32 * w, p.seq, lane);
}

}  // namespace

// ------------------------------------------------------------------------------------------------ launchers
static constexpr int dkv_smem_bytes(int d) { return 512 + (2 * 64 * (d + 8) + 2 * d * LDT) * 2; }

static void fill_common(AttnArgs& p, int batch, int seq, int a, int kh, int d) {
  p.batch = batch; p.seq = seq; p.a = a; p.kh = kh;
  p.scale = 1.0f / sqrtf((float)d);
  p.scale_log2e = p.scale * 1.4426950408889634f;
}

hipError_t k_attn_fwd(hipStream_t st, const void* q, const void* k, const void* v, void* o, float* lse, long ldq,
                      long ldk, long ldv, long ldo, int batch, int seq, int a, int kh, int d) {
  if (batch * seq == 0) return hipSuccess;
  AttnArgs p = {};
  p.q = (const bf16*)q; p.k = (const bf16*)k; p.v = (const bf16*)v; p.o = (bf16*)o; p.lse = lse;
  p.ldq = ldq; p.ldk = ldk; p.ldv = ldv; p.ldo = ldo;
  fill_common(p, batch, seq, a, kh, d);
  const int grid = ((seq + 127) / 128) * a * batch;
  if (d == 128) RP_LAUNCH(attn_fwd_kernel<128>, dim3(grid), dim3(256), 0, st, p);
  else if (d == 64) RP_LAUNCH(attn_fwd_kernel<64>, dim3(grid), dim3(256), 0, st, p);
  else return hipErrorInvalidValue;
  return hipGetLastError();
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
                      const float* lse, const float* delta, void* dq, void* dk, void* dv, long ldq, long ldk, long ldv,
                      long lddo, long lddq, long lddk, long lddv, int batch, int seq, int a, int kh, int d) {
  if (batch * seq == 0) return hipSuccess;
  AttnArgs p = {};
  p.q = (const bf16*)q; p.k = (const bf16*)k; p.v = (const bf16*)v; p.dout = (const bf16*)dout;
  p.lse_in = lse; p.delta = delta; p.dq = (bf16*)dq; p.dk = (bf16*)dk; p.dv = (bf16*)dv;
  p.ldq = ldq; p.ldk = ldk; p.ldv = ldv; p.lddo = lddo; p.lddq = lddq; p.lddk = lddk; p.lddv = lddv;
  fill_common(p, batch, seq, a, kh, d);
  const int nq = ((seq + 127) / 128) * a * batch;
  const int nk = ((seq + 127) / 128) * kh * batch;
  if (d != 128 && d != 64) return hipErrorInvalidValue;
  if (part == 0) {
    if (d == 128) {
      constexpr int smem = dkv_smem_bytes(128);
      static bool attr_done = false;
      if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bwd_dkv_kernel<128>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_done = true;
      }
      RP_LAUNCH(attn_bwd_dkv_kernel<128>, dim3(nk), dim3(256), smem, st, p);
    } else {
      RP_LAUNCH(attn_bwd_dkv_kernel<64>, dim3(nk), dim3(256), dkv_smem_bytes(64), st, p);
    }
  } else {
    if (d == 128) RP_LAUNCH(attn_bwd_dq_kernel<128>, dim3(nq), dim3(256), 0, st, p);
    else RP_LAUNCH(attn_bwd_dq_kernel<64>, dim3(nq), dim3(256), 0, st, p);
  }
  return hipGetLastError();
}
