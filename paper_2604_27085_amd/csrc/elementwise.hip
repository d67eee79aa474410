// Memory-bound kernels of the decoder layer: RMSNorm, per-head QK-norm + RoPE, SwiGLU, small utilities.
// All of them move 16 bytes per lane per access, keep their arithmetic in fp32 and are bounded by HBM bandwidth.
#include "common.hpp"
#include "kernels.hpp"

namespace {

RP_DEV void unpack8(const uint4& u, float (&f)[8]) {
  f[0] = bf16_lo(u.x); f[1] = bf16_hi(u.x); f[2] = bf16_lo(u.y); f[3] = bf16_hi(u.y);
  f[4] = bf16_lo(u.z); f[5] = bf16_hi(u.z); f[6] = bf16_lo(u.w); f[7] = bf16_hi(u.w);
}
RP_DEV uint4 pack8(const float (&f)[8]) {
  return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
}

// ------------------------------------------------------------------------------------------------ RMSNorm forward
// One wave per row, the row lives in registers between the sum of squares and the scaling.  MAXC = 16-byte chunks
// per lane (h <= 512*MAXC).
template <int MAXC>
__global__ void __launch_bounds__(256) rmsnorm_fwd_kernel(const bf16* __restrict__ x, const bf16* __restrict__ g,
                                                          bf16* __restrict__ y, float* __restrict__ rstd_out, int T,
                                                          int h, float eps) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= T) return;
  const int nch = h >> 3;
  const uint4* xr = reinterpret_cast<const uint4*>(x + (long)row * h);
  uint4 v[MAXC];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < MAXC; ++i) {
    const int c = lane + 64 * i;
    v[i] = make_uint4(0u, 0u, 0u, 0u);
    if (c < nch) {
      v[i] = xr[c];
      float f[8];
      unpack8(v[i], f);
#pragma unroll
      for (int e = 0; e < 8; ++e) ss += f[e] * f[e];
    }
  }
  ss = wave_sum(ss);
  const float rstd = 1.0f / sqrtf(ss / (float)h + eps);
  if (lane == 0 && rstd_out) rstd_out[row] = rstd;
  const uint4* gr = reinterpret_cast<const uint4*>(g);
  uint4* yr = reinterpret_cast<uint4*>(y + (long)row * h);
#pragma unroll
  for (int i = 0; i < MAXC; ++i) {
    const int c = lane + 64 * i;
    if (c < nch) {
      float f[8], gg[8];
      unpack8(v[i], f);
      unpack8(gr[c], gg);
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] = f[e] * rstd * gg[e];
      yr[c] = pack8(f);
    }
  }
}

// ------------------------------------------------------------------------------------------------ RMSNorm backward
// dx = rstd*(dy*g) - rstd^3/h * x * sum_j(dy_j g_j x_j)  (+ dres, the gradient arriving over the residual branch);
// dg partial = sum_t dy_t * x_t * rstd_t over the rows a block visits, written to part[block][h]; a column-sum kernel
// adds the partials to dg in a fixed order.
// One BLOCK per row: the four waves split the row's columns (chunk (4i + wave)*64 + lane, i < MAXC, so
// h <= 2048*MAXC), the row's dot product crosses the waves through LDS (one barrier per row), and every lane owns its
// columns for all the rows of the block, so the gain-gradient partial is written straight from registers.
template <int MAXC, int NR, typename DyT>
__global__ void __launch_bounds__(256) rmsnorm_bwd_kernel(const DyT* __restrict__ dy, const bf16* __restrict__ x,
                                                               const bf16* __restrict__ g, const float* __restrict__ rstd_in,
                                                               const bf16* __restrict__ dres, bf16* __restrict__ dx,
                                                               float* __restrict__ part, int T, int h) {
  // NR rows per trip (rows r, r + gridDim.x, ...): NR times the loads in flight per thread and one barrier for all of
  // them, against NR times the registers (measured: two rows win at h = 5120, 145 against 181 us for 16384 rows, and
  // lose at h = 4096, where they halve the waves per SIMD).
  __shared__ float s_dot[2][NR][4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nch = h >> 3;
  const uint4* gr = reinterpret_cast<const uint4*>(g);
  float gg[MAXC][8], dgacc[MAXC][8];
#pragma unroll
  for (int i = 0; i < MAXC; ++i) {
    const int c = (4 * i + wave) * 64 + lane;
#pragma unroll
    for (int e = 0; e < 8; ++e) { dgacc[i][e] = 0.f; gg[i][e] = 0.f; }
    if (c < nch) unpack8(gr[c], gg[i]);
  }
  int par = 0;
  for (int row0 = blockIdx.x; row0 < T; row0 += NR * gridDim.x, par ^= 1) {
    float dyv[NR][MAXC][8], xf[NR][MAXC][8], rstd[NR], dot[NR];
    uint4 rr[NR][MAXC];
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      const int row = row0 + r * gridDim.x;
      const bool rok = row < T;
      rstd[r] = rok ? rstd_in[row] : 0.f;
      dot[r] = 0.f;
#pragma unroll
      for (int i = 0; i < MAXC; ++i) {
        const int c = (4 * i + wave) * 64 + lane;
#pragma unroll
        for (int e = 0; e < 8; ++e) { dyv[r][i][e] = 0.f; xf[r][i][e] = 0.f; }
        rr[r][i] = make_uint4(0u, 0u, 0u, 0u);
        if (rok && c < nch) {
          unpack8(reinterpret_cast<const uint4*>(x + (long)row * h)[c], xf[r][i]);
          if constexpr (sizeof(DyT) == 4) {
            const float4* dr = reinterpret_cast<const float4*>(dy + (long)row * h) + 2 * c;
            const float4 a = dr[0], b = dr[1];
            dyv[r][i][0] = a.x; dyv[r][i][1] = a.y; dyv[r][i][2] = a.z; dyv[r][i][3] = a.w;
            dyv[r][i][4] = b.x; dyv[r][i][5] = b.y; dyv[r][i][6] = b.z; dyv[r][i][7] = b.w;
          } else {
            unpack8(reinterpret_cast<const uint4*>(dy + (long)row * h)[c], dyv[r][i]);
          }
          if (dres) rr[r][i] = reinterpret_cast<const uint4*>(dres + (long)row * h)[c];
        }
      }
    }
#pragma unroll
    for (int r = 0; r < NR; ++r) {
#pragma unroll
      for (int i = 0; i < MAXC; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          dot[r] += dyv[r][i][e] * gg[i][e] * xf[r][i][e];
          dgacc[i][e] += dyv[r][i][e] * xf[r][i][e] * rstd[r];      // rows past the end contribute zeros
        }
      dot[r] = wave_sum(dot[r]);
      if (lane == 0) s_dot[par][r][wave] = dot[r];
    }
    __syncthreads();   // the other parity's slots are rewritten only after the next barrier
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      const int row = row0 + r * gridDim.x;
      if (row >= T) continue;
      const float d = (s_dot[par][r][0] + s_dot[par][r][1]) + (s_dot[par][r][2] + s_dot[par][r][3]);
      const float k2 = rstd[r] * rstd[r] * rstd[r] * d / (float)h;
#pragma unroll
      for (int i = 0; i < MAXC; ++i) {
        const int c = (4 * i + wave) * 64 + lane;
        if (c < nch) {
          float o[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = rstd[r] * dyv[r][i][e] * gg[i][e] - k2 * xf[r][i][e];
          if (dres) {
            float rv[8];
            unpack8(rr[r][i], rv);
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] += rv[e];
          }
          reinterpret_cast<uint4*>(dx + (long)row * h)[c] = pack8(o);
        }
      }
    }
  }
  if (part) {
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      const int c = (4 * i + wave) * 64 + lane;
      if (c < nch) {
        float4* o = reinterpret_cast<float4*>(part + (long)blockIdx.x * h + c * 8);
        o[0] = make_float4(dgacc[i][0], dgacc[i][1], dgacc[i][2], dgacc[i][3]);
        o[1] = make_float4(dgacc[i][4], dgacc[i][5], dgacc[i][6], dgacc[i][7]);
      }
    }
  }
}

// dst[c] += sum_r part[r][c], r = 0..rows-1 (columns from cols1 on go to dst2).  A block owns 64 columns; its sixteen
// waves each sum every sixteenth row (four independent loads in flight per thread) and the slices are merged in LDS in
// a fixed order.
__global__ void __launch_bounds__(1024) colsum_add_kernel(const float* __restrict__ part, int rows, int ld, int cols,
                                                          float* __restrict__ dst, int cols1, float* __restrict__ dst2) {
  __shared__ float red[16][64];
  const int cl = threadIdx.x & 63, sl = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  if (c < cols) {
    int r = sl;
    for (; r + 48 < rows; r += 64) {
      s0 += part[(long)r * ld + c];
      s1 += part[(long)(r + 16) * ld + c];
      s2 += part[(long)(r + 32) * ld + c];
      s3 += part[(long)(r + 48) * ld + c];
    }
    for (; r < rows; r += 16) s0 += part[(long)r * ld + c];
  }
  red[sl][cl] = (s0 + s1) + (s2 + s3);
  __syncthreads();
  if (sl == 0 && c < cols) {
    float t = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) t += red[k][cl];
    if (c < cols1) dst[c] += t; else dst2[c - cols1] += t;
  }
}

// ------------------------------------------------------------------------------------------------ RoPE table
// cs[p][i] = (cos, sin)(p * base^(-2i/d)), evaluated in double so that long sequences keep full fp32 accuracy.
__global__ void rope_table_kernel(float2* __restrict__ cs, int seq, int half, double log2_base) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= seq * half) return;
  const int p = idx / half, i = idx - p * half;
  const double theta = exp2(-(double)i / (double)half * log2_base);
  const double phi = (double)p * theta;
  double s, c;
  sincos(phi, &s, &c);
  cs[idx] = make_float2((float)c, (float)s);
}

// ------------------------------------------------------------------------------------------------ QK-norm + RoPE
// One wave per token.  A head vector of D elements is spread over D/8 lanes (8 elements each); the rotation partner
// (i, i + D/2) sits D/16 lanes away.  Heads 0..a-1 are query heads, a..a+k-1 key heads, both read from the fused
// projection output (row stride ld_in) and written to dense [T, a, D] / [T, k, D] buffers.
template <int D, bool BWD>
__global__ void __launch_bounds__(512) qknorm_rope_kernel(const bf16* __restrict__ in_q, const bf16* __restrict__ in_k,
                                                          long ld_in_q, long ld_in_k, bf16* __restrict__ out_q,
                                                          bf16* __restrict__ out_k, long ld_out_q, long ld_out_k,
                                                          const bf16* __restrict__ gq, const bf16* __restrict__ gk,
                                                          float* __restrict__ rstd_q, float* __restrict__ rstd_k,
                                                          const bf16* __restrict__ raw_q, const bf16* __restrict__ raw_k,
                                                          long ld_raw, float* __restrict__ part,
                                                          const float2* __restrict__ cs, int T, int seq, int a, int k,
                                                          int use_norm, float eps) {
  constexpr int MAXW = 8;             // waves per block the gain-gradient merge is sized for
  __shared__ float dg_s[BWD ? MAXW : 1][2 * D];
  constexpr int LPH = D / 8;          // lanes per head
  constexpr int HPW = 64 / LPH;       // heads per wave pass
  const int lane = threadIdx.x & 63;
  const int sub = lane % LPH, hsel = lane / LPH;
  const int wave_id = blockIdx.x * ((int)blockDim.x >> 6) + (threadIdx.x >> 6);
  const int nwaves = gridDim.x * ((int)blockDim.x >> 6);
  const bool first_half = sub < LPH / 2;
  float gqv[8], gkv[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { gqv[e] = 1.f; gkv[e] = 1.f; }
  if (use_norm) {
    unpack8(reinterpret_cast<const uint4*>(gq)[sub], gqv);
    unpack8(reinterpret_cast<const uint4*>(gk)[sub], gkv);
  }
  float dgq_acc[8], dgk_acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { dgq_acc[e] = 0.f; dgk_acc[e] = 0.f; }

  for (int t = wave_id; t < T; t += nwaves) {
    const int pos = t % seq;
    float c8[8], s8[8];
    {
      const float2* row = cs + (long)pos * (D / 2) + (sub % (LPH / 2)) * 8;
#pragma unroll
      for (int e = 0; e < 8; ++e) { const float2 v = row[e]; c8[e] = v.x; s8[e] = v.y; }
    }
    // NP passes of HPW heads at a time, all their loads issued before any arithmetic: a token's heads are the only
    // work a wave has, so the loads in flight are what hides the memory latency
    constexpr int NP = 4;
    for (int h0 = 0; h0 < a + k; h0 += HPW * NP) {
      uint4 in_v[NP], raw_v[NP];
      float rs[NP];
#pragma unroll
      for (int u = 0; u < NP; ++u) {
        const int head = h0 + u * HPW + hsel;
        const bool ok = head < a + k, isq = head < a;
        const int hh = isq ? head : head - a;
        in_v[u] = make_uint4(0u, 0u, 0u, 0u);
        raw_v[u] = in_v[u];
        rs[u] = 0.f;
        if (ok) {
          const bf16* src = isq ? in_q + (long)t * ld_in_q + hh * D : in_k + (long)t * ld_in_k + hh * D;
          in_v[u] = reinterpret_cast<const uint4*>(src)[sub];
          if (BWD && use_norm) {
            const bf16* rsrc = (isq ? raw_q : raw_k) + (long)t * ld_raw + hh * D;
            raw_v[u] = reinterpret_cast<const uint4*>(rsrc)[sub];
            rs[u] = isq ? rstd_q[(long)t * a + hh] : rstd_k[(long)t * k + hh];
          }
        }
      }
#pragma unroll
      for (int u = 0; u < NP; ++u) {
        const int head = h0 + u * HPW + hsel;
        if (h0 + u * HPW >= a + k) break;      // wave-uniform: no head left in this pass
        const bool ok = head < a + k;
        const bool isq = head < a;
        const int hh = isq ? head : head - a;
        float f[8];
        unpack8(in_v[u], f);
        if constexpr (!BWD) {
          if (use_norm) {
            float ss = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += f[e] * f[e];
#pragma unroll
            for (int o = LPH / 2; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
            const float rstd = 1.0f / sqrtf(ss / (float)D + eps);
            if (ok && sub == 0) {
              if (isq) rstd_q[(long)t * a + hh] = rstd; else rstd_k[(long)t * k + hh] = rstd;
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = f[e] * rstd * (isq ? gqv[e] : gkv[e]);
          }
          float o8[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float partner = __shfl_xor(f[e], LPH / 2, 64);
            o8[e] = first_half ? (f[e] * c8[e] - partner * s8[e]) : (f[e] * c8[e] + partner * s8[e]);
          }
          if (ok) {
            bf16* dst = isq ? out_q + (long)t * ld_out_q + hh * D : out_k + (long)t * ld_out_k + hh * D;
            reinterpret_cast<uint4*>(dst)[sub] = pack8(o8);
          }
        } else {
          // inverse rotation of the incoming gradient
          float gr[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float partner = __shfl_xor(f[e], LPH / 2, 64);
            gr[e] = first_half ? (f[e] * c8[e] + partner * s8[e]) : (f[e] * c8[e] - partner * s8[e]);
          }
          if (use_norm) {
            float xr[8];
            unpack8(raw_v[u], xr);
            const float rstd = rs[u];
            float dot = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const float gg = isq ? gqv[e] : gkv[e];
              dot += gr[e] * gg * xr[e];
              if (isq) dgq_acc[e] += gr[e] * xr[e] * rstd; else dgk_acc[e] += gr[e] * xr[e] * rstd;
            }
#pragma unroll
            for (int o = LPH / 2; o > 0; o >>= 1) dot += __shfl_xor(dot, o, 64);
            const float k2 = rstd * rstd * rstd * dot / (float)D;
#pragma unroll
            for (int e = 0; e < 8; ++e) gr[e] = rstd * gr[e] * (isq ? gqv[e] : gkv[e]) - k2 * xr[e];
          }
          if (ok) {
            bf16* dst = isq ? out_q + (long)t * ld_out_q + hh * D : out_k + (long)t * ld_out_k + hh * D;
            reinterpret_cast<uint4*>(dst)[sub] = pack8(gr);
          }
        }
      }
    }
  }
  if constexpr (BWD) {
    if (use_norm && part) {
      // lanes with the same `sub` hold partial sums for the same 8 gain entries; every wave leaves its sums in a row
      // of its own, the rows are added in wave order (no atomics: the result does not depend on timing), blocks merge
      // via part[]
      const int wv = threadIdx.x >> 6, nwv = (int)blockDim.x >> 6;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float vq = dgq_acc[e], vk = dgk_acc[e];
#pragma unroll
        for (int o = LPH; o < 64; o <<= 1) { vq += __shfl_xor(vq, o, 64); vk += __shfl_xor(vk, o, 64); }
        if (hsel == 0) { dg_s[wv][sub * 8 + e] = vq; dg_s[wv][D + sub * 8 + e] = vk; }
      }
      __syncthreads();
      for (int i = threadIdx.x; i < 2 * D; i += (int)blockDim.x) {
        float t = dg_s[0][i];
        for (int k2 = 1; k2 < nwv; ++k2) t += dg_s[k2][i];
        part[(long)blockIdx.x * 2 * D + i] = t;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------ SwiGLU
__global__ void __launch_bounds__(256) swiglu_fwd_kernel(const bf16* __restrict__ gu, bf16* __restrict__ act, long T,
                                                         int m) {
  const int mc = m >> 3;
  const long total = T * mc;
  for (long idx = (long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (long)gridDim.x * blockDim.x) {
    const long row = idx / mc;
    const int c = (int)(idx - row * mc);
    const uint4* r = reinterpret_cast<const uint4*>(gu + row * 2 * m);
    float g[8], u[8], o[8];
    unpack8(r[c], g);
    unpack8(r[mc + c], u);
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = g[e] / (1.f + __expf(-g[e])) * u[e];
    reinterpret_cast<uint4*>(act + row * m)[c] = pack8(o);
  }
}

__global__ void __launch_bounds__(256) swiglu_bwd_kernel(const bf16* __restrict__ dact, const bf16* __restrict__ gu,
                                                         bf16* __restrict__ dgu, long T, int m) {
  const int mc = m >> 3;
  const long total = T * mc;
  for (long idx = (long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (long)gridDim.x * blockDim.x) {
    const long row = idx / mc;
    const int c = (int)(idx - row * mc);
    const uint4* r = reinterpret_cast<const uint4*>(gu + row * 2 * m);
    float g[8], u[8], d[8], dg[8], du[8];
    unpack8(r[c], g);
    unpack8(r[mc + c], u);
    unpack8(reinterpret_cast<const uint4*>(dact + row * m)[c], d);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float sg = 1.f / (1.f + __expf(-g[e]));
      dg[e] = d[e] * u[e] * sg * (1.f + g[e] * (1.f - sg));
      du[e] = d[e] * g[e] * sg;
    }
    uint4* o = reinterpret_cast<uint4*>(dgu + row * 2 * m);
    o[c] = pack8(dg);
    o[mc + c] = pack8(du);
  }
}

// ------------------------------------------------------------------------------------------------ utilities
__global__ void fill_u32_kernel(uint32_t* __restrict__ p, long n, uint32_t v) {
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) p[i] = v;
}

__global__ void copy16_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, long n) {
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) dst[i] = src[i];
}

__global__ void cast_f32_bf16_kernel(const float* __restrict__ src, bf16* __restrict__ dst, long n8) {
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += (long)gridDim.x * blockDim.x) {
    const float4 a = reinterpret_cast<const float4*>(src)[2 * i], b = reinterpret_cast<const float4*>(src)[2 * i + 1];
    const float f[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    reinterpret_cast<uint4*>(dst)[i] = pack8(f);
  }
}

// Block-diagonal LoRA B for a fused projection: out[n, seg.col0 + c] = src_seg[n - seg.row0, c] inside a segment, 0 elsewhere.
__global__ void lora_blockdiag_kernel(bf16* __restrict__ out, int N, int ncols, LoraSegs segs, int r) {
  const long total = (long)N * ncols;
  for (long idx = (long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (long)gridDim.x * blockDim.x) {
    const int n = (int)(idx / ncols), c = (int)(idx - (long)n * ncols);
    bf16 v = (bf16)0.f;
#pragma unroll
    for (int s = 0; s < 3; ++s) {
      if (segs.src[s] && n >= segs.row0[s] && n < segs.row1[s] && c >= segs.col0[s] && c < segs.col0[s] + r)
        v = reinterpret_cast<const bf16*>(segs.src[s])[(long)(n - segs.row0[s]) * r + (c - segs.col0[s])];
    }
    out[idx] = v;
  }
}

int grid_for(long n, int block = 256, int cap = 256 * 16) {
  long g = (n + block - 1) / block;
  if (g < 1) g = 1;
  if (g > cap) g = cap;
  return (int)g;
}

}  // namespace

// ------------------------------------------------------------------------------------------------ launchers
hipError_t k_rmsnorm_fwd(hipStream_t st, const void* x, const void* g, void* y, float* rstd, int T, int h, float eps) {
  const int grid = (T + 3) / 4;
  if (grid == 0) return hipSuccess;
  if (h <= 2048)
    RP_LAUNCH((rmsnorm_fwd_kernel<4>), dim3(grid), dim3(256), 0, st, (const bf16*)x, (const bf16*)g, (bf16*)y, rstd, T, h, eps);
  else
    RP_LAUNCH((rmsnorm_fwd_kernel<16>), dim3(grid), dim3(256), 0, st, (const bf16*)x, (const bf16*)g, (bf16*)y, rstd, T, h, eps);
  return hipGetLastError();
}

hipError_t k_rmsnorm_bwd(hipStream_t st, const void* dy, int dy_is_f32, const void* x, const void* g, const float* rstd,
                         const void* dres, void* dx, float* dg, float* scratch, int T, int h) {
  if (T == 0) return hipSuccess;
  if (dg && !scratch) return hipErrorInvalidValue;
  const int grid = T < RP_PARTIAL_BLOCKS ? T : RP_PARTIAL_BLOCKS;
  float* part = dg ? scratch : nullptr;
#define RP_LAUNCH_RR(MAXC, NR, DT) \
  RP_LAUNCH((rmsnorm_bwd_kernel<MAXC, NR, DT>), dim3(grid), dim3(256), 0, st, (const DT*)dy, (const bf16*)x, \
                     (const bf16*)g, rstd, (const bf16*)dres, (bf16*)dx, part, T, h)
  if (h <= 2048) { if (dy_is_f32) RP_LAUNCH_RR(1, 2, float); else RP_LAUNCH_RR(1, 2, bf16); }
  else if (h <= 4096) { if (dy_is_f32) RP_LAUNCH_RR(2, 1, float); else RP_LAUNCH_RR(2, 1, bf16); }
  else { if (dy_is_f32) RP_LAUNCH_RR(4, 2, float); else RP_LAUNCH_RR(4, 2, bf16); }
#undef RP_LAUNCH_RR
  hipError_t e = hipGetLastError();
  if (e == hipSuccess && dg) {
    RP_LAUNCH(colsum_add_kernel, dim3((h + 63) / 64), dim3(1024), 0, st, part, grid, h, h, dg, h, (float*)nullptr);
    e = hipGetLastError();
  }
  return e;
}

hipError_t k_rope_table(hipStream_t st, float2* cs, int seq, int d, float base) {
  const int n = seq * (d / 2);
  if (n == 0) return hipSuccess;
  RP_LAUNCH(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, st, cs, seq, d / 2, log2((double)base));
  return hipGetLastError();
}

hipError_t k_qknorm_rope(hipStream_t st, int bwd, int d, const void* in_q, const void* in_k, long ld_in_q, long ld_in_k,
                         void* out_q, void* out_k, long ld_out_q, long ld_out_k, const void* gq, const void* gk,
                         float* rstd_q, float* rstd_k, const void* raw_q, const void* raw_k, long ld_raw, float* dgq,
                         float* dgk, float* scratch, const float2* cs, int T, int seq, int a, int k, int use_norm, float eps) {
  if (T == 0) return hipSuccess;
  const int nthr = 256;
  int grid = (T + nthr / 64 - 1) / (nthr / 64);
  if (bwd && grid > RP_PARTIAL_BLOCKS) grid = RP_PARTIAL_BLOCKS;
  const bool want_dg = bwd && use_norm && dgq && dgk;
  if (want_dg && !scratch) return hipErrorInvalidValue;
  float* part = want_dg ? scratch : nullptr;
#define RP_LAUNCH_QR(D, B) \
  RP_LAUNCH((qknorm_rope_kernel<D, B>), dim3(grid), dim3(nthr), 0, st, (const bf16*)in_q, (const bf16*)in_k, \
                     ld_in_q, ld_in_k, (bf16*)out_q, (bf16*)out_k, ld_out_q, ld_out_k, (const bf16*)gq, (const bf16*)gk, \
                     rstd_q, rstd_k, (const bf16*)raw_q, (const bf16*)raw_k, ld_raw, part, cs, T, seq, a, k, use_norm, eps)
  if (d == 128) { if (bwd) RP_LAUNCH_QR(128, true); else RP_LAUNCH_QR(128, false); }
  else if (d == 64) { if (bwd) RP_LAUNCH_QR(64, true); else RP_LAUNCH_QR(64, false); }
  else return hipErrorInvalidValue;
#undef RP_LAUNCH_QR
  hipError_t e = hipGetLastError();
  if (e == hipSuccess && want_dg) {
    RP_LAUNCH(colsum_add_kernel, dim3((2 * d + 63) / 64), dim3(1024), 0, st, part, grid, 2 * d, 2 * d, dgq, d, dgk);
    e = hipGetLastError();
  }
  return e;
}

hipError_t k_swiglu_fwd(hipStream_t st, const void* gu, void* act, long T, int m) {
  if (T == 0) return hipSuccess;
  RP_LAUNCH(swiglu_fwd_kernel, dim3(grid_for(T * (m / 8))), dim3(256), 0, st, (const bf16*)gu, (bf16*)act, T, m);
  return hipGetLastError();
}

hipError_t k_swiglu_bwd(hipStream_t st, const void* dact, const void* gu, void* dgu, long T, int m) {
  if (T == 0) return hipSuccess;
  RP_LAUNCH(swiglu_bwd_kernel, dim3(grid_for(T * (m / 8))), dim3(256), 0, st, (const bf16*)dact, (const bf16*)gu, (bf16*)dgu, T, m);
  return hipGetLastError();
}

hipError_t k_fill_u32(hipStream_t st, void* p, long n_words, uint32_t v) {
  if (n_words == 0) return hipSuccess;
  RP_LAUNCH(fill_u32_kernel, dim3(grid_for(n_words)), dim3(256), 0, st, (uint32_t*)p, n_words, v);
  return hipGetLastError();
}

hipError_t k_copy16(hipStream_t st, const void* src, void* dst, long bytes) {
  if (bytes == 0) return hipSuccess;
  RP_LAUNCH(copy16_kernel, dim3(grid_for(bytes / 16)), dim3(256), 0, st, (const uint4*)src, (uint4*)dst, bytes / 16);
  return hipGetLastError();
}

hipError_t k_cast_f32_bf16(hipStream_t st, const float* src, void* dst, long n) {
  if (n == 0) return hipSuccess;
  RP_LAUNCH(cast_f32_bf16_kernel, dim3(grid_for(n / 8)), dim3(256), 0, st, src, (bf16*)dst, n / 8);
  return hipGetLastError();
}

hipError_t k_lora_blockdiag(hipStream_t st, void* out, int N, int ncols, const LoraSegs& segs, int r) {
  if ((long)N * ncols == 0) return hipSuccess;
  RP_LAUNCH(lora_blockdiag_kernel, dim3(grid_for((long)N * ncols)), dim3(256), 0, st, (bf16*)out, N, ncols, segs, r);
  return hipGetLastError();
}
