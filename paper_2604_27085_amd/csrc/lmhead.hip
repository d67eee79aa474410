// Cross-entropy bookkeeping around the LM-head GEMMs: the logits are reduced inside the GEMM epilogue to per-token
// (max, sum exp) partials, one per 128 vocabulary rows; these kernels merge the partials and produce the loss and the
// per-token gradient coefficient.
#include "common.hpp"
#include "kernels.hpp"
#include "gemm.hpp"

namespace {

// lse[t] = log sum_v exp(z[t, v]) from P partial (max, sum) pairs per token; part is [P][ld] so reads are coalesced
// over tokens.  A block handles 16 tokens with 64 slices of the partials each (a thread's chain of dependent
// exponentials is P/64 long), merged through LDS in two steps.
__global__ void __launch_bounds__(1024) ce_lse_kernel(const float2* __restrict__ part, int P, long ld, float* __restrict__ lse, int T) {
  constexpr int NS = 64;
  __shared__ float2 red[NS][17];
  const int tl = threadIdx.x & 15, sl = threadIdx.x >> 4;
  const int t = blockIdx.x * 16 + tl;
  float m = -INFINITY, s = 0.f;
  auto merge = [&](const float2 v) {
    if (v.x > -INFINITY) {
      const float mn = fmaxf(m, v.x);
      s = s * __expf(m - mn) + v.y * __expf(v.x - mn);
      m = mn;
    }
  };
  if (t < T)
    for (int i = sl; i < P; i += NS) merge(part[(long)i * ld + t]);
  red[sl][tl] = make_float2(m, s);
  __syncthreads();
  if (sl < 8) {   // slices sl, sl + 8, ..., in a fixed order
    for (int i = sl + 8; i < NS; i += 8) merge(red[i][tl]);
    red[sl][tl] = make_float2(m, s);
  }
  __syncthreads();
  if (sl == 0 && t < T) {
    for (int i = 1; i < 8; ++i) merge(red[i][tl]);
    lse[t] = m + logf(s);
  }
}

// One block: counts the valid tokens, loss = sum(lse - z_label) / n_valid, coef[t] = grad_scale / n_valid or 0.
__global__ void __launch_bounds__(1024) ce_finalize_kernel(const float* __restrict__ lse, const float* __restrict__ zlab,
                                                           const int* __restrict__ labels, float grad_scale,
                                                           float* __restrict__ coef, float* __restrict__ loss_out, int T) {
  __shared__ float red[16];
  __shared__ int redi[16];
  __shared__ float bc;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  int cnt = 0;
  float sum = 0.f;
  for (int t = tid; t < T; t += 1024) {
    if (labels[t] != -100) { ++cnt; sum += lse[t] - zlab[t]; }
  }
  sum = wave_sum(sum);
  float fc = wave_sum((float)cnt);
  if (lane == 0) { red[w] = sum; redi[w] = (int)(fc + 0.5f); }
  __syncthreads();
  if (tid == 0) {
    float s = 0.f;
    int n = 0;
    for (int i = 0; i < 16; ++i) { s += red[i]; n += redi[i]; }
    loss_out[0] = n > 0 ? s / (float)n : 0.f;
    bc = n > 0 ? grad_scale / (float)n : 0.f;
  }
  __syncthreads();
  const float c = bc;
  for (int t = tid; t < T; t += 1024) coef[t] = labels[t] != -100 ? c : 0.f;
}

// ---- frozen head: one sweep over the vocabulary (no dW, so the softmax normaliser is only needed at the end) ---------
// Per vocabulary chunk the logits Z^T [vc, T] (fp32) are turned into p = exp(z - m_t) against a per-token reference
// exponent m_t, and acc_t = sum_v p_tv W_v, l_t = sum_v p_tv are carried from chunk to chunk; when a chunk's maximum
// outgrows the reference by more than 2^8 (in e-units: 8), the reference moves and acc_t, l_t are rescaled.  At the end
// lse_t = m_t + log l_t and dx_t = coef_t (acc_t / l_t - W[y_t]).
//
// After the first chunk the logits GEMM writes p itself (EPI_CE_P) against the reference as it stands, together with the
// chunk's column maxima and sums; only when some token's maximum outgrows its reference by more than RP_CE_P_LIMIT does
// the chunk take the path above (a device flag switches those kernels on; they return at once otherwise).

constexpr int CE_PROB_ROWS = 128;

// Moves the reference exponent of every token if this chunk needs it and rescales l; alpha[t] is the factor acc_t must
// be multiplied with (1 for most tokens and chunks).
__global__ void __launch_bounds__(256) ce_chunk_ref_kernel(const float2* __restrict__ pmax, int nslab, int T, int first,
                                                           float* __restrict__ m, float* __restrict__ l,
                                                           float* __restrict__ alpha, const int* __restrict__ run_flag) {
  if (run_flag && *run_flag == 0) return;
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= T) return;
  float cm = -INFINITY;
  for (int i = 0; i < nslab; ++i) cm = fmaxf(cm, pmax[(long)i * T + t].x);
  if (first) { m[t] = cm; l[t] = 0.f; alpha[t] = 1.f; return; }
  const float mo = m[t];
  if (cm > mo + 8.f) {
    const float a = __expf(mo - cm);
    m[t] = cm; l[t] *= a; alpha[t] = a;
  } else {
    alpha[t] = 1.f;
  }
}

// p[r][t] = exp(z[r][t] - m[t]) as bf16; the fp32 sum over the block's CE_PROB_ROWS rows goes to the .y half of the
// block's row of the partial array (whose .x half holds the column maxima the logits GEMM left there, one row of
// partials per CE_PROB_ROWS vocabulary rows): no atomics, ce_chunk_sum_kernel adds the rows in order.
__global__ void __launch_bounds__(256) ce_chunk_prob_kernel(const float* __restrict__ z, int vc, int T,
                                                            const float* __restrict__ m, bf16* __restrict__ p,
                                                            float2* __restrict__ part, const int* __restrict__ run_flag) {
  if (run_flag && *run_flag == 0) return;
  const int t = (blockIdx.x * 256 + threadIdx.x) * 4;      // four tokens per thread: 16-byte loads, 8-byte stores
  if (t >= T) return;
  const int r0 = blockIdx.y * CE_PROB_ROWS, r1 = min(r0 + CE_PROB_ROWS, vc);
  const float4 mm = *reinterpret_cast<const float4*>(m + t);
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  auto one = [&](const float4& zz, int r) {
    const float p0 = __expf(zz.x - mm.x), p1 = __expf(zz.y - mm.y), p2 = __expf(zz.z - mm.z), p3 = __expf(zz.w - mm.w);
    s.x += p0; s.y += p1; s.z += p2; s.w += p3;
    *reinterpret_cast<uint2*>(p + (long)r * T + t) = make_uint2(pack_bf16x2(p0, p1), pack_bf16x2(p2, p3));
  };
  int r = r0;
  for (; r + 8 <= r1; r += 8) {          // eight rows in flight per thread
    float4 zz[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) zz[k] = *reinterpret_cast<const float4*>(z + (long)(r + k) * T + t);
#pragma unroll
    for (int k = 0; k < 8; ++k) one(zz[k], r + k);
  }
  for (; r < r1; ++r) one(*reinterpret_cast<const float4*>(z + (long)r * T + t), r);
  float2* const row = part + (long)blockIdx.y * T + t;
  row[0].y = s.x; row[1].y = s.y; row[2].y = s.z; row[3].y = s.w;
}

// Sets *flag when a token's maximum over the chunk (the .x halves of the partial rows) lies more than RP_CE_P_LIMIT
// above its reference exponent: the probabilities EPI_CE_P wrote for this chunk are then replaced.
__global__ void __launch_bounds__(256) ce_chunk_check_kernel(const float2* __restrict__ pmax, int nslab, int T,
                                                             const float* __restrict__ m, int* __restrict__ flag) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= T) return;
  const int r0 = blockIdx.y * 8, r1 = min(r0 + 8, nslab);   // eight partial rows per thread
  const float lim = m[t] + RP_CE_P_LIMIT;
  bool over = false;
  for (int i = r0; i < r1; ++i) over |= pmax[(long)i * T + t].x > lim;
  if (over) *flag = 1;   // every writer stores the same value
}

// l[t] += sum over the chunk's partial rows of part[i][t].y, in row order.
__global__ void __launch_bounds__(256) ce_chunk_sum_kernel(const float2* __restrict__ part, int nslab, int T, float* __restrict__ l) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= T) return;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;   // four chains, merged in a fixed order
  int i = 0;
  for (; i + 4 <= nslab; i += 4) {
    s0 += part[(long)i * T + t].y; s1 += part[(long)(i + 1) * T + t].y;
    s2 += part[(long)(i + 2) * T + t].y; s3 += part[(long)(i + 3) * T + t].y;
  }
  for (; i < nslab; ++i) s0 += part[(long)i * T + t].y;
  l[t] += (s0 + s1) + (s2 + s3);
}

// acc[t, :] *= alpha[t] for the rows whose reference moved.  One wave per row.
__global__ void __launch_bounds__(256) ce_rescale_rows_kernel(float* __restrict__ acc, const float* __restrict__ alpha, int T, int h,
                                                              const int* __restrict__ run_flag) {
  if (run_flag && *run_flag == 0) return;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (t >= T) return;
  const float a = alpha[t];
  if (a == 1.f) return;
  float4* row = reinterpret_cast<float4*>(acc + (long)t * h);
  for (int c = lane; c < h / 4; c += 64) { float4 v = row[c]; v.x *= a; v.y *= a; v.z *= a; v.w *= a; row[c] = v; }
}

// One sweep with a trainable head: the probabilities of every chunk stay in memory ([V, T] bf16, against the reference
// exponent), and the weight gradient is formed afterwards as  dW = P'^T^T xs,  P'[v, t] = p[v, t] - l_t [v = y_t],
// xs_t = (coef_t / l_t) xf_t  (= sum_t coef_t (p_tv / l_t - [v = y_t]) xf_t).
//
// p[r, t] *= alpha[t] for the rows r < rows stored so far, where a token's reference moved (alpha != 1).  Grid-stride.
__global__ void __launch_bounds__(256) ce_rescale_p_kernel(bf16* __restrict__ p, long rows, int T, const float* __restrict__ alpha,
                                                           const int* __restrict__ run_flag) {
  if (run_flag && *run_flag == 0) return;
  const int t8 = T >> 3;
  const long total = rows * t8;
  for (long idx = (long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long)gridDim.x * 256) {
    const int c = (int)(idx % t8);
    const float4 a0 = *reinterpret_cast<const float4*>(alpha + c * 8), a1 = *reinterpret_cast<const float4*>(alpha + c * 8 + 4);
    if (a0.x == 1.f && a0.y == 1.f && a0.z == 1.f && a0.w == 1.f && a1.x == 1.f && a1.y == 1.f && a1.z == 1.f && a1.w == 1.f) continue;
    uint4* const q = reinterpret_cast<uint4*>(p) + idx;
    const uint4 v = *q;
    *q = make_uint4(pack_bf16x2(bf16_lo(v.x) * a0.x, bf16_hi(v.x) * a0.y), pack_bf16x2(bf16_lo(v.y) * a0.z, bf16_hi(v.y) * a0.w),
                    pack_bf16x2(bf16_lo(v.z) * a1.x, bf16_hi(v.z) * a1.y), pack_bf16x2(bf16_lo(v.w) * a1.z, bf16_hi(v.w) * a1.w));
  }
}

// p[y_t, t] -= l_t for every token whose label takes part in the loss (coef != 0) and lies inside the vocabulary.  One
// element per token, all in different columns: no two threads touch the same one.
__global__ void __launch_bounds__(256) ce_patch_label_kernel(bf16* __restrict__ p, int T, int V, const int* __restrict__ labels,
                                                             const float* __restrict__ l, const float* __restrict__ coef) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= T) return;
  const int y = labels[t];
  if (coef[t] == 0.f || y < 0 || y >= V) return;
  bf16* const e = p + (long)y * T + t;
  *e = (bf16)((float)*e - l[t]);
}

// xs[t, :] = xf[t, :] * coef[t] / l[t]  (bf16; zero rows for ignored tokens)
__global__ void __launch_bounds__(256) ce_scale_x_kernel(const bf16* __restrict__ xf, const float* __restrict__ coef,
                                                         const float* __restrict__ l, bf16* __restrict__ xs, int T, int h) {
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (t >= T) return;
  const float s = coef[t] == 0.f ? 0.f : coef[t] / l[t];
  const uint4* src = reinterpret_cast<const uint4*>(xf + (long)t * h);
  uint4* dst = reinterpret_cast<uint4*>(xs + (long)t * h);
  for (int c = lane; c < h / 8; c += 64) {
    const uint4 v = src[c];
    dst[c] = make_uint4(pack_bf16x2(bf16_lo(v.x) * s, bf16_hi(v.x) * s), pack_bf16x2(bf16_lo(v.y) * s, bf16_hi(v.y) * s),
                        pack_bf16x2(bf16_lo(v.z) * s, bf16_hi(v.z) * s), pack_bf16x2(bf16_lo(v.w) * s, bf16_hi(v.w) * s));
  }
}

__global__ void __launch_bounds__(256) ce_lse_from_ref_kernel(const float* __restrict__ m, const float* __restrict__ l,
                                                              float* __restrict__ lse, int T) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t < T) lse[t] = m[t] + logf(l[t]);
}

// acc[t, :] = coef[t] * (acc[t, :] / l[t] - W[label_t, :]); rows with coef 0 (ignored labels) become zero.
__global__ void __launch_bounds__(256) ce_frozen_dx_kernel(float* __restrict__ acc, const float* __restrict__ l,
                                                           const float* __restrict__ coef, const int* __restrict__ labels,
                                                           const bf16* __restrict__ W, int T, int h, int V) {
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (t >= T) return;
  const float c = coef[t];
  float4* row = reinterpret_cast<float4*>(acc + (long)t * h);
  if (c == 0.f) {
    for (int q = lane; q < h / 4; q += 64) row[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    return;
  }
  const float il = c / l[t];
  const int lab = labels[t];
  const bool has = lab >= 0 && lab < V;          // a label outside the vocabulary has no logit to subtract
  const uint2* wr = reinterpret_cast<const uint2*>(W + (long)(has ? lab : 0) * h);
  for (int q = lane; q < h / 4; q += 64) {
    float4 v = row[q];
    const uint2 w2 = has ? wr[q] : make_uint2(0u, 0u);
    v.x = v.x * il - c * bf16_lo(w2.x); v.y = v.y * il - c * bf16_hi(w2.x);
    v.z = v.z * il - c * bf16_lo(w2.y); v.w = v.w * il - c * bf16_hi(w2.y);
    row[q] = v;
  }
}

}  // namespace

hipError_t k_ce_chunk_update(hipStream_t st, const float* z, int vc, int T, float2* pmax, int nparts, int first, float* m,
                             float* l, float* alpha, void* p, const int* flag) {
  if (T == 0 || vc == 0) return hipSuccess;
  const int nblk = (vc + CE_PROB_ROWS - 1) / CE_PROB_ROWS;
  if (T % 4 || nblk > nparts) return hipErrorInvalidValue;   // one partial row per CE_PROB_ROWS vocabulary rows
  RP_LAUNCH(ce_chunk_ref_kernel, dim3((T + 255) / 256), dim3(256), 0, st, (const float2*)pmax, nparts, T, first, m, l, alpha, flag);
  RP_LAUNCH(ce_chunk_prob_kernel, dim3((T / 4 + 255) / 256, nblk), dim3(256), 0, st, z, vc, T, (const float*)m, (bf16*)p, pmax, flag);
  RP_LAUNCH(ce_chunk_sum_kernel, dim3((T + 255) / 256), dim3(256), 0, st, (const float2*)pmax, nblk, T, l);
  return hipGetLastError();
}

hipError_t k_ce_ref_init(hipStream_t st, const float2* pmax, int nparts, int T, float* m, float* l, float* alpha) {
  if (T == 0) return hipSuccess;
  RP_LAUNCH(ce_chunk_ref_kernel, dim3((T + 255) / 256), dim3(256), 0, st, pmax, nparts, T, 1, m, l, alpha, (const int*)nullptr);
  return hipGetLastError();
}

hipError_t k_ce_chunk_check(hipStream_t st, const float2* pmax, int nparts, int T, const float* m, int* flag) {
  if (T == 0) return hipSuccess;
  RP_LAUNCH(ce_chunk_check_kernel, dim3((T + 255) / 256, (nparts + 7) / 8), dim3(256), 0, st, pmax, nparts, T, m, flag);
  return hipGetLastError();
}

hipError_t k_ce_rescale_rows(hipStream_t st, float* acc, const float* alpha, int T, int h, const int* flag) {
  if (T == 0) return hipSuccess;
  if (h % 4) return hipErrorInvalidValue;
  RP_LAUNCH(ce_rescale_rows_kernel, dim3((T + 3) / 4), dim3(256), 0, st, acc, alpha, T, h, flag);
  return hipGetLastError();
}

hipError_t k_ce_rescale_p(hipStream_t st, void* p, long rows, int T, const float* alpha, const int* flag) {
  if (T == 0 || rows == 0) return hipSuccess;
  if (T % 8) return hipErrorInvalidValue;
  RP_LAUNCH(ce_rescale_p_kernel, dim3(2048), dim3(256), 0, st, (bf16*)p, rows, T, alpha, flag);
  return hipGetLastError();
}

hipError_t k_ce_patch_label(hipStream_t st, void* p, int T, int V, const int* labels, const float* l, const float* coef) {
  if (T == 0) return hipSuccess;
  RP_LAUNCH(ce_patch_label_kernel, dim3((T + 255) / 256), dim3(256), 0, st, (bf16*)p, T, V, labels, l, coef);
  return hipGetLastError();
}

hipError_t k_ce_scale_x(hipStream_t st, const void* xf, const float* coef, const float* l, void* xs, int T, int h) {
  if (T == 0) return hipSuccess;
  if (h % 8) return hipErrorInvalidValue;
  RP_LAUNCH(ce_scale_x_kernel, dim3((T + 3) / 4), dim3(256), 0, st, (const bf16*)xf, coef, l, (bf16*)xs, T, h);
  return hipGetLastError();
}

hipError_t k_ce_lse_from_ref(hipStream_t st, const float* m, const float* l, float* lse, int T) {
  if (T == 0) return hipSuccess;
  RP_LAUNCH(ce_lse_from_ref_kernel, dim3((T + 255) / 256), dim3(256), 0, st, m, l, lse, T);
  return hipGetLastError();
}

hipError_t k_ce_frozen_dx(hipStream_t st, float* acc, const float* l, const float* coef, const int* labels, const void* W, int T, int h,
                          int V) {
  if (T == 0) return hipSuccess;
  if (h % 4) return hipErrorInvalidValue;
  RP_LAUNCH(ce_frozen_dx_kernel, dim3((T + 3) / 4), dim3(256), 0, st, acc, l, coef, labels, (const bf16*)W, T, h, V);
  return hipGetLastError();
}

hipError_t k_ce_lse(hipStream_t st, const float2* part, int P, long part_ld, float* lse, int T) {
  if (T == 0) return hipSuccess;
  RP_LAUNCH(ce_lse_kernel, dim3((T + 15) / 16), dim3(1024), 0, st, part, P, part_ld, lse, T);
  return hipGetLastError();
}

hipError_t k_ce_finalize(hipStream_t st, const float* lse, const float* zlab, const int* labels, float grad_scale,
                         float* coef, float* loss_out, int T) {
  RP_LAUNCH(ce_finalize_kernel, dim3(1), dim3(1024), 0, st, lse, zlab, labels, grad_scale, coef, loss_out, T);
  return hipGetLastError();
}
