// Cross-entropy bookkeeping around the LM-head GEMMs: the logits are reduced inside the GEMM epilogue to per-token
// (max, sum exp) partials, one per 128 vocabulary rows; these kernels merge the partials and produce the loss and the
// per-token gradient coefficient.
#include "common.hpp"
#include "kernels.hpp"

namespace {

// lse[t] = log sum_v exp(z[t, v]) from P partial (max, sum) pairs per token; part is [P][ld] so reads are coalesced
// over tokens.  A block handles 16 tokens with 16 slices of the partials each, merged through LDS.
__global__ void __launch_bounds__(256) ce_lse_kernel(const float2* __restrict__ part, int P, long ld, float* __restrict__ lse, int T) {
  __shared__ float2 red[16][17];
  const int tl = threadIdx.x & 15, sl = threadIdx.x >> 4;
  const int t = blockIdx.x * 16 + tl;
  float m = -INFINITY, s = 0.f;
  if (t < T) {
    for (int i = sl; i < P; i += 16) {
      const float2 v = part[(long)i * ld + t];
      if (v.x > -INFINITY) {
        const float mn = fmaxf(m, v.x);
        s = s * __expf(m - mn) + v.y * __expf(v.x - mn);
        m = mn;
      }
    }
  }
  red[sl][tl] = make_float2(m, s);
  __syncthreads();
  if (sl == 0 && t < T) {
    for (int i = 1; i < 16; ++i) {
      const float2 v = red[i][tl];
      if (v.x > -INFINITY) {
        const float mn = fmaxf(m, v.x);
        s = s * __expf(m - mn) + v.y * __expf(v.x - mn);
        m = mn;
      }
    }
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

}  // namespace

hipError_t k_ce_lse(hipStream_t st, const float2* part, int P, long part_ld, float* lse, int T) {
  if (T == 0) return hipSuccess;
  RP_LAUNCH(ce_lse_kernel, dim3((T + 15) / 16), dim3(256), 0, st, part, P, part_ld, lse, T);
  return hipGetLastError();
}

hipError_t k_ce_finalize(hipStream_t st, const float* lse, const float* zlab, const int* labels, float grad_scale,
                         float* coef, float* loss_out, int T) {
  RP_LAUNCH(ce_finalize_kernel, dim3(1), dim3(1024), 0, st, lse, zlab, labels, grad_scale, coef, loss_out, T);
  return hipGetLastError();
}
