// Top-k mixture-of-experts FFN (the MoE layer of App. B.2 / C.4): everything around the grouped GEMMs.
//
//   route    : per token the top_k largest router logits (ties -> lower expert index) and the softmax over just those
//   plan     : a stable counting sort of the T*top_k (token, choice) entries by expert.  Entry i = t*top_k + j gets slot
//              seg[e] + (number of earlier entries of the same expert); the grouped GEMMs work on slot-ordered rows, so
//              every expert owns a contiguous row range.  Also writes the table of 256-row tiles the GEMM grid walks.
//              Four small kernels (per-run histograms, their prefix per expert, scan + tile table, assign); the
//              order is a function of the logits alone.
//   combine  : out[t] = (res[t]) + sum_j (w[t,j]) * src[slot_of[t,j]], j in order -- the weighted sum of the expert
//              outputs in the forward pass, the plain sum of the expert input gradients in the backward pass
//   swiglu backward for slot rows: the routing weight scales the incoming gradient, and the gradient of the routing
//              weight, <dz_t, FFN_e(n2_t)> = <dact, act> with dact = Wd_e^T dz_t, falls out of the same pass
//   dlogits  : dlogit[t, e] = w_te (dw_te - sum_e' w_te' dw_te') on the selected experts, zero elsewhere
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

// ------------------------------------------------------------------------------------------------ route
// One wave per token; lane l holds experts l, l+64, ... (EPL of them).  top_k rounds of a wave-wide arg-max.
template <int EPL>
__global__ void __launch_bounds__(256) moe_route_kernel(const float* __restrict__ logits, int* __restrict__ idx,
                                                        float* __restrict__ w, int T, int E, int top_k) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  float v[EPL];
#pragma unroll
  for (int i = 0; i < EPL; ++i) {
    const int e = lane + 64 * i;
    v[i] = e < E ? logits[(long)t * E + e] : -INFINITY;
  }
  float sel_v = 0.f, first = 0.f, sum = 0.f;   // lane j keeps the j-th selected logit
  int sel_e = 0;
  for (int j = 0; j < top_k; ++j) {
    float bv = -INFINITY;
    int be = 0x7fffffff;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      const int e = lane + 64 * i;
      if (v[i] > bv) { bv = v[i]; be = e; }      // ascending e within the lane: ties keep the lower index
    }
    if (bv == -INFINITY) be = 0x7fffffff;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      const float ov = __shfl_xor(bv, off, 64);
      const int oe = __shfl_xor(be, off, 64);
      if (ov > bv || (ov == bv && oe < be)) { bv = ov; be = oe; }
    }
    if (j == 0) first = bv;
    const float ex = __expf(bv - first);          // the first pick is the maximum
    sum += ex;
    if (lane == j) { sel_v = ex; sel_e = be; }
#pragma unroll
    for (int i = 0; i < EPL; ++i)
      if (lane + 64 * i == be) v[i] = -INFINITY;
  }
  if (lane < top_k) {
    idx[(long)t * top_k + lane] = sel_e;
    w[(long)t * top_k + lane] = sel_v / sum;
  }
}

// ------------------------------------------------------------------------------------------------ plan
// The entries are cut into runs of RP_MOE_RUN consecutive entries, one wave per run.
// hist[run][e] = number of entries of run `run` routed to expert e.
__global__ void __launch_bounds__(256) moe_hist_kernel(const int* __restrict__ idx, long n, int E, int* __restrict__ hist) {
  extern __shared__ int s_hist[];   // [4][E]
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  int* const h = s_hist + wv * E;
  for (int e = lane; e < E; e += 64) h[e] = 0;
  __syncthreads();
  const long run = (long)blockIdx.x * 4 + wv;
  const long i0 = run * RP_MOE_RUN;
  for (int k = lane; k < RP_MOE_RUN; k += 64)
    if (i0 + k < n) atomicAdd(&h[idx[i0 + k]], 1);
  __syncthreads();
  if (i0 < n)
    for (int e = lane; e < E; e += 64) hist[run * E + e] = h[e];
}

// Per expert (one block each): hist[run][e] becomes the number of entries of expert e in earlier runs; counts[e] = total.
__global__ void __launch_bounds__(256) moe_prefix_kernel(int* __restrict__ hist, long nruns, int E, int* __restrict__ counts) {
  __shared__ int s_part[256];
  __shared__ int s_carry;
  const int e = blockIdx.x, tid = threadIdx.x;
  if (tid == 0) s_carry = 0;
  __syncthreads();
  for (long r0 = 0; r0 < nruns; r0 += 256) {
    const long r = r0 + tid;
    const int v = r < nruns ? hist[r * E + e] : 0;
    s_part[tid] = v;
    __syncthreads();
    // inclusive scan of 256 values
    for (int off = 1; off < 256; off <<= 1) {
      const int add = tid >= off ? s_part[tid - off] : 0;
      __syncthreads();
      s_part[tid] += add;
      __syncthreads();
    }
    const int carry = s_carry;
    if (r < nruns) hist[r * E + e] = carry + s_part[tid] - v;
    __syncthreads();
    if (tid == 255) s_carry = carry + s_part[255];
    __syncthreads();
  }
  if (tid == 0) counts[e] = s_carry;
}

// seg[e] = first slot of expert e (seg[E] = n); tile table entries {expert, first row, rows, 0} for every 256-row tile
// of every expert, in expert order; *ntiles = their number.  One block, thread e = expert e (E <= 1024).
__global__ void __launch_bounds__(1024) moe_scan_kernel(const int* __restrict__ counts, int E, int* __restrict__ seg,
                                                        int4* __restrict__ tab, int* __restrict__ ntiles) {
  __shared__ int s_cnt[1024];
  const int e = threadIdx.x;
  s_cnt[e] = e < E ? counts[e] : 0;
  __syncthreads();
  if (e < E) {
    int row0 = 0, tile0 = 0;
    for (int i = 0; i < e; ++i) { row0 += s_cnt[i]; tile0 += (s_cnt[i] + 255) >> 8; }
    seg[e] = row0;
    const int n = s_cnt[e];
    for (int i = 0; i * 256 < n; ++i) tab[tile0 + i] = make_int4(e, row0 + i * 256, min(256, n - i * 256), 0);
    if (e == E - 1) { seg[E] = row0 + n; *ntiles = tile0 + ((n + 255) >> 8); }
  }
}

// slot_of[i] = seg[e] + rank of entry i among the entries of its expert (entry order); row_tok[slot] = token of the
// entry.  Every wave walks its own run 64 entries at a time; inside such a group the lanes of one expert are found with
// a ballot per distinct expert, and the wave's running position per expert lives in LDS.
__global__ void __launch_bounds__(256) moe_assign_kernel(const int* __restrict__ idx, long n, int E, int top_k,
                                                         const int* __restrict__ seg, const int* __restrict__ hist,
                                                         int* __restrict__ slot_of, int* __restrict__ row_tok) {
  extern __shared__ int s_pos[];   // [4][E]
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  int* const pos = s_pos + wv * E;
  const long run = (long)blockIdx.x * 4 + wv;
  const long i0 = run * RP_MOE_RUN;
  if (i0 >= n) return;   // no barriers below: the waves are independent
  for (int e = lane; e < E; e += 64) pos[e] = seg[e] + hist[run * E + e];
  const unsigned long long lt = (1ull << lane) - 1ull;
  for (int k0 = 0; k0 < RP_MOE_RUN && i0 + k0 < n; k0 += 64) {
    const long i = i0 + k0 + lane;
    const bool live = i < n;
    const int e = live ? idx[i] : -1;
    int slot = 0;
    unsigned long long todo = __builtin_amdgcn_ballot_w64(live);
    while (todo) {
      const int first = __builtin_ctzll(todo);
      const int e0 = __builtin_amdgcn_readlane(e, first);
      const unsigned long long m = __builtin_amdgcn_ballot_w64(e == e0);
      const int base = pos[e0];                       // wave-uniform address
      if (e == e0) slot = base + __builtin_popcountll(m & lt);
      // every lane has read pos[e0] before it is advanced: LDS operations of one wave execute in order
      if (lane == first) pos[e0] = base + __builtin_popcountll(m);
      todo &= ~m;
    }
    if (live) {
      slot_of[i] = slot;
      row_tok[slot] = (int)(i / top_k);
    }
  }
}

// ------------------------------------------------------------------------------------------------ combine
// One wave per token row; MAXC 16-byte chunks per lane.
template <int MAXC>
__global__ void __launch_bounds__(256) moe_combine_kernel(const bf16* __restrict__ src, const int* __restrict__ slot_of,
                                                          const float* __restrict__ w, const bf16* __restrict__ res,
                                                          bf16* __restrict__ out, int T, int h, int top_k) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  const int nch = h >> 3;
  float acc[MAXC][8];
#pragma unroll
  for (int i = 0; i < MAXC; ++i) {
    const int c = lane + 64 * i;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[i][e] = 0.f;
    if (res && c < nch) unpack8(reinterpret_cast<const uint4*>(res + (long)t * h)[c], acc[i]);
  }
  for (int j = 0; j < top_k; ++j) {
    const int slot = slot_of[(long)t * top_k + j];
    const float wj = w ? w[(long)t * top_k + j] : 1.f;
    const uint4* r = reinterpret_cast<const uint4*>(src + (long)slot * h);
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      const int c = lane + 64 * i;
      if (c < nch) {
        float f[8];
        unpack8(r[c], f);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[i][e] += wj * f[e];
      }
    }
  }
#pragma unroll
  for (int i = 0; i < MAXC; ++i) {
    const int c = lane + 64 * i;
    if (c < nch) reinterpret_cast<uint4*>(out + (long)t * h)[c] = pack8(acc[i]);
  }
}

// ------------------------------------------------------------------------------------------------ SwiGLU backward, slot rows
// dact_in[slot] = Wd_e^T dz_t (unscaled).  dw_slot[slot] = <dact_in, act>; dgu = swiglu'(w * dact_in).  One wave per row.
__global__ void __launch_bounds__(256) moe_swiglu_bwd_kernel(const bf16* __restrict__ dact, const bf16* __restrict__ gu,
                                                             const float* __restrict__ w_slot, bf16* __restrict__ dgu,
                                                             float* __restrict__ dw_slot, long rows, int m) {
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int mc = m >> 3;
  const float wr = w_slot[row];
  const uint4* r = reinterpret_cast<const uint4*>(gu + row * 2 * m);
  const uint4* dr = reinterpret_cast<const uint4*>(dact + row * m);
  uint4* o = reinterpret_cast<uint4*>(dgu + row * 2 * m);
  float dot = 0.f;
  for (int c = lane; c < mc; c += 64) {
    float g[8], u[8], d[8], dg[8], du[8];
    unpack8(r[c], g);
    unpack8(r[mc + c], u);
    unpack8(dr[c], d);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float sg = 1.f / (1.f + __expf(-g[e]));
      dot += d[e] * g[e] * sg * u[e];
      const float ds = d[e] * wr;
      dg[e] = ds * u[e] * sg * (1.f + g[e] * (1.f - sg));
      du[e] = ds * g[e] * sg;
    }
    o[c] = pack8(dg);
    o[mc + c] = pack8(du);
  }
  dot = wave_sum(dot);
  if (lane == 0) dw_slot[row] = dot;
}

// w_slot[slot_of[i]] = w[i]: the routing weight of every slot row.
__global__ void moe_scatter_w_kernel(const float* __restrict__ w, const int* __restrict__ slot_of, float* __restrict__ w_slot, long n) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) w_slot[slot_of[i]] = w[i];
}

// ------------------------------------------------------------------------------------------------ dlogits
// One thread per (token, expert).
__global__ void moe_dlogits_kernel(const int* __restrict__ idx, const float* __restrict__ w, const int* __restrict__ slot_of,
                                   const float* __restrict__ dw_slot, float* __restrict__ dlogits, long T, int E, int top_k) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= T * E) return;
  const long t = i / E;
  const int e = (int)(i - t * E);
  float mean = 0.f, mine = 0.f;
  bool sel = false;
  for (int j = 0; j < top_k; ++j) {
    const float wj = w[t * top_k + j];
    const float dj = dw_slot[slot_of[t * top_k + j]];
    mean += wj * dj;
    if (idx[t * top_k + j] == e) { sel = true; mine = wj * dj; }
  }
  float out = 0.f;
  if (sel) {
    // w_e (dw_e - mean): recover w_e from mine = w_e dw_e without a second pass
    for (int j = 0; j < top_k; ++j)
      if (idx[t * top_k + j] == e) out = mine - w[t * top_k + j] * mean;
  }
  dlogits[i] = out;
}

}  // namespace

// ------------------------------------------------------------------------------------------------ launchers
hipError_t k_moe_route(hipStream_t st, const float* logits, int* idx, float* w, int T, int E, int top_k) {
  if (T == 0) return hipSuccess;
  if (E > 1024 || top_k < 1 || top_k > 64 || top_k > E) return hipErrorInvalidValue;
  const int grid = (T + 3) / 4;
  if (E <= 64) RP_LAUNCH(moe_route_kernel<1>, dim3(grid), dim3(256), 0, st, logits, idx, w, T, E, top_k);
  else if (E <= 128) RP_LAUNCH(moe_route_kernel<2>, dim3(grid), dim3(256), 0, st, logits, idx, w, T, E, top_k);
  else if (E <= 256) RP_LAUNCH(moe_route_kernel<4>, dim3(grid), dim3(256), 0, st, logits, idx, w, T, E, top_k);
  else RP_LAUNCH(moe_route_kernel<16>, dim3(grid), dim3(256), 0, st, logits, idx, w, T, E, top_k);
  return hipGetLastError();
}

hipError_t k_moe_plan(hipStream_t st, const int* idx, int T, int E, int top_k, int* counts, int* seg, void* tile_tab,
                      int* ntiles, int* slot_of, int* row_tok, int* hist) {
  if (T == 0) return hipSuccess;
  if (E > 1024) return hipErrorInvalidValue;
  const long n = (long)T * top_k;
  const long nruns = (n + RP_MOE_RUN - 1) / RP_MOE_RUN;
  const unsigned blocks = (unsigned)((nruns + 3) / 4);
  const size_t lds = (size_t)4 * E * sizeof(int);
  RP_LAUNCH(moe_hist_kernel, dim3(blocks), dim3(256), lds, st, idx, n, E, hist);
  RP_LAUNCH(moe_prefix_kernel, dim3(E), dim3(256), 0, st, hist, nruns, E, counts);
  RP_LAUNCH(moe_scan_kernel, dim3(1), dim3(1024), 0, st, (const int*)counts, E, seg, (int4*)tile_tab, ntiles);
  RP_LAUNCH(moe_assign_kernel, dim3(blocks), dim3(256), lds, st, idx, n, E, top_k, (const int*)seg, (const int*)hist, slot_of, row_tok);
  return hipGetLastError();
}

hipError_t k_moe_combine(hipStream_t st, const void* src, const int* slot_of, const float* w, const void* res, void* out,
                         int T, int h, int top_k) {
  if (T == 0) return hipSuccess;
  if (h % 8 || h > 8192) return hipErrorInvalidValue;
  const int grid = (T + 3) / 4;
  if (h <= 2048)
    RP_LAUNCH(moe_combine_kernel<4>, dim3(grid), dim3(256), 0, st, (const bf16*)src, slot_of, w, (const bf16*)res, (bf16*)out, T, h, top_k);
  else if (h <= 4096)   // half the accumulator registers of the widest variant: more waves, more loads in flight
    RP_LAUNCH(moe_combine_kernel<8>, dim3(grid), dim3(256), 0, st, (const bf16*)src, slot_of, w, (const bf16*)res, (bf16*)out, T, h, top_k);
  else
    RP_LAUNCH(moe_combine_kernel<16>, dim3(grid), dim3(256), 0, st, (const bf16*)src, slot_of, w, (const bf16*)res, (bf16*)out, T, h, top_k);
  return hipGetLastError();
}

hipError_t k_moe_scatter_w(hipStream_t st, const float* w, const int* slot_of, float* w_slot, long n) {
  if (n == 0) return hipSuccess;
  RP_LAUNCH(moe_scatter_w_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, w, slot_of, w_slot, n);
  return hipGetLastError();
}

hipError_t k_moe_swiglu_bwd(hipStream_t st, const void* dact, const void* gu, const float* w_slot, void* dgu, float* dw_slot,
                            long rows, int m) {
  if (rows == 0) return hipSuccess;
  if (m % 8) return hipErrorInvalidValue;
  RP_LAUNCH(moe_swiglu_bwd_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, (const bf16*)dact, (const bf16*)gu,
            w_slot, (bf16*)dgu, dw_slot, rows, m);
  return hipGetLastError();
}

hipError_t k_moe_dlogits(hipStream_t st, const int* idx, const float* w, const int* slot_of, const float* dw_slot,
                         float* dlogits, long T, int E, int top_k) {
  if (T == 0) return hipSuccess;
  const long n = T * E;
  RP_LAUNCH(moe_dlogits_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, idx, w, slot_of, dw_slot, dlogits, T, E, top_k);
  return hipGetLastError();
}
