// Launchers of the non-GEMM kernels.  Every function only enqueues on `st` and returns the launch status.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

struct LoraSegs {           // up to three row segments of a fused projection, each with its own LoRA B [rows, r]
  const void* src[3];
  int row0[3], row1[3], col0[3];
};

// y = x * rstd * g, rstd[T] saved (may be NULL).  x, y bf16 [T, h]; g bf16 [h].
hipError_t k_rmsnorm_fwd(hipStream_t st, const void* x, const void* g, void* y, float* rstd, int T, int h, float eps);
// Gain gradients are reduced block by block into `scratch` and then added to their destination in a fixed order.
#define RP_PARTIAL_BLOCKS 1024
// dx = rmsnorm backward (+ dres if non-NULL); dg (fp32 [h], may be NULL) += its gradient, using scratch
// [RP_PARTIAL_BLOCKS * h] floats.  dy bf16 or fp32.
hipError_t k_rmsnorm_bwd(hipStream_t st, const void* dy, int dy_is_f32, const void* x, const void* g, const float* rstd,
                         const void* dres, void* dx, float* dg, float* scratch, int T, int h);
// cs[seq][d/2] = (cos, sin)(pos * base^(-2i/d))
hipError_t k_rope_table(hipStream_t st, float2* cs, int seq, int d, float base);
// forward: (optional per-head RMSNorm) then RoPE on q heads and k heads.  backward: the transpose.
hipError_t k_qknorm_rope(hipStream_t st, int bwd, int d, const void* in_q, const void* in_k, long ld_in_q, long ld_in_k,
                         void* out_q, void* out_k, long ld_out_q, long ld_out_k, const void* gq, const void* gk,
                         float* rstd_q, float* rstd_k, const void* raw_q, const void* raw_k, long ld_raw, float* dgq,
                         float* dgk, float* scratch /* [RP_PARTIAL_BLOCKS * 2 * d] floats, backward with gains */,
                         const float2* cs, int T, int seq, int a, int k, int use_norm, float eps);
// act[T, m] = silu(gu[:, :m]) * gu[:, m:]
hipError_t k_swiglu_fwd(hipStream_t st, const void* gu, void* act, long T, int m);
hipError_t k_swiglu_bwd(hipStream_t st, const void* dact, const void* gu, void* dgu, long T, int m);
hipError_t k_fill_u32(hipStream_t st, void* p, long n_words, uint32_t v);
hipError_t k_copy16(hipStream_t st, const void* src, void* dst, long bytes);
hipError_t k_cast_f32_bf16(hipStream_t st, const float* src, void* dst, long n);
hipError_t k_lora_blockdiag(hipStream_t st, void* out, int N, int ncols, const LoraSegs& segs, int r);

// Causal GQA attention, flash style.  q [T, a, d] (row stride ldq elements), k, v [T, kh, d] (ldk, ldv), o [T, a, d]
// (ldo); lse fp32 [batch, a, seq].  T = batch*seq; sequences are independent.
hipError_t k_attn_fwd(hipStream_t st, const void* q, const void* k, const void* v, void* o, float* lse, long ldq,
                      long ldk, long ldv, long ldo, int batch, int seq, int a, int kh, int d);
// delta[batch, a, seq] = rowsum(dO * O)
hipError_t k_attn_delta(hipStream_t st, const void* o, const void* dout, float* delta, long ldo, long lddo, int batch,
                        int seq, int a, int d);
// part 0: dk, dv [T, kh, d] (lddk, lddv) when a == kh, else per-query-head fp32 partials into scratch (2*T*a*d
// floats);  part 2: sum of each group's partials into dk, dv (nothing to do when a == kh);  part 1: dq [T, a, d].
hipError_t k_attn_bwd(hipStream_t st, int part, const void* q, const void* k, const void* v, const void* dout, const float* lse,
                      const float* delta, void* dq, void* dk, void* dv, float* scratch, long ldq, long ldk, long ldv,
                      long lddo, long lddq, long lddk, long lddv, int batch, int seq, int a, int kh, int d);

// Mixture-of-experts FFN, everything but the grouped GEMMs.  Entries are (token, choice) pairs, i = t*top_k + j; slots
// are the same entries sorted by expert (stable).
// idx [T, top_k] = experts with the largest logits (descending, ties -> lower index), w = softmax over those logits.
hipError_t k_moe_route(hipStream_t st, const float* logits, int* idx, float* w, int T, int E, int top_k);
// counts [E], seg [E+1] (first slot of every expert), tile_tab (int4 {expert, first row, rows, 0} per 256-row tile, at
// most T*top_k/256 + E of them), *ntiles, slot_of [T*top_k], row_tok [T*top_k] (token of every slot);
// hist: scratch, ceil(T*top_k / RP_MOE_RUN) * E ints (per-run histograms, then their prefix sums).
#define RP_MOE_RUN 512
hipError_t k_moe_plan(hipStream_t st, const int* idx, int T, int E, int top_k, int* counts, int* seg, void* tile_tab,
                      int* ntiles, int* slot_of, int* row_tok, int* hist);
// out[t] = (res[t] if res) + sum_j (w[t,j] if w else 1) * src[slot_of[t,j]];  src bf16 [T*top_k, h], out bf16 [T, h].
hipError_t k_moe_combine(hipStream_t st, const void* src, const int* slot_of, const float* w, const void* res, void* out,
                         int T, int h, int top_k);
hipError_t k_moe_scatter_w(hipStream_t st, const float* w, const int* slot_of, float* w_slot, long n);
// dw_slot[r] = <dact[r], swiglu(gu[r])>;  dgu[r] = swiglu backward of w_slot[r] * dact[r].
hipError_t k_moe_swiglu_bwd(hipStream_t st, const void* dact, const void* gu, const float* w_slot, void* dgu, float* dw_slot,
                            long rows, int m);
// dlogits [T, E] = w_te (dw_te - sum_e' w_te' dw_te') on the selected experts, 0 elsewhere.
hipError_t k_moe_dlogits(hipStream_t st, const int* idx, const float* w, const int* slot_of, const float* dw_slot,
                         float* dlogits, long T, int E, int top_k);

// Cross-entropy helpers.  part [P, T] (max, sumexp) partials -> lse[T]; then loss / coef from lse, label logits, labels.
hipError_t k_ce_lse(hipStream_t st, const float2* part, int P, long part_ld, float* lse, int T);
// Frozen head, one sweep over the vocabulary: per chunk, z [vc, T] fp32 -> p = exp(z - m_t) [vc, T] bf16 against the
// per-token reference exponent m (moved, with l rescaled and alpha set, when the chunk outgrows it by more than e^8),
// l += row sums.  pmax [nparts][T]: the chunk's per-column maxima (.x), as the logits GEMM left them, one row per 128
// vocabulary rows; the .y halves are overwritten (per-block row sums, added to l in row order: no atomics).
// flag (optional, device): the reference and probability kernels return at once when *flag == 0 (the partial sums
// already there are then added to l as they are).
hipError_t k_ce_chunk_update(hipStream_t st, const float* z, int vc, int T, float2* pmax, int nparts, int first, float* m,
                             float* l, float* alpha, void* p, const int* flag);
// m[t] = max over the partial rows' .x, l[t] = 0, alpha[t] = 1: the reference exponents a sweep starts from.
hipError_t k_ce_ref_init(hipStream_t st, const float2* pmax, int nparts, int T, float* m, float* l, float* alpha);
// *flag = 1 when some token's maximum over the chunk (pmax .x) lies more than RP_CE_P_LIMIT above its reference m.
hipError_t k_ce_chunk_check(hipStream_t st, const float2* pmax, int nparts, int T, const float* m, int* flag);
// acc[t, :] *= alpha[t] where alpha[t] != 1 (nothing when flag is given and *flag == 0).
hipError_t k_ce_rescale_rows(hipStream_t st, float* acc, const float* alpha, int T, int h, const int* flag);
hipError_t k_ce_lse_from_ref(hipStream_t st, const float* m, const float* l, float* lse, int T);
// One sweep with a trainable head (the probabilities of all chunks stay in memory, [V, T] bf16):
// p[r, t] *= alpha[t] for r < rows (nothing when flag is given and *flag == 0);
hipError_t k_ce_rescale_p(hipStream_t st, void* p, long rows, int T, const float* alpha, const int* flag);
// p[labels[t], t] -= l[t] for tokens with coef != 0 and a label inside the vocabulary;
hipError_t k_ce_patch_label(hipStream_t st, void* p, int T, int V, const int* labels, const float* l, const float* coef);
// xs[t, :] = xf[t, :] * coef[t] / l[t] (bf16).
hipError_t k_ce_scale_x(hipStream_t st, const void* xf, const float* coef, const float* l, void* xs, int T, int h);
// acc[t, :] = coef[t] * (acc[t, :] / l[t] - W[labels[t], :]) (zero where coef is zero).
hipError_t k_ce_frozen_dx(hipStream_t st, float* acc, const float* l, const float* coef, const int* labels, const void* W, int T, int h,
                          int V);
hipError_t k_ce_finalize(hipStream_t st, const float* lse, const float* zlab, const int* labels, float grad_scale,
                         float* coef, float* loss_out, int T);
