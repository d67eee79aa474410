/*
 * rp_ops.h -- kernel-level entry points of the same library, one per hot-path kernel, so that each kernel can be
 * compared with the CPU oracle on its own.  Same conventions as rp.h: plain C types, all data pointers are device
 * pointers, bf16 row-major unless stated, `stream` is a hipStream_t, calls only enqueue.  Errors: RP_EINVAL for
 * arguments the kernels do not cover, RP_EHIP for launch failures.
 */
#ifndef RP_OPS_H
#define RP_OPS_H
#include "rp.h"
#ifdef __cplusplus
extern "C" {
#endif

/* The projections of a layer (paper App. B.2: Q/K/V/output and gate/up/down products) and their two gradients
 * (App. C.3).  layout 0 (NT): C[M,N] = A[M,K] B[N,K]^T;  1 (NN): C = A[M,K] B[K,N];  2 (TN): C = A[K,M]^T B[K,N].
 * out_f32 0: C bf16 = alpha*acc (+ R, bf16 [M,N], optional);  1: C fp32 = alpha*acc (+ C when beta);  2: atomic +=.
 * (A2, B2, K2): optional second operand pair, same layout, appended to the reduction (LoRA up-projection).
 * K, K2 and all leading dimensions are multiples of 8; N (and M for layout 2) too when that operand is transposed.
 * tile 0 = automatic, 1..4 force 256x256, 256x128, 128x128, 128x64; 5 = 256x128 worked on by two wave groups that
 * split every K tile (for outputs too small to fill the chip with 256x256 tiles); 6 = 256x256 with B (and B2) given
 * in fragment order (rp_op_gemm_arrange; ldb, ldb2 unused; layouts 0 and 1): that operand is streamed into registers
 * without passing through LDS; 7 = 256x256 by four waves of 128x128 whose operands are loaded from memory straight
 * into LDS (what "automatic" picks whenever it picks 256x256 tiles, K + K2 >= 2560 and M, N > 64 -- 1 always names
 * the eight-wave kernel that stages its operands through registers; the two give bit-identical results).
 * split_ws [dev, split_ws_bytes] or NULL: scratch for a reduction split.  An accumulating fp32 product (out_f32 1 with
 * beta) whose 256x256 tiles would leave most compute units idle is cut into up to 16 slices along K when the scratch
 * holds slices * M * N floats; the slices' partial products are added to C in slice order by a second kernel, so the
 * result is reproducible run to run (the weight-gradient accumulation of Sec. 4.1.1).  out_f32 3: as 1, but the merged
 * sum is written to C as bf16 [M, N] (overwritten; needs M * N floats of scratch; one direct pass when nothing splits). */
RP_API rp_status rp_op_gemm(void* stream, int layout, int out_f32, const void* A, const void* B, void* C, int M, int N, int K,
                     long lda, long ldb, long ldc, float alpha, int beta, const void* A2, const void* B2, int K2, long lda2,
                     long ldb2, const void* R, long ldr, int tile, void* split_ws, size_t split_ws_bytes);

/* The B operand of rp_op_gemm in the fragment order of the matrix instruction, for tile 6: B is [N, K] row-major
 * (transposed 0: the operand of layout 0) or [K, N] row-major (transposed 1: layout 1), bf16, row stride ldb.
 * out [dev, out_bytes]: ceil(N/64) * ceil(K/64) * 8192 bytes, columns and reduction indices past the end zero.
 * The weights of the projections (App. B.2) are constant over a stage's micro-batches, so one arrangement per upload
 * serves every call. */
RP_API rp_status rp_op_gemm_arrange(void* stream, const void* B, long ldb, int N, int K, int transposed, void* out, size_t out_bytes);

/* RMSNorm: y = x * rstd * g, rstd_t = (mean_j x_tj^2 + eps)^(-1/2); rstd fp32 [T] (may be NULL). */
RP_API rp_status rp_op_rmsnorm_fwd(void* stream, const void* x, const void* g, void* y, float* rstd, int T, int h, float eps);
/* dx = backward of the above (+ dres, bf16 [T,h], optional); dg fp32 [h] accumulated (optional; then scratch, fp32
 * [1024 * h], is required and overwritten). dy bf16, or fp32 when dy_is_f32. */
RP_API rp_status rp_op_rmsnorm_bwd(void* stream, const void* dy, int dy_is_f32, const void* x, const void* g, const float* rstd,
                            const void* dres, void* dx, float* dg, float* scratch, int T, int h);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): rp_op_rmsnorm_bwd without the scratch argument.  The gain-gradient partials go through a 16 MiB
 * array that is part of the library's code object (one copy per GPU, resident until the process ends); the call
 * allocates and frees nothing.  Limit: h <= 4096 (RP_EINVAL beyond it, with a message; nothing is enqueued).  Same
 * kernels and results as rp_op_rmsnorm_bwd.  All calls on one GPU share that array: calls that overlap on one GPU
 * (different streams, or threads) race on it -- serialise them.  The array's address is looked up once per device, at
 * rp_ctx_create on that device or else at the first call (with the stream's device current); do that first call
 * outside a graph capture. */
RP_API rp_status rp_op_rmsnorm_bwd_noalloc(void* stream, const void* dy, int dy_is_f32, const void* x, const void* g,
                                    const float* rstd, const void* dres, void* dx, float* dg, int T, int h);

/* cs: float2 [seq][d/2] = (cos, sin)(pos * base^(-2i/d)) */
RP_API rp_status rp_op_rope_table(void* stream, void* cs, int seq, int d, float base);
/* Per-head RMSNorm (optional) + rotary embedding with half-split pairs (i, i + d/2) on a query heads and k key heads.
 * forward: in_* -> out_*;  backward (bwd = 1): in_* are gradients of the rotated heads, raw_* the pre-norm heads,
 * out_* the gradients of the raw heads, dgq/dgk fp32 [d] accumulated (scratch: fp32 [1024 * 2 * d], overwritten).
 * rstd_* fp32 [T, heads]. */
RP_API rp_status rp_op_qknorm_rope(void* stream, int bwd, int d, const void* in_q, const void* in_k, long ld_in_q, long ld_in_k,
                            void* out_q, void* out_k, long ld_out_q, long ld_out_k, const void* gq, const void* gk, float* rstd_q,
                            float* rstd_k, const void* raw_q, const void* raw_k, long ld_raw, float* dgq, float* dgk,
                            float* scratch, const void* cs, int T, int seq, int a, int k, int use_norm, float eps);

/* SwiGLU: act[T,m] = silu(gu[:, :m]) * gu[:, m:];  backward gives dgu [T, 2m]. */
RP_API rp_status rp_op_swiglu_fwd(void* stream, const void* gu, void* act, long T, int m);
RP_API rp_status rp_op_swiglu_bwd(void* stream, const void* dact, const void* gu, void* dgu, long T, int m);

/* Routing of a top-k mixture of experts (the MoE layer of App. B.2) and the plan of its grouped products.
 * logits [dev] fp32 [T, E].  idx [dev] int32 [T, top_k]: the top_k largest logits of every token, descending, ties to the
 * lower expert; w [dev] fp32 [T, top_k]: the softmax over them.  counts [dev] int32 [E]: entries per expert; seg [dev]
 * int32 [E + 1]: first slot of every expert (seg[E] = T * top_k); slot_of [dev] int32 [T * top_k]: slot of entry
 * t * top_k + j = seg[e] + number of earlier entries of the same expert (a stable counting sort); row_tok [dev] int32
 * [T * top_k]: token of every slot; tile_tab [dev] 16 bytes x (T * top_k / 256 + E + 1): {expert, first row, rows, 0} of
 * every 256-row tile in expert order, *ntiles [dev] their number; hist [dev] scratch, ceil(T * top_k / 512) * E int32.
 * E <= 1024, top_k <= min(E, 64). */
RP_API rp_status rp_op_moe_route_plan(void* stream, const float* logits, int T, int E, int top_k, int* idx, float* w,
                               int* counts, int* seg, void* tile_tab, int* ntiles, int* slot_of, int* row_tok, int* hist);

/* Causal grouped-query attention (the attention term of App. B.2), flash style.  q, o [T, a, d]; k, v [T, kh, d];
 * row strides ld* in elements; lse fp32 [batch, a, seq] (natural log). */
RP_API rp_status rp_op_attn_fwd(void* stream, const void* q, const void* k, const void* v, void* o, float* lse, long ldq, long ldk,
                         long ldv, long ldo, int batch, int seq, int a, int kh, int d);
/* delta fp32 [batch, a, seq] is scratch (rowsum(dO*O)); dq [T,a,d], dk, dv [T,kh,d] overwritten.  scratch: device
 * fp32 [2, T, a, d], needed when a > kh (per-query-head partials of dk, dv, summed in head order); may be NULL when
 * a == kh. */
RP_API rp_status rp_op_attn_bwd(void* stream, const void* q, const void* k, const void* v, const void* o, const void* dout,
                         const float* lse, float* delta, void* dq, void* dk, void* dv, float* scratch, long ldq, long ldk,
                         long ldv, long ldo, long lddo, long lddq, long lddk, long lddv, int batch, int seq, int a, int kh,
                         int d);

/* Per-kernel timeline of the stage calls on a ctx (measurement aid; the only calls that synchronise).
 * rp_trace_start: from now on every kernel a stage/head call enqueues is preceded by a timing event (at most
 * max_records ops are recorded).  rp_trace_stop: waits for the compute stream, writes up to cap records
 * {kernel name, useful FLOPs, algorithmic HBM bytes, milliseconds} in launch order and the count into *n. */
typedef struct { char name[40]; double flops; double bytes; float ms; } rp_trace_record;
RP_API rp_status rp_trace_start(rp_ctx* ctx, int max_records);
RP_API rp_status rp_trace_stop(rp_ctx* ctx, rp_trace_record* out, int cap, int* n);

#ifdef __cplusplus
}
#endif
#endif
