/*
 * rp.h -- C ABI of the RoundPipe worker hot path on one MI355X (gfx950).
 *
 * A worker in the paper's computation-dispatch scheme is stateless: it is handed one pipeline
 * stage's weights (streamed from pinned host memory) and an activation, runs the stage and hands
 * the result back (Sec. 3.1; Sec. 4.1, "GPU worker"; Sec. 4.2, parameter-upload stream).  A
 * forward stage runs a contiguous range of decoder layers; a backward stage re-runs that forward
 * from the stored stage input keeping the internals, then back-propagates, accumulating weight
 * gradients in place (Sec. 3.2 "asymmetric stage splitting"; Sec. 4.1.1; App. C.3).  The LM head
 * with its loss is the oversized last stage and returns a scalar loss (Sec. 2.3, Sec. 4.1.1).
 *
 * General rules
 *  - Plain C99 types only.  Pointers marked [dev] are device pointers, [host] are host pointers,
 *    [pinned] are page-locked host pointers.  The caller owns every buffer; the library allocates
 *    no device memory and keeps only the configuration, HIP events and slot bookkeeping in rp_ctx.
 *  - All tensors are row-major and token-major: an activation is [T, features], T = batch*seq,
 *    sequences of one batch entry are contiguous.  bf16 unless stated.  Feature sizes (hidden,
 *    heads*head_dim, ffn, vocab, lora_rank) must be multiples of 8; T must be a multiple of 8.
 *  - Every call only enqueues work (compute calls on the compute stream given at creation, uploads
 *    on the copy stream) and returns; no call synchronises the device.  Ordering between an upload
 *    and the stage that uses the slot, and between a stage and the next upload into the same slot,
 *    is enforced on the device with events.
 *  - Return value: RP_OK or an error code; rp_last_error() gives a message.  Argument errors are
 *    detected before anything is enqueued, so a failed call has no side effects.
 *  - A ctx is used from one thread at a time.
 */
#ifndef RP_H
#define RP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#ifndef RP_API
#define RP_API __attribute__((visibility("default")))
#endif

typedef struct rp_ctx rp_ctx;

typedef enum {
  RP_OK = 0,
  RP_EINVAL = 1,       /* NULL pointer, bad size, bad id */
  RP_ENOMEM = 2,       /* workspace or slot too small */
  RP_EHIP = 3,         /* a HIP runtime call failed */
  RP_ESTATE = 4,       /* slot never uploaded / bound */
  RP_EUNSUPPORTED = 5  /* shape the kernels do not cover */
} rp_status;

/* lora_mask bits, in the order the adapters appear in the weight blob */
enum { RP_LORA_Q = 1, RP_LORA_K = 2, RP_LORA_V = 4, RP_LORA_O = 8, RP_LORA_GATE = 16, RP_LORA_UP = 32, RP_LORA_DOWN = 64 };

/* phases of rp_stage_backward */
enum { RP_PHASE_RECOMPUTE = 1, RP_PHASE_BACKWARD = 2, RP_PHASE_BOTH = 3 };

#define RP_MAX_SLOTS 4
#define RP_IGNORE_INDEX (-100)

/* One stage's shape.  Plain data; struct_size = sizeof(rp_stage_cfg) guards against layout drift. */
typedef struct {
  uint32_t struct_size;
  int32_t n_layers;    /* decoder layers in the stage; 0 = head-only stage */
  int32_t hidden;      /* h */
  int32_t n_q_heads;   /* a */
  int32_t n_kv_heads;  /* k; a % k == 0 */
  int32_t head_dim;    /* d in {64, 128} */
  int32_t ffn;         /* m (per expert for MoE) */
  int32_t vocab;       /* V; 0 = stage has no LM head */
  int32_t n_experts;   /* E; 0 = dense FFN */
  int32_t top_k;       /* E_act */
  float rope_base;     /* theta base, e.g. 1e6 */
  float rms_eps;       /* e.g. 1e-6 */
  int32_t qk_norm;     /* 1: per-head RMSNorm on q and k before RoPE */
  int32_t lora_rank;   /* r; 0 = no adapters */
  float lora_scale;    /* s in y = x W^T + s (x A^T) B^T */
  uint32_t lora_mask;  /* RP_LORA_* bits */
  int32_t train_base;  /* 1: base weights and norm gains receive fp32 gradients; 0: frozen */
  int32_t moe_router;  /* MoE only.  1: the layer chunk holds the router Wr [E, h] and the stage computes the router
                          logits n2 Wr^T itself (fp32);  0: the caller supplies the logits */
  int32_t head_chunk;  /* vocabulary rows per pass of the LM head (the logits of one pass are the largest buffer of its
                          workspace); 0 = automatic (32768, or 16384 for more than 4096 tokens), else a multiple of 256.
                          Enters rp_query_sizes like every other field. */
  int32_t head_two_sweeps; /* 0: the LM head makes one sweep over the vocabulary (a trainable head then keeps the
                          bf16 probabilities of the whole vocabulary, 2 * vocab * tokens bytes, in its workspace and
                          forms dW from them afterwards -- only while that is at most 4 GiB, else as 1);  1: the
                          two-sweep schedule (softmax statistics, then the logits
                          again for the gradients): no vocabulary-sized buffer, one more logit-sized product -- same
                          results within bf16 noise */
} rp_stage_cfg;

/* Tensor ids inside one layer's chunk of the weight blob (and of the gradient blob). */
typedef enum {
  RP_T_G1 = 0,   /* [h]                 input RMSNorm gain */
  RP_T_WQKV,     /* [a*d + 2*k*d, h]    rows: q heads, then k heads, then v heads */
  RP_T_GQ,       /* [d]                 per-head q norm gain (present only with qk_norm) */
  RP_T_GK,       /* [d] */
  RP_T_WO,       /* [h, a*d] */
  RP_T_G2,       /* [h]                 post-attention RMSNorm gain */
  RP_T_WGU,      /* dense [2m, h]: gate rows then up rows;  MoE [E, 2m, h] */
  RP_T_WD,       /* dense [h, m];  MoE [E, h, m] */
  RP_T_WR,       /* [E, h]              router (present only with moe_router) */
  RP_T_LA_Q, RP_T_LA_K, RP_T_LA_V,          /* LoRA A [r, h]  (enabled ones are adjacent)      */
  RP_T_LB_Q, RP_T_LB_K, RP_T_LB_V,          /* LoRA B [a*d, r], [k*d, r], [k*d, r]             */
  RP_T_LA_O, RP_T_LB_O,                     /* [r, a*d], [h, r]                                */
  RP_T_LA_GATE, RP_T_LA_UP,                 /* [r, h]                                          */
  RP_T_LB_GATE, RP_T_LB_UP,                 /* [m, r]                                          */
  RP_T_LA_DOWN, RP_T_LB_DOWN,               /* [r, m], [h, r]                                  */
  RP_T_GF,       /* head chunk: final RMSNorm gain [h] */
  RP_T_WV,       /* head chunk: LM head [V, h] */
  RP_T_COUNT
} rp_tensor_id;

/* ---- context ------------------------------------------------------------------------------- */

/* Creates a context for one stage shape on `device`.  compute_stream / copy_stream are hipStream_t
 * handles owned by the caller (both non-NULL, default priority).  Creates the per-slot, per-layer
 * events.  Mixture-of-experts stages (n_experts > 0; the MoE layer of App. B.2): the top_k experts of every token are
 * chosen from router logits the caller supplies; expert weights are frozen (train_base must be 0) and LoRA may adapt
 * the attention projections only -- other combinations return RP_EUNSUPPORTED.
 * Errors: RP_EINVAL (NULL, struct_size mismatch), RP_EUNSUPPORTED (shape), RP_EHIP. */
RP_API rp_status rp_ctx_create(rp_ctx** out, int device, void* compute_stream, void* copy_stream, const rp_stage_cfg* cfg);

/* Destroys events and frees the context.  The caller must have synchronised both streams. */
RP_API rp_status rp_ctx_destroy(rp_ctx* ctx);

/* Message of the last failed call on this ctx (NULL ctx: last failed ctx-less call). Valid until the next call. */
RP_API const char* rp_last_error(const rp_ctx* ctx);

/* ---- sizes and layouts (pure host functions, no HIP calls) ------------------------------------ */

/* weight_blob_bytes: size of the packed stage weights (host blob == device slot, same layout);
 * grad_blob_bytes: size of the fp32 gradient blob; workspace_bytes: device scratch a stage call or a
 * head call needs for (batch, seq).  Any output pointer may be NULL. */
RP_API rp_status rp_query_sizes(const rp_stage_cfg* cfg, int batch, int seq, size_t* weight_blob_bytes,
                         size_t* grad_blob_bytes, size_t* workspace_bytes);

/* Size of a device weight slot: the packed blob followed by the tensors the library derives from it when the weights
 * arrive (the block-diagonal LoRA B matrices of the fused q|k|v and gate|up projections).  Equal to weight_blob_bytes
 * for stages without such adapters. */
RP_API rp_status rp_slot_bytes(const rp_stage_cfg* cfg, size_t* slot_bytes);

/* Byte offset and element count of tensor `id` of layer `layer` (layer == n_layers addresses the head
 * chunk) inside the weight blob (bf16 elements).  n_elems == 0 when the tensor is absent. */
RP_API rp_status rp_weight_layout(const rp_stage_cfg* cfg, int layer, int id, size_t* byte_offset, size_t* n_elems);

/* Same for the fp32 gradient blob.  Base tensors and gains are present only with train_base. */
RP_API rp_status rp_grad_layout(const rp_stage_cfg* cfg, int layer, int id, size_t* byte_offset, size_t* n_elems);

/* Byte range [begin, end) of layer `layer`'s chunk in the weight blob (the unit of upload and of event gating). */
RP_API rp_status rp_weight_chunk(const rp_stage_cfg* cfg, int layer, size_t* begin, size_t* end);

/* ---- the four calls of the hot path ------------------------------------------------------------ */

/* Weight streaming (Sec. 4.2, parameter-upload stream).  Copies the packed stage weights from pinned host
 * memory into the caller-owned device slot, one hipMemcpyAsync per layer chunk on the copy stream, recording
 * one event per chunk so that layer l can start as soon as its own bytes have landed; behind a chunk's copy and before
 * its event, small kernels on the copy stream build the layer's derived tensors (see rp_slot_bytes) behind the blob.
 * Before copying, the copy stream waits for the last stage call that read this slot.  bytes must equal
 * weight_blob_bytes.  host_blob [pinned], dev_slot [dev, at least rp_slot_bytes].  Errors: RP_EINVAL, RP_EHIP. */
RP_API rp_status rp_stage_upload_weights(rp_ctx* ctx, int slot_id, void* dev_slot, const void* host_blob, size_t bytes);

/* Marks a device slot (at least rp_slot_bytes) whose first `bytes` = weight_blob_bytes already hold packed weights
 * (written on the compute stream or before it) as slot `slot_id` without copying; the derived tensors are built on the
 * compute stream; later stage calls on the slot wait for nothing. */
RP_API rp_status rp_stage_bind_weights(rp_ctx* ctx, int slot_id, void* dev_slot, size_t bytes);

/* Forward stage (Sec. 3.2): x_out = layers(x_in).  x_in, x_out [dev] bf16 [T, h] (may not alias).
 * layer_inputs_out [host array of n_layers dev pointers, or NULL]: entry l, when non-NULL, receives a copy of the
 * input of layer l (the activation checkpoint kept under full recomputation, Sec. 2.1.1).
 * router_logits [dev] fp32 [n_layers, T, E] for MoE stages, else NULL: read when the caller supplies the logits,
 * overwritten with the logits the stage computed when cfg.moe_router is set (the library keeps no copy of its own).
 * Waits on the slot's per-layer upload events.  workspace [dev], at least workspace_bytes of rp_query_sizes.
 * Errors: RP_EINVAL, RP_ENOMEM (workspace), RP_ESTATE (slot not uploaded), RP_EHIP. */
RP_API rp_status rp_stage_forward(rp_ctx* ctx, int slot_id, const void* x_in, void* x_out, void* const* layer_inputs_out,
                           float* router_logits, int batch, int seq, void* workspace, size_t workspace_bytes);

/* Backward stage with recomputation (Sec. 3.2; App. C.3).  Phase RP_PHASE_RECOMPUTE re-runs the forward from the
 * stored stage input x_in keeping every layer's internals in the workspace; phase RP_PHASE_BACKWARD runs the backward
 * in reverse layer order from those internals.  RP_PHASE_BOTH is the ordinary backward stage.  The fused stage of the
 * last layers (Sec. 3.2: its forward doubles as the recomputation) calls RECOMPUTE, then the LM head on x_out, then
 * BACKWARD with the head's dx as dy -- with the same workspace, untouched in between, and the same x_in.
 * dy [dev] bf16 [T, h]: gradient of the stage output;  dx [dev] bf16 [T, h]: overwritten with the gradient of x_in;
 * x_out [dev] bf16 [T, h] or NULL: receives the recomputed stage output;  grads [dev]: fp32 gradient blob,
 * ACCUMULATED (+=) -- the in-place accumulation over micro-batches of Sec. 4.1.1;  router_logits / d_router_logits
 * [dev] fp32 [n_layers, T, E] (MoE only; the latter may be NULL, else it is overwritten with the gradient of the
 * router logits: w_e (dw_e - sum_e' w_e' dw_e') on the selected experts, zero elsewhere).  With cfg.moe_router the
 * RECOMPUTE phase writes router_logits, and the BACKWARD phase adds dlogits Wr to the gradient of n2.
 * dy, dx, grads are ignored by RECOMPUTE alone, x_out by BACKWARD alone.  Errors as rp_stage_forward. */
RP_API rp_status rp_stage_backward(rp_ctx* ctx, int slot_id, int phases, const void* x_in, const void* dy, void* dx,
                            void* x_out, void* grads, float* router_logits, float* d_router_logits, int batch,
                            int seq, void* workspace, size_t workspace_bytes);

/* LM head fused with the mean cross-entropy, forward and backward in one call (the oversized last stage, Sec. 2.3;
 * returns a scalar loss, Sec. 4.1.1).  xf = rmsnorm(x; gf); Z = xf Wv^T is produced tile by tile and reduced on
 * the fly, never stored at [T, V] (fp32 logits exist for one vocabulary chunk at most; see cfg.head_two_sweeps for
 * the bf16 probabilities a trainable head may keep);  loss = mean over rows with label != RP_IGNORE_INDEX of (logsumexp Z_t - Z[t, y_t]);
 * dZ = grad_scale (softmax - onehot) / N_valid.
 * x [dev] bf16 [T, h]; labels [dev] int32 [T]; loss_out [dev] one fp32; dx [dev] bf16 [T, h] overwritten;
 * grads [dev]: the stage's fp32 gradient blob (the one rp_stage_backward takes); its head chunk {gf [h], Wv [V, h]}
 * is accumulated when train_base is set; NULL = frozen head.  Uses the head chunk (layer index n_layers) of the
 * slot.  The workspace is overwritten from its start: between the two phases of a fused last stage give the head
 * a workspace of its own.  Errors as rp_stage_forward. */
RP_API rp_status rp_lmhead_ce_fwd_bwd(rp_ctx* ctx, int slot_id, const void* x, const int32_t* labels, float* loss_out,
                               void* dx, void* grads, float grad_scale, int batch, int seq, void* workspace,
                               size_t workspace_bytes);

/* ---- a round: one stage over M micro-batches whose activations live in host memory (Sec. 4.2) ---------------- */

/* One piece of a transfer plan: bytes [offset, offset + bytes) of item `item`, sent in window `window`. */
typedef struct {
  int32_t item;
  int32_t window;
  size_t offset;
  size_t bytes;
} rp_piece;

/* Packing of parameter / gradient transfers into the n_windows data-transfer windows of a round (Sec. 4.2, "Scheduling
 * parameter transfers"): items (tensors) larger than max_piece_bytes are first split into equal pieces (multiples of
 * 256 bytes, the last one shorter); the pieces are taken in descending size (ties: lower item, lower offset) and each
 * goes to the window that holds the fewest bytes so far (ties: lower window) -- longest-processing-time-first.
 * pieces [host, capacity entries] receives them in the order they were assigned; *n_pieces their number.
 * Pure host function.  Errors: RP_EINVAL (NULL, n_windows <= 0, max_piece_bytes 0 or not a multiple of 256),
 * RP_ENOMEM (capacity too small; *n_pieces then holds the number needed). */
RP_API rp_status rp_plan_transfers(const size_t* item_bytes, int n_items, int n_windows, size_t max_piece_bytes,
                            rp_piece* pieces, int capacity, int* n_pieces);

/* The three further transfer streams of the multi-stream worker (Sec. 4.2, "The multi-stream architecture"):
 * activation upload, activation download, gradient download; the copy stream given at creation is the parameter
 * upload stream.  hipStream_t handles owned by the caller, default priority.  Needed by the rp_round_* calls only. */
RP_API rp_status rp_ctx_set_transfer_streams(rp_ctx* ctx, void* act_upload_stream, void* act_download_stream,
                                      void* grad_download_stream);

/* What a round moves.  Every [pinned] array has n_micro entries of bf16 [T, h]; the [dev] staging buffers are bf16
 * [T, h] each, two per direction (micro-batch j uses entry j & 1). */
typedef struct {
  uint32_t struct_size;
  int32_t n_micro;             /* M in [1, 256]: micro-batches the stage processes with one set of weights (Sec. 3.1) */
  const void* const* x_host;   /* [pinned] stage inputs */
  const void* const* dy_host;  /* [pinned] gradients of the stage outputs (backward rounds; else NULL) */
  void* const* out_host;       /* [pinned] forward round: stage outputs;  backward round: gradients of the inputs */
  void* x_dev[2];              /* [dev] */
  void* dy_dev[2];             /* [dev] backward rounds */
  void* out_dev[2];            /* [dev] */
  int32_t next_slot;           /* slot that receives the next stage's weights during this round, or -1 */
  void* next_dev_slot;         /* [dev]    as in rp_stage_upload_weights (at least rp_slot_bytes) */
  const void* next_host_blob;  /* [pinned] */
  const void* done_grads_dev;  /* [dev] fp32 gradient blob of a stage that has finished, to be sent home, or NULL */
  void* done_grads_host;       /* [pinned] receives it */
  size_t max_piece_bytes;      /* tensors above this are split before scheduling; 0 = 64 MiB */
} rp_round_io;

/* Runs the stage in slot `slot_id` over n_micro micro-batches the way the paper's worker does (Sec. 4.2, Fig.
 * "multi-stream workflow"): micro-batch j+1's activations are uploaded while micro-batch j computes (one micro-batch
 * early), results are downloaded while the next one computes (one micro-batch late), the compute stream meets the two
 * activation streams once per micro-batch through events, and the round's M windows each carry one chunk of the next
 * stage's parameters (upload) and of a finished stage's gradients (download), placed behind the window's activation
 * transfer so that they do not compete with it; the chunks are those of rp_plan_transfers over the tensors of the
 * respective blob.  When the call returns everything is enqueued; out_host / done_grads_host are complete once the
 * activation-download / gradient-download streams have drained, next_slot is usable by later calls on this ctx at once
 * (they wait on its events).  Forward round: out = layers(x).  Backward round: recomputation + backward per micro-batch,
 * weight gradients accumulated into `grads` [dev] over the M micro-batches (Sec. 4.1.1).  Dense stages only.
 * Consecutive rounds on the same staging buffers overlap like the micro-batches inside one (the first upload of a
 * round waits only for the predecessor's last use of that buffer); with other buffers the round first waits for
 * everything enqueued on the compute and activation-download streams so far.  A stream may serve several roles (the
 * activation upload may share the parameter-upload stream, the gradient download the activation-download stream):
 * with the runtime's default of four hardware queues per process, one transfer stream per direction is the faster
 * arrangement.
 * Errors: as rp_stage_forward / rp_stage_backward, RP_ESTATE when the transfer streams were not set, RP_EUNSUPPORTED
 * for MoE stages. */
RP_API rp_status rp_round_forward(rp_ctx* ctx, int slot_id, const rp_round_io* io, int batch, int seq, void* workspace,
                           size_t workspace_bytes);
RP_API rp_status rp_round_backward(rp_ctx* ctx, int slot_id, const rp_round_io* io, void* grads, int batch, int seq,
                            void* workspace, size_t workspace_bytes);

/* ---- automatic stage partitioning (Sec. 4.4) ---------------------------------------------------------------- */

/* Splits n_layers consecutive layers (the LM head counts as the last one) into forward stages F_1..F_Sf over the front
 * layers and backward stages B_1..B_Sb over all layers, B_1 being the fused stage of the last layers whose forward
 * doubles as the recomputation (Sec. 3.2, asymmetric stage splitting: sum F_i + B_1 = sum B_j = n_layers), so that
 * (n_micro * (Sf + Sb) + n_gpus * (n_gpus - 1)) * t_max is smallest (the GPU time of Sec. 3.3, bubble analysis; t_max =
 * the longest stage) while no stage's memory exceeds mem_limit.  t_fwd[l]: forward time of layer l; t_bwd[l]: its
 * backward time including recomputation (also its time inside the fused stage); mem_fwd / mem_bwd: what layer l adds to
 * a forward / backward stage's footprint.  Algorithm as in the paper: every contiguous run of forward or of backward
 * times is a candidate for t_max; for a candidate the stages are packed greedily -- the fused stage first, as full as
 * possible, then the other backward stages towards the front, then the forward stages from the front -- which gives
 * the fewest stages for that bound; O(n_layers^3) in all.  Ties in cost: fewer stages, then the candidate met first
 * (forward runs before backward runs, by start then end).
 * fwd_layers, bwd_layers [host, n_layers entries each] receive the stage sizes, *n_fwd / *n_bwd their counts
 * (bwd_layers[0] = B_1, the last layers); t_max, cost may be NULL.  Pure host function.
 * Errors: RP_EINVAL (NULL, non-positive counts, negative or NaN inputs), RP_EUNSUPPORTED (a layer alone exceeds
 * mem_limit). */
RP_API rp_status rp_partition_stages(int n_layers, const double* t_fwd, const double* t_bwd, const double* mem_fwd,
                              const double* mem_bwd, double mem_limit, int n_gpus, int n_micro, int* fwd_layers, int* n_fwd,
                              int* bwd_layers, int* n_bwd, double* t_max, double* cost);

#ifdef __cplusplus
}
#endif
#endif /* RP_H */
