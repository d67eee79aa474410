// Stage executor and C ABI: weight upload with per-layer events, forward stage, backward stage with recomputation,
// LM head fused with cross-entropy.  Host code only enqueues kernels; nothing here synchronises the device.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>
#include <mutex>
#include <new>

#include "../../include/rp.h"
#include "../../include/rp_ops.h"
#include "gemm.hpp"
#include "kernels.hpp"
#include "layout.hpp"
#include "transfers.hpp"

using namespace rp;

// Scratch memory of the entry point that allocates nothing (rp_op_rmsnorm_bwd_noalloc): 16 MiB in the code object.
constexpr int NOALLOC_MAX_H = 4096;                                  // widest row that entry point accepts
constexpr size_t NOALLOC_FLOATS = (size_t)RP_PARTIAL_BLOCKS * NOALLOC_MAX_H;
static __device__ __align__(256) float scratch[NOALLOC_FLOATS];

namespace {

typedef unsigned short bf16_t;   // host code never does bf16 arithmetic; this is only for pointer stepping

struct Slot {
  void* dev = nullptr;
  size_t bytes = 0;
  bool valid = false;     // uploaded or bound
  bool gated = false;     // stage calls must wait on the per-chunk events
  bool used = false;      // a stage call has read the slot since the last upload
  hipEvent_t* ev = nullptr;   // n_layers + 1 events
  hipEvent_t free_ev = nullptr;
};

char g_err[512];

// ---- scratch memory for the entry point that allocates nothing -----------------------------------------------------
// One array per GPU the library runs on, resident until the process ends.  In host code the array's name is only a
// stand-in: its device address is looked up once per device (with that device current) and kept here; kernels, fills
// and copies are always given that pointer.
constexpr int MAX_DEVICES = 64;
float* g_scratch_ptr[MAX_DEVICES];
std::mutex g_scratch_mutex;

// Device address of this GPU's copy of `scratch` (the current device).  No allocation: the symbol lives in the code
// object.  Returns NULL and sets *err when the look-up fails.
float* noalloc_scratch(hipError_t* err) {
  int dev = -1;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= MAX_DEVICES) { *err = hipErrorInvalidDevice; return nullptr; }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    *err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (*err != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = static_cast<float*>(ptr);
  }
  return g_scratch_ptr[dev];
}

}  // namespace

struct TraceRec { char name[40]; double flops, bytes; };

struct rp_ctx {
  rp_stage_cfg cfg;
  int device;
  hipStream_t compute, copy;
  Slot slots[RP_MAX_SLOTS];
  BlobLayout wl, gl;
  DerivedLayout dl;
  char err[512];
  // optional per-kernel timeline: one event before every enqueued op, one after the last
  bool tracing = false;
  int trace_cap = 0, trace_n = 0;
  hipEvent_t* trace_ev = nullptr;   // trace_cap + 1 events
  TraceRec* trace_rec = nullptr;
  // rounds: activation upload / download and gradient download streams, and the events that tie them to compute
  hipStream_t act_up = nullptr, act_down = nullptr, grad_down = nullptr;
  hipEvent_t* round_ev = nullptr;   // two halves, used by alternate rounds, so that a round can wait on its predecessor's
  int round_ev_n = 0;               // events while recording its own
  // the previous round: its staging buffers and the events of the last compute / download that used each of them
  int round_parity = 0;
  bool prev_round = false;
  void* prev_x[2] = {nullptr, nullptr}; void* prev_out[2] = {nullptr, nullptr}; void* prev_dy[2] = {nullptr, nullptr};
  hipEvent_t prev_done[2] = {nullptr, nullptr}, prev_down[2] = {nullptr, nullptr};
};

namespace {

rp_status fail(rp_ctx* ctx, rp_status code, const char* fmt, ...) {
  char* dst = ctx ? ctx->err : g_err;
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(dst, 512, fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(ctx, expr)                                                                              \
  do {                                                                                                  \
    hipError_t e_ = (expr);                                                                             \
    if (e_ != hipSuccess) return fail(ctx, RP_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_));      \
  } while (0)

// Enqueue one non-GEMM op: timeline mark (name, useful FLOPs, algorithmic HBM bytes), then the launch.
#define RUN(X, name, flops, bytes, call) \
  do { (X).mark(name, (double)(flops), (double)(bytes)); (X).chk(call, name); } while (0)

rp_status validate_cfg(const rp_stage_cfg* c, rp_ctx* ctx) {
  if (!c) return fail(ctx, RP_EINVAL, "cfg is NULL");
  if (c->struct_size != sizeof(rp_stage_cfg)) return fail(ctx, RP_EINVAL, "cfg.struct_size %u != %zu", c->struct_size, sizeof(rp_stage_cfg));
  if (c->n_layers < 0 || c->vocab < 0 || (c->n_layers == 0 && c->vocab == 0)) return fail(ctx, RP_EINVAL, "stage has neither layers nor a head");
  if (c->hidden <= 0 || c->hidden % 8 || c->hidden > 8192) return fail(ctx, RP_EUNSUPPORTED, "hidden must be a multiple of 8 in (0, 8192]");
  if (c->vocab % 8) return fail(ctx, RP_EUNSUPPORTED, "vocab must be a multiple of 8");
  if (c->head_chunk < 0 || c->head_chunk % 256) return fail(ctx, RP_EINVAL, "head_chunk must be 0 or a positive multiple of 256");
  if (c->head_two_sweeps != 0 && c->head_two_sweeps != 1) return fail(ctx, RP_EINVAL, "head_two_sweeps must be 0 or 1");
  if (c->n_layers > 0) {
    if (c->head_dim != 64 && c->head_dim != 128) return fail(ctx, RP_EUNSUPPORTED, "head_dim must be 64 or 128");
    if (c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->n_q_heads % c->n_kv_heads) return fail(ctx, RP_EINVAL, "n_q_heads must be a positive multiple of n_kv_heads");
    if (c->ffn <= 0 || c->ffn % 8) return fail(ctx, RP_EUNSUPPORTED, "ffn must be a positive multiple of 8");
    if (c->lora_rank < 0 || c->lora_rank % 8 || c->lora_rank > 64) return fail(ctx, RP_EUNSUPPORTED, "lora_rank must be a multiple of 8, at most 64");
    if (c->lora_mask >> 7) return fail(ctx, RP_EINVAL, "lora_mask has unknown bits");
    if (c->n_experts < 0 || c->top_k < 0 || (c->n_experts > 0 && (c->top_k <= 0 || c->top_k > c->n_experts))) return fail(ctx, RP_EINVAL, "bad n_experts/top_k");
    if (c->n_experts > 1024 || c->top_k > 64) return fail(ctx, RP_EUNSUPPORTED, "at most 1024 experts and top_k 64");
    if (c->n_experts > 0 && c->train_base) return fail(ctx, RP_EUNSUPPORTED, "expert weights are frozen in this build: train_base must be 0 for MoE stages");
    if (c->moe_router != 0 && c->moe_router != 1) return fail(ctx, RP_EINVAL, "moe_router must be 0 or 1");
    if (c->moe_router && c->n_experts == 0) return fail(ctx, RP_EINVAL, "moe_router needs n_experts > 0");
    if (c->moe_router && c->n_experts % 8) return fail(ctx, RP_EUNSUPPORTED, "with moe_router, n_experts must be a multiple of 8");
    if (c->n_experts > 0 && c->lora_rank > 0 && (c->lora_mask & (RP_LORA_GATE | RP_LORA_UP | RP_LORA_DOWN))) return fail(ctx, RP_EUNSUPPORTED, "LoRA on expert projections is not implemented");
    if (!(c->rms_eps >= 0.f) || !(c->rope_base > 1.f)) return fail(ctx, RP_EINVAL, "bad rms_eps / rope_base");
  }
  return RP_OK;
}

rp_status validate_shape(rp_ctx* ctx, int batch, int seq) {
  if (batch <= 0 || seq <= 0) return fail(ctx, RP_EINVAL, "batch and seq must be positive");
  if (((long)batch * seq) % 8) return fail(ctx, RP_EUNSUPPORTED, "batch*seq must be a multiple of 8");
  if ((long)batch * seq > (1L << 24)) return fail(ctx, RP_EUNSUPPORTED, "batch*seq too large");
  return RP_OK;
}

// ---- pointers into one layer's chunk ------------------------------------------------------------------------------
struct LayerW {
  const char* base;
  const BlobLayout* L;
  const char* derived = nullptr;    // this layer's derived tensors (block-diagonal LoRA B) behind the blob in the slot
  const bf16_t* t(int id) const { return L->elems[id] ? reinterpret_cast<const bf16_t*>(base + L->off[id]) : nullptr; }
};
struct LayerG {
  char* base;   // may be NULL (no gradient blob)
  const BlobLayout* L;
  float* t(int id) const { return (base && L->elems[id]) ? reinterpret_cast<float*>(base + L->off[id]) : nullptr; }
};

struct Exec {
  rp_ctx* ctx;
  hipStream_t st;
  Dims D;
  int batch, seq;
  long T;
  char* ws;
  Plan P;
  hipError_t err = hipSuccess;
  const char* where = "";
  bool fwd_only = false;           // the forward-stage plan of the workspace is in use (rp_stage_forward)
  size_t split_off = 0;            // scratch for the partial products of a GEMM reduction split, in the plan in use
  bool has_split = false;
  float* router = nullptr;         // router logits of the layer being run, fp32 [T, E] (mixture of experts): read, or
                                   // written first when the stage holds the router weights
  float* d_router = nullptr;       // their gradient (optional)

  void chk(hipError_t e, const char* w) { if (err == hipSuccess && e != hipSuccess) { err = e; where = w; } }
  // Called right before an op is enqueued when the timeline is on: records the op's start event and its cost model.
  void mark(const char* name, double flops, double bytes) {
    if (!ctx->tracing || ctx->trace_n >= ctx->trace_cap) return;
    const int i = ctx->trace_n++;
    snprintf(ctx->trace_rec[i].name, sizeof(ctx->trace_rec[i].name), "%s", name);
    ctx->trace_rec[i].flops = flops;
    ctx->trace_rec[i].bytes = bytes;
    chk(hipEventRecord(ctx->trace_ev[i], st), "trace event");
  }
  void mark_gemm(int layout, const GemmArgs& g) {
    if (!ctx->tracing) return;
    static const char* lay[3] = {"NT", "NN", "TN"};
    static const char* til[6] = {"", "256x256", "256x128", "128x128", "128x64", "256x128k2"};
    char nm[40];
    snprintf(nm, sizeof(nm), "gemm_%s_%s", til[gemm_pick_tile(g)], lay[layout]);
    const double out_b = (g.epi == EPI_BF16 || g.epi == EPI_CE_DZ || g.epi == EPI_CE_P) ? 2.0
                         : g.epi == EPI_SWIGLU_BWD ? 4.0 : g.epi == EPI_SWIGLU_FWD ? 3.0 : (g.epi == EPI_CE_STATS ? 0.0 : 4.0 * (1 + g.beta));
    mark(nm, 2.0 * g.M * (double)g.N * ((double)g.K + g.K2),
         2.0 * ((double)g.M * g.K + (double)g.N * g.K + (double)g.M * g.K2 + (double)g.N * g.K2) + out_b * g.M * (double)g.N +
             (g.R ? (g.epi == EPI_SWIGLU_BWD ? 4.0 : 2.0) * g.M * (double)g.N : 0.0));
  }
  template <typename Tp> Tp* at(size_t off) const { return reinterpret_cast<Tp*>(ws + off); }
  void give_split_ws(GemmArgs& g) const {
    if (has_split) { g.split_ws = at<float>(split_off); g.split_ws_bytes = RP_SPLITK_WS_BYTES; }
  }

  // C[M,N] (bf16) = alpha * A * op(B) (+ second pair) (+ R)
  void gemm_bf16(int layout, const void* A, long lda, const void* B, long ldb, void* C, long ldc, int M, int N, int K,
                 float alpha = 1.f, const void* A2 = nullptr, long lda2 = 0, const void* B2 = nullptr, long ldb2 = 0,
                 int K2 = 0, const void* R = nullptr, long ldr = 0, int epi = EPI_BF16, void* C2 = nullptr, long ldc2 = 0) {
    GemmArgs g; gemm_zero_args(g);
    g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc; g.M = M; g.N = N; g.K = K; g.alpha = alpha;
    g.A2 = A2; g.lda2 = lda2; g.B2 = B2; g.ldb2 = ldb2; g.K2 = K2; g.R = R; g.ldr = ldr; g.epi = epi; g.C2 = C2; g.ldc2 = ldc2;
    mark_gemm(layout, g);
    chk(gemm_launch(st, layout, g), "gemm_bf16");
  }
  // C[M,N] (bf16) = alpha * A * op(B) for a skinny N (the LoRA down-projections, N = a few ranks): the product is bound by
  // reading A once, and with so few output tiles only a reduction split puts enough workgroups on the chip.  The
  // slices write fp32 partial products that are added in slice order and converted by the merge kernel.
  void gemm_skinny_bf16(int layout, const void* A, long lda, const void* B, long ldb, void* C, int M, int N, int K, float alpha) {
    GemmArgs g; gemm_zero_args(g);
    g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = N; g.M = M; g.N = N; g.K = K; g.alpha = alpha;
    g.epi = EPI_BF16;
    if (has_split && (size_t)M * N * 4 <= RP_SPLITK_WS_BYTES) { g.epi = EPI_F32; g.split_out_bf16 = 1; give_split_ws(g); }
    mark_gemm(layout, g);
    chk(gemm_launch(st, layout, g), "gemm_skinny");
  }
  // Grouped GEMM over expert-sorted slot rows: C[slot, N] = A[row_map ? row_map[slot] : slot, K] * op(B_e), B_e the
  // matrix of the expert that owns the slot.  set = the layer's saved internals (routing plan).
  void gemm_grouped(int layout, const char* set, const void* A, long lda, int a_rows, bool gather, const void* B, long ldb,
                    long strideB, void* C, long ldc, int N, int K, void* act = nullptr) {
    GemmArgs g; gemm_zero_args(g);
    const long Tk = T * D.topk;
    g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc; g.M = (int)Tk; g.N = N; g.K = K; g.epi = EPI_BF16;
    if (act) { g.epi = EPI_SWIGLU_FWD; g.C2 = act; g.ldc2 = N / 2; }   // gate | up columns: silu(gate) * up from the epilogue
    g.grp_tab = reinterpret_cast<const int4*>(set + P.lb.m_tab);
    g.grp_ntiles = reinterpret_cast<const int*>(set + P.lb.m_ntiles);
    g.grp_max_tiles = P.moe_max_tiles;
    g.grp_strideB = strideB;
    if (gather) { g.row_map = reinterpret_cast<const int*>(set + P.lb.m_tok); g.row_map_rows = a_rows; }
    if (ctx->tracing) {
      char nm[40];
      snprintf(nm, sizeof(nm), "gemm_grouped_%s", layout == GEMM_NT ? "NT" : "NN");
      // every expert's weights are read once; rows as in the dense case
      mark(nm, 2.0 * Tk * (double)N * K, 2.0 * ((double)Tk * K + (double)D.E * N * K) + (act ? 3.0 : 2.0) * Tk * (double)N);
    }
    chk(gemm_launch(st, layout, g), "gemm_grouped");
  }
  // C[M,N] (fp32) = A * B^T, overwritten; one pass, no reduction split, so the result does not depend on scheduling
  void gemm_f32_nt(const void* A, long lda, const void* B, long ldb, float* C, long ldc, int M, int N, int K) {
    GemmArgs g; gemm_zero_args(g);
    g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc; g.M = M; g.N = N; g.K = K; g.beta = 0; g.epi = EPI_F32;
    mark_gemm(GEMM_NT, g);
    chk(gemm_launch(st, GEMM_NT, g), "gemm_f32_nt");
  }
  // C[M,N] (fp32) (+)= A^T * B : weight-gradient form, reduction over the rows of A and B
  void gemm_wgrad(const void* A, long lda, const void* B, long ldb, float* C, long ldc, int M, int N, int K) {
    if (!C) return;
    GemmArgs g; gemm_zero_args(g);
    g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc; g.M = M; g.N = N; g.K = K; g.beta = 1; g.epi = EPI_F32;
    give_split_ws(g);
    mark_gemm(GEMM_TN, g);
    chk(gemm_launch(st, GEMM_TN, g), "gemm_wgrad");
  }
};

// Which LoRA adapters feed a fused projection: ids of A/B tensors, row ranges in the fused output.
struct FusedLora {
  int n = 0;               // adapted projections
  int a_id[3], b_id[3], row0[3], row1[3];
};

FusedLora fused_qkv(const Dims& D) {
  FusedLora f;
  const int a_ids[3] = {RP_T_LA_Q, RP_T_LA_K, RP_T_LA_V}, b_ids[3] = {RP_T_LB_Q, RP_T_LB_K, RP_T_LB_V};
  const int r0[3] = {0, D.qd, D.qd + D.kd}, r1[3] = {D.qd, D.qd + D.kd, D.n1};
  for (int i = 0; i < 3; ++i)
    if (D.lora[i]) { f.a_id[f.n] = a_ids[i]; f.b_id[f.n] = b_ids[i]; f.row0[f.n] = r0[i]; f.row1[f.n] = r1[i]; ++f.n; }
  return f;
}
FusedLora fused_gu(const Dims& D) {
  FusedLora f;
  const int a_ids[2] = {RP_T_LA_GATE, RP_T_LA_UP}, b_ids[2] = {RP_T_LB_GATE, RP_T_LB_UP};
  const int r0[2] = {0, D.m}, r1[2] = {D.m, 2 * D.m};
  for (int i = 0; i < 2; ++i)
    if (D.lora[4 + i]) { f.a_id[f.n] = a_ids[i]; f.b_id[f.n] = b_ids[i]; f.row0[f.n] = r0[i]; f.row1[f.n] = r1[i]; ++f.n; }
  return f;
}
FusedLora fused_single(bool on, int a_id, int b_id, int rows) {
  FusedLora f;
  if (on) { f.n = 1; f.a_id[0] = a_id; f.b_id[0] = b_id; f.row0[0] = 0; f.row1[0] = rows; }
  return f;
}

// The B operand of a fused projection's LoRA product: the block-diagonal B [N, n*r] kept behind the blob in the slot
// (derived_off = its offset in the layer's derived tensors), or the plain B when one adapter covers the whole output.
const void* lora_b_matrix(const LayerW& W, const FusedLora& f, int N, size_t derived_off) {
  if (f.n == 0) return nullptr;
  if (f.n == 1 && f.row0[0] == 0 && f.row1[0] == N) return W.t(f.b_id[0]);
  return W.derived + derived_off;
}

// Enqueues on `st` the kernels that build layer `l`'s derived tensors from the layer's chunk in the slot.
hipError_t build_derived(const rp_ctx* ctx, hipStream_t st, char* slot, int l);

// Y[T,N] = X W^T (+ LoRA) (+ R).  u_buf receives U = s * X A^T (kept for the backward).
// act (optional, N = 2m, gate | up): the product's epilogue also writes silu(gate) * up [T, m] there.
void linear_fwd(Exec& X, const LayerW& W, int w_id, const FusedLora& f, size_t bd_off, const void* x, int K, void* y,
                int N, void* u_buf, const void* R, void* act = nullptr) {
  const int nr = f.n * X.D.r;
  const void* Bm = nullptr;
  if (f.n) {
    Bm = lora_b_matrix(W, f, N, bd_off);
    X.gemm_skinny_bf16(GEMM_NT, x, K, W.t(f.a_id[0]), K, u_buf, (int)X.T, nr, K, X.ctx->cfg.lora_scale);
  }
  X.gemm_bf16(GEMM_NT, x, K, W.t(w_id), K, y, N, (int)X.T, N, K, 1.f, f.n ? u_buf : nullptr, nr, Bm, nr, f.n ? nr : 0, R, N,
              act ? EPI_SWIGLU_FWD : EPI_BF16, act, N / 2);
}

// dX[T,K] = dY W (+ LoRA);  dW += dY^T X;  LoRA gradients.  u_buf = U saved by the forward, ud = scratch [T, n*r].
// sw_gu (optional): x = silu(gate) * up of the [T, 2K] buffer sw_gu; instead of dx ([T, K]) the input-gradient GEMM
// then writes d gate | d up into sw_dgu ([T, 2K]) from its epilogue.
void linear_bwd(Exec& X, const LayerW& W, const LayerG& G, int w_id, const FusedLora& f, size_t bd_off, const void* dy,
                int N, const void* x, int K, void* dx, const void* u_buf, const void* sw_gu = nullptr, void* sw_dgu = nullptr) {
  const int nr = f.n * X.D.r;
  void* ud = X.at<void>(X.P.ud);
  const void* Bm = nullptr;
  if (f.n) {
    Bm = lora_b_matrix(W, f, N, bd_off);
    X.gemm_skinny_bf16(GEMM_NN, dy, N, Bm, nr, ud, (int)X.T, nr, N, X.ctx->cfg.lora_scale);
  }
  if (sw_gu)
    X.gemm_bf16(GEMM_NN, dy, N, W.t(w_id), K, sw_dgu, 2 * K, (int)X.T, K, N, 1.f, f.n ? ud : nullptr, nr,
                f.n ? W.t(f.a_id[0]) : nullptr, K, f.n ? nr : 0, sw_gu, 2 * K, EPI_SWIGLU_BWD);
  else
    X.gemm_bf16(GEMM_NN, dy, N, W.t(w_id), K, dx, K, (int)X.T, K, N, 1.f, f.n ? ud : nullptr, nr, f.n ? W.t(f.a_id[0]) : nullptr,
                K, f.n ? nr : 0);
  X.gemm_wgrad(dy, N, x, K, G.t(w_id), K, N, K, (int)X.T);
  if (f.n) {
    // the adapted A matrices are adjacent in both blobs, so one product fills all of them
    X.gemm_wgrad(ud, nr, x, K, G.t(f.a_id[0]), K, nr, K, (int)X.T);
    for (int i = 0; i < f.n; ++i)
      X.gemm_wgrad(reinterpret_cast<const bf16_t*>(dy) + f.row0[i], N, reinterpret_cast<const bf16_t*>(u_buf) + i * X.D.r, nr,
                   G.t(f.b_id[i]), X.D.r, f.row1[i] - f.row0[i], X.D.r, (int)X.T);
  }
}

// moe_f_off: workspace offset of the per-slot expert output buffer of the plan in use (forward or backward stage).
void layer_forward(Exec& X, const LayerW& W, char* set, const void* x, void* z, size_t moe_f_off) {
  const Dims& D = X.D;
  const LayerBuf& b = X.P.lb;
  const rp_stage_cfg& c = X.ctx->cfg;
  const int T = (int)X.T;
  auto S = [&](size_t off) { return reinterpret_cast<void*>(set + off); };
  bf16_t* qkv = reinterpret_cast<bf16_t*>(S(b.qkv));

  const double Td = (double)T;
  RUN(X, "rmsnorm_fwd", 0, 4.0 * Td * D.h, k_rmsnorm_fwd(X.st, x, W.t(RP_T_G1), S(b.n1), (float*)S(b.rstd1), T, D.h, c.rms_eps));
  linear_fwd(X, W, RP_T_WQKV, fused_qkv(D), X.ctx->dl.bd1, S(b.n1), D.h, qkv, D.n1, S(b.u1), nullptr);
  RUN(X, "qknorm_rope_fwd", 0, 4.0 * Td * (D.qd + D.kd),
      k_qknorm_rope(X.st, 0, D.d, qkv, qkv + D.qd, D.n1, D.n1, S(b.qr), S(b.kr), D.qd, D.kd, W.t(RP_T_GQ), W.t(RP_T_GK),
                    (float*)S(b.rstd_q), (float*)S(b.rstd_k), nullptr, nullptr, 0, nullptr, nullptr, nullptr,
                    X.at<float2>(X.P.rope), T, X.seq, D.a, D.kh, c.qk_norm, c.rms_eps));
  const double s2qd = (double)X.batch * X.seq * (double)X.seq * D.qd;   // causal attention: 2 s^2 qd forward per sequence
  RUN(X, "attn_fwd", 2.0 * s2qd, 2.0 * Td * (2 * D.qd + 2 * D.kd),
      k_attn_fwd(X.st, S(b.qr), S(b.kr), qkv + D.qd + D.kd, S(b.o), (float*)S(b.lse), D.qd, D.kd, D.n1, D.qd, X.batch,
                 X.seq, D.a, D.kh, D.d));
  linear_fwd(X, W, RP_T_WO, fused_single(D.lora[3], RP_T_LA_O, RP_T_LB_O, D.h), 0, S(b.o), D.qd, S(b.y), D.h, S(b.u2), x);
  RUN(X, "rmsnorm_fwd", 0, 4.0 * Td * D.h, k_rmsnorm_fwd(X.st, S(b.y), W.t(RP_T_G2), S(b.n2), (float*)S(b.rstd2), T, D.h, c.rms_eps));
  if (D.E > 0) {
    // top-k mixture of experts (App. B.2, MoE layer): route, sort the (token, choice) entries by expert, run the
    // experts' gate/up and down projections as grouped GEMMs over the sorted rows, weighted sum per token + residual
    const long Tk = (long)T * D.topk;
    const double Tkd = (double)Tk;
    int* idx = (int*)S(b.m_idx);
    float* w = (float*)S(b.m_w);
    int* slot_of = (int*)S(b.m_slot);
    void* f = X.at<void>(moe_f_off);
    // router in the stage: logits = n2 Wr^T in fp32 (bf16 operands), so that the selection is a function of n2 alone
    if (c.moe_router) X.gemm_f32_nt(S(b.n2), D.h, W.t(RP_T_WR), D.h, X.router, D.E, T, D.E, D.h);
    RUN(X, "moe_route", 0, 4.0 * Td * D.E + 8.0 * Tkd, k_moe_route(X.st, X.router, idx, w, T, D.E, D.topk));
    RUN(X, "moe_plan", 0, 16.0 * Tkd, k_moe_plan(X.st, idx, T, D.E, D.topk, (int*)S(b.m_cnt), (int*)S(b.m_seg), S(b.m_tab),
                                                     (int*)S(b.m_ntiles), slot_of, (int*)S(b.m_tok), (int*)S(b.m_hist)));
    if (D.m % 128 == 0) {   // SwiGLU in the epilogue, as in the dense layer
      X.gemm_grouped(GEMM_NT, set, S(b.n2), D.h, T, true, W.t(RP_T_WGU), D.h, (long)2 * D.m * D.h, S(b.gu), 2 * D.m, 2 * D.m, D.h, S(b.act));
    } else {
      X.gemm_grouped(GEMM_NT, set, S(b.n2), D.h, T, true, W.t(RP_T_WGU), D.h, (long)2 * D.m * D.h, S(b.gu), 2 * D.m, 2 * D.m, D.h);
      RUN(X, "swiglu_fwd", 0, 6.0 * Tkd * D.m, k_swiglu_fwd(X.st, S(b.gu), S(b.act), Tk, D.m));
    }
    X.gemm_grouped(GEMM_NT, set, S(b.act), D.m, (int)Tk, false, W.t(RP_T_WD), D.m, (long)D.h * D.m, f, D.h, D.h, D.m);
    RUN(X, "moe_combine", 0, 2.0 * Tkd * D.h + 4.0 * Td * D.h, k_moe_combine(X.st, f, slot_of, w, S(b.y), z, T, D.h, D.topk));
    return;
  }
  // SwiGLU rides in the gate/up product's epilogue when the column blocks pair up (m a multiple of 128): gate | up are
  // still stored for the backward, the activation is not read back from them by a kernel of its own
  if (D.m % 128 == 0) {
    linear_fwd(X, W, RP_T_WGU, fused_gu(D), X.ctx->dl.bd3, S(b.n2), D.h, S(b.gu), 2 * D.m, S(b.u3), nullptr, S(b.act));
  } else {
    linear_fwd(X, W, RP_T_WGU, fused_gu(D), X.ctx->dl.bd3, S(b.n2), D.h, S(b.gu), 2 * D.m, S(b.u3), nullptr);
    RUN(X, "swiglu_fwd", 0, 6.0 * Td * D.m, k_swiglu_fwd(X.st, S(b.gu), S(b.act), T, D.m));
  }
  linear_fwd(X, W, RP_T_WD, fused_single(D.lora[6], RP_T_LA_DOWN, RP_T_LB_DOWN, D.h), 0, S(b.act), D.m, z, D.h, S(b.u4), S(b.y));
}

// dz: gradient of the layer output; dx_out receives the gradient of the layer input x.
void layer_backward(Exec& X, const LayerW& W, const LayerG& G, char* set, const void* x, const void* dz, void* dx_out) {
  const Dims& D = X.D;
  const LayerBuf& b = X.P.lb;
  const rp_stage_cfg& c = X.ctx->cfg;
  const int T = (int)X.T;
  auto S = [&](size_t off) { return reinterpret_cast<void*>(set + off); };
  bf16_t* qkv = reinterpret_cast<bf16_t*>(S(b.qkv));
  bf16_t* dqkv = X.at<bf16_t>(X.P.dqkv);
  void* dy = X.at<void>(X.P.tA);

  const double Td = (double)T;
  if (D.E > 0) {
    // z = y + sum_j w_j FFN_ej(n2): per slot dact = Wd_e^T dz_t (the routing weight is applied inside the SwiGLU
    // backward, which also yields dw = <dact, act>), dgu, then the expert input gradients summed per token
    const long Tk = (long)T * D.topk;
    const double Tkd = (double)Tk;
    const int* idx = (const int*)S(b.m_idx);
    const float* w = (const float*)S(b.m_w);
    const int* slot_of = (const int*)S(b.m_slot);
    float* w_slot = X.at<float>(X.P.moe_wslot);
    float* dw_slot = X.at<float>(X.P.moe_dw);
    void* dxp = X.at<void>(X.P.moe_f_bwd);
    X.gemm_grouped(GEMM_NN, set, dz, D.h, T, true, W.t(RP_T_WD), D.m, (long)D.h * D.m, X.at<void>(X.P.dact), D.m, D.m, D.h);
    RUN(X, "moe_scatter_w", 0, 12.0 * Tkd, k_moe_scatter_w(X.st, w, slot_of, w_slot, Tk));
    RUN(X, "moe_swiglu_bwd", 0, 10.0 * Tkd * D.m,
        k_moe_swiglu_bwd(X.st, X.at<void>(X.P.dact), S(b.gu), w_slot, X.at<void>(X.P.dgu), dw_slot, Tk, D.m));
    float* dlog = X.d_router ? X.d_router : (c.moe_router ? X.at<float>(X.P.moe_dlog) : nullptr);
    if (dlog)
      RUN(X, "moe_dlogits", 0, 4.0 * Td * D.E + 12.0 * Tkd, k_moe_dlogits(X.st, idx, w, slot_of, dw_slot, dlog, T, D.E, D.topk));
    X.gemm_grouped(GEMM_NN, set, X.at<void>(X.P.dgu), 2 * D.m, (int)Tk, false, W.t(RP_T_WGU), D.h, (long)2 * D.m * D.h, dxp, D.h,
                   D.h, 2 * D.m);
    RUN(X, "moe_combine", 0, 2.0 * Tkd * D.h + 2.0 * Td * D.h,
        k_moe_combine(X.st, dxp, slot_of, nullptr, nullptr, X.at<void>(X.P.dn), T, D.h, D.topk));
    if (c.moe_router) {
      // logits = n2 Wr^T: the gradient of n2 gains dlogits Wr (bf16 operands like every activation gradient)
      void* dl16 = X.at<void>(X.P.moe_dlog16);
      RUN(X, "cast", 0, 6.0 * Td * D.E, k_cast_f32_bf16(X.st, dlog, dl16, (long)T * D.E));
      X.gemm_bf16(GEMM_NN, dl16, D.E, W.t(RP_T_WR), D.h, X.at<void>(X.P.dn), D.h, T, D.h, D.E, 1.f, nullptr, 0, nullptr, 0, 0,
                  X.at<void>(X.P.dn), D.h);
    }
  } else {
    // z = y + down(act)
    // the SwiGLU backward rides in the epilogue of the down projection's input-gradient GEMM
    linear_bwd(X, W, G, RP_T_WD, fused_single(D.lora[6], RP_T_LA_DOWN, RP_T_LB_DOWN, D.h), 0, dz, D.h, S(b.act), D.m,
               nullptr, S(b.u4), S(b.gu), X.at<void>(X.P.dgu));
    linear_bwd(X, W, G, RP_T_WGU, fused_gu(D), X.ctx->dl.bd3, X.at<void>(X.P.dgu), 2 * D.m, S(b.n2), D.h, X.at<void>(X.P.dn), S(b.u3));
  }
  RUN(X, "rmsnorm_bwd", 0, 8.0 * Td * D.h,
      k_rmsnorm_bwd(X.st, X.at<void>(X.P.dn), 0, S(b.y), W.t(RP_T_G2), (const float*)S(b.rstd2), dz, dy, G.t(RP_T_G2), X.at<float>(X.P.partials), T, D.h));
  // y = x + o_proj(o)
  linear_bwd(X, W, G, RP_T_WO, fused_single(D.lora[3], RP_T_LA_O, RP_T_LB_O, D.h), 0, dy, D.h, S(b.o), D.qd,
             X.at<void>(X.P.dout), S(b.u2));
  RUN(X, "attn_delta", 0, 4.0 * Td * D.qd,
      k_attn_delta(X.st, S(b.o), X.at<void>(X.P.dout), X.at<float>(X.P.delta), D.qd, D.qd, X.batch, X.seq, D.a, D.d));
  const double s2qd = (double)X.batch * X.seq * (double)X.seq * D.qd;
  // useful FLOPs per kernel: dK/dV kernel runs S, dP, dV, dK (4 half-masked products), dQ kernel S, dP, dQ (3)
  static const int parts[3] = {0, 2, 1};
  static const char* const part_name[3] = {"attn_bwd_dkv", "attn_bwd_dq", "attn_dkv_reduce"};
  for (int i = 0; i < 3; ++i) {
    const int part = parts[i];
    if (part == 2 && D.a == D.kh) continue;
    const double fl = part == 0 ? 4.0 * s2qd : part == 1 ? 3.0 * s2qd : 0.0;
    const double by = part == 2 ? Td * (8.0 * D.qd + 4.0 * D.kd) : 2.0 * Td * (3 * D.qd + 4 * D.kd);
    RUN(X, part_name[part], fl, by,
        k_attn_bwd(X.st, part, S(b.qr), S(b.kr), qkv + D.qd + D.kd, X.at<void>(X.P.dout), (const float*)S(b.lse),
                   X.at<float>(X.P.delta), X.at<void>(X.P.dqr), X.at<void>(X.P.dkr), dqkv + D.qd + D.kd,
                   X.at<float>(X.P.dkvp), D.qd, D.kd, D.n1, D.qd, D.qd, D.kd, D.n1, X.batch, X.seq, D.a, D.kh, D.d));
  }
  RUN(X, "qknorm_rope_bwd", 0, 6.0 * Td * (D.qd + D.kd),
      k_qknorm_rope(X.st, 1, D.d, X.at<void>(X.P.dqr), X.at<void>(X.P.dkr), D.qd, D.kd, dqkv, dqkv + D.qd, D.n1, D.n1,
                    W.t(RP_T_GQ), W.t(RP_T_GK), (float*)S(b.rstd_q), (float*)S(b.rstd_k), qkv, qkv + D.qd, D.n1,
                    G.t(RP_T_GQ), G.t(RP_T_GK), X.at<float>(X.P.partials), X.at<float2>(X.P.rope), T, X.seq, D.a, D.kh, c.qk_norm, c.rms_eps));
  linear_bwd(X, W, G, RP_T_WQKV, fused_qkv(D), X.ctx->dl.bd1, dqkv, D.n1, S(b.n1), D.h, X.at<void>(X.P.dn), S(b.u1));
  RUN(X, "rmsnorm_bwd", 0, 8.0 * Td * D.h,
      k_rmsnorm_bwd(X.st, X.at<void>(X.P.dn), 0, x, W.t(RP_T_G1), (const float*)S(b.rstd1), dy, dx_out, G.t(RP_T_G1), X.at<float>(X.P.partials), T, D.h));
}

hipError_t build_derived(const rp_ctx* ctx, hipStream_t st, char* slot, int l) {
  const Dims D = dims_of(ctx->cfg);
  if (ctx->dl.layer_bytes == 0 || l >= ctx->cfg.n_layers) return hipSuccess;
  const LayerW W{slot + ctx->wl.layer_bytes * (size_t)l, &ctx->wl, nullptr};
  char* const out = slot + ctx->wl.total + ctx->dl.layer_bytes * (size_t)l;
  hipError_t e = hipSuccess;
  const FusedLora groups[2] = {fused_qkv(D), fused_gu(D)};
  const int width[2] = {D.n1, 2 * D.m};
  const size_t off[2] = {ctx->dl.bd1, ctx->dl.bd3};
  for (int gi = 0; gi < 2 && e == hipSuccess; ++gi) {
    const FusedLora& f = groups[gi];
    if (f.n == 0) continue;
    LoraSegs sg{};
    for (int i = 0; i < f.n; ++i) { sg.src[i] = W.t(f.b_id[i]); sg.row0[i] = f.row0[i]; sg.row1[i] = f.row1[i]; sg.col0[i] = i * D.r; }
    e = k_lora_blockdiag(st, out + off[gi], width[gi], f.n * D.r, sg, D.r);
  }
  return e;
}

rp_status check_call(rp_ctx* ctx, int slot_id, int batch, int seq, const void* ws, size_t ws_bytes, size_t need) {
  if (!ctx) return fail(nullptr, RP_EINVAL, "ctx is NULL");
  if (slot_id < 0 || slot_id >= RP_MAX_SLOTS) return fail(ctx, RP_EINVAL, "slot_id %d out of range", slot_id);
  rp_status s = validate_shape(ctx, batch, seq);
  if (s != RP_OK) return s;
  if (!ctx->slots[slot_id].valid) return fail(ctx, RP_ESTATE, "slot %d holds no weights (upload or bind first)", slot_id);
  if (!ws) return fail(ctx, RP_EINVAL, "workspace is NULL");
  if (ws_bytes < need) return fail(ctx, RP_ENOMEM, "workspace too small: %zu < %zu", ws_bytes, need);
  if (reinterpret_cast<uintptr_t>(ws) % 256) return fail(ctx, RP_EINVAL, "workspace must be 256-byte aligned");
  return RP_OK;
}

rp_status wait_chunk(rp_ctx* ctx, Slot& sl, int chunk) {
  if (sl.gated) HIP_TRY(ctx, hipStreamWaitEvent(ctx->compute, sl.ev[chunk], 0));
  return RP_OK;
}

rp_status finish_call(rp_ctx* ctx, Slot& sl, Exec& X) {
  if (ctx->tracing && ctx->trace_n <= ctx->trace_cap) X.chk(hipEventRecord(ctx->trace_ev[ctx->trace_n], ctx->compute), "trace event");
  if (X.err != hipSuccess) return fail(ctx, RP_EHIP, "%s: %s", X.where, hipGetErrorString(X.err));
  HIP_TRY(ctx, hipEventRecord(sl.free_ev, ctx->compute));
  sl.used = true;
  return RP_OK;
}

}  // namespace

// ==================================================================================================== C ABI
extern "C" {

const char* rp_last_error(const rp_ctx* ctx) { return ctx ? ctx->err : g_err; }

rp_status rp_query_sizes(const rp_stage_cfg* cfg, int batch, int seq, size_t* weight_blob_bytes, size_t* grad_blob_bytes,
                         size_t* workspace_bytes_out) {
  rp_status s = validate_cfg(cfg, nullptr);
  if (s != RP_OK) return s;
  if (weight_blob_bytes) *weight_blob_bytes = blob_layout(*cfg, false).total;
  if (grad_blob_bytes) *grad_blob_bytes = blob_layout(*cfg, true).total;
  if (workspace_bytes_out) {
    s = validate_shape(nullptr, batch, seq);
    if (s != RP_OK) return s;
    *workspace_bytes_out = workspace_bytes(make_plan(*cfg, batch, seq), *cfg);
  }
  return RP_OK;
}

rp_status rp_slot_bytes(const rp_stage_cfg* cfg, size_t* slot_bytes) {
  rp_status s = validate_cfg(cfg, nullptr);
  if (s != RP_OK) return s;
  if (!slot_bytes) return fail(nullptr, RP_EINVAL, "slot_bytes is NULL");
  *slot_bytes = blob_layout(*cfg, false).total + derived_layout(*cfg).total;
  return RP_OK;
}

static rp_status layout_query(const rp_stage_cfg* cfg, bool grads, int layer, int id, size_t* off, size_t* n) {
  rp_status s = validate_cfg(cfg, nullptr);
  if (s != RP_OK) return s;
  if (id < 0 || id >= RP_T_COUNT || layer < 0 || layer > cfg->n_layers) return fail(nullptr, RP_EINVAL, "bad layer/tensor id");
  const BlobLayout B = blob_layout(*cfg, grads);
  const bool head = is_head_tensor(id);
  if (head != (layer == cfg->n_layers)) { if (off) *off = 0; if (n) *n = 0; return RP_OK; }
  if (off) *off = (head ? B.layer_bytes * (size_t)cfg->n_layers : B.layer_bytes * (size_t)layer) + B.off[id];
  if (n) *n = B.elems[id];
  return RP_OK;
}
rp_status rp_weight_layout(const rp_stage_cfg* cfg, int layer, int id, size_t* off, size_t* n) { return layout_query(cfg, false, layer, id, off, n); }
rp_status rp_grad_layout(const rp_stage_cfg* cfg, int layer, int id, size_t* off, size_t* n) { return layout_query(cfg, true, layer, id, off, n); }

rp_status rp_weight_chunk(const rp_stage_cfg* cfg, int layer, size_t* begin, size_t* end) {
  rp_status s = validate_cfg(cfg, nullptr);
  if (s != RP_OK) return s;
  if (layer < 0 || layer > cfg->n_layers) return fail(nullptr, RP_EINVAL, "bad layer");
  const BlobLayout B = blob_layout(*cfg, false);
  const size_t b0 = B.layer_bytes * (size_t)layer;
  if (begin) *begin = b0;
  if (end) *end = layer == cfg->n_layers ? b0 + B.head_bytes : b0 + B.layer_bytes;
  return RP_OK;
}

rp_status rp_ctx_create(rp_ctx** out, int device, void* compute_stream, void* copy_stream, const rp_stage_cfg* cfg) {
  if (!out) return fail(nullptr, RP_EINVAL, "out is NULL");
  *out = nullptr;
  rp_status s = validate_cfg(cfg, nullptr);
  if (s != RP_OK) return s;
  if (!compute_stream || !copy_stream) return fail(nullptr, RP_EINVAL, "both streams must be non-NULL");
  HIP_TRY(nullptr, hipSetDevice(device));
  {   // set-up of the no-allocation entry point for this device (rp_op_rmsnorm_bwd_noalloc)
    hipError_t se = hipSuccess;
    if (!noalloc_scratch(&se)) return fail(nullptr, RP_EHIP, "hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(se));
  }
  rp_ctx* c = new (std::nothrow) rp_ctx();
  if (!c) return fail(nullptr, RP_ENOMEM, "out of host memory");
  c->cfg = *cfg; c->device = device;
  c->compute = reinterpret_cast<hipStream_t>(compute_stream);
  c->copy = reinterpret_cast<hipStream_t>(copy_stream);
  c->wl = blob_layout(*cfg, false);
  c->gl = blob_layout(*cfg, true);
  c->dl = derived_layout(*cfg);
  c->err[0] = 0;
  const int nev = cfg->n_layers + 1;
  for (int i = 0; i < RP_MAX_SLOTS; ++i) {
    c->slots[i].ev = new (std::nothrow) hipEvent_t[nev]();
    if (!c->slots[i].ev) { rp_ctx_destroy(c); return fail(nullptr, RP_ENOMEM, "out of host memory"); }
    for (int j = 0; j < nev; ++j)
      if (hipEventCreateWithFlags(&c->slots[i].ev[j], hipEventDisableTiming) != hipSuccess) { rp_ctx_destroy(c); return fail(nullptr, RP_EHIP, "hipEventCreate failed"); }
    if (hipEventCreateWithFlags(&c->slots[i].free_ev, hipEventDisableTiming) != hipSuccess) { rp_ctx_destroy(c); return fail(nullptr, RP_EHIP, "hipEventCreate failed"); }
  }
  *out = c;
  return RP_OK;
}

rp_status rp_ctx_destroy(rp_ctx* c) {
  if (!c) return RP_OK;
  for (int i = 0; i < RP_MAX_SLOTS; ++i) {
    if (c->slots[i].ev) {
      for (int j = 0; j <= c->cfg.n_layers; ++j) if (c->slots[i].ev[j]) (void)hipEventDestroy(c->slots[i].ev[j]);
      delete[] c->slots[i].ev;
    }
    if (c->slots[i].free_ev) (void)hipEventDestroy(c->slots[i].free_ev);
  }
  if (c->trace_ev) {
    for (int i = 0; i <= c->trace_cap; ++i) if (c->trace_ev[i]) (void)hipEventDestroy(c->trace_ev[i]);
    delete[] c->trace_ev;
  }
  delete[] c->trace_rec;
  if (c->round_ev) {
    for (int i = 0; i < c->round_ev_n; ++i) if (c->round_ev[i]) (void)hipEventDestroy(c->round_ev[i]);
    delete[] c->round_ev;
  }
  delete c;
  return RP_OK;
}

rp_status rp_stage_upload_weights(rp_ctx* ctx, int slot_id, void* dev_slot, const void* host_blob, size_t bytes) {
  if (!ctx) return fail(nullptr, RP_EINVAL, "ctx is NULL");
  if (slot_id < 0 || slot_id >= RP_MAX_SLOTS) return fail(ctx, RP_EINVAL, "slot_id %d out of range", slot_id);
  if (!dev_slot || !host_blob) return fail(ctx, RP_EINVAL, "NULL buffer");
  if (bytes != ctx->wl.total) return fail(ctx, RP_EINVAL, "bytes %zu != weight blob size %zu", bytes, ctx->wl.total);
  if (reinterpret_cast<uintptr_t>(dev_slot) % 256) return fail(ctx, RP_EINVAL, "dev_slot must be 256-byte aligned");
  Slot& sl = ctx->slots[slot_id];
  if (sl.used) HIP_TRY(ctx, hipStreamWaitEvent(ctx->copy, sl.free_ev, 0));
  const int L = ctx->cfg.n_layers;
  for (int l = 0; l <= L; ++l) {
    const size_t b0 = ctx->wl.layer_bytes * (size_t)l;
    const size_t n = l == L ? ctx->wl.head_bytes : ctx->wl.layer_bytes;
    if (n) HIP_TRY(ctx, hipMemcpyAsync(static_cast<char*>(dev_slot) + b0, static_cast<const char*>(host_blob) + b0, n, hipMemcpyHostToDevice, ctx->copy));
    HIP_TRY(ctx, build_derived(ctx, ctx->copy, static_cast<char*>(dev_slot), l));   // behind the chunk it reads, before its event
    HIP_TRY(ctx, hipEventRecord(sl.ev[l], ctx->copy));
  }
  sl.dev = dev_slot; sl.bytes = bytes; sl.valid = true; sl.gated = true; sl.used = false;
  return RP_OK;
}

rp_status rp_stage_bind_weights(rp_ctx* ctx, int slot_id, void* dev_slot, size_t bytes) {
  if (!ctx) return fail(nullptr, RP_EINVAL, "ctx is NULL");
  if (slot_id < 0 || slot_id >= RP_MAX_SLOTS) return fail(ctx, RP_EINVAL, "slot_id %d out of range", slot_id);
  if (!dev_slot) return fail(ctx, RP_EINVAL, "NULL buffer");
  if (bytes != ctx->wl.total) return fail(ctx, RP_EINVAL, "bytes %zu != weight blob size %zu", bytes, ctx->wl.total);
  if (reinterpret_cast<uintptr_t>(dev_slot) % 256) return fail(ctx, RP_EINVAL, "dev_slot must be 256-byte aligned");
  Slot& sl = ctx->slots[slot_id];
  for (int l = 0; l < ctx->cfg.n_layers; ++l) HIP_TRY(ctx, build_derived(ctx, ctx->compute, static_cast<char*>(dev_slot), l));
  sl.dev = dev_slot; sl.bytes = bytes; sl.valid = true; sl.gated = false; sl.used = false;
  return RP_OK;
}

rp_status rp_stage_forward(rp_ctx* ctx, int slot_id, const void* x_in, void* x_out, void* const* layer_inputs_out,
                           float* router_logits, int batch, int seq, void* workspace, size_t workspace_bytes_in) {
  if (!ctx) return fail(nullptr, RP_EINVAL, "ctx is NULL");
  if (ctx->cfg.n_layers == 0) return fail(ctx, RP_EINVAL, "stage has no decoder layers");
  if (ctx->cfg.n_experts > 0 && !router_logits) return fail(ctx, RP_EINVAL, "MoE stage needs router_logits");
  const Plan P = make_plan(ctx->cfg, batch > 0 ? batch : 1, seq > 0 ? seq : 8);
  rp_status s = check_call(ctx, slot_id, batch, seq, workspace, workspace_bytes_in, P.fwd_bytes);
  if (s != RP_OK) return s;
  if (!x_in || !x_out || x_in == x_out) return fail(ctx, RP_EINVAL, "x_in / x_out must be distinct non-NULL buffers");
  Slot& sl = ctx->slots[slot_id];
  Exec X{ctx, ctx->compute, dims_of(ctx->cfg), batch, seq, (long)batch * seq, static_cast<char*>(workspace), P};
  X.fwd_only = true;
  X.split_off = P.split_fwd; X.has_split = X.D.r > 0;
  const int L = ctx->cfg.n_layers;
  const size_t act_bytes = (size_t)X.T * X.D.h * 2;
  RUN(X, "rope_table", 0, 4.0 * seq * X.D.d, k_rope_table(X.st, X.at<float2>(P.rope), seq, X.D.d, ctx->cfg.rope_base));
  char* set = X.ws + P.layer0;
  void* pp[2] = {set + P.lb.z, X.ws + P.layer0 + P.layer_stride};
  const void* x = x_in;
  for (int l = 0; l < L; ++l) {
    s = wait_chunk(ctx, sl, l);
    if (s != RP_OK) return s;
    if (layer_inputs_out && layer_inputs_out[l] && layer_inputs_out[l] != x) RUN(X, "copy", 0, 2.0 * act_bytes, k_copy16(X.st, x, layer_inputs_out[l], (long)act_bytes));
    void* z = (l == L - 1) ? x_out : pp[l & 1];
    const LayerW W{static_cast<const char*>(sl.dev) + ctx->wl.layer_bytes * (size_t)l, &ctx->wl,
                     static_cast<const char*>(sl.dev) + ctx->wl.total + ctx->dl.layer_bytes * (size_t)l};
    if (router_logits) X.router = router_logits + (size_t)l * X.T * X.D.E;
    layer_forward(X, W, set, x, z, P.moe_f_fwd);
    x = z;
  }
  return finish_call(ctx, sl, X);
}

rp_status rp_stage_backward(rp_ctx* ctx, int slot_id, int phases, const void* x_in, const void* dy, void* dx, void* x_out,
                            void* grads, float* router_logits, float* d_router_logits, int batch, int seq,
                            void* workspace, size_t workspace_bytes_in) {
  if (!ctx) return fail(nullptr, RP_EINVAL, "ctx is NULL");
  if (ctx->cfg.n_layers == 0) return fail(ctx, RP_EINVAL, "stage has no decoder layers");
  if (ctx->cfg.n_experts > 0 && !router_logits) return fail(ctx, RP_EINVAL, "MoE stage needs router_logits");
  const Plan P = make_plan(ctx->cfg, batch > 0 ? batch : 1, seq > 0 ? seq : 8);
  rp_status s = check_call(ctx, slot_id, batch, seq, workspace, workspace_bytes_in, P.bwd_bytes);
  if (s != RP_OK) return s;
  if (phases < 1 || phases > 3) return fail(ctx, RP_EINVAL, "phases must be RP_PHASE_RECOMPUTE, RP_PHASE_BACKWARD or both");
  const bool do_fwd = phases & RP_PHASE_RECOMPUTE, do_bwd = phases & RP_PHASE_BACKWARD;
  if (!x_in) return fail(ctx, RP_EINVAL, "x_in must be non-NULL");
  if (do_bwd) {
    if (!dy || !dx) return fail(ctx, RP_EINVAL, "dy and dx must be non-NULL for the backward phase");
    if (dx == x_in || dx == dy) return fail(ctx, RP_EINVAL, "dx must not alias x_in or dy");
    if (!grads && ctx->gl.total > 0) return fail(ctx, RP_EINVAL, "grads is NULL but the stage has trainable tensors");
  }
  Slot& sl = ctx->slots[slot_id];
  Exec X{ctx, ctx->compute, dims_of(ctx->cfg), batch, seq, (long)batch * seq, static_cast<char*>(workspace), P};
  X.split_off = P.split_bwd; X.has_split = true;
  const int L = ctx->cfg.n_layers;
  const size_t act_bytes = (size_t)X.T * X.D.h * 2;
  if (do_fwd) RUN(X, "rope_table", 0, 4.0 * seq * X.D.d, k_rope_table(X.st, X.at<float2>(P.rope), seq, X.D.d, ctx->cfg.rope_base));
  auto set_of = [&](int l) { return X.ws + P.layer0 + P.layer_stride * (size_t)l; };
  if (do_fwd) {
    // recomputation: forward over the stage keeping every layer's internals; layer l starts as soon as its own chunk
    // of the upload has landed (per-layer events, Sec. 4.3), so the recomputation overlaps the tail of the upload
    const void* x = x_in;
    for (int l = 0; l < L; ++l) {
      s = wait_chunk(ctx, sl, l);
      if (s != RP_OK) return s;
      const LayerW W{static_cast<const char*>(sl.dev) + ctx->wl.layer_bytes * (size_t)l, &ctx->wl,
                     static_cast<const char*>(sl.dev) + ctx->wl.total + ctx->dl.layer_bytes * (size_t)l};
      void* z = set_of(l) + P.lb.z;
      if (router_logits) X.router = router_logits + (size_t)l * X.T * X.D.E;
      layer_forward(X, W, set_of(l), x, z, P.moe_f_bwd);
      x = z;
    }
    if (x_out) RUN(X, "copy", 0, 2.0 * act_bytes, k_copy16(X.st, x, x_out, (long)act_bytes));
  }
  // backward in reverse layer order
  const void* dz = dy;
  for (int l = L - 1; do_bwd && l >= 0; --l) {
    if (!do_fwd) {   // the backward phase alone: wait per layer, in the order the layers are run
      s = wait_chunk(ctx, sl, l);
      if (s != RP_OK) return s;
    }
    const LayerW W{static_cast<const char*>(sl.dev) + ctx->wl.layer_bytes * (size_t)l, &ctx->wl,
                     static_cast<const char*>(sl.dev) + ctx->wl.total + ctx->dl.layer_bytes * (size_t)l};
    const LayerG G{grads ? static_cast<char*>(grads) + ctx->gl.layer_bytes * (size_t)l : nullptr, &ctx->gl};
    const void* xl = l == 0 ? x_in : set_of(l - 1) + P.lb.z;
    void* dxl = l == 0 ? dx : X.at<void>(P.tB);
    X.d_router = (d_router_logits && X.D.E > 0) ? d_router_logits + (size_t)l * X.T * X.D.E : nullptr;
    layer_backward(X, W, G, set_of(l), xl, dz, dxl);
    dz = dxl;
  }
  return finish_call(ctx, sl, X);
}

rp_status rp_lmhead_ce_fwd_bwd(rp_ctx* ctx, int slot_id, const void* x, const int32_t* labels, float* loss_out, void* dx,
                               void* grads, float grad_scale, int batch, int seq, void* workspace, size_t workspace_bytes_in) {
  if (!ctx) return fail(nullptr, RP_EINVAL, "ctx is NULL");
  if (ctx->cfg.vocab == 0) return fail(ctx, RP_EINVAL, "stage has no LM head");
  const Plan P = make_plan(ctx->cfg, batch > 0 ? batch : 1, seq > 0 ? seq : 8);
  rp_status s = check_call(ctx, slot_id, batch, seq, workspace, workspace_bytes_in, P.head_bytes);
  if (s != RP_OK) return s;
  if (!x || !labels || !loss_out || !dx) return fail(ctx, RP_EINVAL, "x, labels, loss_out and dx must be non-NULL");
  if (dx == x) return fail(ctx, RP_EINVAL, "dx must not alias x");
  Slot& sl = ctx->slots[slot_id];
  Exec X{ctx, ctx->compute, dims_of(ctx->cfg), batch, seq, (long)batch * seq, static_cast<char*>(workspace), P};
  X.split_off = P.h_split; X.has_split = true;
  const Dims& D = X.D;
  const int T = (int)X.T, L = ctx->cfg.n_layers;
  s = wait_chunk(ctx, sl, L);
  if (s != RP_OK) return s;
  const char* hb = static_cast<const char*>(sl.dev) + ctx->wl.layer_bytes * (size_t)L;
  const LayerW W{hb, &ctx->wl};
  const bool train = grads && ctx->cfg.train_base;
  const LayerG G{train ? static_cast<char*>(grads) + ctx->gl.layer_bytes * (size_t)L : nullptr, &ctx->gl};
  const bf16_t* Wv = W.t(RP_T_WV);

  const double Td = (double)T;
  RUN(X, "rmsnorm_fwd", 0, 4.0 * Td * D.h, k_rmsnorm_fwd(X.st, x, W.t(RP_T_GF), X.at<void>(P.h_xf), X.at<float>(P.h_rstd), T, D.h, ctx->cfg.rms_eps));
  RUN(X, "fill", 0, 4.0 * Td, k_fill_u32(X.st, X.at<void>(P.h_zlab), T, 0u));
  if (!ctx->cfg.head_two_sweeps && (!ctx->cfg.train_base || P.head_keep_p)) {
    // One sweep over the vocabulary: the softmax normaliser is only needed at the very end.  Per chunk: logits -> p =
    // exp(z - m_t) against a per-token reference exponent that moves (and rescales what has been accumulated) only when
    // a chunk outgrows it -> acc_t += p W_c;  finally lse_t = m_t + log l_t and dx_t = coef_t (acc_t / l_t - W[y_t]).
    // Frozen head: two logit-sized products instead of three, one chunk of p in memory at a time.  Trainable head
    // (keep_p): the p of every chunk stay in memory ([V, T] bf16) and the weight gradient follows from them afterwards,
    // dW = P'^T^T xs with P'[v, t] = p[v, t] - l_t [v = y_t], xs_t = (coef_t / l_t) xf_t: three products instead of the
    // four of the two-sweep schedule, which has to compute the logits twice.
    const bool keep_p = P.head_keep_p;
    bf16_t* const pall = keep_p ? X.at<bf16_t>(P.h_pall) : nullptr;
    float* const zc = X.at<float>(P.h_z);
    float* const acc = X.at<float>(P.h_dxacc);
    int* const flag = X.at<int>(P.h_flag);
    RUN(X, "fill", 0, 4.0 * Td * D.h, k_fill_u32(X.st, acc, (long)T * D.h, 0u));
    RUN(X, "fill", 0, 4.0, k_fill_u32(X.st, flag, 1, 0u));
    {
      // The reference exponents the sweep starts from: every token's largest logit over the first 256 vocabulary rows.
      // Any reference within e^60 of the row's true maximum serves (bf16 keeps its relative precision over that range),
      // so this small product lets every chunk, the first one included, take the path without fp32 logits.
      const int r0 = D.V < 256 ? D.V : 256;
      GemmArgs g; gemm_zero_args(g);
      g.A = Wv; g.lda = D.h; g.B = X.at<void>(P.h_xf); g.ldb = D.h; g.M = r0; g.N = T; g.K = D.h; g.epi = EPI_F32_COLMAX;
      g.C = zc; g.ldc = T; g.labels = labels; g.zlab = X.at<float>(P.h_zlab); g.part = X.at<float2>(P.h_part); g.part_ld = T;
      X.mark_gemm(GEMM_NT, g);
      X.chk(gemm_launch(X.st, GEMM_NT, g), "lm head reference");
      RUN(X, "ce_ref_init", 0, 28.0 * Td,
          k_ce_ref_init(X.st, X.at<float2>(P.h_part), gemm_ce_stats_partials(r0), T, X.at<float>(P.h_m), X.at<float>(P.h_l), X.at<float>(P.h_alpha)));
    }
    for (int v0 = 0; v0 < D.V; v0 += P.head_chunk) {
      const int vc = (D.V - v0 < P.head_chunk) ? (D.V - v0) : P.head_chunk;
      const int nparts = gemm_ce_stats_partials(vc);
      const bf16_t* Wc = Wv + (size_t)v0 * D.h;
      void* const pc = keep_p ? static_cast<void*>(pall + (size_t)v0 * T) : X.at<void>(P.h_dzt);   // this chunk's p [vc, T]
      GemmArgs g; gemm_zero_args(g);
      g.A = Wc; g.lda = D.h; g.B = X.at<void>(P.h_xf); g.ldb = D.h; g.M = vc; g.N = T; g.K = D.h;
      g.ldc = T; g.labels = labels; g.zlab = X.at<float>(P.h_zlab); g.part = X.at<float2>(P.h_part); g.part_ld = T;
      g.row_offset = v0;
      {
        // the probabilities straight from the accumulators, against the reference as it stands; the chunk is redone
        // below only if a token outgrew its reference by too much for that (the flag stays 0 otherwise)
        GemmArgs f = g;
        f.epi = EPI_CE_P; f.C = pc; f.lse = X.at<float>(P.h_m);
        X.mark_gemm(GEMM_NT, f);
        X.chk(gemm_launch(X.st, GEMM_NT, f), "lm head probabilities");
        RUN(X, "ce_chunk_check", 0, 8.0 * nparts * Td, k_ce_chunk_check(X.st, X.at<float2>(P.h_part), nparts, T, X.at<float>(P.h_m), flag));
      }
      // the slow path, behind the flag: fp32 logits, reference move with rescale of what has been accumulated, p again
      g.run_flag = flag; g.epi = EPI_F32_COLMAX; g.C = zc;
      X.mark("ce_slow_path", 0, 0);
      X.chk(gemm_launch(X.st, GEMM_NT, g), "lm head logits");
      RUN(X, "ce_slow_path", 0, 8.0 * nparts * Td,
          k_ce_chunk_update(X.st, zc, vc, T, X.at<float2>(P.h_part), nparts, 0, X.at<float>(P.h_m), X.at<float>(P.h_l),
                            X.at<float>(P.h_alpha), pc, flag));
      RUN(X, "ce_slow_path", 0, 0, k_ce_rescale_rows(X.st, acc, X.at<float>(P.h_alpha), T, D.h, flag));
      if (keep_p && v0 > 0) RUN(X, "ce_slow_path", 0, 0, k_ce_rescale_p(X.st, pall, v0, T, X.at<float>(P.h_alpha), flag));
      RUN(X, "fill", 0, 4.0, k_fill_u32(X.st, flag, 1, 0u));   // every reader of the flag is behind it in the stream
      GemmArgs d; gemm_zero_args(d);   // acc[T, h] += p^T^T . W_c
      d.A = pc; d.lda = T; d.B = Wc; d.ldb = D.h; d.M = T; d.N = D.h; d.K = vc; d.C = acc;
      d.ldc = D.h; d.beta = 1; d.epi = EPI_F32;
      X.give_split_ws(d);
      X.mark_gemm(GEMM_TN, d);
      X.chk(gemm_launch(X.st, GEMM_TN, d), "lm head dX");
    }
    RUN(X, "ce_lse", 0, 12.0 * Td, k_ce_lse_from_ref(X.st, X.at<float>(P.h_m), X.at<float>(P.h_l), X.at<float>(P.h_lse), T));
    RUN(X, "ce_finalize", 0, 16.0 * Td,
        k_ce_finalize(X.st, X.at<float>(P.h_lse), X.at<float>(P.h_zlab), labels, grad_scale, X.at<float>(P.h_coef), loss_out, T));
    if (train && G.t(RP_T_WV)) {
      RUN(X, "ce_patch_label", 0, 16.0 * Td, k_ce_patch_label(X.st, pall, T, D.V, labels, X.at<float>(P.h_l), X.at<float>(P.h_coef)));
      RUN(X, "ce_scale_x", 0, 4.0 * Td * D.h,
          k_ce_scale_x(X.st, X.at<void>(P.h_xf), X.at<float>(P.h_coef), X.at<float>(P.h_l), X.at<void>(P.h_xs), T, D.h));
      for (int v0 = 0; v0 < D.V; v0 += P.head_chunk) {
        const int vc = (D.V - v0 < P.head_chunk) ? (D.V - v0) : P.head_chunk;
        GemmArgs w; gemm_zero_args(w);  // dW_c[vc, h] += P'_c . xs
        w.A = pall + (size_t)v0 * T; w.lda = T; w.B = X.at<void>(P.h_xs); w.ldb = D.h; w.M = vc; w.N = D.h; w.K = T;
        w.C = G.t(RP_T_WV) + (size_t)v0 * D.h; w.ldc = D.h; w.beta = 1; w.epi = EPI_F32;
        X.give_split_ws(w);
        X.mark_gemm(GEMM_NN, w);
        X.chk(gemm_launch(X.st, GEMM_NN, w), "lm head dW");
      }
    }
    RUN(X, "ce_frozen_dx", 0, 8.0 * Td * D.h + 2.0 * Td * D.h,
        k_ce_frozen_dx(X.st, acc, X.at<float>(P.h_l), X.at<float>(P.h_coef), labels, Wv, T, D.h, D.V));
    RUN(X, "rmsnorm_bwd", 0, 8.0 * Td * D.h,
        k_rmsnorm_bwd(X.st, acc, 1, x, W.t(RP_T_GF), X.at<float>(P.h_rstd), nullptr, dx, train ? G.t(RP_T_GF) : nullptr,
                      X.at<float>(P.h_partials), T, D.h));
    return finish_call(ctx, sl, X);
  }
  {  // sweep 1: logits tile by tile, reduced to per-token (max, sum exp) partials; nothing of size T x V is stored
    GemmArgs g; gemm_zero_args(g);
    g.A = Wv; g.lda = D.h; g.B = X.at<void>(P.h_xf); g.ldb = D.h; g.M = D.V; g.N = T; g.K = D.h; g.epi = EPI_CE_STATS;
    g.labels = labels; g.zlab = X.at<float>(P.h_zlab); g.part = X.at<float2>(P.h_part); g.part_ld = T;
    X.mark_gemm(GEMM_NT, g);
    X.chk(gemm_launch(X.st, GEMM_NT, g), "lm head sweep 1");
  }
  RUN(X, "ce_lse", 0, 8.0 * P.head_parts * Td, k_ce_lse(X.st, X.at<float2>(P.h_part), P.head_parts, T, X.at<float>(P.h_lse), T));
  RUN(X, "ce_finalize", 0, 16.0 * Td,
      k_ce_finalize(X.st, X.at<float>(P.h_lse), X.at<float>(P.h_zlab), labels, grad_scale, X.at<float>(P.h_coef), loss_out, T));
  RUN(X, "fill", 0, 4.0 * Td * D.h, k_fill_u32(X.st, X.at<void>(P.h_dxacc), (long)T * D.h, 0u));
  // sweep 2: per vocabulary chunk recompute the logits, turn them into dZ^T (bf16), and feed dX and dW
  for (int v0 = 0, ci = 0; v0 < D.V; v0 += P.head_chunk, ++ci) {
    const int vc = (D.V - v0 < P.head_chunk) ? (D.V - v0) : P.head_chunk;
    const bf16_t* Wc = Wv + (size_t)v0 * D.h;
    GemmArgs g; gemm_zero_args(g);
    g.A = Wc; g.lda = D.h; g.B = X.at<void>(P.h_xf); g.ldb = D.h; g.M = vc; g.N = T; g.K = D.h; g.epi = EPI_CE_DZ;
    g.C = X.at<void>(P.h_dzt); g.ldc = T; g.labels = labels; g.lse = X.at<float>(P.h_lse); g.coef = X.at<float>(P.h_coef);
    g.row_offset = v0;
    X.mark_gemm(GEMM_NT, g);
    X.chk(gemm_launch(X.st, GEMM_NT, g), "lm head sweep 2");
    GemmArgs d; gemm_zero_args(d);   // dXf[T, h] (+)= dZ^T^T . W_c   (reduction over the chunk's vocabulary rows)
    d.A = X.at<void>(P.h_dzt); d.lda = T; d.B = Wc; d.ldb = D.h; d.M = T; d.N = D.h; d.K = vc; d.C = X.at<void>(P.h_dxacc);
    d.ldc = D.h; d.beta = 1; d.epi = EPI_F32;
    X.give_split_ws(d);
    X.mark_gemm(GEMM_TN, d);
    X.chk(gemm_launch(X.st, GEMM_TN, d), "lm head dX");
    if (G.t(RP_T_WV)) {
      GemmArgs w; gemm_zero_args(w);  // dW_c[vc, h] += dZ^T . xf
      w.A = X.at<void>(P.h_dzt); w.lda = T; w.B = X.at<void>(P.h_xf); w.ldb = D.h; w.M = vc; w.N = D.h; w.K = T;
      w.C = G.t(RP_T_WV) + (size_t)v0 * D.h; w.ldc = D.h; w.beta = 1; w.epi = EPI_F32;
      X.give_split_ws(w);
      X.mark_gemm(GEMM_NN, w);
      X.chk(gemm_launch(X.st, GEMM_NN, w), "lm head dW");
    }
  }
  RUN(X, "rmsnorm_bwd", 0, 8.0 * Td * D.h,
      k_rmsnorm_bwd(X.st, X.at<void>(P.h_dxacc), 1, x, W.t(RP_T_GF), X.at<float>(P.h_rstd), nullptr, dx, G.t(RP_T_GF), X.at<float>(P.h_partials), T, D.h));
  return finish_call(ctx, sl, X);
}

// ---- per-kernel timeline ---------------------------------------------------------------------------------------------
rp_status rp_trace_start(rp_ctx* ctx, int max_records) {
  if (!ctx) return fail(nullptr, RP_EINVAL, "ctx is NULL");
  if (max_records <= 0 || max_records > (1 << 20)) return fail(ctx, RP_EINVAL, "bad max_records");
  if (ctx->trace_cap < max_records) {
    if (ctx->trace_ev) {
      for (int i = 0; i <= ctx->trace_cap; ++i) if (ctx->trace_ev[i]) (void)hipEventDestroy(ctx->trace_ev[i]);
      delete[] ctx->trace_ev;
      delete[] ctx->trace_rec;
      ctx->trace_ev = nullptr; ctx->trace_rec = nullptr; ctx->trace_cap = 0;
    }
    ctx->trace_ev = new (std::nothrow) hipEvent_t[max_records + 1]();
    ctx->trace_rec = new (std::nothrow) TraceRec[max_records];
    if (!ctx->trace_ev || !ctx->trace_rec) return fail(ctx, RP_ENOMEM, "out of host memory");
    for (int i = 0; i <= max_records; ++i) HIP_TRY(ctx, hipEventCreate(&ctx->trace_ev[i]));
    ctx->trace_cap = max_records;
  }
  ctx->trace_n = 0;
  ctx->tracing = true;
  return RP_OK;
}

rp_status rp_trace_stop(rp_ctx* ctx, rp_trace_record* out, int cap, int* n_out) {
  if (!ctx || !n_out) return fail(ctx, RP_EINVAL, "NULL argument");
  if (!ctx->tracing) return fail(ctx, RP_ESTATE, "trace not started");
  ctx->tracing = false;
  HIP_TRY(ctx, hipStreamSynchronize(ctx->compute));
  const int n = ctx->trace_n < cap ? ctx->trace_n : cap;
  for (int i = 0; i < n; ++i) {
    float ms = 0.f;
    // the end of op i is the start of op i+1 (or the call's trailing event); ops of one stream run back to back
    HIP_TRY(ctx, hipEventElapsedTime(&ms, ctx->trace_ev[i], ctx->trace_ev[i + 1]));
    if (out) {
      snprintf(out[i].name, sizeof(out[i].name), "%s", ctx->trace_rec[i].name);
      out[i].flops = ctx->trace_rec[i].flops; out[i].bytes = ctx->trace_rec[i].bytes; out[i].ms = ms;
    }
  }
  *n_out = n;
  return RP_OK;
}

// ---- kernel-level entry points (unit parity tests) ----------------------------------------------------------------
#define OP_RET(e) return ((e) == hipSuccess ? RP_OK : fail(nullptr, RP_EHIP, "%s", hipGetErrorString(e)))

rp_status rp_op_gemm(void* stream, int layout, int out_f32, const void* A, const void* B, void* C, int M, int N, int K,
                     long lda, long ldb, long ldc, float alpha, int beta, const void* A2, const void* B2, int K2, long lda2,
                     long ldb2, const void* R, long ldr, int tile, void* split_ws, size_t split_ws_bytes) {
  if (out_f32 < 0 || out_f32 > 3 || (out_f32 == 3 && !split_ws) || (split_ws && reinterpret_cast<uintptr_t>(split_ws) % 16))
    return fail(nullptr, RP_EINVAL, "rp_op_gemm: bad out_f32 / split_ws");
  if (!A || !B || !C || M < 0 || N < 0 || K < 0 || K % 8 || K2 % 8 || lda % 8 || ldb % 8 || layout < 0 || layout > 2 || tile < 0 || tile > 7)
    return fail(nullptr, RP_EINVAL, "rp_op_gemm: bad arguments");
  if ((layout != GEMM_NT) && (N % 8 || (layout == GEMM_TN && M % 8))) return fail(nullptr, RP_EINVAL, "rp_op_gemm: transposed operands need multiples of 8");
  GemmArgs g; gemm_zero_args(g);
  g.A = A; g.B = B; g.C = C; g.M = M; g.N = N; g.K = K; g.lda = lda; g.ldb = ldb; g.ldc = ldc; g.alpha = alpha; g.beta = beta;
  g.A2 = A2; g.B2 = B2; g.K2 = (A2 && B2) ? K2 : 0; g.lda2 = lda2; g.ldb2 = ldb2; g.R = R; g.ldr = ldr;
  g.epi = out_f32 == 2 ? EPI_F32_ATOMIC : (out_f32 ? EPI_F32 : EPI_BF16);
  g.split_ws = static_cast<float*>(split_ws); g.split_ws_bytes = split_ws ? split_ws_bytes : 0; g.split_out_bf16 = out_f32 == 3;
  if (tile == 6) { g.b_direct = 1; tile = 0; }   // B and B2 in fragment order (rp_op_gemm_arrange)
  hipError_t e = gemm_launch(reinterpret_cast<hipStream_t>(stream), layout, g, tile);
  OP_RET(e);
}

rp_status rp_op_gemm_arrange(void* stream, const void* B, long ldb, int N, int K, int transposed, void* out, size_t out_bytes) {
  if (!B || !out || N < 0 || K < 0 || K % 8 || ldb % 8 || (transposed && N % 8)) return fail(nullptr, RP_EINVAL, "rp_op_gemm_arrange: bad arguments");
  if (out_bytes < gemm_arranged_bytes(N, K)) return fail(nullptr, RP_EINVAL, "rp_op_gemm_arrange: out holds %zu bytes, %zu needed", out_bytes, gemm_arranged_bytes(N, K));
  hipError_t e = gemm_arrange(reinterpret_cast<hipStream_t>(stream), B, ldb, N, K, transposed, out);
  OP_RET(e);
}

rp_status rp_op_rmsnorm_fwd(void* stream, const void* x, const void* g, void* y, float* rstd, int T, int h, float eps) {
  if (!x || !g || !y || h % 8 || h > 8192) return fail(nullptr, RP_EINVAL, "rp_op_rmsnorm_fwd: bad arguments");
  hipError_t e = k_rmsnorm_fwd(reinterpret_cast<hipStream_t>(stream), x, g, y, rstd, T, h, eps);
  OP_RET(e);
}

rp_status rp_op_rmsnorm_bwd(void* stream, const void* dy, int dy_is_f32, const void* x, const void* g, const float* rstd,
                            const void* dres, void* dx, float* dg, float* scratch, int T, int h) {
  if (!dy || !x || !g || !rstd || !dx || h % 8 || h > 8192 || (dg && !scratch)) return fail(nullptr, RP_EINVAL, "rp_op_rmsnorm_bwd: bad arguments");
  hipError_t e = k_rmsnorm_bwd(reinterpret_cast<hipStream_t>(stream), dy, dy_is_f32, x, g, rstd, dres, dx, dg, scratch, T, h);
  OP_RET(e);
}

rp_status rp_op_rmsnorm_bwd_noalloc(void* stream, const void* dy, int dy_is_f32, const void* x, const void* g, const float* rstd,
                                    const void* dres, void* dx, float* dg, int T, int h) {
  if (!dy || !x || !g || !rstd || !dx || T < 0 || h <= 0 || h % 8) return fail(nullptr, RP_EINVAL, "rp_op_rmsnorm_bwd_noalloc: bad arguments");
  if (h > NOALLOC_MAX_H)
    return fail(nullptr, RP_EINVAL, "rp_op_rmsnorm_bwd_noalloc: h = %d exceeds the built-in scratch (h <= %d); use rp_op_rmsnorm_bwd with a caller-owned scratch", h, NOALLOC_MAX_H);
  hipError_t e = hipSuccess;
  float* const sp = noalloc_scratch(&e);
  if (!sp) return fail(nullptr, RP_EHIP, "rp_op_rmsnorm_bwd_noalloc: scratch look-up failed: %s", hipGetErrorString(e));
  // every partial row the column sum reads is written by the kernel before it: nothing has to start at zero
  e = k_rmsnorm_bwd(reinterpret_cast<hipStream_t>(stream), dy, dy_is_f32, x, g, rstd, dres, dx, dg, sp, T, h);
  OP_RET(e);
}

rp_status rp_op_rope_table(void* stream, void* cs, int seq, int d, float base) {
  if (!cs || (d != 64 && d != 128)) return fail(nullptr, RP_EINVAL, "rp_op_rope_table: bad arguments");
  hipError_t e = k_rope_table(reinterpret_cast<hipStream_t>(stream), static_cast<float2*>(cs), seq, d, base);
  OP_RET(e);
}

rp_status rp_op_qknorm_rope(void* stream, int bwd, int d, const void* in_q, const void* in_k, long ld_in_q, long ld_in_k,
                            void* out_q, void* out_k, long ld_out_q, long ld_out_k, const void* gq, const void* gk, float* rstd_q,
                            float* rstd_k, const void* raw_q, const void* raw_k, long ld_raw, float* dgq, float* dgk,
                            float* scratch, const void* cs, int T, int seq, int a, int k, int use_norm, float eps) {
  if (!in_q || !in_k || !out_q || !out_k || !cs || (d != 64 && d != 128)) return fail(nullptr, RP_EINVAL, "rp_op_qknorm_rope: bad arguments");
  if (use_norm && (!gq || !gk || !rstd_q || !rstd_k || (bwd && (!raw_q || !raw_k)))) return fail(nullptr, RP_EINVAL, "rp_op_qknorm_rope: norm buffers missing");
  if (bwd && use_norm && dgq && dgk && !scratch) return fail(nullptr, RP_EINVAL, "rp_op_qknorm_rope: scratch missing");
  hipError_t e = k_qknorm_rope(reinterpret_cast<hipStream_t>(stream), bwd, d, in_q, in_k, ld_in_q, ld_in_k, out_q, out_k, ld_out_q,
                               ld_out_k, gq, gk, rstd_q, rstd_k, raw_q, raw_k, ld_raw, dgq, dgk, scratch, static_cast<const float2*>(cs), T,
                               seq, a, k, use_norm, eps);
  OP_RET(e);
}

rp_status rp_op_swiglu_fwd(void* stream, const void* gu, void* act, long T, int m) {
  if (!gu || !act || m % 8) return fail(nullptr, RP_EINVAL, "rp_op_swiglu_fwd: bad arguments");
  hipError_t e = k_swiglu_fwd(reinterpret_cast<hipStream_t>(stream), gu, act, T, m);
  OP_RET(e);
}

rp_status rp_op_swiglu_bwd(void* stream, const void* dact, const void* gu, void* dgu, long T, int m) {
  if (!dact || !gu || !dgu || m % 8) return fail(nullptr, RP_EINVAL, "rp_op_swiglu_bwd: bad arguments");
  hipError_t e = k_swiglu_bwd(reinterpret_cast<hipStream_t>(stream), dact, gu, dgu, T, m);
  OP_RET(e);
}

rp_status rp_op_moe_route_plan(void* stream, const float* logits, int T, int E, int top_k, int* idx, float* w, int* counts,
                               int* seg, void* tile_tab, int* ntiles, int* slot_of, int* row_tok, int* hist) {
  if (!logits || !idx || !w || !counts || !seg || !tile_tab || !ntiles || !slot_of || !row_tok || !hist || T < 0 || E <= 0 ||
      E > 1024 || top_k <= 0 || top_k > E || top_k > 64)
    return fail(nullptr, RP_EINVAL, "rp_op_moe_route_plan: bad arguments");
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  hipError_t e = k_moe_route(st, logits, idx, w, T, E, top_k);
  if (e == hipSuccess) e = k_moe_plan(st, idx, T, E, top_k, counts, seg, tile_tab, ntiles, slot_of, row_tok, hist);
  OP_RET(e);
}

rp_status rp_op_attn_fwd(void* stream, const void* q, const void* k, const void* v, void* o, float* lse, long ldq, long ldk,
                         long ldv, long ldo, int batch, int seq, int a, int kh, int d) {
  if (!q || !k || !v || !o || !lse || (d != 64 && d != 128) || a <= 0 || kh <= 0 || a % kh || ldq % 8 || ldk % 8 || ldv % 8 || ldo % 8)
    return fail(nullptr, RP_EINVAL, "rp_op_attn_fwd: bad arguments");
  hipError_t e = k_attn_fwd(reinterpret_cast<hipStream_t>(stream), q, k, v, o, lse, ldq, ldk, ldv, ldo, batch, seq, a, kh, d);
  OP_RET(e);
}

rp_status rp_op_attn_bwd(void* stream, const void* q, const void* k, const void* v, const void* o, const void* dout,
                         const float* lse, float* delta, void* dq, void* dk, void* dv, float* scratch, long ldq, long ldk,
                         long ldv, long ldo, long lddo, long lddq, long lddk, long lddv, int batch, int seq, int a, int kh,
                         int d) {
  if (!q || !k || !v || !o || !dout || !lse || !delta || !dq || !dk || !dv || (d != 64 && d != 128) || a <= 0 || kh <= 0 || a % kh)
    return fail(nullptr, RP_EINVAL, "rp_op_attn_bwd: bad arguments");
  if (a != kh && !scratch) return fail(nullptr, RP_EINVAL, "rp_op_attn_bwd: grouped queries need the scratch buffer");
  if (ldq % 8 || ldk % 8 || ldv % 8 || ldo % 8 || lddo % 8 || lddq % 8 || lddk % 8 || lddv % 8) return fail(nullptr, RP_EINVAL, "rp_op_attn_bwd: strides must be multiples of 8");
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  hipError_t e = k_attn_delta(st, o, dout, delta, ldo, lddo, batch, seq, a, d);
  static const int parts[3] = {0, 2, 1};
  for (int i = 0; i < 3 && e == hipSuccess; ++i)
    e = k_attn_bwd(st, parts[i], q, k, v, dout, lse, delta, dq, dk, dv, scratch, ldq, ldk, ldv, lddo, lddq, lddk, lddv, batch, seq,
                   a, kh, d);
  OP_RET(e);
}


// ---- rounds ---------------------------------------------------------------------------------------------------------
rp_status rp_ctx_set_transfer_streams(rp_ctx* ctx, void* act_upload_stream, void* act_download_stream, void* grad_download_stream) {
  if (!ctx) return fail(nullptr, RP_EINVAL, "ctx is NULL");
  if (!act_upload_stream || !act_download_stream || !grad_download_stream) return fail(ctx, RP_EINVAL, "all three streams must be non-NULL");
  ctx->act_up = reinterpret_cast<hipStream_t>(act_upload_stream);
  ctx->act_down = reinterpret_cast<hipStream_t>(act_download_stream);
  ctx->grad_down = reinterpret_cast<hipStream_t>(grad_download_stream);
  return RP_OK;
}

namespace {

rp_status ensure_round_events(rp_ctx* ctx, int n) {
  if (ctx->round_ev_n >= n) return RP_OK;
  ctx->prev_round = false;   // the handles move: fall back to waiting for everything enqueued so far
  hipEvent_t* ev = new (std::nothrow) hipEvent_t[n]();
  if (!ev) return fail(ctx, RP_ENOMEM, "out of host memory");
  for (int i = 0; i < ctx->round_ev_n; ++i) ev[i] = ctx->round_ev[i];
  delete[] ctx->round_ev;
  ctx->round_ev = ev;
  for (int i = ctx->round_ev_n; i < n; ++i) {
    if (hipEventCreateWithFlags(&ev[i], hipEventDisableTiming) != hipSuccess) { ctx->round_ev_n = i; return fail(ctx, RP_EHIP, "hipEventCreate failed"); }
  }
  ctx->round_ev_n = n;
  return RP_OK;
}

// Byte ranges of the tensors of a blob (all layer chunks, then the head chunk), in blob order.
void blob_items(const rp_stage_cfg& c, const BlobLayout& B, size_t es, std::vector<size_t>& off, std::vector<size_t>& bytes) {
  for (int l = 0; l <= c.n_layers; ++l)
    for (int id = 0; id < RP_T_COUNT; ++id) {
      if (is_head_tensor(id) != (l == c.n_layers) || B.elems[id] == 0) continue;
      off.push_back(B.layer_bytes * (size_t)l + B.off[id]);
      bytes.push_back(B.elems[id] * es);
    }
}

rp_status round_run(rp_ctx* ctx, int slot_id, const rp_round_io* io, bool backward, void* grads, int batch, int seq,
                    void* workspace, size_t workspace_bytes_in) {
  if (!ctx) return fail(nullptr, RP_EINVAL, "ctx is NULL");
  if (!io || io->struct_size != sizeof(rp_round_io)) return fail(ctx, RP_EINVAL, "io is NULL or io.struct_size != %zu", sizeof(rp_round_io));
  if (!ctx->act_up) return fail(ctx, RP_ESTATE, "rp_ctx_set_transfer_streams has not been called");
  if (ctx->cfg.n_layers == 0) return fail(ctx, RP_EINVAL, "stage has no decoder layers");
  if (ctx->cfg.n_experts > 0) return fail(ctx, RP_EUNSUPPORTED, "rounds cover dense stages only");
  const int M = io->n_micro;
  if (M < 1 || M > 256) return fail(ctx, RP_EINVAL, "n_micro must be in [1, 256]");
  const Plan P = make_plan(ctx->cfg, batch > 0 ? batch : 1, seq > 0 ? seq : 8);
  rp_status s = check_call(ctx, slot_id, batch, seq, workspace, workspace_bytes_in, backward ? P.bwd_bytes : P.fwd_bytes);
  if (s != RP_OK) return s;
  if (!io->x_host || !io->out_host || (backward && !io->dy_host)) return fail(ctx, RP_EINVAL, "host activation arrays must be non-NULL");
  for (int j = 0; j < M; ++j)
    if (!io->x_host[j] || !io->out_host[j] || (backward && !io->dy_host[j])) return fail(ctx, RP_EINVAL, "host activation pointer %d is NULL", j);
  for (int b = 0; b < 2; ++b) {
    if (!io->x_dev[b] || !io->out_dev[b] || (backward && !io->dy_dev[b])) return fail(ctx, RP_EINVAL, "device staging buffers must be non-NULL");
    if (io->x_dev[b] == io->out_dev[b]) return fail(ctx, RP_EINVAL, "x_dev and out_dev must be distinct");
  }
  if (io->x_dev[0] == io->x_dev[1] || io->out_dev[0] == io->out_dev[1] || (backward && io->dy_dev[0] == io->dy_dev[1]))
    return fail(ctx, RP_EINVAL, "the two staging buffers of a direction must be distinct");
  if (backward && !grads && ctx->gl.total > 0) return fail(ctx, RP_EINVAL, "grads is NULL but the stage has trainable tensors");
  const bool up = io->next_slot >= 0;
  if (up) {
    if (io->next_slot >= RP_MAX_SLOTS || io->next_slot == slot_id) return fail(ctx, RP_EINVAL, "next_slot must be another valid slot");
    if (!io->next_dev_slot || !io->next_host_blob) return fail(ctx, RP_EINVAL, "next_dev_slot / next_host_blob are NULL");
    if (reinterpret_cast<uintptr_t>(io->next_dev_slot) % 256) return fail(ctx, RP_EINVAL, "next_dev_slot must be 256-byte aligned");
  }
  const bool down = io->done_grads_dev != nullptr && ctx->gl.total > 0;
  if (down && !io->done_grads_host) return fail(ctx, RP_EINVAL, "done_grads_host is NULL");
  const size_t max_piece = io->max_piece_bytes ? io->max_piece_bytes : ((size_t)64 << 20);
  if (max_piece % 256) return fail(ctx, RP_EINVAL, "max_piece_bytes must be a multiple of 256");
  const int half = 3 * 256 + 2;                      // events of one round at the largest n_micro
  s = ensure_round_events(ctx, 2 * half);
  if (s != RP_OK) return s;
  hipEvent_t* const pool = ctx->round_ev + (ctx->round_parity ? half : 0);
  hipEvent_t* const e_up = pool;                     // activation upload of micro-batch j has landed
  hipEvent_t* const e_done = pool + M;               // compute of micro-batch j has finished
  hipEvent_t* const e_down = pool + 2 * M;           // result of micro-batch j has left its staging buffer
  const hipEvent_t e_start = pool[3 * M], e_start_down = pool[3 * M + 1];
  // Same staging buffers as the round before (the steady state of a worker): the first uploads and results wait only
  // for the predecessor's last use of the very buffer, so the rounds overlap like the micro-batches inside one.
  bool chained = ctx->prev_round;
  for (int b = 0; b < 2 && chained; ++b)
    chained = io->x_dev[b] == ctx->prev_x[b] && io->out_dev[b] == ctx->prev_out[b] && (!backward || io->dy_dev[b] == ctx->prev_dy[b]);

  // transfer plans: the tensors of the next stage's weight blob and of the finished stage's gradient blob, M windows
  std::vector<size_t> w_off, w_bytes, g_off, g_bytes;
  std::vector<rp_piece> w_plan, g_plan;
  if (up) { blob_items(ctx->cfg, ctx->wl, 2, w_off, w_bytes); w_plan = plan_transfers(w_bytes.data(), (int)w_bytes.size(), M, max_piece); }
  if (down) { blob_items(ctx->cfg, ctx->gl, 4, g_off, g_bytes); g_plan = plan_transfers(g_bytes.data(), (int)g_bytes.size(), M, max_piece); }

  const size_t act_bytes = (size_t)batch * seq * ctx->cfg.hidden * 2;
  // work enqueued before this call may still use the staging buffers: the first uploads wait for the compute stream as
  // it stands now, the first results for the activation-download stream as it stands now
  HIP_TRY(ctx, hipEventRecord(e_start, ctx->compute));
  if (!chained) {
    HIP_TRY(ctx, hipStreamWaitEvent(ctx->act_up, e_start, 0));
    HIP_TRY(ctx, hipEventRecord(e_start_down, ctx->act_down));
    HIP_TRY(ctx, hipStreamWaitEvent(ctx->compute, e_start_down, 0));
  }
  if (down) HIP_TRY(ctx, hipStreamWaitEvent(ctx->grad_down, e_start, 0));   // the finished gradients were written on the compute stream
  if (up) {
    Slot& nx = ctx->slots[io->next_slot];
    if (nx.used) HIP_TRY(ctx, hipStreamWaitEvent(ctx->copy, nx.free_ev, 0));
  }
  auto upload = [&](int j) -> rp_status {
    const int b = j & 1;
    if (j >= 2) HIP_TRY(ctx, hipStreamWaitEvent(ctx->act_up, e_done[j - 2], 0));   // the staging buffer's last reader
    else if (chained && ctx->prev_done[b]) HIP_TRY(ctx, hipStreamWaitEvent(ctx->act_up, ctx->prev_done[b], 0));
    HIP_TRY(ctx, hipMemcpyAsync(io->x_dev[b], io->x_host[j], act_bytes, hipMemcpyHostToDevice, ctx->act_up));
    if (backward) HIP_TRY(ctx, hipMemcpyAsync(io->dy_dev[b], io->dy_host[j], act_bytes, hipMemcpyHostToDevice, ctx->act_up));
    HIP_TRY(ctx, hipEventRecord(e_up[j], ctx->act_up));
    return RP_OK;
  };
  s = upload(0);
  if (s != RP_OK) return s;
  for (int j = 0; j < M; ++j) {
    const int b = j & 1;
    // window j opens: the next micro-batch's activations go up while this one computes (one micro-batch early)
    if (j + 1 < M) { s = upload(j + 1); if (s != RP_OK) return s; }
    HIP_TRY(ctx, hipStreamWaitEvent(ctx->compute, e_up[j], 0));
    if (j >= 2) HIP_TRY(ctx, hipStreamWaitEvent(ctx->compute, e_down[j - 2], 0));   // out_dev[b] has been sent home
    else if (chained && ctx->prev_down[b]) HIP_TRY(ctx, hipStreamWaitEvent(ctx->compute, ctx->prev_down[b], 0));
    if (backward)
      s = rp_stage_backward(ctx, slot_id, RP_PHASE_BOTH, io->x_dev[b], io->dy_dev[b], io->out_dev[b], nullptr, grads, nullptr, nullptr,
                            batch, seq, workspace, workspace_bytes_in);
    else
      s = rp_stage_forward(ctx, slot_id, io->x_dev[b], io->out_dev[b], nullptr, nullptr, batch, seq, workspace, workspace_bytes_in);
    if (s != RP_OK) return s;
    HIP_TRY(ctx, hipEventRecord(e_done[j], ctx->compute));
    // the result goes home while the next micro-batch computes (one micro-batch late)
    HIP_TRY(ctx, hipStreamWaitEvent(ctx->act_down, e_done[j], 0));
    HIP_TRY(ctx, hipMemcpyAsync(io->out_host[j], io->out_dev[b], act_bytes, hipMemcpyDeviceToHost, ctx->act_down));
    HIP_TRY(ctx, hipEventRecord(e_down[j], ctx->act_down));
    // window j's chunk of the next stage's parameters: not before the window opens, and behind its activation upload
    if (up) {
      if (j >= 1) HIP_TRY(ctx, hipStreamWaitEvent(ctx->copy, e_done[j - 1], 0));
      HIP_TRY(ctx, hipStreamWaitEvent(ctx->copy, e_up[j + 1 < M ? j + 1 : j], 0));
      for (const rp_piece& pc : w_plan)
        if (pc.window == j) {
          const size_t o = w_off[pc.item] + pc.offset;
          HIP_TRY(ctx, hipMemcpyAsync(static_cast<char*>(io->next_dev_slot) + o, static_cast<const char*>(io->next_host_blob) + o, pc.bytes,
                                      hipMemcpyHostToDevice, ctx->copy));
        }
    }
    // window j's chunk of the finished stage's gradients: behind the activation download that falls into this window
    if (down) {
      if (j >= 1) HIP_TRY(ctx, hipStreamWaitEvent(ctx->grad_down, e_down[j - 1], 0));
      for (const rp_piece& pc : g_plan)
        if (pc.window == j) {
          const size_t o = g_off[pc.item] + pc.offset;
          HIP_TRY(ctx, hipMemcpyAsync(static_cast<char*>(io->done_grads_host) + o, static_cast<const char*>(io->done_grads_dev) + o, pc.bytes,
                                      hipMemcpyDeviceToHost, ctx->grad_down));
        }
    }
  }
  for (int b = 0; b < 2; ++b) {
    // last micro-batch that used staging buffer b.  With one micro-batch buffer 1 was not touched: whoever used it
    // earlier is already ordered before this round's transfers, which waited for later work on the same streams
    const int j = ((M - 1) & 1) == b ? M - 1 : M - 2;
    ctx->prev_done[b] = j >= 0 ? e_done[j] : nullptr;
    ctx->prev_down[b] = j >= 0 ? e_down[j] : nullptr;
    ctx->prev_x[b] = io->x_dev[b]; ctx->prev_out[b] = io->out_dev[b]; ctx->prev_dy[b] = backward ? io->dy_dev[b] : ctx->prev_dy[b];
  }
  ctx->prev_round = true;
  ctx->round_parity ^= 1;
  if (up) {   // every chunk of the next slot is complete once the copy stream gets here
    Slot& nx = ctx->slots[io->next_slot];
    for (int l = 0; l < ctx->cfg.n_layers; ++l) HIP_TRY(ctx, build_derived(ctx, ctx->copy, static_cast<char*>(io->next_dev_slot), l));
    for (int l = 0; l <= ctx->cfg.n_layers; ++l) HIP_TRY(ctx, hipEventRecord(nx.ev[l], ctx->copy));
    nx.dev = io->next_dev_slot; nx.bytes = ctx->wl.total; nx.valid = true; nx.gated = true; nx.used = false;
  }
  return RP_OK;
}

}  // namespace

rp_status rp_round_forward(rp_ctx* ctx, int slot_id, const rp_round_io* io, int batch, int seq, void* workspace, size_t workspace_bytes) {
  return round_run(ctx, slot_id, io, false, nullptr, batch, seq, workspace, workspace_bytes);
}
rp_status rp_round_backward(rp_ctx* ctx, int slot_id, const rp_round_io* io, void* grads, int batch, int seq, void* workspace,
                            size_t workspace_bytes) {
  return round_run(ctx, slot_id, io, true, grads, batch, seq, workspace, workspace_bytes);
}

}  // extern "C"
