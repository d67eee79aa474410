// Blob layouts (weights bf16, gradients fp32) and the workspace plan.  Pure host arithmetic, no HIP calls.
#pragma once
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include "../../include/rp.h"
#include "kernels.hpp"   // RP_PARTIAL_BLOCKS
#include "gemm.hpp"      // RP_SPLITK_WS_BYTES

namespace rp {

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Dims {
  int L, h, a, kh, d, qd, kd, n1, m, V, E, topk, r;
  bool lora[7];     // q k v o gate up down
  int n_qkv, n_gu;  // number of adapted projections in the fused qkv / gate-up GEMMs
};

inline Dims dims_of(const rp_stage_cfg& c) {
  Dims D{};
  D.L = c.n_layers; D.h = c.hidden; D.a = c.n_q_heads; D.kh = c.n_kv_heads; D.d = c.head_dim;
  D.qd = D.a * D.d; D.kd = D.kh * D.d; D.n1 = D.qd + 2 * D.kd; D.m = c.ffn; D.V = c.vocab;
  D.E = c.n_experts; D.topk = c.top_k; D.r = c.lora_rank;
  for (int i = 0; i < 7; ++i) D.lora[i] = D.r > 0 && ((c.lora_mask >> i) & 1u);
  D.n_qkv = (int)D.lora[0] + (int)D.lora[1] + (int)D.lora[2];
  D.n_gu = (int)D.lora[4] + (int)D.lora[5];
  return D;
}

// Element count of a tensor of the weight blob; 0 = absent for this configuration.
inline size_t tensor_elems(const rp_stage_cfg& c, int id) {
  const Dims D = dims_of(c);
  const size_t e = D.E > 0 ? (size_t)D.E : 1;
  const size_t r = (size_t)D.r;
  switch (id) {
    case RP_T_G1: case RP_T_G2: return D.L > 0 ? D.h : 0;
    case RP_T_WQKV: return (size_t)D.n1 * D.h;
    case RP_T_GQ: case RP_T_GK: return c.qk_norm ? D.d : 0;
    case RP_T_WO: return (size_t)D.h * D.qd;
    case RP_T_WGU: return e * 2 * D.m * D.h;
    case RP_T_WD: return e * (size_t)D.h * D.m;
    case RP_T_WR: return (D.E > 0 && c.moe_router) ? (size_t)D.E * D.h : 0;
    case RP_T_LA_Q: return D.lora[0] ? r * D.h : 0;
    case RP_T_LA_K: return D.lora[1] ? r * D.h : 0;
    case RP_T_LA_V: return D.lora[2] ? r * D.h : 0;
    case RP_T_LB_Q: return D.lora[0] ? (size_t)D.qd * r : 0;
    case RP_T_LB_K: return D.lora[1] ? (size_t)D.kd * r : 0;
    case RP_T_LB_V: return D.lora[2] ? (size_t)D.kd * r : 0;
    case RP_T_LA_O: return D.lora[3] ? r * D.qd : 0;
    case RP_T_LB_O: return D.lora[3] ? (size_t)D.h * r : 0;
    case RP_T_LA_GATE: return D.lora[4] ? r * D.h : 0;
    case RP_T_LA_UP: return D.lora[5] ? r * D.h : 0;
    case RP_T_LB_GATE: return D.lora[4] ? (size_t)D.m * r : 0;
    case RP_T_LB_UP: return D.lora[5] ? (size_t)D.m * r : 0;
    case RP_T_LA_DOWN: return D.lora[6] ? r * D.m : 0;
    case RP_T_LB_DOWN: return D.lora[6] ? (size_t)D.h * r : 0;
    case RP_T_GF: return D.V > 0 ? D.h : 0;
    case RP_T_WV: return (size_t)D.V * D.h;
    default: return 0;
  }
}

inline bool is_head_tensor(int id) { return id == RP_T_GF || id == RP_T_WV; }
inline bool is_lora_tensor(int id) { return id >= RP_T_LA_Q && id <= RP_T_LB_DOWN; }

// Tensors are packed back to back in enum order inside a chunk (all sizes are multiples of 16 bytes); chunks start on
// 256-byte boundaries.  elem_size 2 = weight blob, 4 = gradient blob (where frozen tensors are absent).
struct BlobLayout {
  size_t layer_bytes = 0, head_bytes = 0, total = 0;
  size_t off[RP_T_COUNT];    // offset inside its chunk
  size_t elems[RP_T_COUNT];
};

inline BlobLayout blob_layout(const rp_stage_cfg& c, bool grads) {
  BlobLayout B;
  const size_t es = grads ? 4 : 2;
  size_t lo = 0, ho = 0;
  for (int id = 0; id < RP_T_COUNT; ++id) {
    size_t n = tensor_elems(c, id);
    if (grads && !is_lora_tensor(id) && !c.train_base) n = 0;
    if (!is_head_tensor(id) && c.n_layers == 0) n = 0;
    B.elems[id] = n;
    if (is_head_tensor(id)) { B.off[id] = ho; ho += n * es; }
    else { B.off[id] = lo; lo += n * es; }
  }
  B.layer_bytes = align_up(lo, 256);
  B.head_bytes = align_up(ho, 256);
  B.total = B.layer_bytes * (size_t)c.n_layers + B.head_bytes;
  return B;
}

// Tensors the library derives from the uploaded blob and keeps behind it in the device slot, per layer: the
// block-diagonal LoRA B of the fused q|k|v and gate|up projections ([n1, n_qkv*r] and [2m, n_gu*r]; the adapted
// projections' B matrices on the diagonal, zeros elsewhere), built once when the weights arrive instead of in every call.
struct DerivedLayout {
  size_t bd1 = 0, bd3 = 0, layer_bytes = 0, total = 0;
};

inline DerivedLayout derived_layout(const rp_stage_cfg& c) {
  const Dims D = dims_of(c);
  DerivedLayout L;
  size_t o = 0;
  if (D.n_qkv > 0) { L.bd1 = o; o = align_up(o + (size_t)D.n1 * (size_t)(D.n_qkv * D.r) * 2, 256); }
  if (D.n_gu > 0) { L.bd3 = o; o = align_up(o + (size_t)2 * D.m * (size_t)(D.n_gu * D.r) * 2, 256); }
  L.layer_bytes = o;
  L.total = o * (size_t)(c.n_layers > 0 ? c.n_layers : 0);
  return L;
}

// ---- workspace plan ---------------------------------------------------------------------------------------------
struct LayerBuf {   // byte offsets of one layer's saved internals
  size_t z, rstd1, n1, qkv, rstd_q, rstd_k, qr, kr, o, lse, y, rstd2, n2, gu, act, u1, u2, u3, u4;
  // mixture of experts: routing (expert and weight per (token, choice)), the slot of every entry, the token of every
  // slot, per-expert counts and first slots, the tile table of the grouped GEMMs and its length
  size_t m_idx, m_w, m_slot, m_tok, m_cnt, m_seg, m_tab, m_ntiles, m_hist;
  size_t end;
};

struct Plan {
  size_t rope;                                    // RoPE table
  size_t layer0, layer_stride;                    // saved internals, one set per layer (backward) or one set (forward)
  size_t tA, tB, dact, dgu, dn, dout, dqr, dkr, dqkv, delta, ud, partials;   // backward temporaries
  size_t moe_f_fwd, moe_f_bwd;   // expert outputs / expert input gradients per slot [T*top_k, h] (transient in a layer)
  size_t moe_wslot, moe_dw;      // routing weight per slot, its gradient per slot (backward)
  size_t moe_dlog, moe_dlog16;   // router in the stage: gradient of the logits fp32 [T, E] and its bf16 copy
  int moe_max_tiles;             // capacity of the tile table
  size_t split_fwd, split_bwd, h_split;   // partial products of a GEMM reduction split (RP_SPLITK_WS_BYTES each), per plan
  size_t dkvp;   // per-query-head dK/dV partials of grouped attention; shares memory with dact|dgu, dead by then
  size_t fwd_bytes, bwd_bytes;
  // head
  size_t h_xf, h_rstd, h_part, h_zlab, h_lse, h_coef, h_dzt, h_dxacc, h_partials, head_bytes;
  bool head_keep_p;      // trainable head in one sweep (see make_plan)
  size_t h_pall, h_xs;   // then: the probabilities of the whole vocabulary [V, T] bf16, the scaled input
  size_t h_z, h_m, h_l, h_alpha, h_flag;   // frozen head: fp32 logits of one chunk, reference exponent, normaliser, rescale
                                           // factor, the flag that switches a chunk's slow path on
  int head_chunk, head_parts;
  LayerBuf lb;                                    // offsets relative to a layer set
};

inline Plan make_plan(const rp_stage_cfg& c, int batch, int seq) {
  const Dims D = dims_of(c);
  const size_t T = (size_t)batch * seq;
  Plan P{};
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o = align_up(o + bytes, 256); return r; };
  // one layer set
  LayerBuf& b = P.lb;
  b.z = take(T * D.h * 2); b.rstd1 = take(T * 4); b.n1 = take(T * D.h * 2); b.qkv = take(T * D.n1 * 2);
  b.rstd_q = take(T * D.a * 4); b.rstd_k = take(T * D.kh * 4); b.qr = take(T * D.qd * 2); b.kr = take(T * D.kd * 2);
  b.o = take(T * D.qd * 2); b.lse = take(T * D.a * 4); b.y = take(T * D.h * 2); b.rstd2 = take(T * 4);
  // with experts, gate/up and act hold one row per (token, choice), sorted by expert
  const size_t Tk = D.E > 0 ? T * (size_t)D.topk : T;
  const size_t max_tiles = Tk / 256 + (size_t)(D.E > 0 ? D.E : 0) + 1;
  P.moe_max_tiles = (int)max_tiles;
  b.n2 = take(T * D.h * 2); b.gu = take(Tk * 2 * D.m * 2); b.act = take(Tk * D.m * 2);
  b.u1 = take(T * (size_t)(D.n_qkv * D.r) * 2); b.u2 = take(T * (size_t)D.r * 2);
  b.u3 = take(T * (size_t)(D.n_gu * D.r) * 2); b.u4 = take(T * (size_t)D.r * 2);
  if (D.E > 0) {
    b.m_idx = take(Tk * 4); b.m_w = take(Tk * 4); b.m_slot = take(Tk * 4); b.m_tok = take(Tk * 4);
    b.m_cnt = take((size_t)D.E * 4); b.m_seg = take((size_t)(D.E + 1) * 4); b.m_tab = take(max_tiles * 16);
    b.m_ntiles = take(4);
    b.m_hist = take((Tk + RP_MOE_RUN - 1) / RP_MOE_RUN * (size_t)D.E * 4);
  }
  b.end = o;
  const size_t set = o;
  o = 0;
  P.rope = take((size_t)seq * (D.d / 2) * 8);
  P.layer0 = o;
  P.layer_stride = set;
  // forward-only: one set plus a second z buffer for ping-pong
  {
    size_t f = o + set;
    f = align_up(f + T * D.h * 2, 256);
    if (D.E > 0) { P.moe_f_fwd = f; f = align_up(f + Tk * D.h * 2, 256); }
    P.split_fwd = f;
    if (D.r > 0) f = align_up(f + RP_SPLITK_WS_BYTES, 256);   // only the skinny LoRA products split in a forward stage
    P.fwd_bytes = f;
  }
  o += set * (size_t)(D.L > 0 ? D.L : 0);
  P.tA = take(T * D.h * 2); P.tB = take(T * D.h * 2); P.dact = take(Tk * D.m * 2); P.dgu = take(Tk * 2 * D.m * 2);
  if (D.E > 0) { P.moe_f_bwd = take(Tk * D.h * 2); P.moe_wslot = take(Tk * 4); P.moe_dw = take(Tk * 4); }
  if (D.E > 0 && c.moe_router) { P.moe_dlog = take(T * D.E * 4); P.moe_dlog16 = take(T * D.E * 2); }
  P.dkvp = P.dact;
  if (D.a != D.kh && P.dkvp + 2 * T * D.qd * 4 > o) take(P.dkvp + 2 * T * D.qd * 4 - o);
  P.dn = take(T * D.h * 2); P.dout = take(T * D.qd * 2); P.dqr = take(T * D.qd * 2); P.dkr = take(T * D.kd * 2);
  P.dqkv = take(T * D.n1 * 2); P.delta = take(T * D.a * 4);
  P.ud = take(T * (size_t)(3 * D.r) * 2);
  P.split_bwd = take(RP_SPLITK_WS_BYTES);
  P.partials = take((size_t)RP_PARTIAL_BLOCKS * (size_t)(D.h > 2 * D.d ? D.h : 2 * D.d) * 4);
  P.bwd_bytes = o;
  // head
  o = 0;
  if (D.V > 0) {
    // vocabulary rows per pass: 32768 while the transposed dZ chunk stays within 2^27 elements, else 16384, unless the
    // configuration fixes it (the tests use that to put several chunks into a small vocabulary)
    P.head_chunk = (T * 32768 <= ((size_t)1 << 27)) ? 32768 : 16384;
    if (c.head_chunk > 0) P.head_chunk = c.head_chunk;
    if (P.head_chunk > D.V) P.head_chunk = (int)align_up(D.V, 8);
    P.head_parts = 2 * ((D.V + 255) / 256);
    P.h_xf = take(T * D.h * 2); P.h_rstd = take(T * 4); P.h_part = take((size_t)P.head_parts * T * 8);
    P.h_zlab = take(T * 4); P.h_lse = take(T * 4); P.h_coef = take(T * 4);
    // a trainable head in one sweep keeps every chunk's probabilities (h_pall, bf16 [V, T]) instead of one chunk's dZ^T:
    // taken when that buffer stays within 4 GiB (1.2 GB at 151936 x 4096), else the two-sweep schedule
    const bool keep_p = c.train_base && !c.head_two_sweeps && (size_t)D.V * T * 2 <= ((size_t)4 << 30);
    P.head_keep_p = keep_p;
    P.h_dzt = keep_p ? 0 : take((size_t)P.head_chunk * T * 2);
    P.h_dxacc = take(T * D.h * 4);
    P.h_partials = take((size_t)RP_PARTIAL_BLOCKS * D.h * 4);
    P.h_split = take(RP_SPLITK_WS_BYTES);
    if (!c.train_base || keep_p) {
      P.h_z = take((size_t)P.head_chunk * T * 4);
      P.h_m = take(T * 4); P.h_l = take(T * 4); P.h_alpha = take(T * 4); P.h_flag = take(4);
    }
    if (keep_p) { P.h_pall = take((size_t)D.V * T * 2); P.h_xs = take(T * D.h * 2); }
  }
  P.head_bytes = o;
  return P;
}

inline size_t workspace_bytes(const Plan& P, const rp_stage_cfg& c) {
  size_t w = 256;
  if (c.n_layers > 0) { if (P.fwd_bytes > w) w = P.fwd_bytes; if (P.bwd_bytes > w) w = P.bwd_bytes; }
  if (P.head_bytes > w) w = P.head_bytes;
  return w;
}

}  // namespace rp
