// Host-side interface of the bf16 MFMA GEMM family.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// Operand layouts.  "Reduction-contiguous" operands are read as they are; the others are transposed on their way
// into LDS.
//   NT: C[M,N] = A[M,K] * B[N,K]^T      (forward of a linear layer: activations x weights)
//   NN: C[M,N] = A[M,K] * B[K,N]        (activation gradient: dY x W)
//   TN: C[M,N] = A[K,M]^T * B[K,N]      (weight gradient: dY^T x X)
enum { GEMM_NT = 0, GEMM_NN = 1, GEMM_TN = 2 };

enum {
  EPI_BF16 = 0,      // C bf16 = alpha*acc (+ R)
  EPI_F32 = 1,       // C fp32 = alpha*acc (+ C if beta)
  EPI_F32_ATOMIC = 2,// C fp32 atomically += alpha*acc
  EPI_CE_STATS = 3,  // rows = vocab, cols = tokens: per-column (max, sum exp) partials + label logit
  EPI_CE_DZ = 4,     // C bf16 [rows, cols] = (exp(acc - lse[col]) - (row == label[col])) * coef[col]
  EPI_F32_COLMAX = 5,// C fp32 = acc, plus per-column maximum partials (part[...].x, one per 128 rows) and the label logit
  // The product is the gradient of act = silu(gate) * up ([M, N]); R holds gate | up ([M, 2N], row stride ldr) and
  // C ([M, 2N], row stride ldc) receives d gate | d up.  The product itself is rounded to bf16 on the way (as if it
  // had been stored) and never written.
  EPI_SWIGLU_BWD = 6,
  // rows = vocab, cols = tokens: C bf16 [rows, cols] = exp(min(acc - ref[col], CE_P_CLAMP)) against a per-token reference
  // exponent (p.lse holds ref), plus per-column partials (maximum of acc in .x, fp32 sum of the exponentials in .y, one
  // per 128 rows) and the label logit.  The frozen head's later vocabulary chunks: no logits go to memory.
  EPI_CE_P = 7,
  // NT, 256x256 tile, the N = 2m columns are gate | up of a SwiGLU MLP: an output tile takes 128 gate columns and the 128
  // up columns that belong to them (B rows t*128.. and m + t*128..), C [M, 2m] bf16 is written as by EPI_BF16 (no
  // residual) and C2 [M, m] bf16 = silu(gate) * up from the rounded values, as the separate SwiGLU kernel would compute
  // it from C.  m must be a multiple of 128.
  EPI_SWIGLU_FWD = 8
};
// exp argument beyond which EPI_CE_P saturates; a chunk whose maximum exceeds ref + CE_P_LIMIT is redone the slow way
#define RP_CE_P_CLAMP 64.0f
#define RP_CE_P_LIMIT 60.0f

struct GemmArgs {
  const void* A; const void* B;
  long lda, ldb;
  int M, N, K;
  // optional second operand pair appended to the reduction (LoRA up-projection fused into the base GEMM)
  const void* A2; const void* B2;
  long lda2, ldb2;
  int K2;
  void* C; long ldc;
  const void* R; long ldr;     // optional bf16 residual added in the epilogue (EPI_BF16)
  float alpha; int beta;
  int epi;
  // cross-entropy epilogues
  const int* labels; float* zlab; float2* part; long part_ld; const float* lse; const float* coef;
  int row_offset;              // global vocab index of row 0 of A
  // byte extents of the four operands (filled in by gemm_launch; rows beyond them read as zero)
  unsigned bytesA, bytesB, bytesA2, bytesB2;
  // Grouped mode (mixture of experts): the rows of A and C are sorted by group, every group multiplies with its own B.
  // grp_tab[i] = {group, first row, rows (<= 256), 0} for the i-th 256-row tile, *grp_ntiles of them (device memory:
  // the grid is sized for grp_max_tiles and surplus workgroups exit); B of group g starts grp_strideB elements after
  // B.  row_map (optional): row r of A is read from row row_map[r] of the A buffer (gather fused into the loads).
  // 256x256 tiles, NT or NN, no second operand pair.
  const int4* grp_tab; const int* grp_ntiles; int grp_max_tiles; long grp_strideB; const int* row_map;
  int row_map_rows;            // rows of the A buffer that row_map indexes
  void* C2; long ldc2;         // EPI_SWIGLU_FWD: the activation output
  const int* run_flag;         // optional [dev]: the kernel returns at once when *run_flag == 0 (conditional slow paths)
  // B (and B2) are copies in MFMA fragment order made by gemm_arrange (ldb, ldb2 unused): the kernel streams them into
  // registers without passing through LDS.  256x256 tile, NT or NN (the arrangement absorbs the difference), not grouped.
  int b_direct;
  int splits;                  // reduction slices (grid.y), chosen by gemm_launch
  int part_row0;               // first partial row this launch writes (2 per M tile)
  // Reduction split (EPI_F32 with beta): with a scratch buffer of at least splits * M * N floats the slices write
  // their partial products there ([slice][M][N]) and a second kernel adds them to C in slice order, so the result does
  // not depend on scheduling.  Without the buffer the GEMM is not split.  out_bf16: the merged sum is written to C
  // as bf16 (overwritten, not accumulated) -- the skinny LoRA projections.
  float* split_ws; size_t split_ws_bytes; int split_out_bf16;
  long c_slice_stride;         // set by gemm_launch: elements between the partial outputs of consecutive slices
};

// Scratch that lets every reduction split gemm_launch would choose go ahead: splits * tiles <= 256 tiles of 256 x 256.
#define RP_SPLITK_WS_BYTES ((size_t)64 << 20)

// Enqueues one GEMM.  Returns hipSuccess or the launch error.  tile_hint: 0 = choose automatically.
hipError_t gemm_launch(hipStream_t st, int layout, const GemmArgs& a, int tile_hint = 0);
// Number of partial rows an EPI_CE_STATS launch with M vocab rows writes for tile choice made by gemm_launch.
int gemm_ce_stats_partials(int M);
void gemm_zero_args(GemmArgs& a);
// The 256x256 product (layout GEMM_NT, GEMM_NN or GEMM_TN) with operands loaded straight into LDS and four waves of
// 128x128 (gemm_dtl.hip); arguments as prepared by gemm_launch (extents, slices).
hipError_t gemm_dtl_launch(hipStream_t st, const GemmArgs& a, int layout);
// Tile gemm_launch picks for these arguments: 1..4 = 256x256, 256x128, 128x128, 128x64 (8, 4, 2, 1 waves),
// 5 = 256x128 with eight waves in two groups that split every K tile.  (A product on tile 1 with a long enough
// reduction and an output that is not skinny runs gemm_dtl_launch unless tile_hint is 1; hint 7 asks for it by name.)
int gemm_pick_tile(const GemmArgs& a, int tile_hint = 0);

// Fragment order of a B operand for b_direct: blocks of 64 output columns x K tiles of 64, each 8 KB = 4 steps x 2
// column halves x 64 lanes x 8 consecutive reduction indices; columns and reduction indices past the end are zero.
// B is [N, K] row-major (transposed = 0: the NT operand) or [K, N] row-major (transposed = 1: the NN operand).
size_t gemm_arranged_bytes(int N, int K);
hipError_t gemm_arrange(hipStream_t st, const void* B, long ldb, int N, int K, int transposed, void* out);
