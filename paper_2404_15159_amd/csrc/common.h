// Internal declarations shared by the HIP translation units of libmixlora (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/mixlora.h"

namespace mixlora {

typedef __bf16 bf16_t;
typedef bf16_t bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// ---- element access in the storage dtype, arithmetic always in fp32 -------------------
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }
template <typename E> __device__ __forceinline__ E from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }

template <typename E> struct Vec8;  // 8 consecutive elements
template <> struct Vec8<bf16_t> {
  bf16x8_t v;
  __device__ __forceinline__ void load(const bf16_t *p) { v = *reinterpret_cast<const bf16x8_t *>(p); }
  __device__ __forceinline__ void store(bf16_t *p) const { *reinterpret_cast<bf16x8_t *>(p) = v; }
  __device__ __forceinline__ float get(int i) const { return (float)v[i]; }
  __device__ __forceinline__ void set(int i, float f) { v[i] = (bf16_t)f; }
};
template <> struct Vec8<float> {
  float4 a, b;
  __device__ __forceinline__ void load(const float *p) {
    a = *reinterpret_cast<const float4 *>(p);
    b = *reinterpret_cast<const float4 *>(p + 4);
  }
  __device__ __forceinline__ void store(float *p) const {
    *reinterpret_cast<float4 *>(p) = a;
    *reinterpret_cast<float4 *>(p + 4) = b;
  }
  __device__ __forceinline__ float get(int i) const {
    const float *q = i < 4 ? &a.x : &b.x;
    return q[i & 3];
  }
  __device__ __forceinline__ void set(int i, float f) {
    float *q = i < 4 ? &a.x : &b.x;
    q[i & 3] = f;
  }
};

// ---- GEMM engine:  C[M,N] = sum over segments  A_s[M,K_s] * B_s[N,K_s]^T -----------------
// Both operands are K-contiguous ("NT").  K_s % 8 == 0, lda/ldb % 8 == 0, 16-byte aligned
// bases.  C is written in the storage dtype or as float32.
struct GemmSeg {
  const void *A;
  const void *B;
  int64_t lda, ldb;
  int K;
};
struct GemmProblem {
  GemmSeg seg[3];
  int nseg;
  int M, N;
  void *C;
  int64_t ldc;
  int c_f32;  // 1: C is float32 regardless of the storage dtype
};
// Enqueue up to GEMM_MAX_PROBLEMS independent problems in one launch (N and the output type may
// differ per problem; M too when the launch qualifies for the large-tile bf16 kernel, i.e. every
// M > 128, some N > 128 and every K a multiple of 64 - otherwise differing M is an error).
constexpr int GEMM_MAX_PROBLEMS = 8;
hipError_t launch_gemm(int dtype, const GemmProblem *probs, int nprob, hipStream_t st);
// whether problems of different M may share one launch_gemm call
bool gemm_mixed_rows_ok(int dtype, const GemmProblem *probs, int nprob);

// Measurement hook (csrc/prof.hip): HIP-event timing of launches by kind between prof_begin and
// prof_end (events are recorded on the launch stream).  Not thread-safe; off by default.
// Work is floating-point operations for PROF_GEMM (the DMA-ring bf16 MFMA kernels that carry the
// frozen projections) and algorithmic bytes for the bandwidth-bound kinds.
enum ProfKind {
  PROF_GEMM = 0,      // frozen-projection GEMM launches
  PROF_FUSED_FWD,     // per-pair SwiGLU stage, forward
  PROF_FUSED_BWD,     // per-pair SwiGLU stage, backward
  PROF_COMBINE,       // weighted / unweighted sums of a token's pair rows
  PROF_GRAD_SUMS,     // grouped outer-product sums (LoRA and router gradients)
  PROF_ROUTING,       // softmax / top-k, grouping, auxiliary loss, router backward
  PROF_OTHER,         // re-layouts, gathers, small reductions
  PROF_KINDS
};
bool prof_on();
int prof_begin(int max_launches);
int prof_mark_begin(int kind, hipStream_t st);            // returns a slot (or -1 when off / full)
void prof_mark_end(int slot, hipStream_t st, double work);
int prof_end();
int prof_kind(int kind, double *ms_total, int *launches, double *work_total);

// ---- routing -----------------------------------------------------------------------------
// N experts in all; with several adapters (token_model != NULL) token t is routed among the Nl
// experts [token_model[t] * Nl, ... + Nl) of its adapter: probs is 0 elsewhere, idx_out is the
// index inside the adapter, idx_ws the index among all N.
hipError_t launch_router(int dtype, const void *x, const void *W_router, int T, int d, int N,
                         int k, float *probs, int32_t *idx_out, float *w_out, int32_t *idx_ws,
                         float *w_ws, int Nl, const int32_t *token_model, hipStream_t st);
// Same routing from logits Z[t, n] (row pitch ldz) that a GEMM launch produced.
struct RelayoutJob;
// routing from logits plus weight re-layout jobs (bf16 storage) in one launch
hipError_t launch_route_logits_relayout(const float *Z, int ldz, int T, int N, int k, float *probs,
                                        int32_t *idx_out, float *w_out, int32_t *idx_ws,
                                        float *w_ws, int Nl, const int32_t *token_model,
                                        const RelayoutJob *jobs, int njobs, hipStream_t st);
hipError_t launch_route_logits(const float *Z, int ldz, int T, int N, int k, float *probs,
                               int32_t *idx_out, float *w_out, int32_t *idx_ws, float *w_ws,
                               int Nl, const int32_t *token_model, hipStream_t st);
// Stable grouping of the k*T pairs by expert: counts[N], first_counts[N] (slot-0 histogram),
// offs[N+1], row_of_pair[kT], pair_of_row[kT].  counts_out may be NULL.
hipError_t launch_group_pairs(const int32_t *idx, int T, int N, int k, int32_t *counts,
                              int32_t *counts_out, int32_t *first_counts, int32_t *offs,
                              int32_t *row_of_pair, int32_t *pair_of_row, hipStream_t st);
// launch_group_pairs and launch_aux_loss (without dprobs) in one launch; tok_offs gets {0, T}
hipError_t launch_group_pairs_aux(const int32_t *idx, int T, int N, int k, int32_t *counts,
                                  int32_t *counts_out, int32_t *first_counts, int32_t *offs,
                                  int32_t *row_of_pair, int32_t *pair_of_row, int32_t *tok_offs,
                                  const float *probs, float coeff, int mode, float *loss, float *F,
                                  float *P, int Nl, const int32_t *token_model,
                                  int32_t *model_tokens, int32_t *pg_tok, int32_t *pg_tiles,
                                  int32_t *pg_ntiles, hipStream_t st);
// The same over many workgroups, for long token batches (identical row maps; the probability
// sums of Eq. 9 are added in a different, equally fixed order).  scratch:
// group_pairs_scratch_bytes(T, k) bytes.
size_t group_pairs_scratch_bytes(int T, int k);
hipError_t launch_group_pairs_aux_multi(const int32_t *idx, int T, int N, int k, int32_t *counts,
                                        int32_t *counts_out, int32_t *first_counts, int32_t *offs,
                                        int32_t *row_of_pair, int32_t *pair_of_row,
                                        int32_t *tok_offs, const float *probs, float coeff, int mode,
                                        float *loss, float *F, float *P, int Nl,
                                        const int32_t *token_model, int32_t *model_tokens,
                                        void *scratch, hipStream_t st);
// loss[N / Nl], one per adapter (statistics over the adapter's own tokens); model_tokens (may be
// NULL) receives the token count of every adapter.
hipError_t launch_aux_loss(const float *probs, const int32_t *idx, int T, int N, int k,
                           float coeff, int mode, float *loss, float *F, float *P,
                           float *dprobs, int Nl, const int32_t *token_model,
                           int32_t *model_tokens, hipStream_t st);

// ---- element-wise / rank-r pieces -------------------------------------------------------
struct PairCtx {  // device pointers describing the grouped pairs
  const int32_t *offs;         // [N+1]
  const int32_t *pair_of_row;  // [kT]
  const int32_t *row_of_pair;  // [kT]
  const float *w;              // [T,k] routing weights
  const int32_t *idx;          // [T,k]
  int T, N, k, r;
};

// a_grp[row,:] = SiLU(G[t] + s B_gate[e] Pg[t,e]) * (U[t] + s B_up[e] Pu[t,e]),  rows grouped
hipError_t launch_swiglu_fwd(int dtype, const PairCtx &pc, int f, float s, const void *G,
                             const void *U, const float *Pg_all, const float *Pu_all,
                             const void *B_gate, const void *B_up, void *a_grp,
                             hipStream_t st);
// backward of the above; also the per-(row, column tile) partial sums of <H[t], a_row>
hipError_t launch_swiglu_bwd(int dtype, const PairCtx &pc, int f, float s, const void *G,
                             const void *U, const float *Pg_all, const float *Pu_all,
                             const void *B_gate, const void *B_up, const void *H,
                             const float *VB_all, const void *A_down, void *dg_grp,
                             void *du_grp, float *dw_part, int n_col_tiles, hipStream_t st);
int swiglu_col_tiles(int f);

// Per-expert column factors of the weight-decomposed variant (magnitude / row norm), float32
// [N, f] each, and (backward only) per-tile partial sums for the magnitude gradients,
// [row tiles][f] each with row tiles = kT / 32 + N.
struct DoraArgs {
  const float *cg, *cu;
  float *dm_part_g, *dm_part_u;
};
// bf16 MFMA fusion of the above with the A_down projection of the row's expert: writes a_grp,
// Q_all[row, e(row)*r + q] and the non-zero blocks of Qw[t, e*r + q] = w * Q (bf16, pitch ldqw;
// the caller zero-fills Qw first).  Q_part is scratch of fused_splits(f, kT) * kT * r floats.
hipError_t launch_swiglu_fwd_mfma(const PairCtx &pc, int f, float s, const void *G, const void *U,
                                  const float *Pg_all, const float *Pu_all, const void *B_gate,
                                  const void *B_up, const void *A_down, void *a_grp,
                                  float *Q_part, float *Q_all, void *Qw, int ldqw,
                                  hipStream_t st, int rows_mode = 0, const DoraArgs *dora = nullptr,
                                  bool reduce_parts = true);   // false: the caller sums Q_part itself
// rows_mode of the fused stages (for the paper's own schedules, Figure 3): bit 0 = G and U hold
// one row per grouped pair row instead of one per token; bit 1 = H likewise; bit 2 = the
// block-sparse operand has one row per grouped pair row (unweighted) instead of one per token.
constexpr int ROWS_GU = 1, ROWS_H = 2, ROWS_SPARSE = 4;

// bf16 MFMA backward of the same stage: dg_grp, du_grp, dw_part[row][split]
// (split count = fused_splits(f, kT)), TG_all / TU_all at [row, e(row)*r + q].  AdT = A_down re-laid
// [N, f, r]; BgT / BuT = B banks re-laid [N, r, f]; rank_part is scratch of 2 * fused_splits(f, kT) * kT * r floats.
hipError_t launch_swiglu_bwd_mfma(const PairCtx &pc, int f, float s, const void *G, const void *U,
                                  const void *H, const float *Pg_all, const float *Pu_all,
                                  const float *VB_all, const void *B_gate, const void *B_up,
                                  const void *AdT, const void *BgT, const void *BuT, void *dg_grp,
                                  void *du_grp, float *dw_part, float *rank_part, float *TG_all,
                                  float *TU_all, void *S, int lds_, hipStream_t st,
                                  int rows_mode = 0, const DoraArgs *dora = nullptr);
// Pair-grouped token tiles (csrc/fused_pg.hip) for top-2 routing, N <= PG_MAX_EXPERTS, 128 < T <=
// PG_MAX_TOKENS, r <= 16: tokens are grouped by their unordered expert pair, a workgroup handles
// 32 tokens of one pair (forward: one wavefront computes both experts of its columns; backward: one
// set of wavefronts per expert), G / U (/ H) are fetched from HBM once per token and the sums over
// a token's two pairs are written per token (no combine pass).
// Tables: tok_of_pos [T], tile_info [fused_pg_max_tiles(T, N)][4], ntiles [1] (device int32).
// Forward: a_comb[t] = w_t0 a_t0 + w_t1 a_t1, a_grp only when write_a, Q_all / Qw as above;
// Q_part: fused_pg_splits(f, T, N) * kT * r floats.
constexpr int PG_MAX_EXPERTS = 16;
constexpr int PG_TILE_ROWS = 32;
constexpr int PG_MAX_TOKENS = 1 << 16;
bool fused_pg_ok(const PairCtx &pc, int f);
int fused_pg_max_tiles(int T, int N);
int fused_pg_splits(int f, int T, int N);
hipError_t launch_group_token_pairs(const PairCtx &pc, int32_t *tok_of_pos, int32_t *tile_info,
                                    int32_t *ntiles, hipStream_t st);
hipError_t launch_swiglu_fwd_pg(const PairCtx &pc, int f, float s, const int32_t *tok_of_pos,
                                const int32_t *tile_info, const int32_t *ntiles, const void *G,
                                const void *U, const float *Pg_all, const float *Pu_all,
                                const void *B_gate, const void *B_up, const void *A_down,
                                void *a_grp, void *a_comb, float *Q_part, float *Q_all, void *Qw,
                                int ldqw, int write_a, hipStream_t st);
// backward on the same tiles: per-pair dg_grp, du_grp, dw_part [pair row][fused_pg_splits], TG / TU
// (reduced into TG_all, TU_all and the block-sparse operand S) and the per-token sums dgsum, dusum
hipError_t launch_swiglu_bwd_pg(const PairCtx &pc, int f, float s, const int32_t *tok_of_pos,
                                const int32_t *tile_info, const int32_t *ntiles, const void *G,
                                const void *U, const void *H, const float *Pg_all,
                                const float *Pu_all, const float *VB_all, const void *B_gate,
                                const void *B_up, const void *AdT, const void *BgT, const void *BuT,
                                void *dg_grp, void *du_grp, void *dgsum, void *dusum, float *dw_part,
                                float *rank_part, float *TG_all, float *TU_all, void *S, int ld_s,
                                hipStream_t st);
// dense[row, e(row)*r + q] = sum over splits of part[split][row][q] (fixed order) for one bank
// (dense1 == NULL) or two banks bank_stride floats apart; the value (times the routing weight if
// weighted) also goes as bf16 into the block-sparse operand sparse[t(row) or row, bank*N*r + e*r + q]
hipError_t launch_reduce_rank_parts(const PairCtx &pc, const float *part0, int64_t bank_stride,
                                    int nsplit, float *dense0, float *dense1, void *sparse,
                                    int ld_sparse, int weighted, int by_row, hipStream_t st);
int fused_row_tiles(int kT, int N);   // grid.x of the fused stages
int fused_splits(int f, int kT);   // at most FUSED_MAX_SPLITS
constexpr int FUSED_MAX_SPLITS = 32;

// out[t,:] = sum_j (weighted ? w[t,j] : 1) * in_grp[row_of_pair[t,j], :]
// launch_pair_combine (bf16, weighted) and the one-bank weighted per-token launch_reduce_rank_parts
// as one launch (few tokens; k * r <= 256)
hipError_t launch_pair_combine_reduce(const PairCtx &pc, int width, const void *in_grp, void *out,
                                      const float *part, int nsplit, float *dense, void *sparse,
                                      int ld_sparse, hipStream_t st);
hipError_t launch_pair_combine(int dtype, const PairCtx &pc, int width, const void *in_grp,
                               void *out, int weighted, hipStream_t st);
// two combines of the same shape in one launch (in_grp1 == NULL: only the first)
hipError_t launch_pair_combine2(int dtype, const PairCtx &pc, int width, const void *in_grp0,
                                void *out0, const void *in_grp1, void *out1, int weighted,
                                hipStream_t st);
// dst[row, :] = src[token of grouped row, :]   (width a multiple of 8)
hipError_t launch_gather_rows(int dtype, const PairCtx &pc, int width, const void *src, void *dst,
                              hipStream_t st);
// dst[t, col0 + e_j*r + q] = scale_j * src[row_j, (src_dense ? e_j*r : 0) + q] for the kept
// experts, 0 elsewhere; dst is in the storage dtype with leading dimension ldd.  nsrc sources
// (src + b*src_stride, b < nsrc) fill consecutive N*r-column blocks in one launch.
hipError_t launch_scatter_blocks(int dtype, const PairCtx &pc, const float *src, int64_t src_stride,
                                 int nsrc, int lds_, int src_dense, int weighted, void *dst,
                                 int ldd, int col0, hipStream_t st);
// small_grp[row, q] = scale * src[(by_token ? t(row) : row), e(row)*r + q]   (float32)
hipError_t launch_gather_small(const PairCtx &pc, const float *src, int by_token, int weighted,
                               float *small_grp, hipStream_t st);

// io[t, c] += s * sum_q P[t, q] * Wt[c, q]   (io [T,C] storage dtype, P [T,r] f32, Wt [C,r])
hipError_t launch_lowrank_add(int dtype, void *io, const float *P, const void *Wt, int T, int C,
                              int r, float s, hipStream_t st);

// out[i] = sum_{s<S} part[s][i], i < n, fixed order (closing step of a split-K GEMM)
hipError_t launch_splitk_reduce(int dtype, const float *part, int S, int64_t n, void *out,
                                hipStream_t st);

// Weight re-layouts (tiny index permutations), batched into one launch:
//   dst[dst0 + i0*d0 + i1*d1 + i2*d2] = scale * src[i0*s0 + i1*s1 + i2*s2]   (0 where i2 >= valid2)
// or, with batched_transpose set,  dst[dst0 + b*d0 + q*d1 + p] = scale * src[b*s0 + p*n2 + q]  for
// b < n0, p < n1, q < n2 (0 where p >= valid2), tiled through LDS.
struct RelayoutJob {
  const void *src;
  void *dst;
  int64_t s0, s1, s2, dst0, d0, d1, d2;
  int n0, n1, n2, valid2;
  float scale;
  int batched_transpose;
  size_t zero_bytes;   // non-zero: the job is a plain zero fill of that many bytes at dst
};
constexpr int RELAYOUT_MAX_JOBS = 8;
hipError_t launch_relayout(int dtype, const RelayoutJob *jobs, int njobs, hipStream_t st);
// bytes (rounded up to a multiple of 16) of zeros at dst
RelayoutJob job_zero_fill(void *dst, size_t bytes);
// bank [N, rows, r] -> out[i, col0 + e*r + q] = scale * bank[e, i, q]   (out pitch ldo)
RelayoutJob job_bank_cat(const void *bank, int N, int rows, int r, float scale, void *out,
                         int ldo, int col0);
// bank [N, rows, r] -> out[e*r + q, i]                                   (out is [N*r, rows])
RelayoutJob job_bank_T(const void *bank, int N, int rows, int r, void *out);
// A bank with another number of rank entries: [N, r_src, width] -> [N, r_dst, width] when
// rank_major, else [N, width, r_src] -> [N, width, r_dst]; the first min(r_src, r_dst) entries are
// copied, the rest (if any) are zeros.  Pads a bank to a whole multiple of 8 rank entries, or cuts
// a padded gradient back.
RelayoutJob job_rank_resize(const void *src, void *dst, int N, int r_src, int r_dst, int width,
                            bool rank_major);
// A [N, r, cols] -> out[c, col0 + e*r + q] = scale * A[e, q, c]
RelayoutJob job_A_cat(const void *A, int N, int r, int cols, float scale, void *out, int ldo,
                      int col0);
// W_router [N, d] -> out[c, col0 + n] = W_router[n, c] for n < N, 0 for N <= n < ncols
RelayoutJob job_router_T(const void *W_router, int N, int d, void *out, int ldo, int col0,
                         int ncols);
hipError_t launch_transpose(int dtype, const void *in, void *out, int rows, int cols,
                            hipStream_t st);

// ---- gradients --------------------------------------------------------------------------
// out[g][q][c] (layout_qc = 1) or out[g][c][q] (0) = scale * sum over rows of group g of
//   small[row, q] * wide[(tok_of_row ? tok(row) : row), c];   groups from offs[0..G].
hipError_t launch_group_outer(int dtype, const int32_t *offs, int G, int max_rows,
                              const int32_t *pair_of_row, int k, const float *small, int r,
                              const void *wide, int C, float scale, int layout_qc, float *out,
                              float *partials, size_t partial_floats, hipStream_t st);
size_t group_outer_partial_floats(int G, int r, int C);

// bf16 MFMA version: smallT is the transposed bf16 factor [r][ldT] (ldT % 8 == 0, readable up to
// the next multiple of 16 rows past the last group), wide is bf16 with C % 8 == 0.  Up to
// GOM_MAX_JOBS sums of the same shape (groups, C, gather mode, scale) go into one launch and
// one reduction launch; partials must hold njobs * group_outer_mfma_partial_floats(G, r, C).
struct GomJob {
  const void *smallT;
  const void *wide;
  float *out;
  int layout_qc;
};
constexpr int GOM_MAX_JOBS = 3;
hipError_t launch_group_outer_mfma(const int32_t *offs, int G, int nrows,
                                   const int32_t *pair_of_row, int k, const GomJob *jobs, int njobs,
                                   int ldT, int r, int C, float scale, float *partials,
                                   size_t partial_floats, hipStream_t st);
size_t group_outer_mfma_partial_floats(int G, int r, int C);
// outT[q, row] = (w_row or 1) * src[(by_token ? t(row) : row), e(row)*r + q] as bf16, pitch ldT;
// up to GATHER_MAX_JOBS factors in one launch
struct GatherJob {
  const float *src;
  void *outT;
  int by_token, weighted;
};
constexpr int GATHER_MAX_JOBS = 6;
hipError_t launch_gather_small_T(const PairCtx &pc, const GatherJob *jobs, int njobs, int ldT,
                                 hipStream_t st);
hipError_t launch_f32_to_bf16T(const float *src, int rows, int r, void *outT, int ldT,
                               hipStream_t st);

struct AuxUpstream {   // upstream gradient of every adapter's auxiliary loss
  float v[64];
};
hipError_t launch_router_bwd(int dtype, const PairCtx &pc, const float *probs, const float *dw_part,
                             int n_col_tiles, const float *VB_all, const float *Q_all,
                             const float *F, float s, const AuxUpstream &d_aux, float aux_coeff,
                             float *dw_ws, float *dz, void *S, int lds_, int col0, int ncols,
                             int Nl, const int32_t *token_model, const int32_t *model_tokens,
                             void *dzT, int ldTz, hipStream_t st,    // dzT: bf16 [N][ldTz] copy or NULL
                             int s_by_first_pair = 0);   // S has one row per grouped pair row

// ---- weight-decomposed experts (csrc/dora.hip); bf16 storage only --------------------------------
hipError_t launch_row_sqnorm(const void *W, int rows, int cols, float *out, hipStream_t st);
size_t gram_part_floats(int N, int r);   // floats of one bank's Gram slice sums
hipError_t launch_gram(const void *A_bank, int N, int r, int in, float *part, hipStream_t st);
// c = m / n, ninv = 1 / n with n the row norms of W + s B_e A_e (from w2, WA = W A_cat^T, AA)
hipError_t launch_dora_scale(const void *B_bank, const float *WA, const float *AA, const float *w2,
                             const float *m, int shared, int N, int out, int r, float s, float *c,
                             float *ninv, hipStream_t st);
hipError_t launch_scale_bank(void *bank, const float *c, int N, int r, int d, hipStream_t st);
hipError_t launch_gather_rows_scaled(const PairCtx &pc, int width, const void *src, const float *c,
                                     void *dst, hipStream_t st);
hipError_t launch_pair_combine_scaled(const PairCtx &pc, int width, const void *in_grp,
                                      const float *c, void *out, hipStream_t st);
size_t dm_down_part_floats(int N, int d);
hipError_t launch_dm_down(const PairCtx &pc, int d, const void *dy, const void *v, const float *ninv,
                          float *part, float *dm, int shared, hipStream_t st);
hipError_t launch_dm_tiles_reduce(const int32_t *offs, int N, int f, const float *part_g,
                                  const float *part_u, const float *ninv_g, const float *ninv_u,
                                  float *dm_g, float *dm_u, int shared, hipStream_t st);

}  // namespace mixlora
