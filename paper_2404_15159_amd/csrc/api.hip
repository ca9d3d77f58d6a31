// C ABI of libmixlora: argument validation (host only, before any HIP call), workspace
// carving and the stream-ordered kernel sequences of the forward and backward passes.
//
// Schedule (Section 3.3 "Reducing the Computational Complexity (I)", Algorithm 1): the frozen
// gate/up projections run once over all T tokens and are shared by the experts; LoRA deltas,
// SiLU * up and everything per (token, expert) pair run on expert-grouped rows.  Because the
// frozen down projection is linear and shared, it is applied once per token to the
// routing-weighted sum of the pair activations, with the per-expert low-rank part entering as a
// K-extension of the same GEMM; its transpose is used the same way in the backward.
#include "common.h"

#include <mutex>

using namespace mixlora;

namespace {

constexpr size_t ALIGN = 256;
constexpr size_t SPLITK_MAX_ROWS = 128;   // at most this many tokens: the down GEMM is split along K
inline size_t up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }
inline int up64(int v) { return (v + 63) / 64 * 64; }

// Up to this many (token, expert) pairs the grouping runs in one workgroup (bound by its own
// latency); longer batches use the multi-workgroup passes.
constexpr size_t GROUP_SINGLE_WG_PAIRS = 8192;

struct Layout {
  // saved by forward
  size_t probs, Z, idx, w, counts, first_counts, offs, row_of_pair, pair_of_row, F, P, tok_offs,
      model_tokens;
  size_t pg_tok, pg_tiles, pg_ntiles;   // tokens grouped by expert pair (csrc/fused_pg.hip)
  size_t G, U, Pg_all, Pu_all, a_grp, Q_all;
  // forward scratch
  size_t a_comb, Qw, Bd_cat, rank_part, splitk, gp_scratch;
  size_t fwd_end;
  // backward scratch
  size_t WdT, WgT, WuT, H, Bd_T, VB_all, dg_grp, du_grp, dgsum, dusum, dw_part, dw, Bg_T, Bu_T, AdT,
      TG_all, TU_all, small[6], S, Bx, dz, partials, dzT;
  int ldT, ldTz;
  size_t partial_floats;
  size_t bwd_end;
  int Kx, nct;
  // per-pair-row buffers of the paper's own schedules (Section 3.3, Figure 3); size 0 otherwise
  size_t Xp, Gp, Up, Qp, Op;     // forward (Gp, Up are kept for the backward pass)
  size_t dYp, Hp, Sp, dXp;       // backward scratch
  // weight-decomposed experts: W A^T products, Gram matrices, squared row norms of the frozen
  // matrices, factors c = m / n and 1 / n (kept for the backward pass); backward partial sums
  size_t WA_g, WA_u, WA_d, AA, w2, c_g, c_u, c_d, ninv_g, ninv_u, ninv_d;
  size_t dm_part_g, dm_part_u, dmd_part;
  // ranks that are not a multiple of 8 (Section 4.3's rank study goes down to r = 2): the six LoRA
  // banks zero-padded to rp = 8 * ceil(r / 8) rank entries, and their fp32 gradients in that form
  int rp;
  size_t pad_w[6], pad_g[6];
};

inline int pad_rank(int r) { return (r + 7) & ~7; }

// banks in the order A_gate, B_gate, A_up, B_up, A_down, B_down: elements of the rank-padded bank
inline size_t bank_elems(int i, size_t N, size_t rp, size_t d, size_t f) {
  const size_t width[6] = {d, f, d, f, f, d};
  return N * rp * width[i];
}

// Buffers a schedule does not use get size 0 (per-token G, U in the unshared schedule, the
// combined activations where the down projection runs per pair, ...).
Layout make_layout(const mixlora_dims &D, int schedule = MIXLORA_SCHEDULE_LINEAR_DOWN,
                   bool dora = false) {
  Layout L{};
  const bool pair_down = schedule != MIXLORA_SCHEDULE_LINEAR_DOWN;
  const bool vanilla = schedule == MIXLORA_SCHEDULE_VANILLA;
  const size_t T = D.T, d = D.d, f = D.d_ff, N = D.N, k = D.k, r = pad_rank(D.r);
  const size_t R = N * r, kT = k * T;
  const size_t E = D.dtype == MIXLORA_BF16 ? 2 : 4;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = up(o + bytes); return at; };
  L.rp = (int)r;
  for (int i = 0; i < 6; i++) L.pad_w[i] = take((int)r != D.r ? bank_elems(i, N, r, d, f) * E : 0);
  L.probs = take(T * N * 4);
  L.Z = take(T * N * 4);
  L.idx = take(kT * 4);
  L.w = take(kT * 4);
  L.counts = take(N * 4);
  L.first_counts = take(N * 4);
  L.offs = take((N + 1) * 4);
  L.row_of_pair = take(kT * 4);
  L.pair_of_row = take(kT * 4);
  L.F = take(N * 4);
  L.P = take(N * 4);
  L.tok_offs = take(2 * 4);
  L.model_tokens = take(64 * 4);
  L.pg_tok = take(T * 4);
  L.pg_tiles = take((size_t)fused_pg_max_tiles((int)T, (int)(N <= PG_MAX_EXPERTS ? N : 1)) * 16);
  L.pg_ntiles = take(4);
  L.G = take(vanilla ? 0 : T * f * E);
  L.U = take(vanilla ? 0 : T * f * E);
  L.Pg_all = take(T * R * 4);
  L.Pu_all = take(T * R * 4);
  L.a_grp = take(kT * f * E);
  L.Q_all = take(kT * R * 4);
  L.a_comb = take(pair_down ? 0 : T * f * E);
  L.Qw = take(pair_down ? 0 : T * R * E);
  L.Xp = take(vanilla ? kT * d * E : 0);
  L.Gp = take(vanilla ? kT * f * E : 0);
  L.Up = take(vanilla ? kT * f * E : 0);
  L.Qp = take(pair_down ? kT * R * E : 0);
  L.Op = take(pair_down ? kT * d * E : 0);
  L.WA_g = take(dora ? f * R * 4 : 0);
  L.WA_u = take(dora ? f * R * 4 : 0);
  L.WA_d = take(dora ? d * R * 4 : 0);
  L.AA = take(dora ? 3 * gram_part_floats((int)N, (int)r) * 4 : 0);
  L.w2 = take(dora ? (2 * f + d) * 4 : 0);
  L.c_g = take(dora ? N * f * 4 : 0);
  L.c_u = take(dora ? N * f * 4 : 0);
  L.c_d = take(dora ? N * d * 4 : 0);
  L.ninv_g = take(dora ? N * f * 4 : 0);
  L.ninv_u = take(dora ? N * f * 4 : 0);
  L.ninv_d = take(dora ? N * d * 4 : 0);
  L.Bd_cat = take(d * R * E);
  {   // per-split rank-r partial sums (two banks), for the grouped and the token-major stages
    const size_t sp_g = (size_t)fused_splits((int)f, (int)kT), sp_t = (size_t)fused_pg_splits((int)f, (int)T, (int)(N <= PG_MAX_EXPERTS ? N : 1));
    L.rank_part = take(2 * (sp_g > sp_t ? sp_g : sp_t) * kT * r * 4);
  }
  // few tokens (decode-shaped calls): partial outputs of the K-split down projection
  L.splitk = take(T <= SPLITK_MAX_ROWS ? (size_t)GEMM_MAX_PROBLEMS * T * d * 4 : 0);
  L.gp_scratch = take(kT > GROUP_SINGLE_WG_PAIRS ? group_pairs_scratch_bytes((int)T, (int)k) : 0);
  L.fwd_end = o;
  L.Kx = up64((int)(2 * R) + (int)N);   // whole K tiles of the GEMM's DMA path
  L.nct = swiglu_col_tiles((int)f);
  L.WdT = take(f * d * E);
  L.WgT = take(f * d * E);
  L.WuT = take(f * d * E);
  L.H = take(pair_down ? 0 : T * f * E);
  L.dYp = take(pair_down ? kT * d * E : 0);
  L.Hp = take(pair_down ? kT * f * E : 0);
  L.Bd_T = take(R * d * E);
  L.VB_all = take(T * R * 4);
  L.dg_grp = take(kT * f * E);
  L.du_grp = take(kT * f * E);
  L.dgsum = take(vanilla ? 0 : T * f * E);
  L.dusum = take(vanilla ? 0 : T * f * E);
  L.dw_part = take(kT * (size_t)(L.nct > FUSED_MAX_SPLITS ? L.nct : FUSED_MAX_SPLITS) * 4);
  L.dw = take(kT * 4);
  L.Bg_T = take(R * f * E);
  L.Bu_T = take(R * f * E);
  L.AdT = take(R * f * E);
  L.TG_all = take(kT * R * 4);
  L.TU_all = take(kT * R * 4);
  L.ldT = (int)((kT + 15) / 16 * 16 + 16);   // transposed bf16 factors, padded for whole MFMA steps
  L.ldTz = (int)((T + 15) / 16 * 16 + 16);
  for (int i = 0; i < 6; i++) L.small[i] = take(kT * r * 4 > (size_t)L.ldT * r * 2 ? kT * r * 4 : (size_t)L.ldT * r * 2);
  L.dzT = take((size_t)L.ldTz * N * 2);
  L.S = take(vanilla ? 0 : T * (size_t)L.Kx * E);
  L.Sp = take(vanilla ? kT * (size_t)L.Kx * E : 0);
  L.dXp = take(vanilla ? kT * d * E : 0);
  L.dm_part_g = take(dora ? (size_t)fused_row_tiles((int)kT, (int)N) * f * 4 : 0);
  L.dm_part_u = take(dora ? (size_t)fused_row_tiles((int)kT, (int)N) * f * 4 : 0);
  L.dmd_part = take(dora ? dm_down_part_floats((int)N, (int)d) * 4 : 0);
  L.Bx = take(d * (size_t)L.Kx * E);
  for (int i = 0; i < 6; i++) L.pad_g[i] = take((int)r != D.r ? bank_elems(i, N, r, d, f) * 4 : 0);
  L.dz = take(T * N * 4);
  size_t pf = group_outer_partial_floats((int)N, (int)r, (int)f);
  size_t pd = group_outer_partial_floats((int)N, (int)r, (int)d);
  size_t pr = group_outer_partial_floats(1, (int)N, (int)d);
  L.partial_floats = pf > pd ? pf : pd;
  if (pr > L.partial_floats) L.partial_floats = pr;
  for (size_t v : {GOM_MAX_JOBS * group_outer_mfma_partial_floats((int)N, (int)r, (int)f),
                   GOM_MAX_JOBS * group_outer_mfma_partial_floats((int)N, (int)r, (int)d),
                   group_outer_mfma_partial_floats(1, (int)N, (int)d)})
    if (v > L.partial_floats) L.partial_floats = v;
  L.partials = take(L.partial_floats * 4);
  L.bwd_end = o;
  return L;
}

int check_dims(const mixlora_dims *D) {
  if (!D) return MIXLORA_E_NULL;
  if (D->dtype != MIXLORA_F32 && D->dtype != MIXLORA_BF16) return MIXLORA_E_DTYPE;
  if (D->aux_mode != MIXLORA_AUX_TOP1 && D->aux_mode != MIXLORA_AUX_TOPK) return MIXLORA_E_DTYPE;
  if (D->T < 1 || D->d < 8 || D->d_ff < 8 || D->N < 1 || D->N > 64 || D->k < 1 || D->k > D->N ||
      D->r < 1)
    return MIXLORA_E_SHAPE;
  if (D->d % 8 || D->d_ff % 8 || D->r > 64) return MIXLORA_E_SHAPE;
  if ((int64_t)D->N * pad_rank(D->r) > 512) return MIXLORA_E_SHAPE;
  if ((int64_t)D->T * D->k >= (1 << 24)) return MIXLORA_E_SHAPE;
  if ((int64_t)D->T * D->k * D->d_ff >= ((int64_t)1 << 40)) return MIXLORA_E_SHAPE;
  return MIXLORA_OK;
}

inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; }

int check_weights(const mixlora_weights *w) {
  if (!w) return MIXLORA_E_NULL;
  const void *req[] = {w->W_gate, w->W_up,   w->W_down, w->A_gate, w->B_gate,
                       w->A_up,   w->B_up,   w->A_down, w->B_down, w->W_router};
  for (const void *p : req) {
    if (!p) return MIXLORA_E_NULL;
    if (misaligned(p)) return MIXLORA_E_ALIGN;
  }
  const void *opt[] = {w->W_gate_T, w->W_up_T, w->W_down_T};
  for (const void *p : opt)
    if (p && misaligned(p)) return MIXLORA_E_ALIGN;
  return MIXLORA_OK;
}

#define HIP_TRY(expr)                                   \
  do {                                                  \
    hipError_t e_ = (expr);                             \
    if (e_ != hipSuccess) return MIXLORA_E_HIP;         \
  } while (0)

// A launch bracketed for the measurement hook (no cost when the hook is off): kind and the
// algorithmic bytes the launch moves, as stated where each kernel is described.
#define HIP_TRY_AS(kind, bytes, expr)                                     \
  do {                                                                    \
    const int slot_ = prof_on() ? prof_mark_begin((kind), st) : -1;       \
    hipError_t e_ = (expr);                                               \
    if (slot_ >= 0) prof_mark_end(slot_, st, (double)(bytes));            \
    if (e_ != hipSuccess) return MIXLORA_E_HIP;                           \
  } while (0)

GemmProblem problem(int M, int N, void *C, int64_t ldc, int c_f32) {
  GemmProblem p{};
  p.M = M;
  p.N = N;
  p.C = C;
  p.ldc = ldc;
  p.c_f32 = c_f32;
  p.nseg = 0;
  return p;
}
void add_seg(GemmProblem &p, const void *A, int64_t lda, const void *B, int64_t ldb, int K) {
  GemmSeg &s = p.seg[p.nseg++];
  s.A = A;
  s.lda = lda;
  s.B = B;
  s.ldb = ldb;
  s.K = K;
}

}  // namespace

extern "C" {

int mixlora_version(void) { return 100; }

size_t mixlora_workspace_bytes(const mixlora_dims *dims, int for_backward) {
  if (check_dims(dims) != MIXLORA_OK) return 0;
  const Layout L = make_layout(*dims);
  return for_backward ? L.bwd_end : L.fwd_end;
}

// Forward pass on D.N experts in all, of which every adapter owns Nl consecutive ones
// (token_model == NULL: one adapter).  Arguments are already validated.
// Rank padding: bank i of the user's weights ([N, r, width] for the A banks, [N, width, r] for
// the B banks) -> the same bank with rp rank entries, zeros in the added ones.  Zero rank entries
// contribute nothing to any product of the pass, and their gradients come out zero.
static RelayoutJob job_pad_bank(int i, const void *src, void *dst, int N, int r_src, int r_dst, int d, int f) {
  const int width[6] = {d, f, d, f, f, d};
  return job_rank_resize(src, dst, N, r_src, r_dst, width[i], /*rank_major=*/i == 0 || i == 2 || i == 4);
}
static hipError_t pad_weights(const Layout &L, char *ws, const mixlora_dims &Du, const mixlora_weights *w,
                              mixlora_weights *wp, hipStream_t st) {
  *wp = *w;
  const void *src[6] = {w->A_gate, w->B_gate, w->A_up, w->B_up, w->A_down, w->B_down};
  const void **dstp[6] = {&wp->A_gate, &wp->B_gate, &wp->A_up, &wp->B_up, &wp->A_down, &wp->B_down};
  RelayoutJob jobs[6];
  for (int i = 0; i < 6; i++) {
    jobs[i] = job_pad_bank(i, src[i], ws + L.pad_w[i], Du.N, Du.r, L.rp, Du.d, Du.d_ff);
    *dstp[i] = ws + L.pad_w[i];
  }
  return launch_relayout(Du.dtype, jobs, 6, st);
}

// Every re-layout of the LoRA banks and the router that the backward pass needs (eight jobs, the
// last two for bf16 storage only).
static void bwd_relayout_jobs(const Layout &L, char *ws, const mixlora_weights *w, int N, int d,
                              int f, int r, int kT, int T, float s, bool vanilla,
                              RelayoutJob jobs[8]) {
  const int R = N * r, Kx = L.Kx;
  jobs[0] = job_bank_T(w->B_down, N, d, r, ws + L.Bd_T);
  jobs[1] = job_bank_T(w->B_gate, N, f, r, ws + L.Bg_T);
  jobs[2] = job_bank_T(w->B_up, N, f, r, ws + L.Bu_T);
  jobs[3] = job_A_cat(w->A_gate, N, r, d, s, ws + L.Bx, Kx, 0);
  jobs[4] = job_A_cat(w->A_up, N, r, d, s, ws + L.Bx, Kx, R);
  jobs[5] = job_router_T(w->W_router, N, d, ws + L.Bx, Kx, 2 * R, Kx - 2 * R);
  jobs[6] = job_bank_T(w->A_down, N, r, f, ws + L.AdT);   // [N,r,f] -> [N,f,r], bf16 path only
  // bf16 path only: zeros for the block-sparse operand S, filled in by the fused stage
  jobs[7] = vanilla ? job_zero_fill(ws + L.Sp, (size_t)kT * Kx * 2)
                    : job_zero_fill(ws + L.S, (size_t)T * Kx * 2);
}

static int forward_impl(const mixlora_dims &Du, int Nl, const int32_t *token_model,
                        const mixlora_weights *w, const void *x, void *y, int32_t *topk_idx,
                        float *topk_w, int32_t *expert_counts, float *aux_loss, void *workspace,
                        size_t workspace_bytes, void *stream,
                        int schedule = MIXLORA_SCHEDULE_LINEAR_DOWN,
                        const mixlora_dora *dora = nullptr) {
  const Layout L = make_layout(Du, schedule, dora != nullptr);
  const bool pair_down = schedule != MIXLORA_SCHEDULE_LINEAR_DOWN;   // down projection per pair
  const bool vanilla = schedule == MIXLORA_SCHEDULE_VANILLA;         // gate/up per pair as well
  if (workspace_bytes < L.fwd_end) return MIXLORA_E_WORKSPACE;

  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  char *ws = reinterpret_cast<char *>(workspace);
  mixlora_dims D = Du;   // the pass runs on the rank-padded banks
  D.r = L.rp;
  mixlora_weights wpad;
  if (L.rp != Du.r) {
    if (pad_weights(L, ws, Du, w, &wpad, st) != hipSuccess) return MIXLORA_E_HIP;
    w = &wpad;
  }
  const int T = D.T, d = D.d, f = D.d_ff, N = D.N, k = D.k, r = D.r, R = N * r, kT = k * T;
  const int dt = D.dtype;
  const double Eb = dt == MIXLORA_BF16 ? 2.0 : 4.0;   // bytes per stored element (measurement hook)
  float *probs = (float *)(ws + L.probs);
  int32_t *idx = (int32_t *)(ws + L.idx);
  float *wts = (float *)(ws + L.w);
  int32_t *offs = (int32_t *)(ws + L.offs);
  int32_t *row_of_pair = (int32_t *)(ws + L.row_of_pair);
  int32_t *pair_of_row = (int32_t *)(ws + L.pair_of_row);

  // Shared frozen projections, once for all tokens (Algorithm 1 lines 7-8), and in the same
  // launch the LoRA A projections of every expert (rank-r, N*r output columns per bank).  None
  // of them depends on the routing; in bf16 the router logits (Eq. 7) ride along as a fifth,
  // N-column problem, so x is not read a second time.
  {
    GemmProblem p[8] = {problem(T, f, ws + L.G, f, 0), problem(T, f, ws + L.U, f, 0),
                        problem(T, R, ws + L.Pg_all, R, 1), problem(T, R, ws + L.Pu_all, R, 1),
                        problem(T, N, ws + L.Z, N, 1),
                        // weight-decomposed experts only: W A_cat^T for the row norms
                        problem(f, R, ws + L.WA_g, R, 1), problem(f, R, ws + L.WA_u, R, 1),
                        problem(d, R, ws + L.WA_d, R, 1)};
    add_seg(p[0], x, d, w->W_gate, d, d);
    add_seg(p[1], x, d, w->W_up, d, d);
    add_seg(p[2], x, d, w->A_gate, d, d);
    add_seg(p[3], x, d, w->A_up, d, d);
    add_seg(p[4], x, d, w->W_router, d, d);
    add_seg(p[5], w->W_gate, d, w->A_gate, d, d);
    add_seg(p[6], w->W_up, d, w->A_up, d, d);
    add_seg(p[7], w->W_down, f, w->A_down, f, f);
    if (vanilla) {   // unshared schedule: the frozen gate/up products follow the routing, per pair;
      HIP_TRY(launch_gemm(dt, p + 4, 1, st));   // only the router logits are needed up front
    } else if (dora) {
      // the W_down product has the longest K range: its tiles go first so that they do not
      // trail the launch
      const GemmProblem q[8] = {p[7], p[0], p[1], p[2], p[3], p[4], p[5], p[6]};
      if (gemm_mixed_rows_ok(dt, q, 8)) {
        HIP_TRY(launch_gemm(dt, q, 8, st));
      } else {   // shapes outside the large-tile kernel: problems of different M go separately
        HIP_TRY(launch_gemm(dt, p, 5, st));
        HIP_TRY(launch_gemm(dt, p + 5, 2, st));
        HIP_TRY(launch_gemm(dt, p + 7, 1, st));
      }
    } else {
      HIP_TRY(launch_gemm(dt, p, dt == MIXLORA_BF16 ? 5 : 4, st));
    }
  }
  DoraArgs dargs{};
  if (dora) {
    // factors c = m / n of the three projections (n: row norms of W + s B_e A_e)
    float *w2 = (float *)(ws + L.w2), *AA = (float *)(ws + L.AA);
    HIP_TRY_AS(PROF_OTHER, 0, launch_row_sqnorm(w->W_gate, f, d, w2, st));
    HIP_TRY_AS(PROF_OTHER, 0, launch_row_sqnorm(w->W_up, f, d, w2 + f, st));
    HIP_TRY_AS(PROF_OTHER, 0, launch_row_sqnorm(w->W_down, d, f, w2 + 2 * (size_t)f, st));
    HIP_TRY_AS(PROF_OTHER, 0, launch_gram(w->A_gate, N, r, d, AA, st));
    const size_t gpf = gram_part_floats(N, r);
    HIP_TRY_AS(PROF_OTHER, 0, launch_gram(w->A_up, N, r, d, AA + gpf, st));
    HIP_TRY_AS(PROF_OTHER, 0, launch_gram(w->A_down, N, r, f, AA + 2 * gpf, st));
    HIP_TRY_AS(PROF_OTHER, 0, launch_dora_scale(w->B_gate, (float *)(ws + L.WA_g), AA, w2, dora->m_gate, dora->shared, N, f, r,
                              D.lora_scale, (float *)(ws + L.c_g), (float *)(ws + L.ninv_g), st));
    HIP_TRY_AS(PROF_OTHER, 0, launch_dora_scale(w->B_up, (float *)(ws + L.WA_u), AA + gpf, w2 + f,
                              dora->m_up, dora->shared, N, f, r, D.lora_scale, (float *)(ws + L.c_u),
                              (float *)(ws + L.ninv_u), st));
    HIP_TRY_AS(PROF_OTHER, 0, launch_dora_scale(w->B_down, (float *)(ws + L.WA_d), AA + 2 * gpf, w2 + 2 * (size_t)f,
                              dora->m_down, dora->shared, N, d, r, D.lora_scale, (float *)(ws + L.c_d),
                              (float *)(ws + L.ninv_d), st));
    dargs.cg = (float *)(ws + L.c_g);
    dargs.cu = (float *)(ws + L.c_u);
  }
  // Eq. 7 + Norm (Algorithm 1 lines 4-5)
  // s * B_down packed for the K-extension of the down GEMM; in bf16 also zeros for the
  // block-sparse operand Qw, whose non-zero blocks the fused stage fills in.  In bf16 these
  // re-layouts ride in the routing launch.
  const RelayoutJob fwd_jobs[2] = {job_bank_cat(w->B_down, N, d, r, D.lora_scale, ws + L.Bd_cat, R, 0),
                                   pair_down ? job_zero_fill(ws + L.Qp, (size_t)kT * R * 2)
                                             : job_zero_fill(ws + L.Qw, (size_t)T * R * 2)};
  if (dt == MIXLORA_BF16)
    HIP_TRY_AS(PROF_ROUTING, (double)T * N * 8,
               launch_route_logits_relayout((const float *)(ws + L.Z), N, T, N, k, probs, topk_idx,
                                            topk_w, idx, wts, Nl, token_model, fwd_jobs, 2, st));
  else
    HIP_TRY_AS(PROF_ROUTING, (double)T * d * Eb, launch_router(dt, x, w->W_router, T, d, N, k, probs, topk_idx, topk_w, idx, wts, Nl,
                          token_model, st));
  PairCtx pc{offs, pair_of_row, row_of_pair, wts, idx, T, N, k, r};
  // the per-pair stages on tokens grouped by expert pair (csrc/fused_pg.hip), when they apply
  const bool use_pg = dt == MIXLORA_BF16 && !pair_down && !dora && fused_pg_ok(pc, f);
  int32_t *pg_tok = (int32_t *)(ws + L.pg_tok), *pg_tiles = (int32_t *)(ws + L.pg_tiles),
          *pg_ntiles = (int32_t *)(ws + L.pg_ntiles);
  // grouping of the pairs by expert and Eq. 8-9, one launch
  if ((size_t)kT > GROUP_SINGLE_WG_PAIRS) {
    HIP_TRY_AS(PROF_ROUTING, (double)kT * 16, launch_group_pairs_aux_multi(idx, T, N, k, (int32_t *)(ws + L.counts), expert_counts,
                                         (int32_t *)(ws + L.first_counts), offs, row_of_pair,
                                         pair_of_row, (int32_t *)(ws + L.tok_offs), probs,
                                         D.aux_coeff, D.aux_mode, aux_loss, (float *)(ws + L.F),
                                         (float *)(ws + L.P), Nl, token_model,
                                         (int32_t *)(ws + L.model_tokens), ws + L.gp_scratch, st));
    if (use_pg)
      HIP_TRY_AS(PROF_ROUTING, (double)T * 12, launch_group_token_pairs(pc, pg_tok, pg_tiles, pg_ntiles, st));
  } else {
    // (Eq. 8-9 and the tokens' grouping by expert pair run as further workgroups of the launch)
    HIP_TRY_AS(PROF_ROUTING, (double)kT * 16 + (use_pg ? (double)T * 12 : 0.0),
               launch_group_pairs_aux(idx, T, N, k, (int32_t *)(ws + L.counts), expert_counts,
                                      (int32_t *)(ws + L.first_counts), offs, row_of_pair, pair_of_row,
                                      (int32_t *)(ws + L.tok_offs), probs, D.aux_coeff, D.aux_mode,
                                      aux_loss, (float *)(ws + L.F), (float *)(ws + L.P), Nl,
                                      token_model, (int32_t *)(ws + L.model_tokens),
                                      use_pg ? pg_tok : nullptr, pg_tiles, pg_ntiles, st));
  }
  if (dt != MIXLORA_BF16) HIP_TRY_AS(PROF_OTHER, 0, launch_relayout(dt, fwd_jobs, 1, st));
  if (pair_down) {
    // The paper's schedules (Figure 3): every expert runs its own frozen products on its slice of
    // tokens.  (a) unshared: gate and up on the gathered token rows, k rows per token;
    // (b) shared: gate and up once per token (above).  Both: the down projection on every pair
    // row, combined with the routing weights afterwards (Algorithm 1 lines 14-15).
    const char *Gsrc = ws + L.G, *Usrc = ws + L.U;
    int rows_mode = ROWS_SPARSE;
    if (vanilla) {
      HIP_TRY_AS(PROF_OTHER, 2.0 * kT * d * Eb, launch_gather_rows(dt, pc, d, x, ws + L.Xp, st));
      // the LoRA A projections of every expert (per token) ride in the same launch
      GemmProblem p[4] = {problem(kT, f, ws + L.Gp, f, 0), problem(kT, f, ws + L.Up, f, 0),
                          problem(T, R, ws + L.Pg_all, R, 1), problem(T, R, ws + L.Pu_all, R, 1)};
      add_seg(p[0], ws + L.Xp, d, w->W_gate, d, d);
      add_seg(p[1], ws + L.Xp, d, w->W_up, d, d);
      add_seg(p[2], x, d, w->A_gate, d, d);
      add_seg(p[3], x, d, w->A_up, d, d);
      if (gemm_mixed_rows_ok(dt, p, 4)) {
        HIP_TRY(launch_gemm(dt, p, 4, st));
      } else {   // shapes outside the large-tile kernel: problems of different M go separately
        HIP_TRY(launch_gemm(dt, p, 2, st));
        HIP_TRY(launch_gemm(dt, p + 2, 2, st));
      }
      Gsrc = ws + L.Gp;
      Usrc = ws + L.Up;
      rows_mode |= ROWS_GU;
    }
    HIP_TRY_AS(PROF_FUSED_FWD, 3.0 * kT * f * Eb, launch_swiglu_fwd_mfma(pc, f, D.lora_scale, Gsrc, Usrc, (float *)(ws + L.Pg_all),
                                   (float *)(ws + L.Pu_all), w->B_gate, w->B_up, w->A_down,
                                   ws + L.a_grp, (float *)(ws + L.rank_part),
                                   (float *)(ws + L.Q_all), ws + L.Qp, R, st, rows_mode,
                                   dora ? &dargs : nullptr));
    GemmProblem p = problem(kT, d, ws + L.Op, d, 0);
    add_seg(p, ws + L.a_grp, f, w->W_down, f, f);
    add_seg(p, ws + L.Qp, R, ws + L.Bd_cat, R, R);
    HIP_TRY(launch_gemm(dt, &p, 1, st));
    if (!dora) {
      HIP_TRY_AS(PROF_COMBINE, (double)(k + 1) * T * d * Eb, launch_pair_combine(dt, pc, d, ws + L.Op, y, 1, st));
      return MIXLORA_OK;
    }
    // the down projection's factor is applied to every pair's output while combining
    HIP_TRY_AS(PROF_COMBINE, (double)(k + 1) * T * d * Eb, launch_pair_combine_scaled(pc, d, ws + L.Op, (float *)(ws + L.c_d), y, st));
    return MIXLORA_OK;
  }
  if (use_pg) {
    // tokens grouped by expert pair: rank-r deltas, SiLU * up, the weighted combination of a
    // token's two pairs (Algorithm 1 lines 11-13 and 15) and the A_down projections in one pass
    // that fetches G and U once per token; the grouped activations are kept only when a backward
    // pass can follow
    const int write_a = workspace_bytes >= L.bwd_end ? 1 : 0;
    HIP_TRY_AS(PROF_FUSED_FWD, (double)(3 + 2 * write_a) * T * f * Eb,
               launch_swiglu_fwd_pg(pc, f, D.lora_scale, pg_tok, pg_tiles, pg_ntiles,
                                    ws + L.G, ws + L.U, (float *)(ws + L.Pg_all),
                                    (float *)(ws + L.Pu_all), w->B_gate, w->B_up, w->A_down,
                                    ws + L.a_grp, ws + L.a_comb, (float *)(ws + L.rank_part),
                                    (float *)(ws + L.Q_all), ws + L.Qw, R, write_a, st));
    GemmProblem p = problem(T, d, y, d, 0);
    add_seg(p, ws + L.a_comb, f, w->W_down, f, f);
    add_seg(p, ws + L.Qw, R, ws + L.Bd_cat, R, R);
    HIP_TRY(launch_gemm(dt, &p, 1, st));
    return MIXLORA_OK;
  }
  // Algorithm 1 lines 11-13 on the routed pairs, expert-grouped rows
  // (few tokens: the sum of the stage's rank-r partial products rides in the combine's launch;
  // each of the two launches alone is little more than its own latency)
  const bool merge_tail = dt == MIXLORA_BF16 && (size_t)T <= SPLITK_MAX_ROWS && k * r <= 256;
  if (dt == MIXLORA_BF16) {
    // fused: LoRA deltas + SiLU * up + A_down of the row's expert, all on MFMA
    HIP_TRY_AS(PROF_FUSED_FWD, 3.0 * kT * f * Eb, launch_swiglu_fwd_mfma(pc, f, D.lora_scale, ws + L.G, ws + L.U,
                                   (float *)(ws + L.Pg_all), (float *)(ws + L.Pu_all), w->B_gate,
                                   w->B_up, w->A_down, ws + L.a_grp, (float *)(ws + L.rank_part),
                                   (float *)(ws + L.Q_all), ws + L.Qw, R, st, 0, nullptr, !merge_tail));
  } else {
    HIP_TRY_AS(PROF_FUSED_FWD, 3.0 * kT * f * Eb, launch_swiglu_fwd(dt, pc, f, D.lora_scale, ws + L.G, ws + L.U,
                              (float *)(ws + L.Pg_all), (float *)(ws + L.Pu_all), w->B_gate,
                              w->B_up, ws + L.a_grp, st));
    // A_down of every expert on the grouped activations
    GemmProblem p = problem(kT, R, ws + L.Q_all, R, 1);
    add_seg(p, ws + L.a_grp, f, w->A_down, f, f);
    HIP_TRY(launch_gemm(dt, &p, 1, st));
    // the block-sparse low-rank operand
    HIP_TRY_AS(PROF_OTHER, 0, launch_scatter_blocks(dt, pc, (float *)(ws + L.Q_all), 0, 1, R, 1, 1, ws + L.Qw, R, 0, st));
  }
  // weighted combine of the pair activations (Algorithm 1 line 15, moved in front of the linear
  // frozen down projection)
  if (merge_tail)
    HIP_TRY_AS(PROF_COMBINE, (double)(k + 1) * T * f * Eb,
               launch_pair_combine_reduce(pc, f, ws + L.a_grp, ws + L.a_comb, (float *)(ws + L.rank_part),
                                          fused_splits(f, kT), (float *)(ws + L.Q_all), ws + L.Qw, R, st));
  else
    HIP_TRY_AS(PROF_COMBINE, (double)(k + 1) * T * f * Eb,
               launch_pair_combine(dt, pc, f, ws + L.a_grp, ws + L.a_comb, 1, st));
  // down projection (Algorithm 1 line 14): y = a_comb W_down^T + Qw (s B_down)^T
  if (dt == MIXLORA_BF16 && (size_t)T <= SPLITK_MAX_ROWS) {
    // Few rows: the d output columns alone give too few tiles to stream W_down at full rate, so
    // the K range is cut into S slices (whole 64-wide K tiles), one GEMM problem each with an
    // fp32 partial output, and the partial outputs are added in slice order.
    const int tiles_n = (d + 63) / 64, ktiles = (f + 63) / 64;
    int S = 256 / tiles_n;
    S = S < 1 ? 1 : (S > GEMM_MAX_PROBLEMS ? GEMM_MAX_PROBLEMS : S);
    S = S > ktiles ? ktiles : S;
    const int chunk = ((ktiles + S - 1) / S) * 64;
    GemmProblem p[GEMM_MAX_PROBLEMS];
    float *part = (float *)(ws + L.splitk);
    const size_t E = 2;
    int used = 0;
    for (int k0 = 0; k0 < f; k0 += chunk, used++) {
      p[used] = problem(T, d, part + (size_t)used * T * d, d, 1);
      const int klen = f - k0 < chunk ? f - k0 : chunk;
      add_seg(p[used], ws + L.a_comb + (size_t)k0 * E, f, (const char *)w->W_down + (size_t)k0 * E, f, klen);
      if (used == 0) add_seg(p[0], ws + L.Qw, R, ws + L.Bd_cat, R, R);
    }
    HIP_TRY(launch_gemm(dt, p, used, st));
    HIP_TRY_AS(PROF_OTHER, 0, launch_splitk_reduce(dt, part, used, (int64_t)T * d, y, st));
  } else {
    GemmProblem p = problem(T, d, y, d, 0);
    add_seg(p, ws + L.a_comb, f, w->W_down, f, f);
    add_seg(p, ws + L.Qw, R, ws + L.Bd_cat, R, R);
    HIP_TRY(launch_gemm(dt, &p, 1, st));
  }
  return MIXLORA_OK;
}

// Validation shared by the forward entry points; D.N is the number of experts in all.
static int check_forward_args(const mixlora_dims *dims, const mixlora_weights *w, const void *x,
                              const void *y, const int32_t *topk_idx, const float *topk_w,
                              const int32_t *expert_counts, const float *aux_loss,
                              const void *workspace) {
  int rc = check_dims(dims);
  if (rc) return rc;
  rc = check_weights(w);
  if (rc) return rc;
  if (!x || !y || !topk_idx || !topk_w || !expert_counts || !aux_loss || !workspace)
    return MIXLORA_E_NULL;
  if (misaligned(x) || misaligned(y) || misaligned(workspace)) return MIXLORA_E_ALIGN;
  return MIXLORA_OK;
}

int mixlora_ffn_forward(const mixlora_dims *dims, const mixlora_weights *w, const void *x,
                        void *y, int32_t *topk_idx, float *topk_w, int32_t *expert_counts,
                        float *aux_loss, void *workspace, size_t workspace_bytes,
                        void *stream) {
  const int rc = check_forward_args(dims, w, x, y, topk_idx, topk_w, expert_counts, aux_loss, workspace);
  if (rc) return rc;
  return forward_impl(*dims, dims->N, nullptr, w, x, y, topk_idx, topk_w, expert_counts, aux_loss,
                      workspace, workspace_bytes, stream);
}

// dims with N replaced by the number of experts of all adapters together
static int multi_dims(const mixlora_dims *dims, const mixlora_multi *multi, mixlora_dims *all) {
  if (!dims || !multi) return MIXLORA_E_NULL;
  if (multi->M < 1 || multi->M > 64 || dims->N < 1 || dims->k > dims->N) return MIXLORA_E_SHAPE;
  if ((int64_t)multi->M * dims->N > 64) return MIXLORA_E_SHAPE;
  if (!multi->token_model) return MIXLORA_E_NULL;
  *all = *dims;
  all->N = multi->M * dims->N;
  return check_dims(all);
}

size_t mixlora_multi_workspace_bytes(const mixlora_dims *dims, int32_t M, int for_backward) {
  if (!dims || M < 1 || (int64_t)M * dims->N > 64 || dims->k > dims->N) return 0;
  mixlora_dims all = *dims;
  all.N = M * dims->N;
  return mixlora_workspace_bytes(&all, for_backward);
}

int mixlora_multi_forward(const mixlora_dims *dims, const mixlora_multi *multi,
                          const mixlora_weights *w, const void *x, void *y, int32_t *topk_idx,
                          float *topk_w, int32_t *expert_counts, float *aux_loss, void *workspace,
                          size_t workspace_bytes, void *stream) {
  mixlora_dims all;
  int rc = multi_dims(dims, multi, &all);
  if (rc) return rc;
  rc = check_forward_args(&all, w, x, y, topk_idx, topk_w, expert_counts, aux_loss, workspace);
  if (rc) return rc;
  return forward_impl(all, dims->N, multi->token_model, w, x, y, topk_idx, topk_w, expert_counts,
                      aux_loss, workspace, workspace_bytes, stream);
}

static int check_backward_args(const mixlora_dims *dims, const mixlora_weights *w, const void *x,
                               const void *dy, const void *workspace, const void *dx,
                               const mixlora_grads *grads) {
  int rc = check_dims(dims);
  if (rc) return rc;
  rc = check_weights(w);
  if (rc) return rc;
  if (!x || !dy || !dx || !workspace || !grads) return MIXLORA_E_NULL;
  float *gp[] = {grads->dA_gate, grads->dB_gate, grads->dA_up,    grads->dB_up,
                 grads->dA_down, grads->dB_down, grads->dW_router};
  for (float *p : gp) {
    if (!p) return MIXLORA_E_NULL;
    if (misaligned(p)) return MIXLORA_E_ALIGN;
  }
  if (misaligned(x) || misaligned(dy) || misaligned(dx) || misaligned(workspace))
    return MIXLORA_E_ALIGN;
  return MIXLORA_OK;
}

// Backward pass; same conventions as forward_impl.
static int backward_impl(const mixlora_dims &Du, int Nl, const int32_t *token_model,
                         const AuxUpstream &d_aux, const mixlora_weights *w, const void *x,
                         const void *dy, void *workspace, size_t workspace_bytes, void *dx,
                         const mixlora_grads *grads, void *stream,
                         int schedule = MIXLORA_SCHEDULE_LINEAR_DOWN,
                         const mixlora_dora *dora = nullptr,
                         const mixlora_dora_grads *dgrads = nullptr) {
  const Layout L = make_layout(Du, schedule, dora != nullptr);
  const bool pair_down = schedule != MIXLORA_SCHEDULE_LINEAR_DOWN;
  const bool vanilla = schedule == MIXLORA_SCHEDULE_VANILLA;
  if (workspace_bytes < L.bwd_end) return MIXLORA_E_WORKSPACE;

  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  char *ws = reinterpret_cast<char *>(workspace);
  mixlora_dims D = Du;   // rank-padded banks (the forward pass left them in the workspace) and
  D.r = L.rp;            // rank-padded gradients, cut back to r entries at the end
  mixlora_weights wpad;
  mixlora_grads gpad;
  const mixlora_grads *grads_user = grads;
  if (L.rp != Du.r) {
    wpad = *w;
    gpad = *grads;
    const void **wp[6] = {&wpad.A_gate, &wpad.B_gate, &wpad.A_up, &wpad.B_up, &wpad.A_down, &wpad.B_down};
    float **gp[6] = {&gpad.dA_gate, &gpad.dB_gate, &gpad.dA_up, &gpad.dB_up, &gpad.dA_down, &gpad.dB_down};
    for (int i = 0; i < 6; i++) {
      *wp[i] = ws + L.pad_w[i];
      *gp[i] = (float *)(ws + L.pad_g[i]);
    }
    w = &wpad;
    grads = &gpad;
  }
  const int T = D.T, d = D.d, f = D.d_ff, N = D.N, k = D.k, r = D.r, R = N * r, kT = k * T;
  const int dt = D.dtype, Kx = L.Kx;
  const double Eb = dt == MIXLORA_BF16 ? 2.0 : 4.0;   // bytes per stored element (measurement hook)
  const float s = D.lora_scale;
  float *probs = (float *)(ws + L.probs);
  int32_t *idx = (int32_t *)(ws + L.idx);
  float *wts = (float *)(ws + L.w);
  int32_t *offs = (int32_t *)(ws + L.offs);
  int32_t *row_of_pair = (int32_t *)(ws + L.row_of_pair);
  int32_t *pair_of_row = (int32_t *)(ws + L.pair_of_row);
  PairCtx pc{offs, pair_of_row, row_of_pair, wts, idx, T, N, k, r};

  const void *WdT = w->W_down_T, *WgT = w->W_gate_T, *WuT = w->W_up_T;
  if (!WdT) { HIP_TRY_AS(PROF_OTHER, 2.0 * d * f * Eb, launch_transpose(dt, w->W_down, ws + L.WdT, d, f, st)); WdT = ws + L.WdT; }
  if (!WgT) { HIP_TRY_AS(PROF_OTHER, 2.0 * d * f * Eb, launch_transpose(dt, w->W_gate, ws + L.WgT, f, d, st)); WgT = ws + L.WgT; }
  if (!WuT) { HIP_TRY_AS(PROF_OTHER, 2.0 * d * f * Eb, launch_transpose(dt, w->W_up, ws + L.WuT, f, d, st)); WuT = ws + L.WuT; }

  // every re-layout of the LoRA banks and the router that the pass needs, in one launch
  {
    RelayoutJob jobs[8];
    bwd_relayout_jobs(L, ws, w, N, d, f, r, kT, T, s, vanilla, jobs);
    HIP_TRY_AS(PROF_OTHER, 0, launch_relayout(dt, jobs, dt == MIXLORA_BF16 ? 8 : 6, st));
  }
  // H = dy W_down  (once per token: the frozen down projection is shared and linear) and, in
  // the same launch, VB[t, e, :] = B_down[e]^T dy[t]
  if (pair_down) {
    // the paper's schedules: the frozen down projection is differentiated per pair row
    // (k rows per token); the routing weight is applied inside the fused stage as before
    if (dora) {
      // the pair's upstream gradient carries the down projection's factor: c_down[e] * dy[t],
      // and so does the B_down^T product (the transposed bank is scaled in place)
      HIP_TRY_AS(PROF_OTHER, 2.0 * kT * d * Eb, launch_gather_rows_scaled(pc, d, dy, (float *)(ws + L.c_d), ws + L.dYp, st));
      HIP_TRY_AS(PROF_OTHER, 0, launch_scale_bank(ws + L.Bd_T, (float *)(ws + L.c_d), N, r, d, st));
    } else {
      HIP_TRY_AS(PROF_OTHER, 2.0 * kT * d * Eb, launch_gather_rows(dt, pc, d, dy, ws + L.dYp, st));
    }
    GemmProblem p[2] = {problem(kT, f, ws + L.Hp, f, 0), problem(T, R, ws + L.VB_all, R, 1)};
    add_seg(p[0], ws + L.dYp, d, WdT, d, d);
    add_seg(p[1], dy, d, ws + L.Bd_T, d, d);
    if (gemm_mixed_rows_ok(dt, p, 2)) {
      HIP_TRY(launch_gemm(dt, p, 2, st));
    } else {   // shapes outside the large-tile kernel: problems of different M go separately
      HIP_TRY(launch_gemm(dt, p, 1, st));
      HIP_TRY(launch_gemm(dt, p + 1, 1, st));
    }
  } else {
    GemmProblem p[2] = {problem(T, f, ws + L.H, f, 0), problem(T, R, ws + L.VB_all, R, 1)};
    add_seg(p[0], dy, d, WdT, d, d);
    add_seg(p[1], dy, d, ws + L.Bd_T, d, d);
    HIP_TRY(launch_gemm(dt, p, 2, st));
  }
  const int rows_mode = (pair_down ? ROWS_H : 0) | (vanilla ? ROWS_GU | ROWS_SPARSE : 0);
  DoraArgs dargs{};
  if (dora) {
    dargs.cg = (float *)(ws + L.c_g);
    dargs.cu = (float *)(ws + L.c_u);
    dargs.dm_part_g = (float *)(ws + L.dm_part_g);
    dargs.dm_part_u = (float *)(ws + L.dm_part_u);
  }
  char *Sop = vanilla ? ws + L.Sp : ws + L.S;      // K-extension operand of the dx GEMM
  // through SiLU * up and the LoRA deltas, per pair; TG[row, e, :] = B_gate[e]^T dg[row] (and up)
  int nct = L.nct;
  // tokens grouped by expert pair (tables left by the forward pass): the per-token sums of dg and
  // du come out of the same launch
  const bool use_pg = dt == MIXLORA_BF16 && !pair_down && !dora && fused_pg_ok(pc, f);
  if (use_pg) {
    nct = fused_pg_splits(f, T, N);
    HIP_TRY_AS(PROF_FUSED_BWD, 9.0 * T * f * Eb,
               launch_swiglu_bwd_pg(pc, f, s, (int32_t *)(ws + L.pg_tok), (int32_t *)(ws + L.pg_tiles),
                                    (int32_t *)(ws + L.pg_ntiles), ws + L.G, ws + L.U, ws + L.H,
                                    (float *)(ws + L.Pg_all), (float *)(ws + L.Pu_all),
                                    (float *)(ws + L.VB_all), w->B_gate, w->B_up, ws + L.AdT,
                                    ws + L.Bg_T, ws + L.Bu_T, ws + L.dg_grp, ws + L.du_grp,
                                    ws + L.dgsum, ws + L.dusum, (float *)(ws + L.dw_part),
                                    (float *)(ws + L.rank_part), (float *)(ws + L.TG_all),
                                    (float *)(ws + L.TU_all), Sop, Kx, st));
  } else if (dt == MIXLORA_BF16) {
    nct = fused_splits(f, (int)kT);
    HIP_TRY_AS(PROF_FUSED_BWD, 5.0 * kT * f * Eb, launch_swiglu_bwd_mfma(pc, f, s, vanilla ? ws + L.Gp : ws + L.G,
                                   vanilla ? ws + L.Up : ws + L.U, pair_down ? ws + L.Hp : ws + L.H,
                                   (float *)(ws + L.Pg_all),
                                   (float *)(ws + L.Pu_all), (float *)(ws + L.VB_all), w->B_gate,
                                   w->B_up, ws + L.AdT, ws + L.Bg_T, ws + L.Bu_T, ws + L.dg_grp,
                                   ws + L.du_grp, (float *)(ws + L.dw_part),
                                   (float *)(ws + L.rank_part), (float *)(ws + L.TG_all),
                                   (float *)(ws + L.TU_all), Sop, Kx, st, rows_mode,
                                   dora ? &dargs : nullptr));
  } else {
    HIP_TRY_AS(PROF_FUSED_BWD, 5.0 * kT * f * Eb, launch_swiglu_bwd(dt, pc, f, s, ws + L.G, ws + L.U, (float *)(ws + L.Pg_all),
                              (float *)(ws + L.Pu_all), w->B_gate, w->B_up, ws + L.H,
                              (float *)(ws + L.VB_all), w->A_down, ws + L.dg_grp, ws + L.du_grp,
                              (float *)(ws + L.dw_part), L.nct, st));
    GemmProblem p[2] = {problem(kT, R, ws + L.TG_all, R, 1), problem(kT, R, ws + L.TU_all, R, 1)};
    add_seg(p[0], ws + L.dg_grp, f, ws + L.Bg_T, f, f);
    add_seg(p[1], ws + L.du_grp, f, ws + L.Bu_T, f, f);
    HIP_TRY(launch_gemm(dt, p, 2, st));
  }
  if (!vanilla && !use_pg) {   // shared gate/up: their input gradient needs the per-token sums only
    HIP_TRY_AS(PROF_COMBINE, 2.0 * (k + 1) * T * f * Eb, launch_pair_combine2(dt, pc, f, ws + L.dg_grp, ws + L.dgsum, ws + L.du_grp,
                                 ws + L.dusum, 0, st));
  }
  // per-row rank-r factors of the LoRA gradients, then the grouped outer-product sums:
  //   dB_gate[e] = s sum dg (x) Pg ; dA_gate[e] = s sum TG (x) x ; same for up ;
  //   dA_down[e] = s sum (w B_down^T dy) (x) a ; dB_down[e] = s sum dy (x) (w A_down a)
  float *part = (float *)(ws + L.partials);
  const size_t pfl = L.partial_floats;
  const float *fsrc[6] = {(float *)(ws + L.Pg_all), (float *)(ws + L.Pu_all),
                          (float *)(ws + L.TG_all), (float *)(ws + L.TU_all),
                          (float *)(ws + L.VB_all), (float *)(ws + L.Q_all)};
  const int by_token[6] = {1, 1, 0, 0, 1, 0}, weighted[6] = {0, 0, 0, 0, 1, 1};
  const void *wide[6] = {ws + L.dg_grp, ws + L.du_grp, x, x, ws + L.a_grp, dy};
  const int32_t *gat[6] = {nullptr, nullptr, pair_of_row, pair_of_row, nullptr, pair_of_row};
  const int width[6] = {f, f, d, d, f, d}, layout_qc[6] = {0, 0, 1, 1, 1, 0};
  float *gout[6] = {grads->dB_gate, grads->dB_up, grads->dA_gate, grads->dA_up,
                    grads->dA_down, grads->dB_down};
  // router: dw -> dz (also written into the K-extension operand S)
  HIP_TRY_AS(PROF_ROUTING, (double)T * N * 8, launch_router_bwd(dt, pc, probs, (float *)(ws + L.dw_part), nct,
                            (float *)(ws + L.VB_all), (float *)(ws + L.Q_all), (float *)(ws + L.F),
                            s, d_aux, D.aux_coeff, (float *)(ws + L.dw), (float *)(ws + L.dz),
                            Sop, Kx, 2 * R, Kx - 2 * R, Nl, token_model,
                            (const int32_t *)(ws + L.model_tokens),
                            dt == MIXLORA_BF16 ? ws + L.dzT : nullptr, L.ldTz, st, vanilla ? 1 : 0));
  // The input gradient goes before the gradient sums: those stream what the fused stage wrote, and
  // measured 15 us faster behind this long GEMM launch than right behind that stage.
  // dx = dgsum W_gate + dusum W_up + [TG | TU | dz] [s A_gate ; s A_up ; W_router]
  if (dt != MIXLORA_BF16)   // in bf16 the fused stage has already written these blocks
    HIP_TRY_AS(PROF_OTHER, 0, launch_scatter_blocks(dt, pc, (float *)(ws + L.TG_all),
                                  (int64_t)((float *)(ws + L.TU_all) - (float *)(ws + L.TG_all)), 2, R,
                                  1, 0, ws + L.S, Kx, 0, st));
  if (dora) {
    // magnitude gradients: dm = (1 / n) * sum over the expert's rows of (output gradient *
    // unscaled projection output); gate / up sums come from the fused stage per row tile
    HIP_TRY_AS(PROF_OTHER, 0, launch_dm_tiles_reduce(offs, N, f, (float *)(ws + L.dm_part_g),
                                   (float *)(ws + L.dm_part_u), (float *)(ws + L.ninv_g),
                                   (float *)(ws + L.ninv_u), dgrads->dm_gate, dgrads->dm_up, dora->shared, st));
    HIP_TRY_AS(PROF_OTHER, 0, launch_dm_down(pc, d, dy, ws + L.Op, (float *)(ws + L.ninv_d),
                           (float *)(ws + L.dmd_part), dgrads->dm_down, dora->shared, st));
  }
  if (vanilla) {
    // unshared schedule: every pair row goes through W_gate^T / W_up^T on its own, the k rows of
    // a token are added afterwards
    GemmProblem p = problem(kT, d, ws + L.dXp, d, 0);
    add_seg(p, ws + L.dg_grp, f, WgT, f, f);
    add_seg(p, ws + L.du_grp, f, WuT, f, f);
    add_seg(p, ws + L.Sp, Kx, ws + L.Bx, Kx, Kx);
    HIP_TRY(launch_gemm(dt, &p, 1, st));
    HIP_TRY_AS(PROF_COMBINE, (double)(k + 1) * T * d * Eb, launch_pair_combine(dt, pc, d, ws + L.dXp, dx, 0, st));
  } else {
    GemmProblem p = problem(T, d, dx, d, 0);
    add_seg(p, ws + L.dgsum, f, WgT, f, f);
    add_seg(p, ws + L.dusum, f, WuT, f, f);
    add_seg(p, ws + L.S, Kx, ws + L.Bx, Kx, Kx);
    HIP_TRY(launch_gemm(dt, &p, 1, st));
  }
  if (dt == MIXLORA_BF16) {
    GatherJob gj[6];
    for (int i = 0; i < 6; i++) gj[i] = GatherJob{fsrc[i], ws + L.small[i], by_token[i], weighted[i]};
    HIP_TRY_AS(PROF_OTHER, 0, launch_gather_small_T(pc, gj, 6, L.ldT, st));
    // the three sums over d_ff-wide operands in one launch, the three over gathered d-wide
    // operands in another (same groups, width and gather mode within a launch)
    const int wide_f[3] = {0, 1, 4}, wide_d[3] = {2, 3, 5};
    GomJob jf[3], jd[3];
    for (int j = 0; j < 3; j++) {
      jf[j] = GomJob{ws + L.small[wide_f[j]], wide[wide_f[j]], gout[wide_f[j]], layout_qc[wide_f[j]]};
      jd[j] = GomJob{ws + L.small[wide_d[j]], wide[wide_d[j]], gout[wide_d[j]], layout_qc[wide_d[j]]};
    }
    HIP_TRY_AS(PROF_GRAD_SUMS, 3.0 * kT * f * Eb,
               launch_group_outer_mfma(offs, N, kT, nullptr, k, jf, 3, L.ldT, r, f, s, part, pfl, st));
    if (dora) {
      // dB_down sums the factor-carrying pair rows c_down[e] * dy[t] (already gathered)
      HIP_TRY_AS(PROF_GRAD_SUMS, 2.0 * kT * d * Eb,
                 launch_group_outer_mfma(offs, N, kT, pair_of_row, k, jd, 2, L.ldT, r, d, s, part, pfl, st));
      const GomJob jb{ws + L.small[5], ws + L.dYp, gout[5], layout_qc[5]};
      HIP_TRY_AS(PROF_GRAD_SUMS, 1.0 * kT * d * Eb,
                 launch_group_outer_mfma(offs, N, kT, nullptr, k, &jb, 1, L.ldT, r, d, s, part, pfl, st));
    } else {
      HIP_TRY_AS(PROF_GRAD_SUMS, 3.0 * kT * d * Eb,
                 launch_group_outer_mfma(offs, N, kT, pair_of_row, k, jd, 3, L.ldT, r, d, s, part, pfl, st));
    }
    // dW_router = dz^T x  (the transposed bf16 dz comes from the router backward)
    const GomJob jr{ws + L.dzT, x, grads->dW_router, 1};
    HIP_TRY_AS(PROF_GRAD_SUMS, (double)T * d * Eb,
               launch_group_outer_mfma((int32_t *)(ws + L.tok_offs), 1, T, nullptr, 1, &jr, 1, L.ldTz,
                                       N, d, 1.f, part, pfl, st));
  } else {
    for (int i = 0; i < 6; i++) {
      HIP_TRY_AS(PROF_OTHER, 0, launch_gather_small(pc, fsrc[i], by_token[i], weighted[i], (float *)(ws + L.small[i]), st));
      HIP_TRY_AS(PROF_GRAD_SUMS, (double)kT * width[i] * Eb,
                 launch_group_outer(dt, offs, N, kT, gat[i], k, (float *)(ws + L.small[i]), r, wide[i],
                                    width[i], s, layout_qc[i], gout[i], part, pfl, st));
    }
    HIP_TRY_AS(PROF_GRAD_SUMS, (double)T * d * Eb,
               launch_group_outer(dt, (int32_t *)(ws + L.tok_offs), 1, T, nullptr, 1,
                                  (float *)(ws + L.dz), N, x, d, 1.f, 1, grads->dW_router, part, pfl, st));
  }
  if (L.rp != Du.r) {
    float *dst[6] = {grads_user->dA_gate, grads_user->dB_gate, grads_user->dA_up,
                     grads_user->dB_up, grads_user->dA_down, grads_user->dB_down};
    RelayoutJob jobs[6];
    for (int i = 0; i < 6; i++)
      jobs[i] = job_pad_bank(i, ws + L.pad_g[i], dst[i], N, L.rp, Du.r, d, f);
    HIP_TRY_AS(PROF_OTHER, 0, launch_relayout(MIXLORA_F32, jobs, 6, st));
  }
  return MIXLORA_OK;
}

int mixlora_ffn_backward(const mixlora_dims *dims, const mixlora_weights *w, const void *x,
                         const void *dy, float d_aux, void *workspace,
                         size_t workspace_bytes, void *dx, const mixlora_grads *grads,
                         void *stream) {
  const int rc = check_backward_args(dims, w, x, dy, workspace, dx, grads);
  if (rc) return rc;
  AuxUpstream up{};
  up.v[0] = d_aux;
  return backward_impl(*dims, dims->N, nullptr, up, w, x, dy, workspace, workspace_bytes, dx, grads,
                       stream);
}

int mixlora_multi_backward(const mixlora_dims *dims, const mixlora_multi *multi,
                           const mixlora_weights *w, const void *x, const void *dy,
                           void *workspace, size_t workspace_bytes, void *dx,
                           const mixlora_grads *grads, void *stream) {
  mixlora_dims all;
  int rc = multi_dims(dims, multi, &all);
  if (rc) return rc;
  rc = check_backward_args(&all, w, x, dy, workspace, dx, grads);
  if (rc) return rc;
  AuxUpstream up{};
  for (int m = 0; m < multi->M; m++) up.v[m] = multi->d_aux ? multi->d_aux[m] : 1.f;
  return backward_impl(all, dims->N, multi->token_model, up, w, x, dy, workspace, workspace_bytes,
                       dx, grads, stream);
}

static int check_schedule(const mixlora_dims *dims, int32_t schedule) {
  if (!dims) return MIXLORA_E_NULL;
  if (schedule < MIXLORA_SCHEDULE_LINEAR_DOWN || schedule > MIXLORA_SCHEDULE_VANILLA)
    return MIXLORA_E_SHAPE;
  if (schedule != MIXLORA_SCHEDULE_LINEAR_DOWN && dims->dtype != MIXLORA_BF16) return MIXLORA_E_DTYPE;
  return MIXLORA_OK;
}

size_t mixlora_schedule_workspace_bytes(const mixlora_dims *dims, int32_t schedule,
                                        int for_backward) {
  if (check_dims(dims) != MIXLORA_OK || check_schedule(dims, schedule) != MIXLORA_OK) return 0;
  const Layout L = make_layout(*dims, schedule);
  return for_backward ? L.bwd_end : L.fwd_end;
}

int mixlora_ffn_forward_schedule(const mixlora_dims *dims, int32_t schedule,
                                 const mixlora_weights *w, const void *x, void *y,
                                 int32_t *topk_idx, float *topk_w, int32_t *expert_counts,
                                 float *aux_loss, void *workspace, size_t workspace_bytes,
                                 void *stream) {
  int rc = check_forward_args(dims, w, x, y, topk_idx, topk_w, expert_counts, aux_loss, workspace);
  if (rc) return rc;
  rc = check_schedule(dims, schedule);
  if (rc) return rc;
  return forward_impl(*dims, dims->N, nullptr, w, x, y, topk_idx, topk_w, expert_counts, aux_loss,
                      workspace, workspace_bytes, stream, schedule);
}

int mixlora_ffn_backward_schedule(const mixlora_dims *dims, int32_t schedule,
                                  const mixlora_weights *w, const void *x, const void *dy,
                                  float d_aux, void *workspace, size_t workspace_bytes, void *dx,
                                  const mixlora_grads *grads, void *stream) {
  int rc = check_backward_args(dims, w, x, dy, workspace, dx, grads);
  if (rc) return rc;
  rc = check_schedule(dims, schedule);
  if (rc) return rc;
  AuxUpstream up{};
  up.v[0] = d_aux;
  return backward_impl(*dims, dims->N, nullptr, up, w, x, dy, workspace, workspace_bytes, dx, grads,
                       stream, schedule);
}

static int check_dora(const mixlora_dims *dims, const mixlora_dora *dora) {
  if (!dims || !dora) return MIXLORA_E_NULL;
  if (dims->dtype != MIXLORA_BF16) return MIXLORA_E_DTYPE;
  if (dora->shared != 0 && dora->shared != 1) return MIXLORA_E_SHAPE;
  const float *req[] = {dora->m_gate, dora->m_up, dora->m_down};
  for (const float *p : req) {
    if (!p) return MIXLORA_E_NULL;
    if (misaligned(p)) return MIXLORA_E_ALIGN;
  }
  return MIXLORA_OK;
}

size_t mixlora_dora_workspace_bytes(const mixlora_dims *dims, int for_backward) {
  if (check_dims(dims) != MIXLORA_OK || dims->dtype != MIXLORA_BF16) return 0;
  const Layout L = make_layout(*dims, MIXLORA_SCHEDULE_SHARED, true);
  return for_backward ? L.bwd_end : L.fwd_end;
}

int mixlora_dora_forward(const mixlora_dims *dims, const mixlora_weights *w,
                         const mixlora_dora *dora, const void *x, void *y, int32_t *topk_idx,
                         float *topk_w, int32_t *expert_counts, float *aux_loss, void *workspace,
                         size_t workspace_bytes, void *stream) {
  int rc = check_forward_args(dims, w, x, y, topk_idx, topk_w, expert_counts, aux_loss, workspace);
  if (rc) return rc;
  rc = check_dora(dims, dora);
  if (rc) return rc;
  return forward_impl(*dims, dims->N, nullptr, w, x, y, topk_idx, topk_w, expert_counts, aux_loss,
                      workspace, workspace_bytes, stream, MIXLORA_SCHEDULE_SHARED, dora);
}

int mixlora_dora_backward(const mixlora_dims *dims, const mixlora_weights *w,
                          const mixlora_dora *dora, const void *x, const void *dy, float d_aux,
                          void *workspace, size_t workspace_bytes, void *dx,
                          const mixlora_grads *grads, const mixlora_dora_grads *dora_grads,
                          void *stream) {
  int rc = check_backward_args(dims, w, x, dy, workspace, dx, grads);
  if (rc) return rc;
  rc = check_dora(dims, dora);
  if (rc) return rc;
  if (!dora_grads) return MIXLORA_E_NULL;
  float *gp[] = {dora_grads->dm_gate, dora_grads->dm_up, dora_grads->dm_down};
  for (float *p : gp) {
    if (!p) return MIXLORA_E_NULL;
    if (misaligned(p)) return MIXLORA_E_ALIGN;
  }
  AuxUpstream up{};
  up.v[0] = d_aux;
  return backward_impl(*dims, dims->N, nullptr, up, w, x, dy, workspace, workspace_bytes, dx, grads,
                       stream, MIXLORA_SCHEDULE_SHARED, dora, dora_grads);
}

// ---- forward without a caller workspace ---------------------------------------------------------
// The workspace of this entry point is a file-scope device array: every GPU the library runs on
// holds its own copy at its own address until the process ends.  The array's name is only a
// host-side handle; the device address is looked up once per device and used from then on.
}  // extern "C"

namespace {
static __device__ __align__(256) unsigned char scratch[MIXLORA_STATIC_SCRATCH_BYTES];
constexpr int STATIC_MAX_DEVICES = 64;
void *g_scratch_ptr[STATIC_MAX_DEVICES] = {};
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (NULL on failure).
void *static_scratch_ptr() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_MAX_DEVICES) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

extern "C" {

int mixlora_ffn_forward_static(const mixlora_dims *dims, const mixlora_weights *w, const void *x,
                               void *y, int32_t *topk_idx, float *topk_w, int32_t *expert_counts,
                               float *aux_loss, void *stream) {
  // host-only checks first: a non-NULL stand-in passes the workspace pointer test
  const int rc = check_forward_args(dims, w, x, y, topk_idx, topk_w, expert_counts, aux_loss,
                                    reinterpret_cast<const void *>(uintptr_t{256}));
  if (rc) return rc;
  const Layout L = make_layout(*dims);
  if (L.fwd_end > (size_t)MIXLORA_STATIC_SCRATCH_BYTES) return MIXLORA_E_SCRATCH;
  void *ws = static_scratch_ptr();
  if (!ws) return MIXLORA_E_HIP;
  return forward_impl(*dims, dims->N, nullptr, w, x, y, topk_idx, topk_w, expert_counts, aux_loss,
                      ws, (size_t)MIXLORA_STATIC_SCRATCH_BYTES, stream);
}

int mixlora_aux_loss(const float *probs, const int32_t *topk_idx, int32_t T, int32_t N,
                     int32_t k, float coeff, int32_t mode, float *loss, float *F, float *P,
                     float *dprobs, void *stream) {
  if (!probs || !topk_idx || !loss) return MIXLORA_E_NULL;
  if (mode != MIXLORA_AUX_TOP1 && mode != MIXLORA_AUX_TOPK) return MIXLORA_E_DTYPE;
  if (T < 1 || N < 1 || N > 64 || k < 1 || k > N || (int64_t)T * k >= (1 << 24))
    return MIXLORA_E_SHAPE;
  HIP_TRY(launch_aux_loss(probs, topk_idx, T, N, k, coeff, mode, loss, F, P, dprobs, N, nullptr,
                          nullptr, reinterpret_cast<hipStream_t>(stream)));
  return MIXLORA_OK;
}

int mixlora_profile_begin(int32_t max_launches) {
  return prof_begin(max_launches) == 0 ? MIXLORA_OK : MIXLORA_E_HIP;
}

int mixlora_profile_end(double *ms_total, int32_t *launches, double *flops_total) {
  if (!ms_total || !launches || !flops_total) return MIXLORA_E_NULL;
  if (prof_end() != 0) return MIXLORA_E_HIP;
  int n = 0;
  (void)prof_kind(PROF_GEMM, ms_total, &n, flops_total);
  *launches = n;
  return MIXLORA_OK;
}

int mixlora_profile_kind(int32_t kind, double *ms_total, int32_t *launches, double *work_total) {
  if (!ms_total || !launches || !work_total) return MIXLORA_E_NULL;
  int n = 0;
  if (prof_kind(kind, ms_total, &n, work_total) != 0) return MIXLORA_E_SHAPE;
  *launches = n;
  return MIXLORA_OK;
}

int mixlora_transpose(const void *in, void *out, int32_t rows, int32_t cols, int32_t dtype,
                      void *stream) {
  if (!in || !out) return MIXLORA_E_NULL;
  if (dtype != MIXLORA_F32 && dtype != MIXLORA_BF16) return MIXLORA_E_DTYPE;
  if (rows < 1 || cols < 1) return MIXLORA_E_SHAPE;
  HIP_TRY(launch_transpose(dtype, in, out, rows, cols, reinterpret_cast<hipStream_t>(stream)));
  return MIXLORA_OK;
}

}  // extern "C"
