// Plain LoRA linear (Eq. 1 with the scale alpha / r), the form the method puts on the attention
// projections (Section 3.2):  y = x W^T + s (x A^T) B^T  with W frozen.  Built from the same
// pieces as the feed-forward block: the frozen product and the rank-r projection share one GEMM
// launch, the rank-r update is added in place in fp32 before the result is rounded, and the
// gradients of A and B are outer-product sums over all tokens as one group.
#include "common.h"

using namespace mixlora;

namespace {

constexpr size_t ALIGN = 256;
inline size_t up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }
inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; }

inline int pad_rank(int r) { return (r + 7) & ~7; }

struct LinLayout {
  int rp;                         // rank entries the pass runs on: r rounded up to a multiple of 8
  size_t padA, padB, padgA, padgB;   // zero-padded copies of A, B (kept for the backward) and of dA, dB
  size_t P, tok_offs, slices, fwd_end;
  size_t W_T, Bt, At, VB, VB_T, P_T, partials, bwd_end;
  size_t partial_floats;
  int ldT;
};

LinLayout make_layout(const mixlora_linear_dims &D) {
  LinLayout L{};
  const size_t T = D.T, di = D.d_in, dn = D.d_out, r = pad_rank(D.r);
  const size_t E = D.dtype == MIXLORA_BF16 ? 2 : 4;
  const bool padded = (int)r != D.r;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = up(o + bytes); return at; };
  L.rp = (int)r;
  L.padA = take(padded ? r * di * E : 0);
  L.padB = take(padded ? dn * r * E : 0);
  L.P = take(T * r * 4);
  L.tok_offs = take(2 * 4);
  L.slices = take((size_t)(GEMM_MAX_PROBLEMS - 1) * T * r * 4);   // K-slice partial sums of a rank-r projection
  L.fwd_end = o;
  L.W_T = take(di * dn * E);
  L.Bt = take(r * dn * E);
  L.At = take(di * r * E);
  L.VB = take(T * r * 4);
  L.ldT = (int)((T + 15) / 16 * 16 + 16);
  L.VB_T = take((size_t)L.ldT * r * 2);
  L.P_T = take((size_t)L.ldT * r * 2);
  const int big = (int)(di > dn ? di : dn);
  size_t pf = group_outer_partial_floats(1, (int)r, big);
  const size_t pm = group_outer_mfma_partial_floats(1, (int)r, big);
  for (size_t v : {group_outer_partial_floats(1, (int)r, (int)di), group_outer_partial_floats(1, (int)r, (int)dn),
                   group_outer_mfma_partial_floats(1, (int)r, (int)di),
                   group_outer_mfma_partial_floats(1, (int)r, (int)dn), pm})
    pf = v > pf ? v : pf;
  L.partial_floats = pf;
  L.partials = take(pf * 4);
  L.padgA = take(padded ? r * di * 4 : 0);
  L.padgB = take(padded ? dn * r * 4 : 0);
  L.bwd_end = o;
  return L;
}

int check_dims(const mixlora_linear_dims *D) {
  if (!D) return MIXLORA_E_NULL;
  if (D->dtype != MIXLORA_F32 && D->dtype != MIXLORA_BF16) return MIXLORA_E_DTYPE;
  if (D->T < 1 || D->d_in < 8 || D->d_out < 8 || D->r < 1 || D->r > 64) return MIXLORA_E_SHAPE;
  if (D->d_in % 8 || D->d_out % 8) return MIXLORA_E_SHAPE;
  if ((int64_t)D->T >= (1 << 24)) return MIXLORA_E_SHAPE;
  return MIXLORA_OK;
}

__global__ void set_pair_kernel(int32_t *p, int a, int b) {
  if (threadIdx.x == 0 && blockIdx.x == 0) { p[0] = a; p[1] = b; }
}

#define HIP_TRY(expr)                                   \
  do {                                                  \
    hipError_t e_ = (expr);                             \
    if (e_ != hipSuccess) return MIXLORA_E_HIP;         \
  } while (0)

GemmProblem problem(int M, int N, void *C, int64_t ldc, int c_f32, const void *A, int64_t lda,
                    const void *B, int64_t ldb, int K) {
  GemmProblem p{};
  p.M = M; p.N = N; p.C = C; p.ldc = ldc; p.c_f32 = c_f32; p.nseg = 1;
  p.seg[0].A = A; p.seg[0].lda = lda; p.seg[0].B = B; p.seg[0].ldb = ldb; p.seg[0].K = K;
  return p;
}

// One launch for  C_main = X Wmain^T  (storage dtype)  and the rank-r projection
// C_small = X Wsmall^T  (float32, r columns), both with contraction length K.  The frozen product of
// a square projection fills the chip exactly once, so a second problem whose few tiles run the
// whole K range would add a second round almost as long as the first; the small problem is
// therefore cut into K slices (one problem each, fp32 partial outputs) that finish in a fraction
// of a round, and the slices are added in order afterwards.
int gemm_with_sliced_projection(int dtype, int T, int Nmain, int r, int K, const void *X,
                                const void *Wmain, void *Cmain, const void *Wsmall, float *Csmall,
                                float *slices, hipStream_t st) {
  const size_t E = dtype == MIXLORA_BF16 ? 2 : 4;
  const int ktiles = (K + 63) / 64;
  int S = GEMM_MAX_PROBLEMS - 1;
  if (dtype != MIXLORA_BF16 || T <= 128 || ktiles < 2 * S) S = 1;
  GemmProblem p[GEMM_MAX_PROBLEMS];
  p[0] = problem(T, Nmain, Cmain, Nmain, 0, X, K, Wmain, K, K);
  if (S == 1) {
    p[1] = problem(T, r, Csmall, r, 1, X, K, Wsmall, K, K);
    HIP_TRY(launch_gemm(dtype, p, 2, st));
    return MIXLORA_OK;
  }
  const int chunk = ((ktiles + S - 1) / S) * 64;
  int used = 0;
  for (int k0 = 0; k0 < K; k0 += chunk, used++) {
    const int klen = K - k0 < chunk ? K - k0 : chunk;
    p[1 + used] = problem(T, r, slices + (size_t)used * T * r, r, 1, (const char *)X + (size_t)k0 * E, K,
                          (const char *)Wsmall + (size_t)k0 * E, K, klen);
  }
  HIP_TRY(launch_gemm(dtype, p, 1 + used, st));
  HIP_TRY(launch_splitk_reduce(MIXLORA_F32, slices, used, (int64_t)T * r, Csmall, st));
  return MIXLORA_OK;
}

}  // namespace

extern "C" {

size_t mixlora_lora_linear_workspace_bytes(const mixlora_linear_dims *dims, int for_backward) {
  if (check_dims(dims) != MIXLORA_OK) return 0;
  const LinLayout L = make_layout(*dims);
  return for_backward ? L.bwd_end : L.fwd_end;
}

int mixlora_lora_linear_forward(const mixlora_linear_dims *dims, const void *W, const void *A,
                                const void *B, const void *x, void *y, void *workspace,
                                size_t workspace_bytes, void *stream) {
  const int rc = check_dims(dims);
  if (rc) return rc;
  if (!W || !A || !B || !x || !y || !workspace) return MIXLORA_E_NULL;
  for (const void *p : {W, A, B, x, (const void *)y, (const void *)workspace})
    if (misaligned(p)) return MIXLORA_E_ALIGN;
  mixlora_linear_dims D = *dims;
  const LinLayout L = make_layout(D);
  if (workspace_bytes < L.fwd_end) return MIXLORA_E_WORKSPACE;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  char *ws = reinterpret_cast<char *>(workspace);
  if (L.rp != D.r) {   // run on zero-padded banks (they stay in the workspace for the backward)
    const RelayoutJob jobs[2] = {job_rank_resize(A, ws + L.padA, 1, D.r, L.rp, D.d_in, true),
                                 job_rank_resize(B, ws + L.padB, 1, D.r, L.rp, D.d_out, false)};
    HIP_TRY(launch_relayout(D.dtype, jobs, 2, st));
    A = ws + L.padA;
    B = ws + L.padB;
    D.r = L.rp;
  }
  // y0 = x W^T and P = x A^T in one launch (both read x), then y = y0 + s P B^T in place
  const int grc = gemm_with_sliced_projection(D.dtype, D.T, D.d_out, D.r, D.d_in, x, W, y, A,
                                              (float *)(ws + L.P), (float *)(ws + L.slices), st);
  if (grc) return grc;
  HIP_TRY(launch_lowrank_add(D.dtype, y, (const float *)(ws + L.P), B, D.T, D.d_out, D.r,
                             D.lora_scale, st));
  return MIXLORA_OK;
}

int mixlora_lora_linear_backward(const mixlora_linear_dims *dims, const void *W, const void *W_T,
                                 const void *A, const void *B, const void *x, const void *dy,
                                 void *workspace, size_t workspace_bytes, void *dx, float *dA,
                                 float *dB, void *stream) {
  const int rc = check_dims(dims);
  if (rc) return rc;
  if (!W || !A || !B || !x || !dy || !workspace || !dx || !dA || !dB) return MIXLORA_E_NULL;
  for (const void *p : {W, A, B, x, dy, (const void *)workspace, (const void *)dx, (const void *)dA,
                        (const void *)dB})
    if (misaligned(p)) return MIXLORA_E_ALIGN;
  if (W_T && misaligned(W_T)) return MIXLORA_E_ALIGN;
  const mixlora_linear_dims &D = *dims;
  const LinLayout L = make_layout(D);
  if (workspace_bytes < L.bwd_end) return MIXLORA_E_WORKSPACE;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  char *ws = reinterpret_cast<char *>(workspace);
  const int T = D.T, di = D.d_in, dn = D.d_out, r = L.rp, dt = D.dtype;
  float *dA_user = dA, *dB_user = dB;
  if (L.rp != D.r) {   // padded banks from the forward pass; padded gradients, cut back at the end
    A = ws + L.padA;
    B = ws + L.padB;
    dA = (float *)(ws + L.padgA);
    dB = (float *)(ws + L.padgB);
  }
  const float s = D.lora_scale;
  if (!W_T) {
    HIP_TRY(launch_transpose(dt, W, ws + L.W_T, dn, di, st));
    W_T = ws + L.W_T;
  }
  {
    const RelayoutJob jobs[2] = {job_bank_T(B, 1, dn, r, ws + L.Bt),     // [d_out, r] -> [r, d_out]
                                 job_bank_T(A, 1, r, di, ws + L.At)};    // [r, d_in]  -> [d_in, r]
    HIP_TRY(launch_relayout(dt, jobs, 2, st));
  }
  hipLaunchKernelGGL(set_pair_kernel, dim3(1), dim3(64), 0, st, (int32_t *)(ws + L.tok_offs), 0, T);
  HIP_TRY(hipGetLastError());
  // dx0 = dy W and VB = dy B in one launch (both read dy), then dx = dx0 + s VB A in place
  const int grc = gemm_with_sliced_projection(dt, T, di, r, dn, dy, W_T, dx, ws + L.Bt,
                                              (float *)(ws + L.VB), (float *)(ws + L.slices), st);
  if (grc) return grc;
  HIP_TRY(launch_lowrank_add(dt, dx, (const float *)(ws + L.VB), ws + L.At, T, di, r, s, st));
  // dA = s VB^T x  [r, d_in];  dB = s dy^T P  [d_out, r]: outer-product sums over all tokens
  const int32_t *tok = (const int32_t *)(ws + L.tok_offs);
  float *part = (float *)(ws + L.partials);
  if (dt == MIXLORA_BF16) {
    HIP_TRY(launch_f32_to_bf16T((const float *)(ws + L.VB), T, r, ws + L.VB_T, L.ldT, st));
    const GomJob ja{ws + L.VB_T, x, dA, 1};
    HIP_TRY(launch_group_outer_mfma(tok, 1, T, nullptr, 1, &ja, 1, L.ldT, r, di, s, part,
                                    L.partial_floats, st));
    HIP_TRY(launch_f32_to_bf16T((const float *)(ws + L.P), T, r, ws + L.P_T, L.ldT, st));
    const GomJob jb{ws + L.P_T, dy, dB, 0};
    HIP_TRY(launch_group_outer_mfma(tok, 1, T, nullptr, 1, &jb, 1, L.ldT, r, dn, s, part,
                                    L.partial_floats, st));
  } else {
    HIP_TRY(launch_group_outer(dt, tok, 1, T, nullptr, 1, (const float *)(ws + L.VB), r, x, di, s, 1,
                               dA, part, L.partial_floats, st));
    HIP_TRY(launch_group_outer(dt, tok, 1, T, nullptr, 1, (const float *)(ws + L.P), r, dy, dn, s, 0,
                               dB, part, L.partial_floats, st));
  }
  if (L.rp != D.r) {
    const RelayoutJob jobs[2] = {job_rank_resize(dA, dA_user, 1, L.rp, D.r, di, true),
                                 job_rank_resize(dB, dB_user, 1, L.rp, D.r, dn, false)};
    HIP_TRY(launch_relayout(MIXLORA_F32, jobs, 2, st));
  }
  return MIXLORA_OK;
}

}  // extern "C"
