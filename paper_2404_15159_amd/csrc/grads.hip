// Gradient kernels: sums of outer products over the rows of each expert group (the LoRA A/B
// gradients and the router weight gradient), and the router's backward (top-k renormalised
// softmax of Eq. 7 / Algorithm 1 plus the auxiliary term of Eq. 8-9).
//
// Each LoRA gradient has the form  out[g] = scale * sum_{rows of group g} small[row] (x) wide[row']
// with `small` an r-vector per grouped row and `wide` a d- or d_ff-wide row (grouped, or the
// token's row).  The sum over rows is split into fixed slices whose partial results are added
// in a fixed order by a second kernel: no floating-point atomics, bit-reproducible.
#include "common.h"

namespace mixlora {

constexpr int GO_COLS = 512;   // 256 threads x 2 adjacent columns
constexpr int GO_STAGE = 64;   // rows staged per pass

__device__ __forceinline__ float2 ld2(const float *p) { return *reinterpret_cast<const float2 *>(p); }
__device__ __forceinline__ float2 ld2(const bf16_t *p) {
  typedef bf16_t bf16x2_t __attribute__((ext_vector_type(2)));
  const bf16x2_t v = *reinterpret_cast<const bf16x2_t *>(p);
  return make_float2((float)v[0], (float)v[1]);
}

// partial[split][g][q][c], q < r.  RQ = rank chunk held in registers.
template <typename E, int RQ>
__global__ __launch_bounds__(256) void group_outer_kernel(
    const int32_t *__restrict__ offs, const int32_t *__restrict__ pair_of_row, int k,
    const float *__restrict__ small, int r, const E *__restrict__ wide, int C, int nsplit,
    float *__restrict__ partial) {
  __shared__ float sm[GO_STAGE][RQ];
  __shared__ int src_s[GO_STAGE];
  const int g = blockIdx.y, sp = blockIdx.z, G = gridDim.y;
  const int lo = offs[g], hi = offs[g + 1];
  const int len = (hi - lo + nsplit - 1) / nsplit;
  const int r_lo = lo + sp * len;
  const int r_hi = r_lo + len < hi ? r_lo + len : hi;
  const int c = blockIdx.x * GO_COLS + threadIdx.x * 2;
  const bool active = c < C;
  for (int q0 = 0; q0 < r; q0 += RQ) {
    float acc[RQ][2];
#pragma unroll
    for (int q = 0; q < RQ; q++) acc[q][0] = acc[q][1] = 0.f;
    for (int rb = r_lo; rb < r_hi; rb += GO_STAGE) {
      const int n = r_hi - rb < GO_STAGE ? r_hi - rb : GO_STAGE;
      __syncthreads();
      for (int i = threadIdx.x; i < GO_STAGE * RQ; i += 256) {
        const int rr = i / RQ, q = i % RQ;
        sm[rr][q] = (rr < n && q0 + q < r) ? small[(int64_t)(rb + rr) * r + q0 + q] : 0.f;
      }
      if (threadIdx.x < GO_STAGE && threadIdx.x < n)
        src_s[threadIdx.x] = pair_of_row ? pair_of_row[rb + threadIdx.x] / k : rb + threadIdx.x;
      __syncthreads();
      if (active) {
        for (int rr = 0; rr < n; rr++) {
          const float2 v = ld2(wide + (int64_t)src_s[rr] * C + c);
#pragma unroll
          for (int q = 0; q < RQ; q++) {
            const float sv = sm[rr][q];
            acc[q][0] = fmaf(sv, v.x, acc[q][0]);
            acc[q][1] = fmaf(sv, v.y, acc[q][1]);
          }
        }
      }
    }
    if (active) {
#pragma unroll
      for (int q = 0; q < RQ; q++) {
        if (q0 + q < r) {
          float *o = partial + (((int64_t)sp * G + g) * r + q0 + q) * C + c;
          *reinterpret_cast<float2 *>(o) = make_float2(acc[q][0], acc[q][1]);
        }
      }
    }
  }
}

// out = scale * sum_split partial, written as [g][q][c] (layout_qc) or [g][c][q]; blockIdx.y picks
// one of up to GOM_MAX_JOBS reductions of the same shape.
struct ReduceBatch {
  const float *partial[GOM_MAX_JOBS];
  float *out[GOM_MAX_JOBS];
  int layout_qc[GOM_MAX_JOBS];
};

__global__ void group_outer_reduce_kernel(ReduceBatch batch, int G, int r, int C, int nsplit,
                                          float scale) {
  const float *__restrict__ partial = batch.partial[blockIdx.y];
  float *__restrict__ out = batch.out[blockIdx.y];
  const int layout_qc = batch.layout_qc[blockIdx.y];
  const int64_t n = (int64_t)G * r * C;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  // four loads in flight at a time; the additions keep the split order
  float acc = 0.f;
  int sp = 0;
  for (; sp + 4 <= nsplit; sp += 4) {
    const float a0 = partial[(int64_t)sp * n + i], a1 = partial[(int64_t)(sp + 1) * n + i];
    const float a2 = partial[(int64_t)(sp + 2) * n + i], a3 = partial[(int64_t)(sp + 3) * n + i];
    acc += a0; acc += a1; acc += a2; acc += a3;
  }
  for (; sp < nsplit; sp++) acc += partial[(int64_t)sp * n + i];
  acc *= scale;
  if (layout_qc) {
    out[i] = acc;
  } else {
    const int c = (int)(i % C);
    const int q = (int)((i / C) % r);
    const int g = (int)(i / ((int64_t)C * r));
    out[((int64_t)g * C + c) * r + q] = acc;
  }
}

static int go_splits(int G, int C) {
  const int col_tiles = (C + GO_COLS - 1) / GO_COLS;
  int s = 1024 / (col_tiles * G);
  if (s < 1) s = 1;
  if (s > 32) s = 32;
  return s;
}

size_t group_outer_partial_floats(int G, int r, int C) {
  return (size_t)go_splits(G, C) * G * r * C;
}

hipError_t launch_group_outer(int dtype, const int32_t *offs, int G, int max_rows,
                              const int32_t *pair_of_row, int k, const float *small, int r,
                              const void *wide, int C, float scale, int layout_qc, float *out,
                              float *partials, size_t partial_floats, hipStream_t st) {
  (void)max_rows;
  const int nsplit = go_splits(G, C);
  if ((size_t)nsplit * G * r * C > partial_floats) return hipErrorInvalidValue;
  const dim3 grid((C + GO_COLS - 1) / GO_COLS, G, nsplit), block(256);
  const bool r16 = r > 8;
#define MIXLORA_GO(E_, RQ_)                                                                   \
  hipLaunchKernelGGL((group_outer_kernel<E_, RQ_>), grid, block, 0, st, offs, pair_of_row, k,   \
                     small, r, (const E_ *)wide, C, nsplit, partials)
  if (dtype == MIXLORA_BF16) {
    if (r16) MIXLORA_GO(bf16_t, 16); else MIXLORA_GO(bf16_t, 8);
  } else {
    if (r16) MIXLORA_GO(float, 16); else MIXLORA_GO(float, 8);
  }
#undef MIXLORA_GO
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int64_t n = (int64_t)G * r * C;
  ReduceBatch rb{};
  rb.partial[0] = partials;
  rb.out[0] = out;
  rb.layout_qc[0] = layout_qc;
  hipLaunchKernelGGL(group_outer_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                     st, rb, G, r, C, nsplit, scale);
  return hipGetLastError();
}

// ---- bf16 MFMA version of the grouped outer-product sums ----------------------------------------
// out[g][q][c] partial = sum over a slice of group g's rows of smallT[q][row] * wide[src(row)][c].
// The contraction index is the row: first MFMA operand = wide (index = column, 8 rows per
// lane, read as 2-byte-pair loads whose even/odd halves feed two column-interleaved MFMA
// blocks), second operand = smallT (index = q, 8 consecutive rows = one 16-byte load from the
// transposed bf16 copy).  Rows outside the group are masked in the small operand.
constexpr int GOM_CB = 8;     // column blocks per wave: a lane reads 8 adjacent columns (16 bytes)

// A wave covers 256 columns: lane (l31, hi) reads, for each of its 8 rows, the 16-byte run of
// columns c0 + 8*l31 .. +7; element b of the run feeds MFMA block b, whose operand index i = l31
// therefore stands for column c0 + 8*i + b.  In the result, lane (q, hi) register 4*gg + m of
// block b is column c0 + 8*(8*gg + 4*hi + m) + b: for fixed (gg, m) the 8 blocks give 8
// consecutive columns, stored as two float4.
// Several sums of the same shape (same groups, same C, same gather mode) share one launch:
// blockIdx.y = job * G + group.
struct GomBatch {
  const bf16_t *smallT[GOM_MAX_JOBS];
  const bf16_t *wide[GOM_MAX_JOBS];
  float *partial[GOM_MAX_JOBS];
  float *out[GOM_MAX_JOBS];      // used when the rows are not split: the result is final
  int layout_qc[GOM_MAX_JOBS];
};

template <bool GATHER, int NQ>
__global__ __launch_bounds__(256, NQ == 1 ? 2 : 1) void group_outer_mfma_kernel(
    const int32_t *__restrict__ offs, const int32_t *__restrict__ pair_of_row, int k, int nrows,
    GomBatch batch, int G, int ldT, int r, int C, int nsplit, float scale) {
  const int job = blockIdx.y / G, g = blockIdx.y % G, sp = blockIdx.z;
  const bf16_t *__restrict__ smallT = batch.smallT[job];
  const bf16_t *__restrict__ wide = batch.wide[job];
  float *__restrict__ partial = batch.partial[job];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l31 = lane & 31, hi = lane >> 5;
  const int lo = offs[g], hi_ = offs[g + 1];
  const int base = lo & ~15;
  const int nsteps = hi_ > lo ? (hi_ - base + 15) >> 4 : 0;
  const int per = (nsteps + nsplit - 1) / nsplit;
  const int st_lo = sp * per;
  const int st_hi = st_lo + per < nsteps ? st_lo + per : nsteps;
  const int c0 = (blockIdx.x * 4 + wave) * (32 * GOM_CB);
  if (c0 >= C) return;   // whole wave out of range (no barriers in this kernel)
  int ccol = c0 + 8 * l31;
  if (ccol >= C) ccol = C - 8;
  f32x16_t acc[GOM_CB][NQ];
#pragma unroll
  for (int b = 0; b < GOM_CB; b++)
#pragma unroll
    for (int j = 0; j < NQ; j++)
#pragma unroll
      for (int i = 0; i < 16; i++) acc[b][j][i] = 0.f;

  for (int st = st_lo; st < st_hi; st++) {
    const int rbase = base + st * 16 + hi * 8;
    bf16x8_t bq[NQ];
#pragma unroll
    for (int j = 0; j < NQ; j++) {
      const int q = j * 32 + l31;
      const bf16x8_t ld = *reinterpret_cast<const bf16x8_t *>(smallT + (int64_t)(q < r ? q : 0) * ldT + rbase);
      bf16x8_t v;
#pragma unroll
      for (int p = 0; p < 8; p++) {
        const int row = rbase + p;
        v[p] = (q < r && row >= lo && row < hi_) ? ld[p] : (bf16_t)0.f;
      }
      bq[j] = v;
    }
    bf16x8_t wrow[8];
#pragma unroll
    for (int p = 0; p < 8; p++) {
      int row = rbase + p;
      row = row < nrows ? row : nrows - 1;
      const int64_t src = GATHER ? pair_of_row[row] / k : row;
      // rows read in place are read exactly once per step: a streaming (non-temporal) load keeps
      // them from displacing the gathered rows and partial results other kernels reuse (the
      // launch over the d_ff-wide operands measured 28 % faster); gathered token rows are read by
      // k groups and stay cached
      const bf16x8_t *wp = reinterpret_cast<const bf16x8_t *>(wide + src * C + ccol);
      wrow[p] = GATHER ? *wp : __builtin_nontemporal_load(wp);
    }
#pragma unroll
    for (int b = 0; b < GOM_CB; b++) {
      bf16x8_t fa;
#pragma unroll
      for (int p = 0; p < 8; p++) fa[p] = wrow[p][b];
#pragma unroll
      for (int j = 0; j < NQ; j++)
        acc[b][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, bq[j], acc[b][j], 0, 0, 0);
    }
  }
#pragma unroll
  for (int j = 0; j < NQ; j++) {
    const int q = j * 32 + l31;
    if (q < r) {
      if (nsplit == 1) {
        // rows not split: scale and write the result itself, [g][q][c] or [g][c][q]
        float *out = batch.out[job];
        const bool qc = batch.layout_qc[job] != 0;
#pragma unroll
        for (int gg = 0; gg < 4; gg++)
#pragma unroll
          for (int m = 0; m < 4; m++) {
            const int c = c0 + 8 * (8 * gg + 4 * hi + m);
            if (c + 7 < C) {
              if (qc) {
                float *o = out + ((int64_t)g * r + q) * C + c;
                *reinterpret_cast<float4 *>(o) =
                    make_float4(scale * acc[0][j][gg * 4 + m], scale * acc[1][j][gg * 4 + m],
                                scale * acc[2][j][gg * 4 + m], scale * acc[3][j][gg * 4 + m]);
                *reinterpret_cast<float4 *>(o + 4) =
                    make_float4(scale * acc[4][j][gg * 4 + m], scale * acc[5][j][gg * 4 + m],
                                scale * acc[6][j][gg * 4 + m], scale * acc[7][j][gg * 4 + m]);
              } else {
                float *o = out + ((int64_t)g * C + c) * r + q;
#pragma unroll
                for (int b = 0; b < GOM_CB; b++) o[(int64_t)b * r] = scale * acc[b][j][gg * 4 + m];
              }
            }
          }
        continue;
      }
      float *o = partial + (((int64_t)sp * G + g) * r + q) * C;
#pragma unroll
      for (int gg = 0; gg < 4; gg++)
#pragma unroll
        for (int m = 0; m < 4; m++) {
          const int c = c0 + 8 * (8 * gg + 4 * hi + m);
          if (c + 7 < C) {
            *reinterpret_cast<float4 *>(o + c) = make_float4(acc[0][j][gg * 4 + m], acc[1][j][gg * 4 + m],
                                                             acc[2][j][gg * 4 + m], acc[3][j][gg * 4 + m]);
            *reinterpret_cast<float4 *>(o + c + 4) = make_float4(acc[4][j][gg * 4 + m], acc[5][j][gg * 4 + m],
                                                                 acc[6][j][gg * 4 + m], acc[7][j][gg * 4 + m]);
          }
        }
    }
  }
}

static int gom_splits(int G, int C, int njobs = 1) {
  // one resident round: 256 CUs x 2 workgroups of 4 waves (the kernel runs 2 waves per SIMD)
  const int col_groups = (C + 1023) / 1024;
  int s = 512 / (col_groups * G * njobs);
  if (s < 1) s = 1;
  if (s > 8 && G > 1) s = 8;     // partial sums cost HBM traffic: nsplit * G * r * C floats
  if (s > 32) s = 32;
  return s;
}

size_t group_outer_mfma_partial_floats(int G, int r, int C) {
  return (size_t)gom_splits(G, C) * G * r * C;
}

hipError_t launch_group_outer_mfma(const int32_t *offs, int G, int nrows,
                                   const int32_t *pair_of_row, int k, const GomJob *jobs, int njobs,
                                   int ldT, int r, int C, float scale, float *partials,
                                   size_t partial_floats, hipStream_t st) {
  if (njobs < 1 || njobs > GOM_MAX_JOBS) return hipErrorInvalidValue;
  const int nsplit = gom_splits(G, C, njobs);
  const size_t per_job = (size_t)nsplit * G * r * C;
  if (per_job * njobs > partial_floats) return hipErrorInvalidValue;
  GomBatch b{};
  ReduceBatch rb{};
  for (int i = 0; i < njobs; i++) {
    b.smallT[i] = (const bf16_t *)jobs[i].smallT;
    b.wide[i] = (const bf16_t *)jobs[i].wide;
    b.partial[i] = partials + per_job * i;
    b.out[i] = jobs[i].out;
    b.layout_qc[i] = jobs[i].layout_qc;
    rb.partial[i] = b.partial[i];
    rb.out[i] = jobs[i].out;
    rb.layout_qc[i] = jobs[i].layout_qc;
  }
  const dim3 grid((C + 1023) / 1024, G * njobs, nsplit), block(256);
#define MIXLORA_GOM(GA_, NQ_)                                                                   \
  hipLaunchKernelGGL((group_outer_mfma_kernel<GA_, NQ_>), grid, block, 0, st, offs, pair_of_row, \
                     k, nrows, b, G, ldT, r, C, nsplit, scale)
  if (pair_of_row) { if (r <= 32) MIXLORA_GOM(true, 1); else MIXLORA_GOM(true, 2); }
  else { if (r <= 32) MIXLORA_GOM(false, 1); else MIXLORA_GOM(false, 2); }
#undef MIXLORA_GOM
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || nsplit == 1) return e;   // unsplit rows: the kernel wrote the results
  const int64_t n = (int64_t)G * r * C;
  hipLaunchKernelGGL(group_outer_reduce_kernel, dim3((unsigned)((n + 255) / 256), njobs), dim3(256),
                     0, st, rb, G, r, C, nsplit, scale);
  return hipGetLastError();
}

// Transposed bf16 row factors for the MFMA gradient sums, several factors per launch:
//   outT[q, row] = (w_row or 1) * src[(by_token ? t(row) : row), e(row)*r + q]
struct GatherBatch {
  GatherJob job[GATHER_MAX_JOBS];
};

__global__ void gather_small_T_kernel(PairCtx pc, GatherBatch batch, int ldT) {
  const GatherJob &J = batch.job[blockIdx.y];
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int nP = pc.T * pc.k;
  if (i >= (int64_t)nP * pc.r) return;
  const int q = (int)(i / nP), row = (int)(i % nP);
  const int p = pc.pair_of_row[row];
  const int e = pc.idx[p];
  const int64_t srow = J.by_token ? p / pc.k : row;
  const float w = J.weighted ? pc.w[p] : 1.f;
  reinterpret_cast<bf16_t *>(J.outT)[(int64_t)q * ldT + row] =
      (bf16_t)(w * J.src[srow * (pc.N * pc.r) + e * pc.r + q]);
}

hipError_t launch_gather_small_T(const PairCtx &pc, const GatherJob *jobs, int njobs, int ldT,
                                 hipStream_t st) {
  if (njobs < 1 || njobs > GATHER_MAX_JOBS) return hipErrorInvalidValue;
  GatherBatch b;
  for (int i = 0; i < GATHER_MAX_JOBS; i++) b.job[i] = jobs[i < njobs ? i : 0];
  const int64_t n = (int64_t)pc.T * pc.k * pc.r;
  hipLaunchKernelGGL(gather_small_T_kernel, dim3((unsigned)((n + 255) / 256), njobs), dim3(256), 0,
                     st, pc, b, ldT);
  return hipGetLastError();
}

// outT[q][row] (bf16) = src[row][q] (fp32, [rows, r])
__global__ void f32_to_bf16T_kernel(const float *__restrict__ src, int rows, int r,
                                    bf16_t *__restrict__ outT, int ldT) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)rows * r) return;
  const int q = (int)(i / rows), row = (int)(i % rows);
  outT[(int64_t)q * ldT + row] = (bf16_t)src[(int64_t)row * r + q];
}

hipError_t launch_f32_to_bf16T(const float *src, int rows, int r, void *outT, int ldT,
                               hipStream_t st) {
  const int64_t n = (int64_t)rows * r;
  hipLaunchKernelGGL(f32_to_bf16T_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, src,
                     rows, r, (bf16_t *)outT, ldT);
  return hipGetLastError();
}

// ---- router backward -------------------------------------------------------------------------
// One wavefront per token.  dw_j = <dy_t, o_pair> is assembled from the column-tile partials of
// <H[t], a_row> plus the low-rank part  s <B_down[e]^T dy_t, A_down[e] a_row>  (lanes split the
// terms, a butterfly adds them).  Then, with w_j = p_j / sum_kept p (Norm of Algorithm 1):
// dp_j = (dw_j - sum_i w_i dw_i) / sum_kept p on the kept experts, plus the auxiliary term
// d_aux * a * N * F_e / T  on every expert (Eq. 8-9; F is piecewise constant; evaluated as its
// deviation from 1/N, see below), and
// dz = p * (dp - <p, dp>) through the softmax of Eq. 7 (lane e holds expert e).  With several
// adapters p is zero outside the token's adapter, so dz is too; T and the upstream gradient of
// the auxiliary loss are those of the token's adapter.
__device__ __forceinline__ float rb_wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

template <typename E>
__global__ __launch_bounds__(256) void router_bwd_kernel(
    PairCtx pc, const float *__restrict__ probs, const float *__restrict__ dw_part,
    int n_col_tiles, const float *__restrict__ VB_all, const float *__restrict__ Q_all,
    const float *__restrict__ F, float s, AuxUpstream d_aux, float aux_coeff,
    float *__restrict__ dw_ws, float *__restrict__ dz, E *__restrict__ S, int lds_, int col0,
    int ncols, int Nl, const int32_t *__restrict__ token_model,
    const int32_t *__restrict__ model_tokens, bf16_t *__restrict__ dzT, int ldTz,
    int s_by_first_pair) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= pc.T) return;   // whole wave leaves together
  const int N = pc.N, k = pc.k, r = pc.r, R = N * r;
  float my_dw = 0.f, my_w = 0.f, my_p = 0.f;   // lane j < k: slot j of the token
  int my_e = -1;
  for (int j = 0; j < k; j++) {
    const int p = t * k + j;
    const int row = pc.row_of_pair[p];
    const int e = pc.idx[p];
    float part = 0.f;
    for (int ct = lane; ct < n_col_tiles; ct += 64) part += dw_part[(int64_t)row * n_col_tiles + ct];
    float lr = 0.f;
    for (int q = lane; q < r; q += 64)
      lr = fmaf(VB_all[(int64_t)t * R + e * r + q], Q_all[(int64_t)row * R + e * r + q], lr);
    const float dwj = rb_wave_sum(part + s * lr);
    if (lane == j) {
      my_dw = dwj;
      my_e = e;
      my_w = pc.w[p];
      my_p = probs[(int64_t)t * N + e];
      dw_ws[p] = dwj;
    }
  }
  const float wdw = rb_wave_sum(my_w * my_dw);
  const float ssum = rb_wave_sum(my_p);
  // auxiliary term of the token's adapter: statistics over that adapter's own tokens
  const int m = __builtin_amdgcn_readfirstlane(token_model ? token_model[t] : 0);   // wave-uniform
  const float auxg = d_aux.v[m] * aux_coeff * (float)Nl / (float)model_tokens[m];
  // The softmax Jacobian ignores a constant added to dp, so F_e - 1/Nl stands in for F_e: with
  // nearly balanced loads (what the loss drives towards) p * (F_e - <p, F>) would otherwise be a
  // difference of nearly equal numbers.  F_e * (k * tokens) is an integer in both modes of Eq. 9
  // (k times the first-slot count, or the kept count), recovered exactly by rounding, so the
  // deviation (num_e * Nl - k * tokens) / (k * tokens * Nl) has an exact numerator.
  float dp = 0.f;
  if (lane < N) {
    const float kt = (float)k * (float)model_tokens[m];
    const int64_t num = (int64_t)rintf(F[lane] * kt);
    const int64_t dev = num * Nl - (int64_t)k * model_tokens[m];
    dp = auxg * ((float)dev / (kt * (float)Nl));
  }
  for (int j = 0; j < k; j++) {
    const int ej = __shfl(my_e, j, 64);
    const float dwj = __shfl(my_dw, j, 64);
    if (ej == lane) dp += (dwj - wdw) / ssum;
  }
  const float pe = lane < N ? probs[(int64_t)t * N + lane] : 0.f;
  const float dot = rb_wave_sum(pe * dp);
  const float v = pe * (dp - dot);   // 0 on lanes >= N
  if (lane < N) {
    dz[(int64_t)t * N + lane] = v;
    // transposed bf16 copy: the row factor of the dW_router outer-product sum
    if (dzT) dzT[(int64_t)lane * ldTz + t] = (bf16_t)v;
  }
  // row of the K-extension operand: the token's, or (operand with one row per grouped pair row)
  // the row of the token's first slot, whose other rows keep zeros in these columns
  const int64_t srow = s_by_first_pair ? pc.row_of_pair[t * pc.k] : t;
  for (int e = lane; e < ncols; e += 64)
    S[srow * lds_ + col0 + e] = from_f32<E>(e < N ? v : 0.f);
}

hipError_t launch_router_bwd(int dtype, const PairCtx &pc, const float *probs, const float *dw_part,
                             int n_col_tiles, const float *VB_all, const float *Q_all,
                             const float *F, float s, const AuxUpstream &d_aux, float aux_coeff,
                             float *dw_ws, float *dz, void *S, int lds_, int col0, int ncols,
                             int Nl, const int32_t *token_model, const int32_t *model_tokens,
                             void *dzT, int ldTz, hipStream_t st, int s_by_first_pair) {
  const dim3 grid((pc.T + 3) / 4), block(256);
  if (dtype == MIXLORA_BF16)
    hipLaunchKernelGGL(router_bwd_kernel<bf16_t>, grid, block, 0, st, pc, probs, dw_part,
                       n_col_tiles, VB_all, Q_all, F, s, d_aux, aux_coeff, dw_ws, dz, (bf16_t *)S,
                       lds_, col0, ncols, Nl, token_model, model_tokens, (bf16_t *)dzT, ldTz,
                       s_by_first_pair);
  else
    hipLaunchKernelGGL(router_bwd_kernel<float>, grid, block, 0, st, pc, probs, dw_part,
                       n_col_tiles, VB_all, Q_all, F, s, d_aux, aux_coeff, dw_ws, dz, (float *)S,
                       lds_, col0, ncols, Nl, token_model, model_tokens, (bf16_t *)dzT, ldTz,
                       s_by_first_pair);
  return hipGetLastError();
}

}  // namespace mixlora
