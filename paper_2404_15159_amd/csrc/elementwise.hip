// Element-wise and rank-r kernels of the MixLoRA block.
//
// Pairs (token, slot) are processed in expert-grouped row order: every row tile belongs to one
// expert, so the tile's threads keep that expert's LoRA B columns in registers while they walk
// the tile's rows (Algorithm 1 lines 11-13: add the LoRA deltas to the shared gate/up
// projections, then SiLU * up).
#include "common.h"
#include "relayout_body.h"

namespace mixlora {

// ---- two adjacent elements ------------------------------------------------------------------
__device__ __forceinline__ float2 load2(const float *p) { return *reinterpret_cast<const float2 *>(p); }
__device__ __forceinline__ float2 load2(const bf16_t *p) {
  typedef bf16_t bf16x2_t __attribute__((ext_vector_type(2)));
  const bf16x2_t v = *reinterpret_cast<const bf16x2_t *>(p);
  return make_float2((float)v[0], (float)v[1]);
}
__device__ __forceinline__ void store2(float *p, float a, float b) {
  *reinterpret_cast<float2 *>(p) = make_float2(a, b);
}
__device__ __forceinline__ void store2(bf16_t *p, float a, float b) {
  typedef bf16_t bf16x2_t __attribute__((ext_vector_type(2)));
  bf16x2_t v;
  v[0] = (bf16_t)a;
  v[1] = (bf16_t)b;
  *reinterpret_cast<bf16x2_t *>(p) = v;
}

// Row tile `b` (of RM rows) in the grouped order: which expert, first row, number of rows.
__device__ __forceinline__ bool tile_rows(const int32_t *offs, int N, int RM, int b, int &e,
                                          int &row0, int &rows) {
  for (e = 0; e < N; e++) {
    const int lo = offs[e], hi = offs[e + 1];
    const int nt = (hi - lo + RM - 1) / RM;
    if (b < nt) {
      row0 = lo + b * RM;
      rows = hi - row0 < RM ? hi - row0 : RM;
      return true;
    }
    b -= nt;
  }
  return false;
}

constexpr int SW_COLS = 512;   // columns per block: 256 threads x 2 adjacent columns
constexpr int SW_RMAX = 64;    // largest LoRA rank

int swiglu_col_tiles(int f) { return (f + SW_COLS - 1) / SW_COLS; }

__device__ __forceinline__ float sigmoidf_(float v) { return 1.f / (1.f + expf(-v)); }

// a_grp[row, c] = SiLU(g) * u with  g = G[t,c] + s * <B_gate[e,c,:], Pg[t,e,:]>  (same for u)
template <typename E, int RM>
__global__ __launch_bounds__(256) void swiglu_fwd_kernel(
    PairCtx pc, int f, float s, const E *__restrict__ G, const E *__restrict__ U,
    const float *__restrict__ Pg_all, const float *__restrict__ Pu_all,
    const E *__restrict__ B_gate, const E *__restrict__ B_up, E *__restrict__ a_grp) {
  __shared__ float Pg_s[RM][SW_RMAX];
  __shared__ float Pu_s[RM][SW_RMAX];
  __shared__ int tok_s[RM];
  int e, row0, rows;
  if (!tile_rows(pc.offs, pc.N, RM, blockIdx.x, e, row0, rows)) return;
  const int r = pc.r, R = pc.N * pc.r;
  for (int i = threadIdx.x; i < RM * r; i += 256) {
    const int rr = i / r, q = i % r;
    float vg = 0.f, vu = 0.f;
    if (rr < rows) {
      const int t = pc.pair_of_row[row0 + rr] / pc.k;
      vg = Pg_all[(int64_t)t * R + e * r + q];
      vu = Pu_all[(int64_t)t * R + e * r + q];
      if (q == 0) tok_s[rr] = t;
    }
    Pg_s[rr][q] = vg;
    Pu_s[rr][q] = vu;
  }
  __syncthreads();
  const int c = blockIdx.y * SW_COLS + threadIdx.x * 2;
  if (c >= f) return;
  float ag[RM][2], au[RM][2];
#pragma unroll
  for (int i = 0; i < RM; i++) ag[i][0] = ag[i][1] = au[i][0] = au[i][1] = 0.f;
  const E *bg = B_gate + ((int64_t)e * f + c) * r;
  const E *bu = B_up + ((int64_t)e * f + c) * r;
  for (int q0 = 0; q0 < r; q0 += 8) {
    Vec8<E> g0, g1, u0, u1;
    g0.load(bg + q0);
    g1.load(bg + r + q0);
    u0.load(bu + q0);
    u1.load(bu + r + q0);
#pragma unroll
    for (int q = 0; q < 8; q++) {
      const float b0 = g0.get(q), b1 = g1.get(q), c0 = u0.get(q), c1 = u1.get(q);
#pragma unroll
      for (int i = 0; i < RM; i++) {
        const float pg = Pg_s[i][q0 + q], pu = Pu_s[i][q0 + q];
        ag[i][0] = fmaf(b0, pg, ag[i][0]);
        ag[i][1] = fmaf(b1, pg, ag[i][1]);
        au[i][0] = fmaf(c0, pu, au[i][0]);
        au[i][1] = fmaf(c1, pu, au[i][1]);
      }
    }
  }
#pragma unroll
  for (int i = 0; i < RM; i++) {
    if (i < rows) {
      const int64_t t = tok_s[i];
      const float2 gv = load2(G + t * f + c), uv = load2(U + t * f + c);
      const float g0 = gv.x + s * ag[i][0], g1 = gv.y + s * ag[i][1];
      const float u0 = uv.x + s * au[i][0], u1 = uv.y + s * au[i][1];
      store2(a_grp + (int64_t)(row0 + i) * f + c, g0 * sigmoidf_(g0) * u0, g1 * sigmoidf_(g1) * u1);
    }
  }
}

// Backward of the tile above.  With H[t] = W_down^T dy[t] (shared by the token's pairs, since
// the frozen down projection is linear) and Vw[row] = w_row * B_down[e]^T dy[t]:
//   da = w_row * H[t] + s * A_down[e]^T Vw[row];   dg = da * u * sig(g) * (1 + g (1 - sig(g)));
//   du = da * g * sig(g);   dw_part[row, column tile] = sum over the tile's columns of H * a.
template <typename E, int RM>
__global__ __launch_bounds__(256) void swiglu_bwd_kernel(
    PairCtx pc, int f, float s, const E *__restrict__ G, const E *__restrict__ U,
    const float *__restrict__ Pg_all, const float *__restrict__ Pu_all,
    const E *__restrict__ B_gate, const E *__restrict__ B_up, const E *__restrict__ H,
    const float *__restrict__ VB_all, const E *__restrict__ A_down, E *__restrict__ dg_grp,
    E *__restrict__ du_grp, float *__restrict__ dw_part, int n_col_tiles) {
  __shared__ float Pg_s[RM][SW_RMAX];
  __shared__ float Pu_s[RM][SW_RMAX];
  __shared__ float Vw_s[RM][SW_RMAX];
  __shared__ int tok_s[RM];
  __shared__ float wrow_s[RM];
  __shared__ float red[4][RM];
  int e, row0, rows;
  if (!tile_rows(pc.offs, pc.N, RM, blockIdx.x, e, row0, rows)) return;
  const int r = pc.r, R = pc.N * pc.r;
  for (int i = threadIdx.x; i < RM * r; i += 256) {
    const int rr = i / r, q = i % r;
    float vg = 0.f, vu = 0.f, vv = 0.f;
    if (rr < rows) {
      const int p = pc.pair_of_row[row0 + rr];
      const int t = p / pc.k;
      const float w = pc.w[p];
      vg = Pg_all[(int64_t)t * R + e * r + q];
      vu = Pu_all[(int64_t)t * R + e * r + q];
      vv = w * VB_all[(int64_t)t * R + e * r + q];
      if (q == 0) { tok_s[rr] = t; wrow_s[rr] = w; }
    }
    Pg_s[rr][q] = vg;
    Pu_s[rr][q] = vu;
    Vw_s[rr][q] = vv;
  }
  __syncthreads();
  const int c = blockIdx.y * SW_COLS + threadIdx.x * 2;
  const bool active = c < f;
  float ag[RM][2], au[RM][2], ad[RM][2];
#pragma unroll
  for (int i = 0; i < RM; i++)
    ag[i][0] = ag[i][1] = au[i][0] = au[i][1] = ad[i][0] = ad[i][1] = 0.f;
  if (active) {
    const E *bg = B_gate + ((int64_t)e * f + c) * r;
    const E *bu = B_up + ((int64_t)e * f + c) * r;
    const E *adn = A_down + (int64_t)e * r * f + c;
    for (int q0 = 0; q0 < r; q0 += 8) {
      Vec8<E> g0, g1, u0, u1;
      g0.load(bg + q0);
      g1.load(bg + r + q0);
      u0.load(bu + q0);
      u1.load(bu + r + q0);
#pragma unroll
      for (int q = 0; q < 8; q++) {
        const float b0 = g0.get(q), b1 = g1.get(q), c0 = u0.get(q), c1 = u1.get(q);
        const float2 av = load2(adn + (int64_t)(q0 + q) * f);
#pragma unroll
        for (int i = 0; i < RM; i++) {
          const float pg = Pg_s[i][q0 + q], pu = Pu_s[i][q0 + q], vw = Vw_s[i][q0 + q];
          ag[i][0] = fmaf(b0, pg, ag[i][0]);
          ag[i][1] = fmaf(b1, pg, ag[i][1]);
          au[i][0] = fmaf(c0, pu, au[i][0]);
          au[i][1] = fmaf(c1, pu, au[i][1]);
          ad[i][0] = fmaf(av.x, vw, ad[i][0]);
          ad[i][1] = fmaf(av.y, vw, ad[i][1]);
        }
      }
    }
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < RM; i++) {
    float part = 0.f;
    if (active && i < rows) {
      const int64_t t = tok_s[i];
      const float w = wrow_s[i];
      const float2 gv = load2(G + t * f + c), uv = load2(U + t * f + c), hv = load2(H + t * f + c);
      const float g0 = gv.x + s * ag[i][0], g1 = gv.y + s * ag[i][1];
      const float u0 = uv.x + s * au[i][0], u1 = uv.y + s * au[i][1];
      const float s0 = sigmoidf_(g0), s1 = sigmoidf_(g1);
      const float da0 = w * hv.x + s * ad[i][0], da1 = w * hv.y + s * ad[i][1];
      part = hv.x * (g0 * s0 * u0) + hv.y * (g1 * s1 * u1);
      store2(dg_grp + (int64_t)(row0 + i) * f + c, da0 * u0 * s0 * (1.f + g0 * (1.f - s0)),
             da1 * u1 * s1 * (1.f + g1 * (1.f - s1)));
      store2(du_grp + (int64_t)(row0 + i) * f + c, da0 * g0 * s0, da1 * g1 * s1);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) part += __shfl_xor(part, o, 64);
    if (lane == 0) red[wave][i] = part;
  }
  __syncthreads();
  if (threadIdx.x < rows)
    dw_part[(int64_t)(row0 + threadIdx.x) * n_col_tiles + blockIdx.y] =
        (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
}

constexpr int FWD_RM = 16, BWD_RM = 8;

hipError_t launch_swiglu_fwd(int dtype, const PairCtx &pc, int f, float s, const void *G,
                             const void *U, const float *Pg_all, const float *Pu_all,
                             const void *B_gate, const void *B_up, void *a_grp,
                             hipStream_t st) {
  const int nP = pc.T * pc.k;
  const dim3 grid((nP + FWD_RM - 1) / FWD_RM + pc.N, swiglu_col_tiles(f)), block(256);
  if (dtype == MIXLORA_BF16)
    hipLaunchKernelGGL((swiglu_fwd_kernel<bf16_t, FWD_RM>), grid, block, 0, st, pc, f, s,
                       (const bf16_t *)G, (const bf16_t *)U, Pg_all, Pu_all,
                       (const bf16_t *)B_gate, (const bf16_t *)B_up, (bf16_t *)a_grp);
  else
    hipLaunchKernelGGL((swiglu_fwd_kernel<float, FWD_RM>), grid, block, 0, st, pc, f, s,
                       (const float *)G, (const float *)U, Pg_all, Pu_all, (const float *)B_gate,
                       (const float *)B_up, (float *)a_grp);
  return hipGetLastError();
}

hipError_t launch_swiglu_bwd(int dtype, const PairCtx &pc, int f, float s, const void *G,
                             const void *U, const float *Pg_all, const float *Pu_all,
                             const void *B_gate, const void *B_up, const void *H,
                             const float *VB_all, const void *A_down, void *dg_grp,
                             void *du_grp, float *dw_part, int n_col_tiles, hipStream_t st) {
  const int nP = pc.T * pc.k;
  const dim3 grid((nP + BWD_RM - 1) / BWD_RM + pc.N, swiglu_col_tiles(f)), block(256);
  if (dtype == MIXLORA_BF16)
    hipLaunchKernelGGL((swiglu_bwd_kernel<bf16_t, BWD_RM>), grid, block, 0, st, pc, f, s,
                       (const bf16_t *)G, (const bf16_t *)U, Pg_all, Pu_all,
                       (const bf16_t *)B_gate, (const bf16_t *)B_up, (const bf16_t *)H, VB_all,
                       (const bf16_t *)A_down, (bf16_t *)dg_grp, (bf16_t *)du_grp, dw_part,
                       n_col_tiles);
  else
    hipLaunchKernelGGL((swiglu_bwd_kernel<float, BWD_RM>), grid, block, 0, st, pc, f, s,
                       (const float *)G, (const float *)U, Pg_all, Pu_all, (const float *)B_gate,
                       (const float *)B_up, (const float *)H, VB_all, (const float *)A_down,
                       (float *)dg_grp, (float *)du_grp, dw_part, n_col_tiles);
  return hipGetLastError();
}

// ---- out[t, :] = sum_j (w[t,j] or 1) * in_grp[row_of_pair[t,j], :] ------------------------------
// Gather form of the weighted combine (Eq. 6; Algorithm 1 line 15): each output row is written
// once, by one thread per 8 columns, slots added in ascending order (deterministic).
template <typename E>
__device__ __forceinline__ void pair_combine_body(const PairCtx &pc, int width,
                                                  const E *__restrict__ in_grp,
                                                  E *__restrict__ out, int weighted, int t, int by) {
  // a thread owns two 8-column chunks, 2048 columns apart: 2k independent loads in flight
  const int c0 = (by * 512 + threadIdx.x) * 8;
  const int c1 = c0 + 2048;
  if (c0 >= width) return;
  const bool two = c1 < width;
  float acc0[8] = {0, 0, 0, 0, 0, 0, 0, 0}, acc1[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int j = 0; j < pc.k; j++) {
    const int p = t * pc.k + j;
    const float w = weighted ? pc.w[p] : 1.f;
    const E *src = in_grp + (int64_t)pc.row_of_pair[p] * width;
    Vec8<E> v0, v1;
    v0.load(src + c0);
    if (two) v1.load(src + c1);
#pragma unroll
    for (int i = 0; i < 8; i++) acc0[i] = fmaf(w, v0.get(i), acc0[i]);
    if (two) {
#pragma unroll
      for (int i = 0; i < 8; i++) acc1[i] = fmaf(w, v1.get(i), acc1[i]);
    }
  }
  Vec8<E> o;
#pragma unroll
  for (int i = 0; i < 8; i++) o.set(i, acc0[i]);
  o.store(out + (int64_t)t * width + c0);
  if (two) {
#pragma unroll
    for (int i = 0; i < 8; i++) o.set(i, acc1[i]);
    o.store(out + (int64_t)t * width + c1);
  }
}

template <typename E>
__global__ __launch_bounds__(256) void pair_combine_kernel(PairCtx pc, int width,
                                                           const E *__restrict__ in_grp0,
                                                           E *__restrict__ out0,
                                                           const E *__restrict__ in_grp1,
                                                           E *__restrict__ out1, int weighted) {
  // blockIdx.z picks one of two combines of the same shape that share the launch
  pair_combine_body<E>(pc, width, blockIdx.z ? in_grp1 : in_grp0, blockIdx.z ? out1 : out0, weighted,
                       blockIdx.x, blockIdx.y);
}

// Few tokens: the weighted combine and, as one more slice of workgroups (blockIdx.y == ny), the sum
// over column splits of the per-pair rank-r partial products of a token's k pairs - what
// reduce_rank_parts_kernel (csrc/fused.hip) does for one bank, weighted, per token, with the same
// order of additions.  Needs k * r <= 256.
__global__ __launch_bounds__(256) void pair_combine_reduce_kernel(
    PairCtx pc, int width, const bf16_t *__restrict__ in_grp, bf16_t *__restrict__ out, int ny,
    const float *__restrict__ part, int nsplit, float *__restrict__ dense,
    bf16_t *__restrict__ sparse, int ld_sparse) {
  const int t = blockIdx.x;
  if ((int)blockIdx.y < ny) {
    pair_combine_body<bf16_t>(pc, width, in_grp, out, 1, t, blockIdx.y);
    return;
  }
  const int r = pc.r, i = threadIdx.x;
  if (i >= pc.k * r) return;
  const int pair = t * pc.k + i / r, q = i % r, row = pc.row_of_pair[pair];
  const int64_t n = (int64_t)pc.T * pc.k * r, at = (int64_t)row * r + q;
  float acc = 0.f;
  int sp = 0;
  for (; sp + 8 <= nsplit; sp += 8) {   // eight loads in flight; additions in split order
    float a[8];
#pragma unroll
    for (int u = 0; u < 8; u++) a[u] = part[(sp + u) * n + at];
#pragma unroll
    for (int u = 0; u < 8; u++) acc += a[u];
  }
  for (; sp < nsplit; sp++) acc += part[sp * n + at];
  const int e = pc.idx[pair], R = pc.N * r;
  dense[(int64_t)row * R + e * r + q] = acc;
  sparse[(int64_t)t * ld_sparse + e * r + q] = (bf16_t)(pc.w[pair] * acc);
}

hipError_t launch_pair_combine_reduce(const PairCtx &pc, int width, const void *in_grp, void *out,
                                      const float *part, int nsplit, float *dense, void *sparse,
                                      int ld_sparse, hipStream_t st) {
  if (pc.k * pc.r > 256) return hipErrorInvalidValue;
  const int ny = (width / 8 + 511) / 512;
  hipLaunchKernelGGL(pair_combine_reduce_kernel, dim3(pc.T, ny + 1), dim3(256), 0, st, pc, width,
                     (const bf16_t *)in_grp, (bf16_t *)out, ny, part, nsplit, dense,
                     (bf16_t *)sparse, ld_sparse);
  return hipGetLastError();
}

hipError_t launch_pair_combine2(int dtype, const PairCtx &pc, int width, const void *in_grp0,
                                void *out0, const void *in_grp1, void *out1, int weighted,
                                hipStream_t st) {
  const dim3 grid(pc.T, (width / 8 + 511) / 512, in_grp1 ? 2 : 1), block(256);
  if (dtype == MIXLORA_BF16)
    hipLaunchKernelGGL(pair_combine_kernel<bf16_t>, grid, block, 0, st, pc, width,
                       (const bf16_t *)in_grp0, (bf16_t *)out0, (const bf16_t *)in_grp1,
                       (bf16_t *)out1, weighted);
  else
    hipLaunchKernelGGL(pair_combine_kernel<float>, grid, block, 0, st, pc, width,
                       (const float *)in_grp0, (float *)out0, (const float *)in_grp1,
                       (float *)out1, weighted);
  return hipGetLastError();
}

hipError_t launch_pair_combine(int dtype, const PairCtx &pc, int width, const void *in_grp,
                               void *out, int weighted, hipStream_t st) {
  return launch_pair_combine2(dtype, pc, width, in_grp, out, nullptr, nullptr, weighted, st);
}

// ---- dst[row, :] = src[token of grouped row, :] : the routed tokens' rows in expert-grouped order
// (the per-expert input slices of the unshared schedule, Section 3.3 / Figure 3a)
template <typename E>
__global__ __launch_bounds__(256) void gather_rows_kernel(PairCtx pc, int width,
                                                          const E *__restrict__ src,
                                                          E *__restrict__ dst) {
  const int row = blockIdx.x;
  const int c = (blockIdx.y * 256 + threadIdx.x) * 8;
  if (c >= width) return;
  const int t = pc.pair_of_row[row] / pc.k;
  Vec8<E> v;
  v.load(src + (int64_t)t * width + c);
  v.store(dst + (int64_t)row * width + c);
}

hipError_t launch_gather_rows(int dtype, const PairCtx &pc, int width, const void *src, void *dst,
                              hipStream_t st) {
  const dim3 grid(pc.T * pc.k, (width / 8 + 255) / 256), block(256);
  if (dtype == MIXLORA_BF16)
    hipLaunchKernelGGL(gather_rows_kernel<bf16_t>, grid, block, 0, st, pc, width, (const bf16_t *)src,
                       (bf16_t *)dst);
  else
    hipLaunchKernelGGL(gather_rows_kernel<float>, grid, block, 0, st, pc, width, (const float *)src,
                       (float *)dst);
  return hipGetLastError();
}

// dst[t, col0 + e*r + q] = (w[t,j] or 1) * src[row_j, (src_dense ? e*r : 0) + q] when expert e is
// slot j of token t, else 0.  Builds the block-sparse low-rank operand of a K-extension.
// blockIdx.y = b handles a further source src + b*src_stride into columns col0 + b*N*r.
template <typename E>
__global__ void scatter_blocks_kernel(PairCtx pc, const float *__restrict__ src0,
                                      int64_t src_stride, int lds_, int src_dense, int weighted,
                                      E *__restrict__ dst, int ldd, int col00) {
  const int R = pc.N * pc.r;
  const float *__restrict__ src = src0 + blockIdx.y * src_stride;
  const int col0 = col00 + blockIdx.y * R;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)pc.T * R) return;
  const int t = (int)(i / R), er = (int)(i % R);
  const int e = er / pc.r, q = er % pc.r;
  float v = 0.f;
  for (int j = 0; j < pc.k; j++) {
    const int p = t * pc.k + j;
    if (pc.idx[p] == e) {
      const float w = weighted ? pc.w[p] : 1.f;
      v = w * src[(int64_t)pc.row_of_pair[p] * lds_ + (src_dense ? e * pc.r : 0) + q];
    }
  }
  dst[(int64_t)t * ldd + col0 + er] = from_f32<E>(v);
}

hipError_t launch_scatter_blocks(int dtype, const PairCtx &pc, const float *src, int64_t src_stride,
                                 int nsrc, int lds_, int src_dense, int weighted, void *dst,
                                 int ldd, int col0, hipStream_t st) {
  const int64_t n = (int64_t)pc.T * pc.N * pc.r;
  const dim3 grid((unsigned)((n + 255) / 256), nsrc), block(256);
  if (dtype == MIXLORA_BF16)
    hipLaunchKernelGGL(scatter_blocks_kernel<bf16_t>, grid, block, 0, st, pc, src, src_stride, lds_,
                       src_dense, weighted, (bf16_t *)dst, ldd, col0);
  else
    hipLaunchKernelGGL(scatter_blocks_kernel<float>, grid, block, 0, st, pc, src, src_stride, lds_,
                       src_dense, weighted, (float *)dst, ldd, col0);
  return hipGetLastError();
}

// small_grp[row, q] = (w_row or 1) * src[(by_token ? t(row) : row), e(row)*r + q]
__global__ void gather_small_kernel(PairCtx pc, const float *__restrict__ src, int by_token,
                                    int weighted, float *__restrict__ small_grp) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int nP = pc.T * pc.k;
  if (i >= (int64_t)nP * pc.r) return;
  const int row = (int)(i / pc.r), q = (int)(i % pc.r);
  const int p = pc.pair_of_row[row];
  const int e = pc.idx[p];
  const int64_t srow = by_token ? p / pc.k : row;
  const float w = weighted ? pc.w[p] : 1.f;
  small_grp[i] = w * src[srow * (pc.N * pc.r) + e * pc.r + q];
}

hipError_t launch_gather_small(const PairCtx &pc, const float *src, int by_token, int weighted,
                               float *small_grp, hipStream_t st) {
  const int64_t n = (int64_t)pc.T * pc.k * pc.r;
  hipLaunchKernelGGL(gather_small_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, pc,
                     src, by_token, weighted, small_grp);
  return hipGetLastError();
}

// Rank-r update of a GEMM result (Eq. 1):  io[t, c] += s * sum_q P[t, q] * Wt[c, q]
// io [T, C] storage dtype (in place), P [T, r] float32, Wt [C, r] storage dtype.  A thread owns 8
// columns of LRA_ROWS consecutive rows; its 8 rows of Wt stay in registers 16 rank entries at a time.
constexpr int LRA_ROWS = 4;

template <typename E>
__global__ __launch_bounds__(256) void lowrank_add_kernel(E *__restrict__ io,
                                                          const float *__restrict__ P,
                                                          const E *__restrict__ Wt, int T, int C,
                                                          int r, float s) {
  const int cv = C / 8;                                    // 8-column chunks per row
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int chunk = (int)(id % cv);
  const int t0 = (int)(id / cv) * LRA_ROWS;
  if (t0 >= T) return;
  const int c0 = chunk * 8;
  // the rows to update are requested first, so their latency overlaps the rank-r arithmetic
  Vec8<E> cur[LRA_ROWS];
#pragma unroll
  for (int i = 0; i < LRA_ROWS; i++) {
    const int t = t0 + i < T ? t0 + i : T - 1;
    cur[i].load(io + (int64_t)t * C + c0);
  }
  float acc[LRA_ROWS][8];
#pragma unroll
  for (int i = 0; i < LRA_ROWS; i++)
#pragma unroll
    for (int j = 0; j < 8; j++) acc[i][j] = 0.f;
  for (int q0 = 0; q0 < r; q0 += 8) {
    float wv[8][8];
#pragma unroll
    for (int j = 0; j < 8; j++) {
      Vec8<E> v;
      v.load(Wt + (int64_t)(c0 + j) * r + q0);
#pragma unroll
      for (int q = 0; q < 8; q++) wv[j][q] = v.get(q);
    }
#pragma unroll
    for (int i = 0; i < LRA_ROWS; i++) {
      const int t = t0 + i < T ? t0 + i : T - 1;
      Vec8<float> pv;
      pv.load(P + (int64_t)t * r + q0);
#pragma unroll
      for (int q = 0; q < 8; q++)
#pragma unroll
        for (int j = 0; j < 8; j++) acc[i][j] = fmaf(pv.get(q), wv[j][q], acc[i][j]);
    }
  }
#pragma unroll
  for (int i = 0; i < LRA_ROWS; i++) {
    if (t0 + i < T) {
      Vec8<E> v = cur[i];
#pragma unroll
      for (int j = 0; j < 8; j++) v.set(j, v.get(j) + s * acc[i][j]);
      v.store(io + (int64_t)(t0 + i) * C + c0);
    }
  }
}

// Same update for r <= 16: a thread keeps the 16 rank entries of its 8 columns in registers and
// walks LRB_ROWS rows (P[t, :] is uniform over the workgroup: scalar loads), so the weight rows
// are read once per workgroup instead of once per 4 rows.
constexpr int LRB_ROWS = 8;

template <typename E>
__global__ __launch_bounds__(256) void lowrank_add_r16_kernel(E *__restrict__ io,
                                                              const float *__restrict__ P,
                                                              const E *__restrict__ Wt, int T, int C,
                                                              int r, float s) {
  const int c0 = (blockIdx.x * 256 + threadIdx.x) * 8;
  if (c0 >= C) return;
  const int t0 = blockIdx.y * LRB_ROWS;
  const int t1 = t0 + LRB_ROWS < T ? t0 + LRB_ROWS : T;
  float w[8][16];
#pragma unroll
  for (int j = 0; j < 8; j++) {
    Vec8<E> a, b;
    a.load(Wt + (int64_t)(c0 + j) * r);
    if (r > 8) b.load(Wt + (int64_t)(c0 + j) * r + 8);
#pragma unroll
    for (int q = 0; q < 8; q++) {
      w[j][q] = s * a.get(q);
      w[j][8 + q] = r > 8 ? s * b.get(q) : 0.f;
    }
  }
  // four rows per step, the next four requested before the arithmetic of the current ones
  Vec8<E> cur[4], nxt[4];
  auto load4 = [&](int t, Vec8<E> (&v)[4]) {
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int tt = t + i < T ? t + i : T - 1;
      v[i].load(io + (int64_t)tt * C + c0);
    }
  };
  load4(t0, cur);
  for (int t = t0; t < t1; t += 4) {
    if (t + 4 < t1) load4(t + 4, nxt);
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int tt = t + i < T ? t + i : T - 1;
      const float *pt = P + (int64_t)tt * r;
      float acc[8];
#pragma unroll
      for (int j = 0; j < 8; j++) acc[j] = cur[i].get(j);
#pragma unroll
      for (int q = 0; q < 16; q++) {
        const float pq = q < r ? pt[q] : 0.f;
#pragma unroll
        for (int j = 0; j < 8; j++) acc[j] = fmaf(pq, w[j][q], acc[j]);
      }
      if (t + i < t1) {
        Vec8<E> o;
#pragma unroll
        for (int j = 0; j < 8; j++) o.set(j, acc[j]);
        o.store(io + (int64_t)(t + i) * C + c0);
      }
    }
#pragma unroll
    for (int i = 0; i < 4; i++) cur[i] = nxt[i];
  }
}

hipError_t launch_lowrank_add(int dtype, void *io, const float *P, const void *Wt, int T, int C,
                              int r, float s, hipStream_t st) {
  if (C % 8 || r % 8) return hipErrorInvalidValue;
  if (r <= 16) {
    const dim3 grid((C / 8 + 255) / 256, (T + LRB_ROWS - 1) / LRB_ROWS), block(256);
    if (dtype == MIXLORA_BF16)
      hipLaunchKernelGGL(lowrank_add_r16_kernel<bf16_t>, grid, block, 0, st, (bf16_t *)io, P,
                         (const bf16_t *)Wt, T, C, r, s);
    else
      hipLaunchKernelGGL(lowrank_add_r16_kernel<float>, grid, block, 0, st, (float *)io, P,
                         (const float *)Wt, T, C, r, s);
    return hipGetLastError();
  }
  const int64_t n = (int64_t)((T + LRA_ROWS - 1) / LRA_ROWS) * (C / 8);
  const dim3 grid((unsigned)((n + 255) / 256)), block(256);
  if (dtype == MIXLORA_BF16)
    hipLaunchKernelGGL(lowrank_add_kernel<bf16_t>, grid, block, 0, st, (bf16_t *)io, P,
                       (const bf16_t *)Wt, T, C, r, s);
  else
    hipLaunchKernelGGL(lowrank_add_kernel<float>, grid, block, 0, st, (float *)io, P,
                       (const float *)Wt, T, C, r, s);
  return hipGetLastError();
}

// out[i] = sum over s < S of part[s][i]  (fixed order): closes a GEMM whose K range was split
// over several workgroups because its output alone has too few tiles to cover the chip
template <typename E>
__global__ void splitk_reduce_kernel(const float *__restrict__ part, int S, int64_t n,
                                     E *__restrict__ out) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float acc = 0.f;
  for (int sp = 0; sp < S; sp++) acc += part[(int64_t)sp * n + i];
  out[i] = from_f32<E>(acc);
}

hipError_t launch_splitk_reduce(int dtype, const float *part, int S, int64_t n, void *out,
                                hipStream_t st) {
  const dim3 grid((unsigned)((n + 255) / 256)), block(256);
  if (dtype == MIXLORA_BF16)
    hipLaunchKernelGGL(splitk_reduce_kernel<bf16_t>, grid, block, 0, st, part, S, n, (bf16_t *)out);
  else
    hipLaunchKernelGGL(splitk_reduce_kernel<float>, grid, block, 0, st, part, S, n, (float *)out);
  return hipGetLastError();
}

// ---- weight re-layouts (all tiny next to the frozen matrices) -------------------------------
// Every re-layout is an index permutation of at most three loop dimensions (i2 fastest over the
// threads):  dst[dst0 + i0*d0 + i1*d1 + i2*d2] = scale * src[i0*s0 + i1*s1 + i2*s2], with zeros
// written where i2 >= valid2.  Up to RELAYOUT_MAX_JOBS of them run in one launch (blockIdx.y
// picks the job), since each alone is dominated by its launch.
template <typename E>
__global__ __launch_bounds__(256) void relayout_kernel(RelayoutBatch batch) {
  relayout_body<E>(batch.job[blockIdx.y], blockIdx.x, gridDim.x);
}

hipError_t launch_relayout(int dtype, const RelayoutJob *jobs, int njobs, hipStream_t st) {
  if (njobs < 1 || njobs > RELAYOUT_MAX_JOBS) return hipErrorInvalidValue;
  RelayoutBatch b;
  for (int i = 0; i < RELAYOUT_MAX_JOBS; i++) b.job[i] = jobs[i < njobs ? i : 0];
  const int64_t blocks = relayout_blocks(jobs, njobs);
  if (blocks == 0) return hipErrorInvalidValue;
  const dim3 grid((unsigned)blocks, njobs), block(256);
  if (dtype == MIXLORA_BF16) hipLaunchKernelGGL(relayout_kernel<bf16_t>, grid, block, 0, st, b);
  else hipLaunchKernelGGL(relayout_kernel<float>, grid, block, 0, st, b);
  return hipGetLastError();
}

// bytes (rounded up to a multiple of 16; the buffer must have that room) of zeros at dst
RelayoutJob job_zero_fill(void *dst, size_t bytes) {
  RelayoutJob j{};
  j.dst = dst;
  j.zero_bytes = (bytes + 15) / 16 * 16;
  j.n0 = j.n1 = j.n2 = 1;
  return j;
}
// bank [N, rows, r]  ->  out[i, col0 + e*r + q] = scale * bank[e, i, q]     (out pitch ldo)
RelayoutJob job_bank_cat(const void *bank, int N, int rows, int r, float scale, void *out,
                         int ldo, int col0) {
  RelayoutJob j{};
  j.src = bank; j.dst = out; j.scale = scale;
  j.n0 = N; j.n1 = rows; j.n2 = r; j.valid2 = r;
  j.s0 = (int64_t)rows * r; j.s1 = r; j.s2 = 1;
  j.dst0 = col0; j.d0 = r; j.d1 = ldo; j.d2 = 1;
  return j;
}
// bank [N, rows, r]  ->  out[e*r + q, i] = bank[e, i, q]                     (out is [N*r, rows])
RelayoutJob job_bank_T(const void *bank, int N, int rows, int r, void *out) {
  RelayoutJob j{};
  j.src = bank; j.dst = out; j.scale = 1.f;
  j.batched_transpose = 1;
  j.n0 = N; j.n1 = rows; j.n2 = r; j.valid2 = rows;
  j.s0 = (int64_t)rows * r;
  j.dst0 = 0; j.d0 = (int64_t)r * rows; j.d1 = rows;
  return j;
}
// [N, r_src, width] -> [N, r_dst, width] (rank_major) or [N, width, r_src] -> [N, width, r_dst]
RelayoutJob job_rank_resize(const void *src, void *dst, int N, int r_src, int r_dst, int width,
                            bool rank_major) {
  RelayoutJob j{};
  j.src = src; j.dst = dst; j.scale = 1.f;
  j.n0 = N; j.n1 = width; j.n2 = r_dst;          // i2 walks the rank entries
  j.valid2 = r_src < r_dst ? r_src : r_dst;
  j.s0 = (int64_t)r_src * width;
  j.d0 = (int64_t)r_dst * width;
  if (rank_major) { j.s1 = 1; j.s2 = width; j.d1 = 1; j.d2 = width; }
  else            { j.s1 = r_src; j.s2 = 1; j.d1 = r_dst; j.d2 = 1; }
  return j;
}
// A [N, r, cols]  ->  out[c, col0 + e*r + q] = scale * A[e, q, c]
RelayoutJob job_A_cat(const void *A, int N, int r, int cols, float scale, void *out, int ldo,
                      int col0) {
  RelayoutJob j{};
  j.src = A; j.dst = out; j.scale = scale;
  j.batched_transpose = 1;   // one [N*r, cols] matrix -> [cols, N*r] at pitch ldo
  j.n0 = 1; j.n1 = N * r; j.n2 = cols; j.valid2 = N * r;
  j.s0 = 0;
  j.dst0 = col0; j.d0 = 0; j.d1 = ldo;
  return j;
}
// W_router [N, d]  ->  out[c, col0 + n] = W_router[n, c] for n < N, 0 for N <= n < ncols
RelayoutJob job_router_T(const void *W_router, int N, int d, void *out, int ldo, int col0,
                         int ncols) {
  RelayoutJob j{};
  j.src = W_router; j.dst = out; j.scale = 1.f;
  j.batched_transpose = 1;   // [N, d] -> [d, ncols] at pitch ldo, zero-filled past N
  j.n0 = 1; j.n1 = ncols; j.n2 = d; j.valid2 = N;
  j.s0 = 0;
  j.dst0 = col0; j.d0 = 0; j.d1 = ldo;
  return j;
}

// out[cols, rows] = in[rows, cols]^T through a padded 64x64 LDS tile
template <typename E>
__global__ __launch_bounds__(256) void transpose_kernel(const E *__restrict__ in,
                                                        E *__restrict__ out, int rows, int cols) {
  __shared__ E tile[64][64 + 2];
  const int c0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int i = ty; i < 64; i += 4) {
    const int r = r0 + i, c = c0 + tx;
    if (r < rows && c < cols) tile[i][tx] = in[(int64_t)r * cols + c];
  }
  __syncthreads();
  for (int i = ty; i < 64; i += 4) {
    const int c = c0 + i, r = r0 + tx;
    if (r < rows && c < cols) out[(int64_t)c * rows + r] = tile[tx][i];
  }
}

hipError_t launch_transpose(int dtype, const void *in, void *out, int rows, int cols,
                            hipStream_t st) {
  const dim3 grid((cols + 63) / 64, (rows + 63) / 64), block(256);
  if (dtype == MIXLORA_BF16)
    hipLaunchKernelGGL(transpose_kernel<bf16_t>, grid, block, 0, st, (const bf16_t *)in,
                       (bf16_t *)out, rows, cols);
  else
    hipLaunchKernelGGL(transpose_kernel<float>, grid, block, 0, st, (const float *)in,
                       (float *)out, rows, cols);
  return hipGetLastError();
}

}  // namespace mixlora
