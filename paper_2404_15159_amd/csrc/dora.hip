// Pieces of the weight-decomposed expert variant ("MixDoRA" in the paper's experiments, which
// gives no formula; the reading follows the cited weight-decomposition method): every expert
// projection is  diag(m_e / n_e) (W + s B_e A_e),  n_e = row norms of W + s B_e A_e, held constant
// in the backward pass.  The frozen product stays shared; the per-expert factor c_e = m_e / n_e is
// applied to the rows of the routed pairs.  bf16 storage only.
//
// Row norms without forming W + s B_e A_e:
//   n_e[j]^2 = |W[j,:]|^2 + 2 s B_e[j,:] . (W A_e^T)[j,:] + s^2 B_e[j,:] (A_e A_e^T) B_e[j,:]^T
// with W A_e^T from the GEMM engine (rank-r output columns) and the r x r Gram matrices and the
// squared row norms of W from the small kernels below.
#include "common.h"

namespace mixlora {

// ---- w2[j] = sum_i W[j, i]^2, one wavefront per row, lanes in a fixed order ---------------------
__global__ __launch_bounds__(256) void row_sqnorm_kernel(const bf16_t *__restrict__ W, int rows,
                                                         int cols, float *__restrict__ out) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const bf16_t *p = W + (int64_t)row * cols;
  float acc = 0.f;
  for (int c = lane * 8; c < cols; c += 64 * 8) {
    const bf16x8_t v = *reinterpret_cast<const bf16x8_t *>(p + c);
#pragma unroll
    for (int i = 0; i < 8; i++) acc = fmaf((float)v[i], (float)v[i], acc);
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o, 64);
  if (lane == 0) out[row] = acc;
}

hipError_t launch_row_sqnorm(const void *W, int rows, int cols, float *out, hipStream_t st) {
  hipLaunchKernelGGL(row_sqnorm_kernel, dim3((rows + 3) / 4), dim3(256), 0, st, (const bf16_t *)W,
                     rows, cols, out);
  return hipGetLastError();
}

// ---- AA[e][q][q'] = sum_i A[e, q, i] A[e, q', i]  (A bank [N, r, in]) ----------------------------
// The input dimension is cut into GRAM_SLICES slices (blockIdx.y); slice sums go to
// part[slice][e][q][q'] and are added in slice order by the consumer.
constexpr int GRAM_SLICES = 16;

__global__ __launch_bounds__(256) void gram_kernel(const bf16_t *__restrict__ A, int r, int in,
                                                   int N, float *__restrict__ part) {
  __shared__ float t[64][65];
  const int e = blockIdx.x, sl = blockIdx.y;
  const bf16_t *Ae = A + (int64_t)e * r * in;
  const int per = ((in + GRAM_SLICES - 1) / GRAM_SLICES + 63) / 64 * 64;
  const int lo = sl * per, hi = lo + per < in ? lo + per : in;
  float acc[16];   // r <= 64: at most 4096 outputs over 256 threads
#pragma unroll
  for (int o = 0; o < 16; o++) acc[o] = 0.f;
  for (int i0 = lo; i0 < hi; i0 += 64) {
    for (int idx = threadIdx.x; idx < r * 64; idx += 256) {
      const int q = idx / 64, i = idx % 64;
      t[q][i] = i0 + i < hi ? (float)Ae[(int64_t)q * in + i0 + i] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int o = 0; o < 16; o++) {
      const int out = threadIdx.x + o * 256;
      if (out < r * r) {
        const int q = out / r, q2 = out % r;
        float a = acc[o];
        for (int i = 0; i < 64; i++) a = fmaf(t[q][i], t[q2][i], a);
        acc[o] = a;
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int o = 0; o < 16; o++) {
    const int out = threadIdx.x + o * 256;
    if (out < r * r) part[((int64_t)sl * N + e) * r * r + out] = acc[o];
  }
}

size_t gram_part_floats(int N, int r) { return (size_t)GRAM_SLICES * N * r * r; }

hipError_t launch_gram(const void *A_bank, int N, int r, int in, float *part, hipStream_t st) {
  hipLaunchKernelGGL(gram_kernel, dim3(N, GRAM_SLICES), dim3(256), 0, st, (const bf16_t *)A_bank, r,
                     in, N, part);
  return hipGetLastError();
}

// ---- c[e, j] = m[e, j] / n_e[j],  ninv[e, j] = 1 / n_e[j] ----------------------------------------
// B bank [N, out, r] bf16; WA [out, N*r] float32; AA: the Gram kernel's slice sums
// [GRAM_SLICES][N][r][r]; w2 [out]; c, ninv [N, out]; m [N, out] (m_stride = out) or one [out]
// vector shared by the experts (m_stride = 0).
__global__ __launch_bounds__(256) void dora_scale_kernel(const bf16_t *__restrict__ B,
                                                         const float *__restrict__ WA,
                                                         const float *__restrict__ AA,
                                                         const float *__restrict__ w2,
                                                         const float *__restrict__ m,
                                                         int64_t m_stride, int N, int out,
                                                         int r, float s, float *__restrict__ c,
                                                         float *__restrict__ ninv) {
  __shared__ float aa[64 * 64];
  const int e = blockIdx.y;
  for (int i = threadIdx.x; i < r * r; i += 256) {
    float a = 0.f;
    for (int sl = 0; sl < GRAM_SLICES; sl++) a += AA[((int64_t)sl * N + e) * r * r + i];
    aa[i] = a;
  }
  __syncthreads();
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= out) return;
  const bf16_t *b = B + ((int64_t)e * out + j) * r;
  const float *wa = WA + (int64_t)j * N * r + e * r;
  float cross = 0.f, quad = 0.f;
  for (int q = 0; q < r; q++) {
    const float bq = (float)b[q];
    cross = fmaf(bq, wa[q], cross);
    float row = 0.f;
    for (int q2 = 0; q2 < r; q2++) row = fmaf(aa[q * r + q2], (float)b[q2], row);
    quad = fmaf(bq, row, quad);
  }
  const float n2 = w2[j] + 2.f * s * cross + s * s * quad;
  const float inv = n2 > 0.f ? 1.f / sqrtf(n2) : 0.f;
  ninv[(int64_t)e * out + j] = inv;
  c[(int64_t)e * out + j] = m[e * m_stride + j] * inv;
}

hipError_t launch_dora_scale(const void *B_bank, const float *WA, const float *AA, const float *w2,
                             const float *m, int shared, int N, int out, int r, float s, float *c,
                             float *ninv, hipStream_t st) {
  hipLaunchKernelGGL(dora_scale_kernel, dim3((out + 255) / 256, N), dim3(256), 0, st,
                     (const bf16_t *)B_bank, WA, AA, w2, m, (int64_t)(shared ? 0 : out), N, out, r, s,
                     c, ninv);
  return hipGetLastError();
}

// ---- bank[(e*r + q), j] *= c[e, j]   (transposed B_down bank [N*r, d]) ---------------------------
__global__ void scale_bank_kernel(bf16_t *__restrict__ bank, const float *__restrict__ c, int N,
                                  int r, int d) {
  const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 8;
  if (i >= (int64_t)N * r * d) return;
  const int row = (int)(i / d), j = (int)(i % d);
  const int e = row / r;
  bf16x8_t v = *reinterpret_cast<bf16x8_t *>(bank + i);
#pragma unroll
  for (int q = 0; q < 8; q++) v[q] = (bf16_t)((float)v[q] * c[(int64_t)e * d + j + q]);
  *reinterpret_cast<bf16x8_t *>(bank + i) = v;
}

hipError_t launch_scale_bank(void *bank, const float *c, int N, int r, int d, hipStream_t st) {
  const int64_t n = (int64_t)N * r * d / 8;
  hipLaunchKernelGGL(scale_bank_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                     (bf16_t *)bank, c, N, r, d);
  return hipGetLastError();
}

// ---- dst[row, :] = c[e(row), :] * src[token of row, :] -------------------------------------------
__global__ __launch_bounds__(256) void gather_rows_scaled_kernel(PairCtx pc, int width,
                                                                 const bf16_t *__restrict__ src,
                                                                 const float *__restrict__ c,
                                                                 bf16_t *__restrict__ dst) {
  const int row = blockIdx.x;
  const int col = (blockIdx.y * 256 + threadIdx.x) * 8;
  if (col >= width) return;
  const int pair = pc.pair_of_row[row];
  const int e = pc.idx[pair];
  bf16x8_t v = *reinterpret_cast<const bf16x8_t *>(src + (int64_t)(pair / pc.k) * width + col);
#pragma unroll
  for (int q = 0; q < 8; q++) v[q] = (bf16_t)((float)v[q] * c[(int64_t)e * width + col + q]);
  *reinterpret_cast<bf16x8_t *>(dst + (int64_t)row * width + col) = v;
}

hipError_t launch_gather_rows_scaled(const PairCtx &pc, int width, const void *src, const float *c,
                                     void *dst, hipStream_t st) {
  const dim3 grid(pc.T * pc.k, (width / 8 + 255) / 256), block(256);
  hipLaunchKernelGGL(gather_rows_scaled_kernel, grid, block, 0, st, pc, width, (const bf16_t *)src,
                     c, (bf16_t *)dst);
  return hipGetLastError();
}

// ---- out[t, :] = sum_j w[t, j] * c[e_j, :] * in_grp[row_of_pair[t, j], :]  (slots ascending) -----
__global__ __launch_bounds__(256) void pair_combine_scaled_kernel(PairCtx pc, int width,
                                                                  const bf16_t *__restrict__ in_grp,
                                                                  const float *__restrict__ c,
                                                                  bf16_t *__restrict__ out) {
  const int t = blockIdx.x;
  const int col = (blockIdx.y * 256 + threadIdx.x) * 8;
  if (col >= width) return;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int j = 0; j < pc.k; j++) {
    const int p = t * pc.k + j;
    const float w = pc.w[p];
    const float *ce = c + (int64_t)pc.idx[p] * width + col;
    const bf16x8_t v = *reinterpret_cast<const bf16x8_t *>(in_grp + (int64_t)pc.row_of_pair[p] * width + col);
#pragma unroll
    for (int i = 0; i < 8; i++) acc[i] = fmaf(w * ce[i], (float)v[i], acc[i]);
  }
  bf16x8_t o;
#pragma unroll
  for (int i = 0; i < 8; i++) o[i] = (bf16_t)acc[i];
  *reinterpret_cast<bf16x8_t *>(out + (int64_t)t * width + col) = o;
}

hipError_t launch_pair_combine_scaled(const PairCtx &pc, int width, const void *in_grp,
                                      const float *c, void *out, hipStream_t st) {
  const dim3 grid(pc.T, (width / 8 + 255) / 256), block(256);
  hipLaunchKernelGGL(pair_combine_scaled_kernel, grid, block, 0, st, pc, width,
                     (const bf16_t *)in_grp, c, (bf16_t *)out);
  return hipGetLastError();
}

// ---- magnitude gradient of the down projection ---------------------------------------------------
// dm[e, j] = ninv[e, j] * sum over the rows of expert e of  w_row * dy[token, j] * v[row, j]
// (v = unscaled output of the per-pair down projection).  Rows are cut into DMD_SLICES slices per
// expert; slice sums are written to part[slice][e][j] and added in slice order afterwards.
constexpr int DMD_SLICES = 16;

__global__ __launch_bounds__(256) void dm_down_part_kernel(PairCtx pc, int d,
                                                           const bf16_t *__restrict__ dy,
                                                           const bf16_t *__restrict__ v,
                                                           float *__restrict__ part) {
  const int e = blockIdx.y, sl = blockIdx.z;
  const int col = (blockIdx.x * 256 + threadIdx.x) * 8;
  if (col >= d) return;
  const int lo = pc.offs[e], hi = pc.offs[e + 1];
  const int per = (hi - lo + DMD_SLICES - 1) / DMD_SLICES;
  const int r0 = lo + sl * per, r1 = r0 + per < hi ? r0 + per : hi;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int row = r0; row < r1; row++) {
    const int pair = pc.pair_of_row[row];
    const float w = pc.w[pair];
    const bf16x8_t a = *reinterpret_cast<const bf16x8_t *>(dy + (int64_t)(pair / pc.k) * d + col);
    const bf16x8_t b = *reinterpret_cast<const bf16x8_t *>(v + (int64_t)row * d + col);
#pragma unroll
    for (int i = 0; i < 8; i++) acc[i] = fmaf(w * (float)a[i], (float)b[i], acc[i]);
  }
  float *o = part + ((int64_t)sl * pc.N + e) * d + col;
#pragma unroll
  for (int i = 0; i < 8; i++) o[i] = acc[i];
}

// per expert: dm [N, d]; shared magnitude: dm [d] = sum over the experts in ascending order
__global__ void dm_down_reduce_kernel(const float *__restrict__ part, const float *__restrict__ ninv,
                                      int N, int d, int shared, float *__restrict__ dm) {
  const int64_t n = (int64_t)N * d;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (shared ? d : n)) return;
  float tot = 0.f;
  for (int e = 0; e < (shared ? N : 1); e++) {
    const int64_t o = i + (int64_t)e * d;
    float acc = 0.f;
    for (int sl = 0; sl < DMD_SLICES; sl++) acc += part[(int64_t)sl * n + o];
    tot += acc * ninv[o];
  }
  dm[i] = tot;
}

size_t dm_down_part_floats(int N, int d) { return (size_t)DMD_SLICES * N * d; }

hipError_t launch_dm_down(const PairCtx &pc, int d, const void *dy, const void *v, const float *ninv,
                          float *part, float *dm, int shared, hipStream_t st) {
  hipLaunchKernelGGL(dm_down_part_kernel, dim3((d / 8 + 255) / 256, pc.N, DMD_SLICES), dim3(256), 0,
                     st, pc, d, (const bf16_t *)dy, (const bf16_t *)v, part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int64_t n = shared ? (int64_t)d : (int64_t)pc.N * d;
  hipLaunchKernelGGL(dm_down_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, part,
                     ninv, pc.N, d, shared, dm);
  return hipGetLastError();
}

// ---- magnitude gradients of gate / up from the fused stage's per-tile sums -----------------------
// dm[e, c] = ninv[e, c] * sum over the row tiles of expert e (ascending) of part[tile][c];
// blockIdx.z picks gate (0) or up (1).  The tiles of an expert are consecutive, 32 rows each.
// With a magnitude shared by the experts (grid y = 1, N experts walked here) dm[c] is the sum of
// the experts' terms in ascending order.
__global__ __launch_bounds__(256) void dm_tiles_reduce_kernel(
    const int32_t *__restrict__ offs, int f, int N, int shared, const float *__restrict__ part_g,
    const float *__restrict__ part_u, const float *__restrict__ ninv_g,
    const float *__restrict__ ninv_u, float *__restrict__ dm_g, float *__restrict__ dm_u) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= f) return;
  const float *part = blockIdx.z ? part_u : part_g;
  const float *ninv = blockIdx.z ? ninv_u : ninv_g;
  float *dm = blockIdx.z ? dm_u : dm_g;
  const int e_lo = shared ? 0 : blockIdx.y, e_hi = shared ? N : blockIdx.y + 1;
  int tile0 = 0;
  for (int q = 0; q < e_lo; q++) tile0 += (offs[q + 1] - offs[q] + 31) / 32;
  float tot = 0.f;
  for (int e = e_lo; e < e_hi; e++) {
    const int nt = (offs[e + 1] - offs[e] + 31) / 32;
    float acc = 0.f;
    for (int t = 0; t < nt; t++) acc += part[(int64_t)(tile0 + t) * f + c];
    tile0 += nt;
    tot += acc * ninv[(int64_t)e * f + c];
  }
  dm[shared ? c : (int64_t)e_lo * f + c] = tot;
}

hipError_t launch_dm_tiles_reduce(const int32_t *offs, int N, int f, const float *part_g,
                                  const float *part_u, const float *ninv_g, const float *ninv_u,
                                  float *dm_g, float *dm_u, int shared, hipStream_t st) {
  hipLaunchKernelGGL(dm_tiles_reduce_kernel, dim3((f + 255) / 256, shared ? 1 : N, 2), dim3(256), 0,
                     st, offs, f, N, shared, part_g, part_u, ninv_g, ninv_u, dm_g, dm_u);
  return hipGetLastError();
}

}  // namespace mixlora
