// bf16 MFMA versions of the per-pair (token, expert) stages, on expert-grouped rows.
//
// A workgroup owns one tile of 32 grouped rows (all of one expert) and a range of 32-column
// blocks; each of its 4 wavefronts walks every 4th block.  Per block the LoRA deltas of
// Algorithm 1 lines 11-12 are one rank-r MFMA each (B_e[cols, r] x P[rows, r]^T added to the
// shared gate/up projections gathered by token), SiLU * up follows in registers (line 13), and
// the activation tile - still in registers, whose MFMA result layout is also a valid MFMA
// operand layout with the columns as the contraction index - is multiplied by A_down_e to
// accumulate the rank-r input of the down projection's LoRA (line 14) without re-reading it.
//
// MFMA 32x32x16 layout used throughout: operand lanes carry index (lane % 32) and the 8
// contraction elements of half (lane / 32); result register e of a lane holds
// D[8*(e/4) + 4*(lane/32) + e%4][lane % 32].  Here the FIRST operand is the weight fragment
// (index = column), the SECOND the per-row fragment (index = row), so a lane holds, for its row,
// the 16 columns c0 + 8g + 4*(lane/32) + m (g, m < 4): four 8-byte runs.
#include "common.h"

namespace mixlora {

typedef bf16_t bf16x4_t __attribute__((ext_vector_type(4)));

constexpr int FT_ROWS = 32;    // grouped rows per tile
constexpr int FT_WAVES = 4;

__device__ __forceinline__ bool fused_tile_rows(const int32_t *offs, int N, int b, int &e,
                                                int &row0, int &rows) {
  for (e = 0; e < N; e++) {
    const int lo = offs[e], hi = offs[e + 1];
    const int nt = (hi - lo + FT_ROWS - 1) / FT_ROWS;
    if (b < nt) {
      row0 = lo + b * FT_ROWS;
      rows = hi - row0 < FT_ROWS ? hi - row0 : FT_ROWS;
      return true;
    }
    b -= nt;
  }
  return false;
}

// v_exp_f32 + v_rcp_f32 (about 1 ulp each): far inside the bf16 tolerance, a tenth of the
// instructions of an IEEE division
__device__ __forceinline__ float fsigmoid(float v) { return __builtin_amdgcn_rcpf(1.f + __expf(-v)); }

// 8 consecutive fp32 -> bf16x8 (or zeros)
__device__ __forceinline__ bf16x8_t cvt8(const float *p, bool valid, float scale) {
  bf16x8_t o;
  if (valid) {
    const float4 a = *reinterpret_cast<const float4 *>(p);
    const float4 b = *reinterpret_cast<const float4 *>(p + 4);
    o[0] = (bf16_t)(a.x * scale); o[1] = (bf16_t)(a.y * scale);
    o[2] = (bf16_t)(a.z * scale); o[3] = (bf16_t)(a.w * scale);
    o[4] = (bf16_t)(b.x * scale); o[5] = (bf16_t)(b.y * scale);
    o[6] = (bf16_t)(b.z * scale); o[7] = (bf16_t)(b.w * scale);
  } else {
#pragma unroll
    for (int i = 0; i < 8; i++) o[i] = (bf16_t)0.f;
  }
  return o;
}

__device__ __forceinline__ bf16x8_t zero8() {
  bf16x8_t o;
#pragma unroll
  for (int i = 0; i < 8; i++) o[i] = (bf16_t)0.f;
  return o;
}

// two 8-byte runs -> one 8-element fragment
__device__ __forceinline__ bf16x8_t join44(const bf16_t *p0, const bf16_t *p1) {
  const bf16x4_t a = *reinterpret_cast<const bf16x4_t *>(p0);
  const bf16x4_t b = *reinterpret_cast<const bf16x4_t *>(p1);
  bf16x8_t o;
  o[0] = a[0]; o[1] = a[1]; o[2] = a[2]; o[3] = a[3];
  o[4] = b[0]; o[5] = b[1]; o[6] = b[2]; o[7] = b[3];
  return o;
}

// Forward: a_grp[row, :] and the per-split partial sums  Q_part[split][row][q] = sum over the
// split's columns of a[row, c] * A_down[e, q, c].
template <int KSR, int NQ>
__global__ __launch_bounds__(FT_WAVES * 64) void swiglu_fwd_mfma_kernel(
    PairCtx pc, int f, float s, const bf16_t *__restrict__ G, const bf16_t *__restrict__ U,
    const float *__restrict__ Pg_all, const float *__restrict__ Pu_all,
    const bf16_t *__restrict__ B_gate, const bf16_t *__restrict__ B_up,
    const bf16_t *__restrict__ A_down, bf16_t *__restrict__ a_grp, float *__restrict__ Q_part,
    int nsplit) {
  __shared__ float red[FT_WAVES][NQ][16][64];
  int e, row0, rows;
  if (!fused_tile_rows(pc.offs, pc.N, blockIdx.x, e, row0, rows)) return;
  const int r = pc.r, R = pc.N * r, nP = pc.T * pc.k;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l31 = lane & 31, hi = lane >> 5;
  const bool rvalid = l31 < rows;
  const int row = row0 + (rvalid ? l31 : 0);
  const int64_t t = pc.pair_of_row[row] / pc.k;

  // per-row LoRA-A projections of this expert as second-operand fragments
  bf16x8_t pg[KSR], pu[KSR];
#pragma unroll
  for (int ks = 0; ks < KSR; ks++) {
    const int q0 = ks * 16 + hi * 8;
    const bool v = q0 < r;
    pg[ks] = cvt8(Pg_all + t * R + e * r + (v ? q0 : 0), v, 1.f);
    pu[ks] = cvt8(Pu_all + t * R + e * r + (v ? q0 : 0), v, 1.f);
  }
  f32x16_t accq[NQ];
#pragma unroll
  for (int j = 0; j < NQ; j++)
#pragma unroll
    for (int i = 0; i < 16; i++) accq[j][i] = 0.f;

  const int nblk = f / 32;                       // f % 32 == 0 is required by the launcher
  const int per = (nblk + nsplit - 1) / nsplit;
  const int b_lo = blockIdx.y * per;
  const int b_hi = b_lo + per < nblk ? b_lo + per : nblk;
  const bf16_t *bg_e = B_gate + (int64_t)e * f * r;
  const bf16_t *bu_e = B_up + (int64_t)e * f * r;
  const bf16_t *ad_e = A_down + (int64_t)e * r * f;

  bf16x4_t gnx[4], unx[4];
  {
    const int cbf = b_lo + wave < b_hi ? b_lo + wave : 0;   // any valid block if this wave has none
#pragma unroll
    for (int g = 0; g < 4; g++) {
      gnx[g] = *reinterpret_cast<const bf16x4_t *>(G + t * f + cbf * 32 + hi * 4 + g * 8);
      unx[g] = *reinterpret_cast<const bf16x4_t *>(U + t * f + cbf * 32 + hi * 4 + g * 8);
    }
  }
  for (int cb = b_lo + wave; cb < b_hi; cb += FT_WAVES) {
    const int c0 = cb * 32;
    // (1) this block's weight fragments (L2-resident banks), (2) the NEXT block's gathered G/U
    // runs.  Loads return in order, so waiting for (1) leaves (2) in flight during the math.
    bf16x8_t wg[KSR], wu[KSR], wf[2][NQ];
#pragma unroll
    for (int ks = 0; ks < KSR; ks++) {
      const int q0 = ks * 16 + hi * 8;
      const int64_t o = (int64_t)(c0 + l31) * r + (q0 < r ? q0 : 0);
      wg[ks] = *reinterpret_cast<const bf16x8_t *>(bg_e + o);
      wu[ks] = *reinterpret_cast<const bf16x8_t *>(bu_e + o);
    }
#pragma unroll
    for (int s2 = 0; s2 < 2; s2++)
#pragma unroll
      for (int j = 0; j < NQ; j++) {
        const int q = j * 32 + l31;
        const bf16_t *wp = ad_e + (int64_t)(q < r ? q : 0) * f + c0 + 16 * s2 + hi * 4;
        wf[s2][j] = join44(wp, wp + 8);
      }
    bf16x4_t gcur[4], ucur[4];
#pragma unroll
    for (int g = 0; g < 4; g++) { gcur[g] = gnx[g]; ucur[g] = unx[g]; }
    {   // unconditional (the last iteration re-reads its own block) so that the wait counts
        // the compiler derives are the same on every path
      const int cn = cb + FT_WAVES < b_hi ? c0 + FT_WAVES * 32 : c0;
#pragma unroll
      for (int g = 0; g < 4; g++) {
        gnx[g] = *reinterpret_cast<const bf16x4_t *>(G + t * f + cn + hi * 4 + g * 8);
        unx[g] = *reinterpret_cast<const bf16x4_t *>(U + t * f + cn + hi * 4 + g * 8);
      }
    }
    f32x16_t dg, du;
#pragma unroll
    for (int i = 0; i < 16; i++) dg[i] = du[i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KSR; ks++) {
      const bool v = ks * 16 + hi * 8 < r;
      dg = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v ? wg[ks] : zero8(), pg[ks], dg, 0, 0, 0);
      du = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v ? wu[ks] : zero8(), pu[ks], du, 0, 0, 0);
    }
    bf16_t *ap = a_grp + (int64_t)row * f + c0 + hi * 4;
    bf16x4_t av[4];
#pragma unroll
    for (int g = 0; g < 4; g++) {
      const bf16x4_t gv = gcur[g];
      const bf16x4_t uv = ucur[g];
#pragma unroll
      for (int m = 0; m < 4; m++) {
        const float gg = (float)gv[m] + s * dg[g * 4 + m];
        const float uu = (float)uv[m] + s * du[g * 4 + m];
        av[g][m] = (bf16_t)(gg * fsigmoid(gg) * uu);
      }
      if (rvalid) *reinterpret_cast<bf16x4_t *>(ap + g * 8) = av[g];
    }
    // Q += a[rows, 32 cols] * A_down[e, q, same cols]^T : two K steps of 16 columns
#pragma unroll
    for (int s2 = 0; s2 < 2; s2++) {
      bf16x8_t af;
#pragma unroll
      for (int m = 0; m < 4; m++) { af[m] = av[2 * s2][m]; af[4 + m] = av[2 * s2 + 1][m]; }
#pragma unroll
      for (int j = 0; j < NQ; j++) {
        const bool v = j * 32 + l31 < r;
        accq[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, v ? wf[s2][j] : zero8(), accq[j], 0, 0, 0);
      }
    }
  }
  // accq[j][i]: row 8*(i/4) + 4*hi + i%4 of the tile, q = j*32 + l31.  Sum the 4 waves.
#pragma unroll
  for (int j = 0; j < NQ; j++)
#pragma unroll
    for (int i = 0; i < 16; i++) red[wave][j][i][lane] = accq[j][i];
  __syncthreads();
  for (int idx = threadIdx.x; idx < NQ * 16 * 64; idx += FT_WAVES * 64) {
    const int j = idx / (16 * 64), i = (idx / 64) % 16, ln = idx % 64;
    const int q = j * 32 + (ln & 31);
    const int rr = 8 * (i >> 2) + 4 * (ln >> 5) + (i & 3);
    if (q < r && rr < rows) {
      const float v = (red[0][j][i][ln] + red[1][j][i][ln]) + (red[2][j][i][ln] + red[3][j][i][ln]);
      Q_part[((int64_t)blockIdx.y * nP + row0 + rr) * r + q] = v;
    }
  }
}

// Backward of the tile above, same ownership (32 grouped rows x a range of 32-column blocks).
// With H[t] = W_down^T dy[t] and Vw[row] = w_row * B_down[e]^T dy[t]:
//   da = w_row * H[t] + s * A_down[e]^T Vw[row]      (rank-r MFMA on the transposed bank AdT)
//   dg = da * u * sig(g) * (1 + g (1 - sig(g))),  du = da * g * sig(g)   -> dg_grp, du_grp
//   dw_part[row][split]   = sum over the split's columns of H * a
//   TG_part[split][row][q] = sum_c dg[row, c] * B_gate[e, c, q]   (and TU with du, B_up)
// BgT / BuT are the banks re-laid as [N, r, f] so that the column index is contiguous.
template <int KSR, int NQ>
__global__ __launch_bounds__(FT_WAVES * 64) void swiglu_bwd_mfma_kernel(
    PairCtx pc, int f, float s, const bf16_t *__restrict__ G, const bf16_t *__restrict__ U,
    const bf16_t *__restrict__ H, const float *__restrict__ Pg_all,
    const float *__restrict__ Pu_all, const float *__restrict__ VB_all,
    const bf16_t *__restrict__ B_gate, const bf16_t *__restrict__ B_up,
    const bf16_t *__restrict__ AdT, const bf16_t *__restrict__ BgT, const bf16_t *__restrict__ BuT,
    bf16_t *__restrict__ dg_grp, bf16_t *__restrict__ du_grp, float *__restrict__ dw_part,
    float *__restrict__ TG_part, float *__restrict__ TU_part, int nsplit) {
  __shared__ float red[FT_WAVES][NQ][16][64];
  __shared__ float dwred[FT_WAVES][32];
  int e, row0, rows;
  if (!fused_tile_rows(pc.offs, pc.N, blockIdx.x, e, row0, rows)) return;
  const int r = pc.r, R = pc.N * r, nP = pc.T * pc.k;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l31 = lane & 31, hi = lane >> 5;
  const bool rvalid = l31 < rows;
  const int row = row0 + (rvalid ? l31 : 0);
  const int pair = pc.pair_of_row[row];
  const int64_t t = pair / pc.k;
  const float wrow = pc.w[pair];

  bf16x8_t pg[KSR], pu[KSR], vw[KSR];
#pragma unroll
  for (int ks = 0; ks < KSR; ks++) {
    const int q0 = ks * 16 + hi * 8;
    const bool v = q0 < r;
    const int64_t o = t * R + e * r + (v ? q0 : 0);
    pg[ks] = cvt8(Pg_all + o, v, 1.f);
    pu[ks] = cvt8(Pu_all + o, v, 1.f);
    vw[ks] = cvt8(VB_all + o, v, wrow);
  }
  f32x16_t acctg[NQ], acctu[NQ];
#pragma unroll
  for (int j = 0; j < NQ; j++)
#pragma unroll
    for (int i = 0; i < 16; i++) acctg[j][i] = acctu[j][i] = 0.f;
  float dwacc = 0.f;

  const int nblk = f / 32;
  const int per = (nblk + nsplit - 1) / nsplit;
  const int b_lo = blockIdx.y * per;
  const int b_hi = b_lo + per < nblk ? b_lo + per : nblk;
  const bf16_t *bg_e = B_gate + (int64_t)e * f * r;
  const bf16_t *bu_e = B_up + (int64_t)e * f * r;
  const bf16_t *ad_e = AdT + (int64_t)e * f * r;
  const bf16_t *bgt_e = BgT + (int64_t)e * r * f;
  const bf16_t *but_e = BuT + (int64_t)e * r * f;

  bf16x4_t gnx[4], unx[4], hnx[4];
  {
    const int cbf = b_lo + wave < b_hi ? b_lo + wave : 0;
#pragma unroll
    for (int g = 0; g < 4; g++) {
      gnx[g] = *reinterpret_cast<const bf16x4_t *>(G + t * f + cbf * 32 + hi * 4 + g * 8);
      unx[g] = *reinterpret_cast<const bf16x4_t *>(U + t * f + cbf * 32 + hi * 4 + g * 8);
      hnx[g] = *reinterpret_cast<const bf16x4_t *>(H + t * f + cbf * 32 + hi * 4 + g * 8);
    }
  }
  for (int cb = b_lo + wave; cb < b_hi; cb += FT_WAVES) {
    const int c0 = cb * 32;
    // weight fragments of this block first, then the next block's gathered runs (see forward)
    bf16x8_t wg[KSR], wu[KSR], wd[KSR], tg[2][NQ], tu[2][NQ];
#pragma unroll
    for (int ks = 0; ks < KSR; ks++) {
      const int q0 = ks * 16 + hi * 8;
      const int64_t o = (int64_t)(c0 + l31) * r + (q0 < r ? q0 : 0);
      wg[ks] = *reinterpret_cast<const bf16x8_t *>(bg_e + o);
      wu[ks] = *reinterpret_cast<const bf16x8_t *>(bu_e + o);
      wd[ks] = *reinterpret_cast<const bf16x8_t *>(ad_e + o);
    }
#pragma unroll
    for (int s2 = 0; s2 < 2; s2++)
#pragma unroll
      for (int j = 0; j < NQ; j++) {
        const int q = j * 32 + l31;
        const int64_t o = (int64_t)(q < r ? q : 0) * f + c0 + 16 * s2 + hi * 4;
        tg[s2][j] = join44(bgt_e + o, bgt_e + o + 8);
        tu[s2][j] = join44(but_e + o, but_e + o + 8);
      }
    bf16x4_t gcur[4], ucur[4], hcur[4];
#pragma unroll
    for (int g = 0; g < 4; g++) { gcur[g] = gnx[g]; ucur[g] = unx[g]; hcur[g] = hnx[g]; }
    {
      const int64_t nx = t * f + (cb + FT_WAVES < b_hi ? c0 + FT_WAVES * 32 : c0) + hi * 4;
#pragma unroll
      for (int g = 0; g < 4; g++) {
        gnx[g] = *reinterpret_cast<const bf16x4_t *>(G + nx + g * 8);
        unx[g] = *reinterpret_cast<const bf16x4_t *>(U + nx + g * 8);
        hnx[g] = *reinterpret_cast<const bf16x4_t *>(H + nx + g * 8);
      }
    }
    f32x16_t dgm, dum, ddm;
#pragma unroll
    for (int i = 0; i < 16; i++) dgm[i] = dum[i] = ddm[i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KSR; ks++) {
      const bool v = ks * 16 + hi * 8 < r;
      dgm = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v ? wg[ks] : zero8(), pg[ks], dgm, 0, 0, 0);
      dum = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v ? wu[ks] : zero8(), pu[ks], dum, 0, 0, 0);
      ddm = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v ? wd[ks] : zero8(), vw[ks], ddm, 0, 0, 0);
    }
    const int64_t rout = (int64_t)row * f + c0 + hi * 4;
    bf16x4_t dgv[4], duv[4];
#pragma unroll
    for (int g = 0; g < 4; g++) {
      const bf16x4_t gv = gcur[g], uv = ucur[g], hv = hcur[g];
#pragma unroll
      for (int m = 0; m < 4; m++) {
        const float gg = (float)gv[m] + s * dgm[g * 4 + m];
        const float uu = (float)uv[m] + s * dum[g * 4 + m];
        const float hh = (float)hv[m];
        const float sg = fsigmoid(gg);
        const float da = wrow * hh + s * ddm[g * 4 + m];
        dwacc = fmaf(hh, gg * sg * uu, dwacc);
        dgv[g][m] = (bf16_t)(da * uu * sg * (1.f + gg * (1.f - sg)));
        duv[g][m] = (bf16_t)(da * gg * sg);
      }
      if (rvalid) {
        *reinterpret_cast<bf16x4_t *>(dg_grp + rout + g * 8) = dgv[g];
        *reinterpret_cast<bf16x4_t *>(du_grp + rout + g * 8) = duv[g];
      }
    }
#pragma unroll
    for (int s2 = 0; s2 < 2; s2++) {
      bf16x8_t fg, fu;
#pragma unroll
      for (int m = 0; m < 4; m++) {
        fg[m] = dgv[2 * s2][m]; fg[4 + m] = dgv[2 * s2 + 1][m];
        fu[m] = duv[2 * s2][m]; fu[4 + m] = duv[2 * s2 + 1][m];
      }
#pragma unroll
      for (int j = 0; j < NQ; j++) {
        const bool v = j * 32 + l31 < r;
        acctg[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fg, v ? tg[s2][j] : zero8(), acctg[j], 0, 0, 0);
        acctu[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fu, v ? tu[s2][j] : zero8(), acctu[j], 0, 0, 0);
      }
    }
  }
  // <H, a> per row: the two half-waves hold complementary columns of the same row
  dwacc += __shfl_xor(dwacc, 32, 64);
  if (hi == 0) dwred[wave][l31] = dwacc;
  // rank-r sums: add the 4 waves in a fixed order, gate bank first, then up
  for (int bank = 0; bank < 2; bank++) {
    __syncthreads();
#pragma unroll
    for (int j = 0; j < NQ; j++)
#pragma unroll
      for (int i = 0; i < 16; i++) red[wave][j][i][lane] = bank == 0 ? acctg[j][i] : acctu[j][i];
    __syncthreads();
    float *out = bank == 0 ? TG_part : TU_part;
    for (int idx = threadIdx.x; idx < NQ * 16 * 64; idx += FT_WAVES * 64) {
      const int j = idx / (16 * 64), i = (idx / 64) % 16, ln = idx % 64;
      const int q = j * 32 + (ln & 31);
      const int rr = 8 * (i >> 2) + 4 * (ln >> 5) + (i & 3);
      if (q < r && rr < rows) {
        const float v = (red[0][j][i][ln] + red[1][j][i][ln]) + (red[2][j][i][ln] + red[3][j][i][ln]);
        out[((int64_t)blockIdx.y * nP + row0 + rr) * r + q] = v;
      }
    }
  }
  if (threadIdx.x < rows)
    dw_part[(int64_t)(row0 + threadIdx.x) * nsplit + blockIdx.y] =
        (dwred[0][threadIdx.x] + dwred[1][threadIdx.x]) + (dwred[2][threadIdx.x] + dwred[3][threadIdx.x]);
}

// dense[row, e(row)*r + q] = sum over splits of part[split][row][q]   (fixed order)
__global__ void reduce_rank_parts_kernel(PairCtx pc, const float *__restrict__ part, int nsplit,
                                         float *__restrict__ dense) {
  const int nP = pc.T * pc.k, r = pc.r;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)nP * r) return;
  const int row = (int)(i / r), q = (int)(i % r);
  float acc = 0.f;
  for (int sp = 0; sp < nsplit; sp++) acc += part[(int64_t)sp * nP * r + i];
  const int e = pc.idx[pc.pair_of_row[row]];
  dense[(int64_t)row * (pc.N * r) + e * r + q] = acc;
}

int fused_splits(int f) {
  const int nblk = f / 32;
  int s = 8;
  while (s > 1 && nblk / s < FT_WAVES) s >>= 1;
  return s;
}

hipError_t launch_swiglu_fwd_mfma(const PairCtx &pc, int f, float s, const void *G, const void *U,
                                  const float *Pg_all, const float *Pu_all, const void *B_gate,
                                  const void *B_up, const void *A_down, void *a_grp,
                                  float *Q_part, float *Q_all, hipStream_t st) {
  const int nP = pc.T * pc.k, nsplit = fused_splits(f);
  const dim3 grid((nP + FT_ROWS - 1) / FT_ROWS + pc.N, nsplit), block(FT_WAVES * 64);
#define MIXLORA_FWD(KSR_, NQ_)                                                                   \
  hipLaunchKernelGGL((swiglu_fwd_mfma_kernel<KSR_, NQ_>), grid, block, 0, st, pc, f, s,           \
                     (const bf16_t *)G, (const bf16_t *)U, Pg_all, Pu_all, (const bf16_t *)B_gate, \
                     (const bf16_t *)B_up, (const bf16_t *)A_down, (bf16_t *)a_grp, Q_part, nsplit)
  if (pc.r <= 16) MIXLORA_FWD(1, 1);
  else if (pc.r <= 32) MIXLORA_FWD(2, 1);
  else MIXLORA_FWD(4, 2);
#undef MIXLORA_FWD
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int64_t n = (int64_t)nP * pc.r;
  hipLaunchKernelGGL(reduce_rank_parts_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                     pc, Q_part, nsplit, Q_all);
  return hipGetLastError();
}

hipError_t launch_swiglu_bwd_mfma(const PairCtx &pc, int f, float s, const void *G, const void *U,
                                  const void *H, const float *Pg_all, const float *Pu_all,
                                  const float *VB_all, const void *B_gate, const void *B_up,
                                  const void *AdT, const void *BgT, const void *BuT, void *dg_grp,
                                  void *du_grp, float *dw_part, float *rank_part, float *TG_all,
                                  float *TU_all, hipStream_t st) {
  const int nP = pc.T * pc.k, nsplit = fused_splits(f);
  float *TG_part = rank_part, *TU_part = rank_part + (size_t)8 * nP * pc.r;
  const dim3 grid((nP + FT_ROWS - 1) / FT_ROWS + pc.N, nsplit), block(FT_WAVES * 64);
#define MIXLORA_BWD(KSR_, NQ_)                                                                   \
  hipLaunchKernelGGL((swiglu_bwd_mfma_kernel<KSR_, NQ_>), grid, block, 0, st, pc, f, s,           \
                     (const bf16_t *)G, (const bf16_t *)U, (const bf16_t *)H, Pg_all, Pu_all,      \
                     VB_all, (const bf16_t *)B_gate, (const bf16_t *)B_up, (const bf16_t *)AdT,    \
                     (const bf16_t *)BgT, (const bf16_t *)BuT, (bf16_t *)dg_grp, (bf16_t *)du_grp, \
                     dw_part, TG_part, TU_part, nsplit)
  if (pc.r <= 16) MIXLORA_BWD(1, 1);
  else if (pc.r <= 32) MIXLORA_BWD(2, 1);
  else MIXLORA_BWD(4, 2);
#undef MIXLORA_BWD
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int64_t n = (int64_t)nP * pc.r;
  const dim3 rgrid((unsigned)((n + 255) / 256));
  hipLaunchKernelGGL(reduce_rank_parts_kernel, rgrid, dim3(256), 0, st, pc, TG_part, nsplit, TG_all);
  hipLaunchKernelGGL(reduce_rank_parts_kernel, rgrid, dim3(256), 0, st, pc, TU_part, nsplit, TU_all);
  return hipGetLastError();
}

}  // namespace mixlora
