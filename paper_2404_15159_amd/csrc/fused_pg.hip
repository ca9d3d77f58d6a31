// Per-pair stages (Algorithm 1 lines 11-15 and their backward) on token tiles whose tokens all
// share one unordered pair of experts {a, b} (top-2 routing, bf16, MFMA).
//
// The grouped stages of csrc/fused.hip work on rows grouped by expert: a token's two pairs fall
// into different tiles, so the shared projections G, U of a token are read twice and the weighted
// combination of its two pairs (Eq. 6, moved in front of the linear frozen down projection) needs
// another pass over the grouped rows.  Here the TOKENS are grouped by their unordered expert pair
// instead (csrc/router.hip), 32 tokens of one group to a tile.  A wavefront owns a 32-token x
// 64-column piece for both experts: G and U are fetched and unpacked once, each expert's rank-r
// deltas are one MFMA per 32-column block, and the two activations are still in registers when
// their weighted sum is formed.  Per-pair outputs (a, rank-r partial sums) go to the
// expert-grouped rows that the backward stages and gradient sums read.
//
// The forward kernel spends about 31 vector instructions per token and column for both experts
// and the combination, where the expert-grouped kernel plus the combine pass spent about 56; what
// it mostly does, though, is wait for memory (its time does not change with the shader clock), so
// the next piece's operands are requested a whole piece ahead and the grid is cut into few, long
// workgroups (fused_pg_splits).  The backward kernel keeps one wavefront per expert (two roles per
// tile) and forms the per-token sums of dg and du from the two roles' LDS tiles.
//
// Lane roles, LDS tiles and MFMA fragment layout are those of csrc/fused.hip.
#include "fused_common.h"

namespace mixlora {

// Uniform base + 32-bit BYTE offset: the form the hardware addresses with a scalar base and one
// vector register, so the loop carries no 64-bit address arithmetic.
__device__ __forceinline__ bf16x8_t ldg8(const bf16_t *base, uint32_t byte_off) {
  return *reinterpret_cast<const bf16x8_t *>(reinterpret_cast<const char *>(base) + byte_off);
}
__device__ __forceinline__ void stg8(bf16_t *base, uint32_t byte_off, const bf16x8_t &v) {
  *reinterpret_cast<bf16x8_t *>(reinterpret_cast<char *>(base) + byte_off) = v;
}

static_assert(PG_TILE_ROWS == FT_ROWS, "the grouping kernel cuts tiles of FT_ROWS tokens");

// Forward.  Per pair: a_grp[row(t, j), :] (when write_a), Q_part[split][row(t, j)][q]; per token:
// a_comb[t, :] = w_ta a_ta + w_tb a_tb (the lower-numbered expert's term first, fp32, one rounding).
//
// One wavefront owns a 32-token x 64-column piece for BOTH experts of the tile: G and U are loaded
// and unpacked once, the two experts' rank-r deltas come from four LDS tiles, the two activations
// stay in registers until their weighted sum is stored.  Wavefronts never wait for each other
// inside the loop.  Offsets into the [T, f] / [2T, f] arrays are 32-bit (host check).
template <int KSR, int NQ>
__global__ __launch_bounds__(FT_WAVES * 64, 2) void swiglu_fwd_pg_kernel(
    PairCtx pc, int f, float s, const int32_t *__restrict__ tok_of_pos,
    const int32_t *__restrict__ tile_info, const int32_t *__restrict__ ntiles,
    const bf16_t *__restrict__ G, const bf16_t *__restrict__ U, const float *__restrict__ Pg_all,
    const float *__restrict__ Pu_all, const bf16_t *__restrict__ B_gate,
    const bf16_t *__restrict__ B_up, const bf16_t *__restrict__ A_down, bf16_t *__restrict__ a_grp,
    bf16_t *__restrict__ a_comb, float *__restrict__ Q_part, int nsplit, int write_a) {
  constexpr int TILES = 4;   // per wavefront: gate and up delta tiles of expert a, then of expert b
  extern __shared__ __align__(16) unsigned char lds[];   // pg_fwd_lds(NQ) bytes
  __shared__ int growmap[2][FT_ROWS];   // expert-grouped row of every tile row, per expert
  if ((int)blockIdx.x >= ntiles[0]) return;
  const int32_t *ti = tile_info + (int64_t)blockIdx.x * 4;
  const int r = pc.r, R = pc.N * r, nP = pc.T * 2;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l31 = lane & 31, hi = lane >> 5, rr = lane >> 3, cc = lane & 7;
  const int gid = ti[0], row0 = ti[1], rows = ti[2];
  const int ex[2] = {gid / pc.N, gid % pc.N};
  bf16_t *tiles = reinterpret_cast<bf16_t *>(lds) + wave * TILES * FT_TILE;

  // MFMA role: second-operand fragments of this lane's row (token), per expert
  bf16x8_t pg[2][KSR], pu[2][KSR];
  {
    const int64_t tm = tok_of_pos[row0 + (l31 < rows ? l31 : 0)];
#pragma unroll
    for (int x = 0; x < 2; x++)
#pragma unroll
      for (int ks = 0; ks < KSR; ks++) {
        const int q0 = ks * 16 + hi * 8;
        const bool v = q0 < r;
        pg[x][ks] = cvt8(Pg_all + tm * R + ex[x] * r + (v ? q0 : 0), v, s);
        pu[x][ks] = cvt8(Pu_all + tm * R + ex[x] * r + (v ? q0 : 0), v, s);
      }
  }
  // row-major role: the four rows (8p + rr) this lane serves
  uint32_t gsrc[4], adst[2][4];
  float wx[2][4];
  bool rvalid[4];
#pragma unroll
  for (int p = 0; p < 4; p++) {
    const int rl = 8 * p + rr;
    rvalid[p] = rl < rows;
    const int64_t tok = tok_of_pos[row0 + (rvalid[p] ? rl : 0)];
    const int slot_a = pc.idx[tok * 2] == ex[0] ? 0 : 1;   // expert a's slot of this token
    gsrc[p] = (uint32_t)(tok * f) * 2u;   // bytes
#pragma unroll
    for (int x = 0; x < 2; x++) {
      const int64_t pair = tok * 2 + (slot_a ^ x);
      const int grow = pc.row_of_pair[pair];
      adst[x][p] = (uint32_t)grow * (uint32_t)f * 2u;
      wx[x][p] = pc.w[pair];
      if (cc == 0 && wave == 0) growmap[x][rl] = grow;
    }
  }
  f32x16_t accq[2][NQ];
#pragma unroll
  for (int x = 0; x < 2; x++)
#pragma unroll
    for (int j = 0; j < NQ; j++)
#pragma unroll
      for (int i = 0; i < 16; i++) accq[x][j][i] = 0.f;

  const int nsb = (f + FT_SB - 1) / FT_SB;
  const int per = (nsb + nsplit - 1) / nsplit;
  const int sb_lo = blockIdx.y * per;
  const int sb_hi = sb_lo + per < nsb ? sb_lo + per : nsb;
  const bf16_t *bg_e[2], *bu_e[2], *ad_e[2];
#pragma unroll
  for (int x = 0; x < 2; x++) {
    bg_e[x] = B_gate + (int64_t)ex[x] * f * r;
    bu_e[x] = B_up + (int64_t)ex[x] * f * r;
    ad_e[x] = A_down + (int64_t)ex[x] * r * f;
  }

  bf16x8_t wg[2][2][KSR], wu[2][2][KSR], wf[2][4][NQ], gnx[4], unx[4];
  auto load_w = [&](int c0) {
#pragma unroll
    for (int b = 0; b < 2; b++) {
      int col = c0 + 32 * b + l31;
      col = col < f ? col : f - 1;
#pragma unroll
      for (int ks = 0; ks < KSR; ks++) {
        const int q0 = ks * 16 + hi * 8;
        const uint32_t o = ((uint32_t)col * (uint32_t)r + (q0 < r ? q0 : 0)) * 2u;
#pragma unroll
        for (int x = 0; x < 2; x++) {
          wg[x][b][ks] = ldg8(bg_e[x], o);
          wu[x][b][ks] = ldg8(bu_e[x], o);
        }
      }
    }
  };
  auto load_wf = [&](int c0) {
#pragma unroll
    for (int s4 = 0; s4 < 4; s4++)
#pragma unroll
      for (int j = 0; j < NQ; j++) {
        const int q = j * 32 + l31;
        int col = c0 + 16 * s4 + 8 * hi;
        col = col < f ? col : f - 8;
        const uint32_t o = ((uint32_t)(q < r ? q : 0) * (uint32_t)f + col) * 2u;
#pragma unroll
        for (int x = 0; x < 2; x++) wf[x][s4][j] = ldg8(ad_e[x], o);
      }
  };
  auto col_of = [&](int c0) { const int c = c0 + 8 * cc; return (uint32_t)(c < f ? c : f - 8) * 2u; };   // bytes
  if (sb_lo + wave < sb_hi) {
    const int cf = (sb_lo + wave) * FT_SB;
    load_w(cf);
#pragma unroll
    for (int p = 0; p < 4; p++) {
      gnx[p] = ldg8(G, gsrc[p] + col_of(cf));
      unx[p] = ldg8(U, gsrc[p] + col_of(cf));
    }
    load_wf(cf);
  }
  for (int sb = sb_lo + wave; sb < sb_hi; sb += FT_WAVES) {
    const int c0 = sb * FT_SB;
    const int cn = sb + FT_WAVES < sb_hi ? c0 + FT_WAVES * FT_SB : c0;   // next (or again this)
    const bool tail = c0 + FT_SB > f;
    const uint32_t col = (c0 + 8 * cc) * 2u;   // bytes
    const bool cvalid = c0 + 8 * cc < f;
    // The next piece's shared projections, requested a whole piece before they are needed and
    // moved into (gnx, unx) at the end of this one.  Requested inside the row loop instead (into
    // the registers each row frees) they are copied into place at the loop's back edge while
    // still in flight, and the wavefront waits there: measured 156 against 148 us.
    bf16x8_t gny[4], uny[4];
#pragma unroll
    for (int p = 0; p < 4; p++) {
      gny[p] = ldg8(G, gsrc[p] + col_of(cn));
      uny[p] = ldg8(U, gsrc[p] + col_of(cn));
    }
    __builtin_amdgcn_sched_barrier(0);
    // rank-r deltas of both experts and both 32-column blocks -> LDS tiles
#pragma unroll
    for (int x = 0; x < 2; x++)
#pragma unroll
      for (int b = 0; b < 2; b++) {
        f32x16_t dg, du;
#pragma unroll
        for (int i = 0; i < 16; i++) dg[i] = du[i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KSR; ks++) {
          dg = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wg[x][b][ks], pg[x][ks], dg, 0, 0, 0);
          du = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wu[x][b][ks], pu[x][ks], du, 0, 0, 0);
        }
        tile_put(tiles + (2 * x) * FT_TILE, l31, hi, 32 * b, dg);
        tile_put(tiles + (2 * x + 1) * FT_TILE, l31, hi, 32 * b, du);
      }
    load_w(cn);
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int p = 0; p < 4; p++) {
      const int toff = (8 * p + rr) * FT_PITCH + 8 * cc;
      const bf16x8_t gv = gnx[p], uv = unx[p];
      float gf[8], uf[8], comb[8];
#pragma unroll
      for (int m = 0; m < 8; m++) {
        gf[m] = (float)gv[m];
        uf[m] = (float)uv[m];
      }
#pragma unroll
      for (int x = 0; x < 2; x++) {
        bf16_t *tp = tiles + (2 * x) * FT_TILE + toff;
        const bf16x8_t dgl = ld8(tp), dul = ld8(tp + FT_TILE);
        bf16x8_t av;
#pragma unroll
        for (int m = 0; m < 8; m++) {
          const float gg = gf[m] + (float)dgl[m];
          const float uu = uf[m] + (float)dul[m];
          const float a = gg * fsigmoid(gg) * uu;   // columns past f: finite, meet zeroed weights
          av[m] = (bf16_t)a;
          comb[m] = x == 0 ? wx[0][p] * a : fmaf(wx[1][p], a, comb[m]);
        }
        if (write_a && rvalid[p] && cvalid) stg8(a_grp, adst[x][p] + col, av);
        *reinterpret_cast<bf16x8_t *>(tp) = av;
      }
      if (rvalid[p] && cvalid) {
        bf16x8_t o;
#pragma unroll
        for (int m = 0; m < 8; m++) o[m] = (bf16_t)comb[m];
        stg8(a_comb, gsrc[p] + col, o);
      }
    }
    __builtin_amdgcn_wave_barrier();
    // Q_x += a_x[rows, 64 cols] * A_down[e_x, q, same cols]^T : four K steps of 16 columns
#pragma unroll
    for (int s4 = 0; s4 < 4; s4++) {
      const bool zero_w = tail && c0 + 16 * s4 + 8 * hi >= f;
#pragma unroll
      for (int x = 0; x < 2; x++) {
        const bf16x8_t af = ld8(tiles + (2 * x) * FT_TILE + l31 * FT_PITCH + 16 * s4 + 8 * hi);
#pragma unroll
        for (int j = 0; j < NQ; j++) {
          bf16x8_t w = wf[x][s4][j];
          if (zero_w) w = zero8();
          accq[x][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, w, accq[x][j], 0, 0, 0);
        }
      }
    }
    load_wf(cn);
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int p = 0; p < 4; p++) {
      gnx[p] = gny[p];
      unx[p] = uny[p];
    }
  }
  // accq[x][j][i]: row 8*(i/4) + 4*hi + i%4 of the tile, q = j*32 + l31.  Each wavefront parks its
  // sums in its own (now dead) tile space; then the four are added in a fixed order.
  static_assert(sizeof(float) * 2 * NQ * 16 * 64 <= sizeof(bf16_t) * TILES * FT_TILE, "reduction space");
  float *mine = reinterpret_cast<float *>(tiles);
#pragma unroll
  for (int x = 0; x < 2; x++)
#pragma unroll
    for (int j = 0; j < NQ; j++)
#pragma unroll
      for (int i = 0; i < 16; i++) mine[((x * NQ + j) * 16 + i) * 64 + lane] = accq[x][j][i];
  __syncthreads();
  const int wstride = TILES * FT_TILE / 2;   // floats between two wavefronts' spaces
  const float *base = reinterpret_cast<const float *>(lds);
  for (int idx2 = threadIdx.x; idx2 < 2 * NQ * 16 * 64; idx2 += FT_WAVES * 64) {
    const int x = idx2 / (NQ * 16 * 64), j = (idx2 / (16 * 64)) % NQ, i = (idx2 / 64) % 16, ln = idx2 % 64;
    const int q = j * 32 + (ln & 31);
    const int rl = 8 * (i >> 2) + 4 * (ln >> 5) + (i & 3);
    if (q < r && rl < rows) {
      const float v = (base[idx2] + base[wstride + idx2]) + (base[2 * wstride + idx2] + base[3 * wstride + idx2]);
      Q_part[((int64_t)blockIdx.y * nP + growmap[x][rl]) * r + q] = v;
    }
  }
}

static size_t pg_fwd_lds(int) { return (size_t)FT_WAVES * 4 * FT_TILE * sizeof(bf16_t); }

// Backward of the stage above on the same token tiles.  A workgroup of eight wavefronts owns a
// tile: wavefronts 0-3 ("role A") treat it as 32 rows of expert a, wavefronts 4-7 ("role B") as 32
// rows of expert b, each exactly as the expert-grouped kernel of csrc/fused.hip treats a row tile
// (same MFMA products, same element math, same per-pair outputs dg_grp, du_grp, dw_part, TG_part,
// TU_part on the expert-grouped rows); wavefront w of either role walks super-blocks w, w + 4, ...
// of the workgroup's column range, so both roles hold the same 32 x 64 piece at the same time.
// After a workgroup barrier role A adds role B's dg and du tiles (LDS) to its own and writes the
// per-token sums  dgsum[t] = dg_ta + dg_tb, dusum[t] = du_ta + du_tb  that the input-gradient GEMM
// reads: no pass over the grouped rows follows, and the second fetch of G, U, H hits in cache.
template <int KSR, int NQ>
__global__ __launch_bounds__(2 * FT_WAVES * 64, 1) void swiglu_bwd_pg_kernel(
    PairCtx pc, int f, float s, const int32_t *__restrict__ tok_of_pos,
    const int32_t *__restrict__ tile_info, const int32_t *__restrict__ ntiles,
    const bf16_t *__restrict__ G, const bf16_t *__restrict__ U, const bf16_t *__restrict__ H,
    const float *__restrict__ Pg_all, const float *__restrict__ Pu_all,
    const float *__restrict__ VB_all, const bf16_t *__restrict__ B_gate,
    const bf16_t *__restrict__ B_up, const bf16_t *__restrict__ AdT, const bf16_t *__restrict__ BgT,
    const bf16_t *__restrict__ BuT, bf16_t *__restrict__ dg_grp, bf16_t *__restrict__ du_grp,
    bf16_t *__restrict__ dgsum, bf16_t *__restrict__ dusum, float *__restrict__ dw_part,
    float *__restrict__ TG_part, float *__restrict__ TU_part, int nsplit) {
  constexpr int TILES = 3;
  extern __shared__ __align__(16) unsigned char lds[];   // pg_bwd_lds(NQ) bytes
  __shared__ float dwred[2 * FT_WAVES][FT_ROWS];
  __shared__ int growmap[2][FT_ROWS];
  if ((int)blockIdx.x >= ntiles[0]) return;
  const int32_t *ti = tile_info + (int64_t)blockIdx.x * 4;
  const int r = pc.r, R = pc.N * r, nP = pc.T * 2;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int role = wave >> 2, w4 = wave & 3;
  const int l31 = lane & 31, hi = lane >> 5, rr = lane >> 3, cc = lane & 7;
  const int gid = ti[0], row0 = ti[1], rows = ti[2];
  const int e = role ? gid % pc.N : gid / pc.N;
  bf16_t *tg = reinterpret_cast<bf16_t *>(lds) + wave * TILES * FT_TILE;
  bf16_t *tu = tg + FT_TILE, *td = tu + FT_TILE;
  const bf16_t *tg_b = reinterpret_cast<const bf16_t *>(lds) + (wave ^ 4) * TILES * FT_TILE;
  const bf16_t *tu_b = tg_b + FT_TILE;

  bf16x8_t pg[KSR], pu[KSR], vw[KSR];
  {
    const int64_t tm = tok_of_pos[row0 + (l31 < rows ? l31 : 0)];
    const float wm = pc.w[tm * 2 + (pc.idx[tm * 2] == e ? 0 : 1)];
#pragma unroll
    for (int ks = 0; ks < KSR; ks++) {
      const int q0 = ks * 16 + hi * 8;
      const bool v = q0 < r;
      const int64_t o = tm * R + e * r + (v ? q0 : 0);
      pg[ks] = cvt8(Pg_all + o, v, s);
      pu[ks] = cvt8(Pu_all + o, v, s);
      vw[ks] = cvt8(VB_all + o, v, wm * s);
    }
  }
  uint32_t gsrc[4], odst[4];   // byte offsets of the token row / the pair's grouped row
  float wrow[4], dwacc[4];
  bool rvalid[4];
#pragma unroll
  for (int p = 0; p < 4; p++) {
    const int rl = 8 * p + rr;
    rvalid[p] = rl < rows;
    const int64_t tok = tok_of_pos[row0 + (rvalid[p] ? rl : 0)];
    const int64_t pair = tok * 2 + (pc.idx[tok * 2] == e ? 0 : 1);
    const int grow = pc.row_of_pair[pair];
    gsrc[p] = (uint32_t)(tok * f) * 2u;
    odst[p] = (uint32_t)grow * (uint32_t)f * 2u;
    wrow[p] = pc.w[pair];
    dwacc[p] = 0.f;
    if (cc == 0 && w4 == 0) growmap[role][rl] = grow;
  }
  f32x16_t acctg[NQ], acctu[NQ];
#pragma unroll
  for (int j = 0; j < NQ; j++)
#pragma unroll
    for (int i = 0; i < 16; i++) acctg[j][i] = acctu[j][i] = 0.f;

  const int nsb = (f + FT_SB - 1) / FT_SB;
  const int per = (nsb + nsplit - 1) / nsplit;
  const int sb_lo = blockIdx.y * per;
  const int sb_hi = sb_lo + per < nsb ? sb_lo + per : nsb;
  const int iters = (per + FT_WAVES - 1) / FT_WAVES;   // the same for every wavefront: barriers inside
  const bf16_t *bg_e = B_gate + (int64_t)e * f * r;
  const bf16_t *bu_e = B_up + (int64_t)e * f * r;
  const bf16_t *ad_e = AdT + (int64_t)e * f * r;
  const bf16_t *bgt_e = BgT + (int64_t)e * r * f;
  const bf16_t *but_e = BuT + (int64_t)e * r * f;

  bf16x8_t wg[2][KSR], wu[2][KSR], wd[2][KSR], tgw[4][NQ], tuw[4][NQ], gnx[4], unx[4], hnx[4];
  auto load_w = [&](int c0) {
#pragma unroll
    for (int b = 0; b < 2; b++) {
      int col = c0 + 32 * b + l31;
      col = col < f ? col : f - 1;
#pragma unroll
      for (int ks = 0; ks < KSR; ks++) {
        const int q0 = ks * 16 + hi * 8;
        const uint32_t o = ((uint32_t)col * (uint32_t)r + (q0 < r ? q0 : 0)) * 2u;
        wg[b][ks] = ldg8(bg_e, o);
        wu[b][ks] = ldg8(bu_e, o);
        wd[b][ks] = ldg8(ad_e, o);
      }
    }
  };
  auto load_wt = [&](int c0) {
#pragma unroll
    for (int s4 = 0; s4 < 4; s4++)
#pragma unroll
      for (int j = 0; j < NQ; j++) {
        const int q = j * 32 + l31;
        int col = c0 + 16 * s4 + 8 * hi;
        col = col < f ? col : f - 8;
        const uint32_t o = ((uint32_t)(q < r ? q : 0) * (uint32_t)f + col) * 2u;
        tgw[s4][j] = ldg8(bgt_e, o);
        tuw[s4][j] = ldg8(but_e, o);
      }
  };
  auto col_of = [&](int c0) { const int c = c0 + 8 * cc; return (uint32_t)(c < f ? c : f - 8) * 2u; };
  {
    const int sb_first = sb_lo + w4 < sb_hi ? sb_lo + w4 : (nsb - 1);
    load_w(sb_first * FT_SB);
#pragma unroll
    for (int p = 0; p < 4; p++) {
      const uint32_t o = gsrc[p] + col_of(sb_first * FT_SB);
      gnx[p] = ldg8(G, o);
      unx[p] = ldg8(U, o);
      hnx[p] = ldg8(H, o);
    }
    load_wt(sb_first * FT_SB);
  }

  for (int it = 0; it < iters; it++) {
    const int sb = sb_lo + w4 + it * FT_WAVES;
    const bool live = sb < sb_hi;            // wave-uniform; the same for both roles of a pair
    const int c0 = (live ? sb : nsb - 1) * FT_SB;
    const int cn = sb + FT_WAVES < sb_hi ? c0 + FT_WAVES * FT_SB : c0;
    const bool tail = c0 + FT_SB > f;
    const uint32_t col = (uint32_t)(c0 + 8 * cc) * 2u;
    const bool cvalid = c0 + 8 * cc < f;
    if (live) {
#pragma unroll
      for (int b = 0; b < 2; b++) {
        f32x16_t dgm, dum, ddm;
#pragma unroll
        for (int i = 0; i < 16; i++) dgm[i] = dum[i] = ddm[i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KSR; ks++) {
          dgm = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wg[b][ks], pg[ks], dgm, 0, 0, 0);
          dum = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wu[b][ks], pu[ks], dum, 0, 0, 0);
          ddm = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wd[b][ks], vw[ks], ddm, 0, 0, 0);
        }
        tile_put(tg, l31, hi, 32 * b, dgm);
        tile_put(tu, l31, hi, 32 * b, dum);
        tile_put(td, l31, hi, 32 * b, ddm);
      }
      load_w(cn);
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int p = 0; p < 4; p++) {
        const int lo = (8 * p + rr) * FT_PITCH + 8 * cc;
        const bf16x8_t dgl = ld8(tg + lo), dul = ld8(tu + lo), ddl = ld8(td + lo);
        const bf16x8_t gv = gnx[p], uv = unx[p], hv = hnx[p];
        bf16x8_t dgv, duv;
        float part = 0.f;
#pragma unroll
        for (int m = 0; m < 8; m++) {
          const float gg = (float)gv[m] + (float)dgl[m];
          const float uu = (float)uv[m] + (float)dul[m];
          const float hh = (float)hv[m];
          const float sg = fsigmoid(gg);
          const float da = wrow[p] * hh + (float)ddl[m];
          const float gs = gg * sg;                       // SiLU(g)
          part = fmaf(hh, gs * uu, part);
          // d SiLU / dg = sig (1 + g (1 - sig)) = sig + SiLU(g) (1 - sig)
          dgv[m] = (bf16_t)((da * uu) * fmaf(gs, 1.f - sg, sg));
          duv[m] = (bf16_t)(da * gs);
          // columns past f hold finite values of clamped loads; they meet zeroed weights in the
          // rank-r products below and are never stored
        }
        if (cvalid) dwacc[p] += part;
        {
          const uint32_t o = gsrc[p] + col_of(cn);
          gnx[p] = ldg8(G, o);
          unx[p] = ldg8(U, o);
          hnx[p] = ldg8(H, o);
        }
        if (rvalid[p] && cvalid) {
          stg8(dg_grp, odst[p] + col, dgv);
          stg8(du_grp, odst[p] + col, duv);
        }
        *reinterpret_cast<bf16x8_t *>(tg + lo) = dgv;
        *reinterpret_cast<bf16x8_t *>(tu + lo) = duv;
      }
    }
    __syncthreads();   // both roles' dg / du tiles of this piece are complete
    if (live) {
      if (role == 0) {
        // per-token sums over the two pairs (bf16 values added in fp32, rounded once)
#pragma unroll
        for (int p = 0; p < 4; p++) {
          if (rvalid[p] && cvalid) {
            const int lo = (8 * p + rr) * FT_PITCH + 8 * cc;
            const bf16x8_t ga = ld8(tg + lo), gb = ld8(tg_b + lo), ua = ld8(tu + lo), ub = ld8(tu_b + lo);
            bf16x8_t gs8, us8;
#pragma unroll
            for (int m = 0; m < 8; m++) {
              gs8[m] = (bf16_t)((float)ga[m] + (float)gb[m]);
              us8[m] = (bf16_t)((float)ua[m] + (float)ub[m]);
            }
            stg8(dgsum, gsrc[p] + col, gs8);
            stg8(dusum, gsrc[p] + col, us8);
          }
        }
      }
#pragma unroll
      for (int s4 = 0; s4 < 4; s4++) {
        const bf16x8_t fg = ld8(tg + l31 * FT_PITCH + 16 * s4 + 8 * hi);
        const bf16x8_t fu = ld8(tu + l31 * FT_PITCH + 16 * s4 + 8 * hi);
#pragma unroll
        for (int j = 0; j < NQ; j++) {
          bf16x8_t wgt = tgw[s4][j], wut = tuw[s4][j];
          if (tail && c0 + 16 * s4 + 8 * hi >= f) wgt = wut = zero8();
          acctg[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fg, wgt, acctg[j], 0, 0, 0);
          acctu[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fu, wut, acctu[j], 0, 0, 0);
        }
      }
      load_wt(cn);
    }
    __syncthreads();   // the tiles may be overwritten by the next piece
  }
  // <H, a> per row: add the 8 column chunks (lanes cc = 0..7 of a row), then the role's 4 waves
#pragma unroll
  for (int p = 0; p < 4; p++) {
    float v = dwacc[p];
    v += __shfl_xor(v, 1, 64);
    v += __shfl_xor(v, 2, 64);
    v += __shfl_xor(v, 4, 64);
    if (cc == 0) dwred[wave][8 * p + rr] = v;
  }
  float(*red)[NQ][16][64] = reinterpret_cast<float(*)[NQ][16][64]>(lds);
  const int t4 = threadIdx.x & (FT_WAVES * 64 - 1);   // thread within the role
  const int wv0 = role * FT_WAVES;
  for (int bank = 0; bank < 2; bank++) {
    __syncthreads();   // tiles (first pass) or the previous bank's sums are no longer read
#pragma unroll
    for (int j = 0; j < NQ; j++)
#pragma unroll
      for (int i = 0; i < 16; i++) red[wave][j][i][lane] = bank == 0 ? acctg[j][i] : acctu[j][i];
    __syncthreads();
    float *out = bank == 0 ? TG_part : TU_part;
    for (int idx2 = t4; idx2 < NQ * 16 * 64; idx2 += FT_WAVES * 64) {
      const int j = idx2 / (16 * 64), i = (idx2 / 64) % 16, ln = idx2 % 64;
      const int q = j * 32 + (ln & 31);
      const int rl = 8 * (i >> 2) + 4 * (ln >> 5) + (i & 3);
      if (q < r && rl < rows) {
        const float v = (red[wv0][j][i][ln] + red[wv0 + 1][j][i][ln]) +
                        (red[wv0 + 2][j][i][ln] + red[wv0 + 3][j][i][ln]);
        out[((int64_t)blockIdx.y * nP + growmap[role][rl]) * r + q] = v;
      }
    }
  }
  if (t4 < rows)
    dw_part[(int64_t)growmap[role][t4] * nsplit + blockIdx.y] =
        (dwred[wv0][t4] + dwred[wv0 + 1][t4]) + (dwred[wv0 + 2][t4] + dwred[wv0 + 3][t4]);
}

static size_t pg_bwd_lds(int NQ) {
  const size_t tiles = (size_t)2 * FT_WAVES * 3 * FT_TILE * sizeof(bf16_t);
  const size_t red = (size_t)2 * FT_WAVES * NQ * 16 * 64 * sizeof(float);
  return tiles > red ? tiles : red;
}

bool fused_pg_ok(const PairCtx &pc, int f) {
  return pc.k == 2 && pc.N <= PG_MAX_EXPERTS && pc.r <= 16 && pc.T > 128 && pc.T <= PG_MAX_TOKENS &&
         f >= 64 && (int64_t)2 * pc.T * f < ((int64_t)1 << 31);
}

int fused_pg_max_tiles(int T, int N) { return (T + FT_ROWS - 1) / FT_ROWS + N * N; }

// Column splits (grid.y).  Measured at the LLaMA shapes: a workgroup pays a few microseconds of
// set-up (metadata chain, first fetches) and of final reduction, so few long workgroups beat many
// short ones, and best of all is a grid that fits the chip in one round (two 4-wave workgroups
// per compute unit: 512 slots).  tiles = T / 32 plus half a ragged tile per pair group.
int fused_pg_splits(int f, int T, int N) {
  const int nblk = (f + FT_SB - 1) / FT_SB;
  const int tiles = (T + FT_ROWS - 1) / FT_ROWS + N * (N - 1) / 4;
  const int fit = 512 / (tiles > 0 ? tiles : 1);
  int s = fit >= 3 ? (fit < 16 ? fit : 16) : 4;
  while (s > 1 && nblk / s < FT_WAVES) s--;
  return s;
}

hipError_t launch_swiglu_fwd_pg(const PairCtx &pc, int f, float s, const int32_t *tok_of_pos,
                                const int32_t *tile_info, const int32_t *ntiles, const void *G,
                                const void *U, const float *Pg_all, const float *Pu_all,
                                const void *B_gate, const void *B_up, const void *A_down,
                                void *a_grp, void *a_comb, float *Q_part, float *Q_all, void *Qw,
                                int ldqw, int write_a, hipStream_t st) {
  if (!fused_pg_ok(pc, f)) return hipErrorInvalidValue;
  const int nsplit = fused_pg_splits(f, pc.T, pc.N);
  const dim3 grid(fused_pg_max_tiles(pc.T, pc.N), nsplit), block(FT_WAVES * 64);
#define MIXLORA_PGF(KSR_, NQ_)                                                                    \
  do {                                                                                            \
    auto kern = swiglu_fwd_pg_kernel<KSR_, NQ_>;                                                  \
    const size_t lds_ = pg_fwd_lds(NQ_);                                                          \
    static bool attr_set = false;                                                                 \
    if (!attr_set) {                                                                              \
      hipError_t e_ = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),                   \
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_); \
      if (e_ != hipSuccess) return e_;                                                            \
      attr_set = true;                                                                            \
    }                                                                                             \
    hipLaunchKernelGGL(kern, grid, block, lds_, st, pc, f, s, tok_of_pos, tile_info, ntiles,      \
                       (const bf16_t *)G, (const bf16_t *)U, Pg_all, Pu_all,                      \
                       (const bf16_t *)B_gate, (const bf16_t *)B_up, (const bf16_t *)A_down,      \
                       (bf16_t *)a_grp, (bf16_t *)a_comb, Q_part, nsplit, write_a);               \
  } while (0)
  MIXLORA_PGF(1, 1);
#undef MIXLORA_PGF
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_reduce_rank_parts(pc, Q_part, 0, nsplit, Q_all, nullptr, Qw, ldqw, 1, 0, st);
}

hipError_t launch_swiglu_bwd_pg(const PairCtx &pc, int f, float s, const int32_t *tok_of_pos,
                                const int32_t *tile_info, const int32_t *ntiles, const void *G,
                                const void *U, const void *H, const float *Pg_all,
                                const float *Pu_all, const float *VB_all, const void *B_gate,
                                const void *B_up, const void *AdT, const void *BgT, const void *BuT,
                                void *dg_grp, void *du_grp, void *dgsum, void *dusum, float *dw_part,
                                float *rank_part, float *TG_all, float *TU_all, void *S, int ld_s,
                                hipStream_t st) {
  if (!fused_pg_ok(pc, f)) return hipErrorInvalidValue;
  const int nP = pc.T * 2, nsplit = fused_pg_splits(f, pc.T, pc.N);
  float *TG_part = rank_part, *TU_part = rank_part + (size_t)nsplit * nP * pc.r;
  const dim3 grid(fused_pg_max_tiles(pc.T, pc.N), nsplit), block(2 * FT_WAVES * 64);
  auto kern = swiglu_bwd_pg_kernel<1, 1>;   // fused_pg_ok: r <= 16
  const size_t lds_ = pg_bwd_lds(1);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e_ = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_);
    if (e_ != hipSuccess) return e_;
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, grid, block, lds_, st, pc, f, s, tok_of_pos, tile_info, ntiles,
                     (const bf16_t *)G, (const bf16_t *)U, (const bf16_t *)H, Pg_all, Pu_all, VB_all,
                     (const bf16_t *)B_gate, (const bf16_t *)B_up, (const bf16_t *)AdT,
                     (const bf16_t *)BgT, (const bf16_t *)BuT, (bf16_t *)dg_grp, (bf16_t *)du_grp,
                     (bf16_t *)dgsum, (bf16_t *)dusum, dw_part, TG_part, TU_part, nsplit);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_reduce_rank_parts(pc, TG_part, (int64_t)(TU_part - TG_part), nsplit, TG_all, TU_all, S,
                                  ld_s, 0, 0, st);
}

}  // namespace mixlora
