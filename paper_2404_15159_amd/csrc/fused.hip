// bf16 MFMA versions of the per-pair (token, expert) stages, on expert-grouped rows.
//
// A workgroup owns one tile of 32 grouped rows (all of one expert) and a range of 64-column
// super-blocks; each of its 4 wavefronts walks every 4th super-block.  Per 32x32 block the LoRA
// deltas of Algorithm 1 lines 11-12 are one rank-r MFMA each (B_e[cols, r] x P[rows, r]^T, added
// to the shared gate/up projections gathered by token), SiLU * up follows (line 13), and the
// activation tile is multiplied by A_down_e to accumulate the rank-r input of the down
// projection's LoRA (line 14) without re-reading it from memory.
//
// MFMA 32x32x16 layout used throughout: operand lanes carry index (lane % 32) and the 8
// contraction elements of half (lane / 32); result register e of a lane holds
// D[8*(e/4) + 4*(lane/32) + e%4][lane % 32].  For the deltas the FIRST operand is the weight
// fragment (index = column), the SECOND the per-row fragment (index = row), so a lane holds, for
// its row, the 16 columns c0 + 8g + 4*(lane/32) + m (g, m < 4): four 8-byte runs, which go into
// an LDS tile (see below).
#include "fused_common.h"

namespace mixlora {

// Forward: a_grp[row, :] and the per-split partial sums  Q_part[split][row][q] = sum over the
// split's columns of a[row, c] * A_down[e, q, c].
// DORA: g and u are multiplied by the per-expert, per-column factors cg[e, c], cu[e, c]
// (magnitude / row norm of the weight-decomposed projections) before SiLU * up.
template <int KSR, int NQ, bool DORA>
__global__ __launch_bounds__(FT_WAVES * 64, KSR == 1 ? 3 : 1) void swiglu_fwd_mfma_kernel(
    PairCtx pc, int f, float s, const bf16_t *__restrict__ G, const bf16_t *__restrict__ U,
    const float *__restrict__ Pg_all, const float *__restrict__ Pu_all,
    const bf16_t *__restrict__ B_gate, const bf16_t *__restrict__ B_up,
    const bf16_t *__restrict__ A_down, bf16_t *__restrict__ a_grp, float *__restrict__ Q_part,
    int nsplit, int rows_mode, DoraArgs dora) {
  constexpr int TILES = 2;
  constexpr int LDS_BYTES = FT_WAVES * TILES * FT_TILE * 2 > FT_WAVES * NQ * 16 * 64 * 4
                                ? FT_WAVES * TILES * FT_TILE * 2 : FT_WAVES * NQ * 16 * 64 * 4;
  __shared__ __align__(16) unsigned char lds[LDS_BYTES];
  int e, row0, rows;
  if (!fused_tile_rows(pc.offs, pc.N, blockIdx.x, e, row0, rows)) return;
  const int r = pc.r, R = pc.N * r, nP = pc.T * pc.k;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l31 = lane & 31, hi = lane >> 5, rr = lane >> 3, cc = lane & 7;
  bf16_t *tg = reinterpret_cast<bf16_t *>(lds) + wave * TILES * FT_TILE;
  bf16_t *tu = tg + FT_TILE;

  // MFMA role: second-operand fragments of this lane's row
  bf16x8_t pg[KSR], pu[KSR];
  {
    const int64_t tm = pc.pair_of_row[row0 + (l31 < rows ? l31 : 0)] / pc.k;
#pragma unroll
    for (int ks = 0; ks < KSR; ks++) {
      const int q0 = ks * 16 + hi * 8;
      const bool v = q0 < r;
      pg[ks] = cvt8(Pg_all + tm * R + e * r + (v ? q0 : 0), v, s);
      pu[ks] = cvt8(Pu_all + tm * R + e * r + (v ? q0 : 0), v, s);
    }
  }
  // row-major role: the four rows (8p + rr) this lane serves
  int64_t gsrc[4], adst[4];
  bool rvalid[4];
#pragma unroll
  for (int p = 0; p < 4; p++) {
    const int rl = 8 * p + rr;
    rvalid[p] = rl < rows;
    const int row = row0 + (rvalid[p] ? rl : 0);
    gsrc[p] = (int64_t)((rows_mode & ROWS_GU) ? row : pc.pair_of_row[row] / pc.k) * f;
    adst[p] = (int64_t)row * f;
  }
  f32x16_t accq[NQ];
#pragma unroll
  for (int j = 0; j < NQ; j++)
#pragma unroll
    for (int i = 0; i < 16; i++) accq[j][i] = 0.f;

  const int nsb = (f + FT_SB - 1) / FT_SB;
  const int per = (nsb + nsplit - 1) / nsplit;
  const int sb_lo = blockIdx.y * per;
  const int sb_hi = sb_lo + per < nsb ? sb_lo + per : nsb;
  const bf16_t *bg_e = B_gate + (int64_t)e * f * r;
  const bf16_t *bu_e = B_up + (int64_t)e * f * r;
  const bf16_t *ad_e = A_down + (int64_t)e * r * f;

  // software pipeline: everything a super-block needs from memory is requested one iteration
  // ahead, weights first (they are consumed first; loads complete in order)
  bf16x8_t wg[2][KSR], wu[2][KSR], wf[4][NQ], gnx[4], unx[4];
  auto load_w = [&](int c0) {
#pragma unroll
    for (int b = 0; b < 2; b++) {
      int col = c0 + 32 * b + l31;
      col = col < f ? col : f - 1;
#pragma unroll
      for (int ks = 0; ks < KSR; ks++) {
        const int q0 = ks * 16 + hi * 8;
        const int64_t o = (int64_t)col * r + (q0 < r ? q0 : 0);
        wg[b][ks] = ld8(bg_e + o);
        wu[b][ks] = ld8(bu_e + o);
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
        wf[s4][j] = ld8(ad_e + (int64_t)(q < r ? q : 0) * f + col);
      }
  };
  auto col_of = [&](int c0) { const int c = c0 + 8 * cc; return c < f ? c : f - 8; };
  const int sb_first = sb_lo + wave < sb_hi ? sb_lo + wave : (nsb - 1);
  load_w(sb_first * FT_SB);
#pragma unroll
  for (int p = 0; p < 4; p++) {
    gnx[p] = ld8(G + gsrc[p] + col_of(sb_first * FT_SB));
    unx[p] = ld8(U + gsrc[p] + col_of(sb_first * FT_SB));
  }
  load_wf(sb_first * FT_SB);

  for (int sb = sb_lo + wave; sb < sb_hi; sb += FT_WAVES) {
    const int c0 = sb * FT_SB;
    const int cn = sb + FT_WAVES < sb_hi ? c0 + FT_WAVES * FT_SB : c0;   // next (or again this)
    const bool tail = c0 + FT_SB > f;                                    // wave-uniform
    // rank-r deltas of both 32-column blocks -> LDS tiles
#pragma unroll
    for (int b = 0; b < 2; b++) {
      f32x16_t dg, du;
#pragma unroll
      for (int i = 0; i < 16; i++) dg[i] = du[i] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KSR; ks++) {
        // rank entries past r: the row fragments hold zeros there, the weight fragments finite
        // values of clamped loads
        dg = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wg[b][ks], pg[ks], dg, 0, 0, 0);
        du = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wu[b][ks], pu[ks], du, 0, 0, 0);
      }
      tile_put(tg, l31, hi, 32 * b, dg);
      tile_put(tu, l31, hi, 32 * b, du);
    }
    load_w(cn);   // next iteration's delta weights: oldest outstanding loads from here on
    __builtin_amdgcn_wave_barrier();
    // row-major phase
    const int col = c0 + 8 * cc;
    const bool cvalid = col < f;
    float cgv[8], cuv[8];
    if constexpr (DORA) {
      const int64_t o = (int64_t)e * f + col_of(c0);
#pragma unroll
      for (int m = 0; m < 8; m++) { cgv[m] = dora.cg[o + m]; cuv[m] = dora.cu[o + m]; }
    }
#pragma unroll
    for (int p = 0; p < 4; p++) {
      bf16_t *tp = tg + (8 * p + rr) * FT_PITCH + 8 * cc;
      const bf16x8_t dgl = ld8(tp), dul = ld8(tu + (8 * p + rr) * FT_PITCH + 8 * cc);
      const bf16x8_t gv = gnx[p], uv = unx[p];
      bf16x8_t av;
#pragma unroll
      for (int m = 0; m < 8; m++) {
        float gg = (float)gv[m] + (float)dgl[m];
        float uu = (float)uv[m] + (float)dul[m];
        if constexpr (DORA) { gg *= cgv[m]; uu *= cuv[m]; }
        av[m] = (bf16_t)(gg * fsigmoid(gg) * uu);   // columns past f: finite, meet zeroed weights
      }
      gnx[p] = ld8(G + gsrc[p] + col_of(cn));
      unx[p] = ld8(U + gsrc[p] + col_of(cn));
      if (rvalid[p] && cvalid) *reinterpret_cast<bf16x8_t *>(a_grp + adst[p] + col) = av;
      *reinterpret_cast<bf16x8_t *>(tp) = av;
    }
    __builtin_amdgcn_wave_barrier();
    // Q += a[rows, 64 cols] * A_down[e, q, same cols]^T : four K steps of 16 columns
#pragma unroll
    for (int s4 = 0; s4 < 4; s4++) {
      const bf16x8_t af = ld8(tg + l31 * FT_PITCH + 16 * s4 + 8 * hi);
#pragma unroll
      for (int j = 0; j < NQ; j++) {
        // outputs with q >= r are never stored; columns past f (last super-block only) hold
        // finite values in the tile and must meet zeros
        bf16x8_t w = wf[s4][j];
        if (tail && c0 + 16 * s4 + 8 * hi >= f) w = zero8();
        accq[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, w, accq[j], 0, 0, 0);
      }
    }
    load_wf(cn);
    __builtin_amdgcn_wave_barrier();
  }
  // accq[j][i]: row 8*(i/4) + 4*hi + i%4 of the tile, q = j*32 + l31.  Sum the 4 waves.
  __syncthreads();   // the tiles are dead; their space becomes the reduction buffer
  float(*red)[NQ][16][64] = reinterpret_cast<float(*)[NQ][16][64]>(lds);
#pragma unroll
  for (int j = 0; j < NQ; j++)
#pragma unroll
    for (int i = 0; i < 16; i++) red[wave][j][i][lane] = accq[j][i];
  __syncthreads();
  for (int idx = threadIdx.x; idx < NQ * 16 * 64; idx += FT_WAVES * 64) {
    const int j = idx / (16 * 64), i = (idx / 64) % 16, ln = idx % 64;
    const int q = j * 32 + (ln & 31);
    const int rl = 8 * (i >> 2) + 4 * (ln >> 5) + (i & 3);
    if (q < r && rl < rows) {
      const float v = (red[0][j][i][ln] + red[1][j][i][ln]) + (red[2][j][i][ln] + red[3][j][i][ln]);
      Q_part[((int64_t)blockIdx.y * nP + row0 + rl) * r + q] = v;
    }
  }
}

// Backward of the tile above, same ownership and lane roles.
// With H[t] = W_down^T dy[t] and Vw[row] = w_row * B_down[e]^T dy[t]:
//   da = w_row * H[t] + s * A_down[e]^T Vw[row]      (rank-r MFMA on the transposed bank AdT)
//   dg = da * u * sig(g) * (1 + g (1 - sig(g))),  du = da * g * sig(g)   -> dg_grp, du_grp
//   dw_part[row][split]   = sum over the split's columns of H * a
//   TG_part[split][row][q] = sum_c dg[row, c] * B_gate[e, c, q]   (and TU with du, B_up)
// AdT is A_down re-laid [N, f, r]; BgT / BuT are the B banks re-laid [N, r, f].
// DORA: g = cg * (G + delta), u = cu * (U + delta); the gradients written (and used for TG / TU)
// are those of the unscaled projections, cg * dg and cu * du; the sums over the tile's rows of
// dg * (G + delta) and du * (U + delta) go to dm_part_g / dm_part_u [tile][column].
template <int KSR, int NQ, bool DORA>
__global__ __launch_bounds__(FT_WAVES * 64, (KSR == 1 && !DORA) ? 2 : 1) void swiglu_bwd_mfma_kernel(
    PairCtx pc, int f, float s, const bf16_t *__restrict__ G, const bf16_t *__restrict__ U,
    const bf16_t *__restrict__ H, const float *__restrict__ Pg_all,
    const float *__restrict__ Pu_all, const float *__restrict__ VB_all,
    const bf16_t *__restrict__ B_gate, const bf16_t *__restrict__ B_up,
    const bf16_t *__restrict__ AdT, const bf16_t *__restrict__ BgT, const bf16_t *__restrict__ BuT,
    bf16_t *__restrict__ dg_grp, bf16_t *__restrict__ du_grp, float *__restrict__ dw_part,
    float *__restrict__ TG_part, float *__restrict__ TU_part, int nsplit, int rows_mode,
    DoraArgs dora) {
  constexpr int TILES = 3;
  constexpr int LDS_BYTES = FT_WAVES * TILES * FT_TILE * 2 > FT_WAVES * NQ * 16 * 64 * 4
                                ? FT_WAVES * TILES * FT_TILE * 2 : FT_WAVES * NQ * 16 * 64 * 4;
  __shared__ __align__(16) unsigned char lds[LDS_BYTES];
  __shared__ float dwred[FT_WAVES][32];
  int e, row0, rows;
  if (!fused_tile_rows(pc.offs, pc.N, blockIdx.x, e, row0, rows)) return;
  const int r = pc.r, R = pc.N * r, nP = pc.T * pc.k;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l31 = lane & 31, hi = lane >> 5, rr = lane >> 3, cc = lane & 7;
  bf16_t *tg = reinterpret_cast<bf16_t *>(lds) + wave * TILES * FT_TILE;
  bf16_t *tu = tg + FT_TILE, *td = tu + FT_TILE;

  bf16x8_t pg[KSR], pu[KSR], vw[KSR];
  {
    const int pair = pc.pair_of_row[row0 + (l31 < rows ? l31 : 0)];
    const int64_t tm = pair / pc.k;
    const float wm = pc.w[pair];
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
  int64_t gsrc[4], odst[4];
  float wrow[4], dwacc[4];
  bool rvalid[4];
#pragma unroll
  for (int p = 0; p < 4; p++) {
    const int rl = 8 * p + rr;
    rvalid[p] = rl < rows;
    const int row = row0 + (rvalid[p] ? rl : 0);
    const int pair = pc.pair_of_row[row];
    gsrc[p] = (int64_t)((rows_mode & ROWS_GU) ? row : pair / pc.k) * f;
    odst[p] = (int64_t)row * f;
    wrow[p] = pc.w[pair];
    dwacc[p] = 0.f;
  }
  const bool h_by_row = (rows_mode & ROWS_H) != 0;
  f32x16_t acctg[NQ], acctu[NQ];
#pragma unroll
  for (int j = 0; j < NQ; j++)
#pragma unroll
    for (int i = 0; i < 16; i++) acctg[j][i] = acctu[j][i] = 0.f;

  const int nsb = (f + FT_SB - 1) / FT_SB;
  const int per = (nsb + nsplit - 1) / nsplit;
  const int sb_lo = blockIdx.y * per;
  const int sb_hi = sb_lo + per < nsb ? sb_lo + per : nsb;
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
        const int64_t o = (int64_t)col * r + (q0 < r ? q0 : 0);
        wg[b][ks] = ld8(bg_e + o);
        wu[b][ks] = ld8(bu_e + o);
        wd[b][ks] = ld8(ad_e + o);
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
        const int64_t o = (int64_t)(q < r ? q : 0) * f + col;
        tgw[s4][j] = ld8(bgt_e + o);
        tuw[s4][j] = ld8(but_e + o);
      }
  };
  auto col_of = [&](int c0) { const int c = c0 + 8 * cc; return c < f ? c : f - 8; };
  const int sb_first = sb_lo + wave < sb_hi ? sb_lo + wave : (nsb - 1);
  load_w(sb_first * FT_SB);
#pragma unroll
  for (int p = 0; p < 4; p++) {
    const int64_t o = gsrc[p] + col_of(sb_first * FT_SB);
    gnx[p] = ld8(G + o);
    unx[p] = ld8(U + o);
    hnx[p] = ld8(H + (h_by_row ? odst[p] : gsrc[p]) + col_of(sb_first * FT_SB));
  }
  load_wt(sb_first * FT_SB);

  for (int sb = sb_lo + wave; sb < sb_hi; sb += FT_WAVES) {
    const int c0 = sb * FT_SB;
    const int cn = sb + FT_WAVES < sb_hi ? c0 + FT_WAVES * FT_SB : c0;
    const bool tail = c0 + FT_SB > f;   // wave-uniform
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
    const int col = c0 + 8 * cc;
    const bool cvalid = col < f;
    float cgv[8], cuv[8], dmg[8], dmu[8];
    if constexpr (DORA) {
      const int64_t o = (int64_t)e * f + col_of(c0);
#pragma unroll
      for (int m = 0; m < 8; m++) {
        cgv[m] = dora.cg[o + m];
        cuv[m] = dora.cu[o + m];
        dmg[m] = dmu[m] = 0.f;
      }
    }
#pragma unroll
    for (int p = 0; p < 4; p++) {
      const int lo = (8 * p + rr) * FT_PITCH + 8 * cc;
      const bf16x8_t dgl = ld8(tg + lo), dul = ld8(tu + lo), ddl = ld8(td + lo);
      const bf16x8_t gv = gnx[p], uv = unx[p], hv = hnx[p];
      bf16x8_t dgv, duv;
      float part = 0.f;
#pragma unroll
      for (int m = 0; m < 8; m++) {
        float gg = (float)gv[m] + (float)dgl[m];
        float uu = (float)uv[m] + (float)dul[m];
        const float vg = gg, vu = uu;
        if constexpr (DORA) { gg *= cgv[m]; uu *= cuv[m]; }
        const float hh = (float)hv[m];
        const float sg = fsigmoid(gg);
        const float da = wrow[p] * hh + (float)ddl[m];
        const float gs = gg * sg;                       // SiLU(g)
        part = fmaf(hh, gs * uu, part);
        // d SiLU / dg = sig (1 + g (1 - sig)) = sig + SiLU(g) (1 - sig)
        float dgr = (da * uu) * fmaf(gs, 1.f - sg, sg);
        float dur = da * gs;
        if constexpr (DORA) {
          if (rvalid[p]) { dmg[m] = fmaf(dgr, vg, dmg[m]); dmu[m] = fmaf(dur, vu, dmu[m]); }
          dgr *= cgv[m];
          dur *= cuv[m];
        }
        // columns past f hold finite values of clamped loads; they meet zeroed weights in the
        // rank-r products below and are never stored
        dgv[m] = (bf16_t)dgr;
        duv[m] = (bf16_t)dur;
      }
      if (cvalid) dwacc[p] += part;
      {
        const int64_t o = gsrc[p] + col_of(cn);
        gnx[p] = ld8(G + o);
        unx[p] = ld8(U + o);
        hnx[p] = ld8(H + (h_by_row ? odst[p] : gsrc[p]) + col_of(cn));
      }
      if (rvalid[p] && cvalid) {
        *reinterpret_cast<bf16x8_t *>(dg_grp + odst[p] + col) = dgv;
        *reinterpret_cast<bf16x8_t *>(du_grp + odst[p] + col) = duv;
      }
      *reinterpret_cast<bf16x8_t *>(tg + lo) = dgv;
      *reinterpret_cast<bf16x8_t *>(tu + lo) = duv;
    }
    if constexpr (DORA) {
      // add the 8 row lanes (rr = lane / 8) of every 8-column chunk in a fixed order; this
      // wave is the only one that handles these columns of this tile
#pragma unroll
      for (int m = 0; m < 8; m++) {
        float a = dmg[m], b = dmu[m];
        a += __shfl_xor(a, 8, 64);  b += __shfl_xor(b, 8, 64);
        a += __shfl_xor(a, 16, 64); b += __shfl_xor(b, 16, 64);
        a += __shfl_xor(a, 32, 64); b += __shfl_xor(b, 32, 64);
        dmg[m] = a;
        dmu[m] = b;
      }
      if (rr == 0 && cvalid) {
        const int64_t o = (int64_t)blockIdx.x * f + col;
#pragma unroll
        for (int m = 0; m < 8; m++) { dora.dm_part_g[o + m] = dmg[m]; dora.dm_part_u[o + m] = dmu[m]; }
      }
    }
    __builtin_amdgcn_wave_barrier();
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
    __builtin_amdgcn_wave_barrier();
  }
  // <H, a> per row: add the 8 column chunks (lanes cc = 0..7 of a row), then the 4 waves
#pragma unroll
  for (int p = 0; p < 4; p++) {
    float v = dwacc[p];
    v += __shfl_xor(v, 1, 64);
    v += __shfl_xor(v, 2, 64);
    v += __shfl_xor(v, 4, 64);
    if (cc == 0) dwred[wave][8 * p + rr] = v;
  }
  float(*red)[NQ][16][64] = reinterpret_cast<float(*)[NQ][16][64]>(lds);
  for (int bank = 0; bank < 2; bank++) {
    __syncthreads();   // tiles (first pass) or the previous bank's sums are no longer read
#pragma unroll
    for (int j = 0; j < NQ; j++)
#pragma unroll
      for (int i = 0; i < 16; i++) red[wave][j][i][lane] = bank == 0 ? acctg[j][i] : acctu[j][i];
    __syncthreads();
    float *out = bank == 0 ? TG_part : TU_part;
    for (int idx = threadIdx.x; idx < NQ * 16 * 64; idx += FT_WAVES * 64) {
      const int j = idx / (16 * 64), i = (idx / 64) % 16, ln = idx % 64;
      const int q = j * 32 + (ln & 31);
      const int rl = 8 * (i >> 2) + 4 * (ln >> 5) + (i & 3);
      if (q < r && rl < rows) {
        const float v = (red[0][j][i][ln] + red[1][j][i][ln]) + (red[2][j][i][ln] + red[3][j][i][ln]);
        out[((int64_t)blockIdx.y * nP + row0 + rl) * r + q] = v;
      }
    }
  }
  if (threadIdx.x < rows)
    dw_part[(int64_t)(row0 + threadIdx.x) * nsplit + blockIdx.y] =
        (dwred[0][threadIdx.x] + dwred[1][threadIdx.x]) + (dwred[2][threadIdx.x] + dwred[3][threadIdx.x]);
}

// dense[row, e(row)*r + q] = sum over splits of part[split][row][q]   (fixed order); blockIdx.y
// picks the bank (partials bank_stride floats apart, outputs dense0 / dense1).  The same value
// (times the routing weight if weighted) also goes, as bf16, into the block-sparse per-token
// operand of a K-extension:  sparse[t(row), col0 + bank*N*r + e*r + q]; the rest of that
// operand was zero-filled beforehand.  With by_row the operand has one row per grouped pair row
// (sparse[row, ...]) instead of one per token.
__global__ void reduce_rank_parts_kernel(PairCtx pc, const float *__restrict__ part0,
                                         int64_t bank_stride, int nsplit,
                                         float *__restrict__ dense0, float *__restrict__ dense1,
                                         bf16_t *__restrict__ sparse, int ld_sparse, int col0,
                                         int weighted, int by_row) {
  const int nP = pc.T * pc.k, r = pc.r;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)nP * r) return;
  const float *part = part0 + blockIdx.y * bank_stride;
  float *dense = blockIdx.y ? dense1 : dense0;
  const int row = (int)(i / r), q = (int)(i % r);
  float acc = 0.f;
  int sp = 0;
  for (; sp + 4 <= nsplit; sp += 4) {   // four loads in flight; additions in split order
    const float a0 = part[(int64_t)sp * nP * r + i], a1 = part[(int64_t)(sp + 1) * nP * r + i];
    const float a2 = part[(int64_t)(sp + 2) * nP * r + i], a3 = part[(int64_t)(sp + 3) * nP * r + i];
    acc += a0; acc += a1; acc += a2; acc += a3;
  }
  for (; sp < nsplit; sp++) acc += part[(int64_t)sp * nP * r + i];
  const int pair = pc.pair_of_row[row];
  const int e = pc.idx[pair];
  const int R = pc.N * r;
  dense[(int64_t)row * R + e * r + q] = acc;
  const float wv = weighted ? pc.w[pair] : 1.f;
  sparse[(int64_t)(by_row ? row : pair / pc.k) * ld_sparse + col0 + blockIdx.y * R + e * r + q] =
      (bf16_t)(wv * acc);
}

// one bank (dense1 == NULL) or two banks bank_stride floats apart, as described above
hipError_t launch_reduce_rank_parts(const PairCtx &pc, const float *part0, int64_t bank_stride,
                                    int nsplit, float *dense0, float *dense1, void *sparse,
                                    int ld_sparse, int weighted, int by_row, hipStream_t st) {
  const int64_t n = (int64_t)pc.T * pc.k * pc.r;
  const dim3 grid((unsigned)((n + 255) / 256), dense1 ? 2 : 1);
  hipLaunchKernelGGL(reduce_rank_parts_kernel, grid, dim3(256), 0, st, pc, part0, bank_stride, nsplit,
                     dense0, dense1 ? dense1 : dense0, (bf16_t *)sparse, ld_sparse, 0, weighted,
                     by_row);
  return hipGetLastError();
}

int fused_row_tiles(int kT, int N) { return (kT + FT_ROWS - 1) / FT_ROWS + N; }

int fused_splits(int f, int kT) {
  const int nblk = (f + FT_SB - 1) / FT_SB;
  // with few pairs (decode-shaped calls) the row tiles alone cannot fill the chip: finer column cuts
  int s = kT <= 1024 ? FUSED_MAX_SPLITS : kT <= 2048 ? 16 : 8;
  while (s > 1 && nblk / s < FT_WAVES) s >>= 1;
  return s;
}

hipError_t launch_swiglu_fwd_mfma(const PairCtx &pc, int f, float s, const void *G, const void *U,
                                  const float *Pg_all, const float *Pu_all, const void *B_gate,
                                  const void *B_up, const void *A_down, void *a_grp,
                                  float *Q_part, float *Q_all, void *Qw, int ldqw,
                                  hipStream_t st, int rows_mode, const DoraArgs *dora,
                                  bool reduce_parts) {
  const int nP = pc.T * pc.k, nsplit = fused_splits(f, nP);
  const dim3 grid((nP + FT_ROWS - 1) / FT_ROWS + pc.N, nsplit), block(FT_WAVES * 64);
  const DoraArgs da = dora ? *dora : DoraArgs{};
#define MIXLORA_FWD(KSR_, NQ_, DORA_)                                                            \
  hipLaunchKernelGGL((swiglu_fwd_mfma_kernel<KSR_, NQ_, DORA_>), grid, block, 0, st, pc, f, s,    \
                     (const bf16_t *)G, (const bf16_t *)U, Pg_all, Pu_all, (const bf16_t *)B_gate, \
                     (const bf16_t *)B_up, (const bf16_t *)A_down, (bf16_t *)a_grp, Q_part, nsplit, \
                     rows_mode, da)
  if (dora) {
    if (pc.r <= 16) MIXLORA_FWD(1, 1, true);
    else if (pc.r <= 32) MIXLORA_FWD(2, 1, true);
    else MIXLORA_FWD(4, 2, true);
  } else {
    if (pc.r <= 16) MIXLORA_FWD(1, 1, false);
    else if (pc.r <= 32) MIXLORA_FWD(2, 1, false);
    else MIXLORA_FWD(4, 2, false);
  }
#undef MIXLORA_FWD
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !reduce_parts) return e;
  const int64_t n = (int64_t)nP * pc.r;
  hipLaunchKernelGGL(reduce_rank_parts_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                     pc, Q_part, (int64_t)0, nsplit, Q_all, Q_all, (bf16_t *)Qw, ldqw, 0,
                     (rows_mode & ROWS_SPARSE) ? 0 : 1, (rows_mode & ROWS_SPARSE) ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_swiglu_bwd_mfma(const PairCtx &pc, int f, float s, const void *G, const void *U,
                                  const void *H, const float *Pg_all, const float *Pu_all,
                                  const float *VB_all, const void *B_gate, const void *B_up,
                                  const void *AdT, const void *BgT, const void *BuT, void *dg_grp,
                                  void *du_grp, float *dw_part, float *rank_part, float *TG_all,
                                  float *TU_all, void *S, int lds_, hipStream_t st, int rows_mode,
                                  const DoraArgs *dora) {
  const int nP = pc.T * pc.k, nsplit = fused_splits(f, nP);
  float *TG_part = rank_part, *TU_part = rank_part + (size_t)nsplit * nP * pc.r;
  const dim3 grid((nP + FT_ROWS - 1) / FT_ROWS + pc.N, nsplit), block(FT_WAVES * 64);
  const DoraArgs da = dora ? *dora : DoraArgs{};
#define MIXLORA_BWD(KSR_, NQ_, DORA_)                                                            \
  hipLaunchKernelGGL((swiglu_bwd_mfma_kernel<KSR_, NQ_, DORA_>), grid, block, 0, st, pc, f, s,    \
                     (const bf16_t *)G, (const bf16_t *)U, (const bf16_t *)H, Pg_all, Pu_all,      \
                     VB_all, (const bf16_t *)B_gate, (const bf16_t *)B_up, (const bf16_t *)AdT,    \
                     (const bf16_t *)BgT, (const bf16_t *)BuT, (bf16_t *)dg_grp, (bf16_t *)du_grp, \
                     dw_part, TG_part, TU_part, nsplit, rows_mode, da)
  if (dora) {
    if (pc.r <= 16) MIXLORA_BWD(1, 1, true);
    else if (pc.r <= 32) MIXLORA_BWD(2, 1, true);
    else MIXLORA_BWD(4, 2, true);
  } else {
    if (pc.r <= 16) MIXLORA_BWD(1, 1, false);
    else if (pc.r <= 32) MIXLORA_BWD(2, 1, false);
    else MIXLORA_BWD(4, 2, false);
  }
#undef MIXLORA_BWD
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int64_t n = (int64_t)nP * pc.r;
  const dim3 rgrid((unsigned)((n + 255) / 256), 2);
  hipLaunchKernelGGL(reduce_rank_parts_kernel, rgrid, dim3(256), 0, st, pc, TG_part,
                     (int64_t)(TU_part - TG_part), nsplit, TG_all, TU_all, (bf16_t *)S, lds_, 0, 0,
                     (rows_mode & ROWS_SPARSE) ? 1 : 0);
  return hipGetLastError();
}

}  // namespace mixlora
