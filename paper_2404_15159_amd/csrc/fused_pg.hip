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
// The stage is bound by vector-ALU issue (exp and rcp of the sigmoid run at quarter rate), not by
// memory: per token and column it now spends about 31 vector instructions for both experts where
// the expert-grouped kernel plus the combine pass spent about 56.
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
      gnx[p] = ldg8(G, gsrc[p] + col_of(cn));
      unx[p] = ldg8(U, gsrc[p] + col_of(cn));
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

bool fused_pg_ok(const PairCtx &pc, int f) {
  return pc.k == 2 && pc.N <= PG_MAX_EXPERTS && pc.r <= 16 && pc.T > 128 && pc.T <= PG_MAX_TOKENS &&
         f >= 64 && (int64_t)2 * pc.T * f < ((int64_t)1 << 31);
}

int fused_pg_max_tiles(int T, int N) { return (T + FT_ROWS - 1) / FT_ROWS + N * N; }

int fused_pg_splits(int f, int T) {
  const int nblk = (f + FT_SB - 1) / FT_SB;
  int s = T <= 1024 ? 16 : 8;
  while (s > 1 && nblk / s < FT_WAVES) s >>= 1;
  return s;
}

hipError_t launch_swiglu_fwd_pg(const PairCtx &pc, int f, float s, const int32_t *tok_of_pos,
                                const int32_t *tile_info, const int32_t *ntiles, const void *G,
                                const void *U, const float *Pg_all, const float *Pu_all,
                                const void *B_gate, const void *B_up, const void *A_down,
                                void *a_grp, void *a_comb, float *Q_part, float *Q_all, void *Qw,
                                int ldqw, int write_a, hipStream_t st) {
  if (!fused_pg_ok(pc, f)) return hipErrorInvalidValue;
  const int nsplit = fused_pg_splits(f, pc.T);
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

}  // namespace mixlora
