// Routing kernels: router logits + softmax + top-k + renormalisation (Eq. 7, Norm step of
// Algorithm 1), stable grouping of the (token, expert) pairs by expert with wavefront ballots
// and prefix counts, and the auxiliary load-balance loss (Eq. 8-9).
#include "common.h"
#include "relayout_body.h"

namespace mixlora {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Softmax over the logits of token t (lane n holds logit n), restricted to the experts
// [lo, lo + N) of the token's adapter, top-k on the logits (monotone with the probabilities; equal
// logits go to the lower expert index; slots in descending order) and renormalisation of the kept
// probabilities.  probs gets all Ntot columns (0 outside the adapter); idx_out is the index
// inside the adapter, idx_ws the index among all Ntot experts.
__device__ __forceinline__ void route_token(float z, int lane, int t, int lo, int N, int Ntot,
                                            int k, float *__restrict__ probs,
                                            int32_t *__restrict__ idx_out,
                                            float *__restrict__ w_out,
                                            int32_t *__restrict__ idx_ws,
                                            float *__restrict__ w_ws) {
  const bool own = lane >= lo && lane < lo + N;
  if (!own) z = -INFINITY;
  const float zmax = wave_max(z);
  const float ez = own ? expf(z - zmax) : 0.f;
  const float p = ez / wave_sum(ez);
  if (lane < Ntot) probs[(int64_t)t * Ntot + lane] = p;
  // k rounds of arg-max with ties to the lowest lane
  float zc = z;
  float psel = 0.f;     // lane j keeps the probability of slot j
  int esel = 0;
  float ksum = 0.f;
  for (int j = 0; j < k; j++) {
    const float m = wave_max(zc);
    const unsigned long long b = __ballot(zc == m && own);
    const int e = __ffsll((long long)b) - 1;
    const float pe = __shfl(p, e, 64);
    ksum += pe;
    if (lane == j) { psel = pe; esel = e; }
    if (lane == e) zc = -INFINITY;
  }
  if (lane < k) {
    const float w = psel / ksum;
    const int64_t o = (int64_t)t * k + lane;
    idx_out[o] = esel - lo;
    w_out[o] = w;
    idx_ws[o] = esel;
    w_ws[o] = w;
  }
}

// One wavefront per token.  Lane l accumulates, for every expert, the products of the 8-wide
// chunks l, l+64, ... of the row; a butterfly then gives every lane the full logit.
template <typename E, int NMAX>
__global__ __launch_bounds__(256) void router_kernel(const E *__restrict__ x,
                                                     const E *__restrict__ Wr, int T, int d,
                                                     int N, int k, float *__restrict__ probs,
                                                     int32_t *__restrict__ idx_out,
                                                     float *__restrict__ w_out,
                                                     int32_t *__restrict__ idx_ws,
                                                     float *__restrict__ w_ws, int Nl,
                                                     const int32_t *__restrict__ token_model) {
  __shared__ float zbuf[4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t = blockIdx.x * 4 + wave;
  if (t >= T) return;   // whole wave leaves together; no block-wide barrier below
  float acc[NMAX];
#pragma unroll
  for (int e = 0; e < NMAX; e++) acc[e] = 0.f;
  const E *xr = x + (int64_t)t * d;
  for (int c = lane * 8; c < d; c += 64 * 8) {
    Vec8<E> xv;
    xv.load(xr + c);
#pragma unroll
    for (int e = 0; e < NMAX; e++) {
      if (e < N) {
        Vec8<E> wv;
        wv.load(Wr + (int64_t)e * d + c);
#pragma unroll
        for (int i = 0; i < 8; i++) acc[e] = fmaf(xv.get(i), wv.get(i), acc[e]);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < NMAX; e++) {
    const float s = wave_sum(acc[e]);
    if (lane == e) zbuf[wave][e] = s;
  }
  __builtin_amdgcn_wave_barrier();
  const float z = lane < N ? zbuf[wave][lane] : -INFINITY;
  const int lo = token_model ? token_model[t] * Nl : 0;
  route_token(z, lane, t, lo, Nl, N, k, probs, idx_out, w_out, idx_ws, w_ws);
}

// Routing from logits that a GEMM launch has already produced: Z[t, n], row pitch ldz.
__global__ __launch_bounds__(256) void route_logits_kernel(const float *__restrict__ Z, int ldz,
                                                           int T, int N, int k,
                                                           float *__restrict__ probs,
                                                           int32_t *__restrict__ idx_out,
                                                           float *__restrict__ w_out,
                                                           int32_t *__restrict__ idx_ws,
                                                           float *__restrict__ w_ws, int Nl,
                                                           const int32_t *__restrict__ token_model) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  const float z = lane < N ? Z[(int64_t)t * ldz + lane] : -INFINITY;
  const int lo = token_model ? token_model[t] * Nl : 0;
  route_token(z, lane, t, lo, Nl, N, k, probs, idx_out, w_out, idx_ws, w_ws);
}

template <typename E>
static hipError_t launch_router_t(const void *x, const void *Wr, int T, int d, int N, int k,
                                  float *probs, int32_t *idx_out, float *w_out, int32_t *idx_ws,
                                  float *w_ws, int Nl, const int32_t *token_model,
                                  hipStream_t st) {
  const dim3 grid((T + 3) / 4), block(256);
  const E *xe = reinterpret_cast<const E *>(x), *we = reinterpret_cast<const E *>(Wr);
#define MIXLORA_ROUTER(NM)                                                                    \
  hipLaunchKernelGGL((router_kernel<E, NM>), grid, block, 0, st, xe, we, T, d, N, k, probs,   \
                     idx_out, w_out, idx_ws, w_ws, Nl, token_model)
  if (N <= 8) MIXLORA_ROUTER(8);
  else if (N <= 16) MIXLORA_ROUTER(16);
  else if (N <= 32) MIXLORA_ROUTER(32);
  else MIXLORA_ROUTER(64);
#undef MIXLORA_ROUTER
  return hipGetLastError();
}

hipError_t launch_router(int dtype, const void *x, const void *W_router, int T, int d, int N,
                         int k, float *probs, int32_t *idx_out, float *w_out, int32_t *idx_ws,
                         float *w_ws, int Nl, const int32_t *token_model, hipStream_t st) {
  return dtype == MIXLORA_BF16
             ? launch_router_t<bf16_t>(x, W_router, T, d, N, k, probs, idx_out, w_out, idx_ws, w_ws,
                                       Nl, token_model, st)
             : launch_router_t<float>(x, W_router, T, d, N, k, probs, idx_out, w_out, idx_ws, w_ws,
                                      Nl, token_model, st);
}

// The same routing with up to RELAYOUT_MAX_JOBS weight re-layout jobs (bf16) in the trailing
// workgroups of the launch: the re-layouts of a forward pass depend on the weights only, and each
// of the two launches alone is dominated by its own latency.
__global__ __launch_bounds__(256) void route_logits_relayout_kernel(
    const float *__restrict__ Z, int ldz, int T, int N, int k, float *__restrict__ probs,
    int32_t *__restrict__ idx_out, float *__restrict__ w_out, int32_t *__restrict__ idx_ws,
    float *__restrict__ w_ws, int Nl, const int32_t *__restrict__ token_model, int route_blocks,
    RelayoutBatch batch, int rblocks) {
  if ((int)blockIdx.x >= route_blocks) {   // workgroup-uniform
    const int b = blockIdx.x - route_blocks;
    relayout_body<bf16_t>(batch.job[b / rblocks], b % rblocks, rblocks);
    return;
  }
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  const float z = lane < N ? Z[(int64_t)t * ldz + lane] : -INFINITY;
  const int lo = token_model ? token_model[t] * Nl : 0;
  route_token(z, lane, t, lo, Nl, N, k, probs, idx_out, w_out, idx_ws, w_ws);
}

hipError_t launch_route_logits_relayout(const float *Z, int ldz, int T, int N, int k, float *probs,
                                        int32_t *idx_out, float *w_out, int32_t *idx_ws,
                                        float *w_ws, int Nl, const int32_t *token_model,
                                        const RelayoutJob *jobs, int njobs, hipStream_t st) {
  if (njobs < 1 || njobs > RELAYOUT_MAX_JOBS) return hipErrorInvalidValue;
  RelayoutBatch b;
  for (int i = 0; i < RELAYOUT_MAX_JOBS; i++) b.job[i] = jobs[i < njobs ? i : 0];
  const int64_t rblocks = relayout_blocks(jobs, njobs);
  if (rblocks == 0) return hipErrorInvalidValue;
  const int route_blocks = (T + 3) / 4;
  hipLaunchKernelGGL(route_logits_relayout_kernel, dim3((unsigned)(route_blocks + njobs * rblocks)),
                     dim3(256), 0, st, Z, ldz, T, N, k, probs, idx_out, w_out, idx_ws, w_ws, Nl,
                     token_model, route_blocks, b, (int)rblocks);
  return hipGetLastError();
}

hipError_t launch_route_logits(const float *Z, int ldz, int T, int N, int k, float *probs,
                               int32_t *idx_out, float *w_out, int32_t *idx_ws, float *w_ws,
                               int Nl, const int32_t *token_model, hipStream_t st) {
  hipLaunchKernelGGL(route_logits_kernel, dim3((T + 3) / 4), dim3(256), 0, st, Z, ldz, T, N, k,
                     probs, idx_out, w_out, idx_ws, w_ws, Nl, token_model);
  return hipGetLastError();
}

// ---- grouping of pairs by expert ---------------------------------------------------------
// One workgroup of 16 wavefronts.  Wave w owns a contiguous range of pairs.  Pass 1 counts the
// range's pairs per expert (lane n keeps the count of expert n: one ballot + popcount per
// expert per 64 pairs).  After an exclusive scan over (expert, wave), pass 2 walks the range
// again and gives each pair the row  base[expert] + (number of earlier pairs of that expert),
// i.e. a stable counting sort: rows of one expert are in ascending pair order.
constexpr int GP_WAVES = 16;
constexpr int GP_CACHE = 16;   // 64-pair steps of a wave's range kept in registers

__device__ __forceinline__ void group_pairs_block(
    const int32_t *__restrict__ idx, int nP, int N, int k, int32_t *__restrict__ counts,
    int32_t *__restrict__ counts_out, int32_t *__restrict__ first_counts,
    int32_t *__restrict__ offs, int32_t *__restrict__ row_of_pair,
    int32_t *__restrict__ pair_of_row) {
  __shared__ int tot[GP_WAVES][64];
  __shared__ int first[GP_WAVES][64];
  __shared__ int base[GP_WAVES][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int per = (((nP + GP_WAVES - 1) / GP_WAVES) + 63) & ~63;
  const int lo = wave * per;
  const int hi = lo + per < nP ? lo + per : nP;
  // the first GP_CACHE 64-pair steps of the range are loaded up front (all loads in flight at
  // once) and kept in registers for both passes; longer ranges read the rest as they go
  int ec[GP_CACHE];
#pragma unroll
  for (int c = 0; c < GP_CACHE; c++) {
    const int p = lo + c * 64 + lane;
    ec[c] = p < hi ? idx[p] : -1;
  }
  int cnt = 0, fcnt = 0;
  auto count_step = [&](int e, int p) {
    const bool is_first = (p % k) == 0;
    for (int n = 0; n < N; n++) {
      const unsigned long long b = __ballot(e == n);
      const unsigned long long bf = __ballot(e == n && is_first);
      if (lane == n) { cnt += __popcll(b); fcnt += __popcll(bf); }
    }
  };
#pragma unroll
  for (int c = 0; c < GP_CACHE; c++)
    if (lo + c * 64 < hi) count_step(ec[c], lo + c * 64 + lane);
  for (int p0 = lo + GP_CACHE * 64; p0 < hi; p0 += 64) {
    const int p = p0 + lane;
    count_step(p < hi ? idx[p] : -1, p);
  }
  tot[wave][lane] = cnt;
  first[wave][lane] = fcnt;
  __syncthreads();
  if (threadIdx.x < 64) {
    // lane n: totals of expert n over the waves, then an exclusive scan over experts
    int c = 0, fc = 0;
    for (int w = 0; w < GP_WAVES; w++) { c += tot[w][lane]; fc += first[w][lane]; }
    if (lane >= N) c = 0;
    int incl = c;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int v = __shfl_up(incl, o, 64);
      if (lane >= o) incl += v;
    }
    const int excl = incl - c;
    if (lane < N) {
      counts[lane] = c;
      if (counts_out) counts_out[lane] = c;
      first_counts[lane] = fc;
      offs[lane] = excl;
      if (lane == N - 1) offs[N] = incl;
    }
    int run = excl;
    for (int w = 0; w < GP_WAVES; w++) { base[w][lane] = run; run += tot[w][lane]; }
  }
  __syncthreads();
  int running = base[wave][lane];   // lane n: next free row of expert n for this wave
  const unsigned long long lt = lane == 0 ? 0ull : (~0ull >> (64 - lane));
  auto place_step = [&](int e, int p) {
    unsigned long long mine = 0;
    int add = 0;
    for (int n = 0; n < N; n++) {
      const unsigned long long b = __ballot(e == n);
      if (e == n) mine = b;
      if (lane == n) add = __popcll(b);
    }
    const int start = __shfl(running, e < 0 ? 0 : e, 64);
    if (e >= 0) {
      const int row = start + __popcll(mine & lt);
      row_of_pair[p] = row;
      pair_of_row[row] = p;
    }
    running += add;
  };
#pragma unroll
  for (int c = 0; c < GP_CACHE; c++)
    if (lo + c * 64 < hi) place_step(ec[c], lo + c * 64 + lane);
  for (int p0 = lo + GP_CACHE * 64; p0 < hi; p0 += 64) {
    const int p = p0 + lane;
    place_step(p < hi ? idx[p] : -1, p);
  }
}

__global__ __launch_bounds__(GP_WAVES * 64) void group_pairs_kernel(
    const int32_t *__restrict__ idx, int nP, int N, int k, int32_t *__restrict__ counts,
    int32_t *__restrict__ counts_out, int32_t *__restrict__ first_counts,
    int32_t *__restrict__ offs, int32_t *__restrict__ row_of_pair,
    int32_t *__restrict__ pair_of_row) {
  group_pairs_block(idx, nP, N, k, counts, counts_out, first_counts, offs, row_of_pair, pair_of_row);
}

hipError_t launch_group_pairs(const int32_t *idx, int T, int N, int k, int32_t *counts,
                              int32_t *counts_out, int32_t *first_counts, int32_t *offs,
                              int32_t *row_of_pair, int32_t *pair_of_row, hipStream_t st) {
  hipLaunchKernelGGL(group_pairs_kernel, dim3(1), dim3(GP_WAVES * 64), 0, st, idx, T * k, N, k,
                     counts, counts_out, first_counts, offs, row_of_pair, pair_of_row);
  return hipGetLastError();
}

// ---- auxiliary loss (Eq. 8-9) -------------------------------------------------------------
// One workgroup.  F from an integer histogram of the kept experts (first slot only, or all k
// slots divided by k); P from column sums taken in a fixed order (thread (g, e) sums rows
// g, g + G, ...; thread e then adds the G partials in ascending g), so the result is
// bit-reproducible.  With several adapters (N = M * Nl experts, expert e belongs to adapter
// e / Nl, probs is zero outside a token's adapter) every adapter's F, P and loss are taken over
// its own T_m tokens; an adapter without tokens has loss 0.
__device__ __forceinline__ void aux_loss_block(const float *__restrict__ probs,
                                               const int32_t *__restrict__ idx, int T, int N,
                                               int k, float coeff, int mode,
                                               float *__restrict__ loss,
                                               float *__restrict__ F_out,
                                               float *__restrict__ P_out, int Nl,
                                               const int32_t *__restrict__ token_model,
                                               int32_t *__restrict__ model_tokens) {
  __shared__ int hist[64];
  __shared__ int tm[64];
  __shared__ float part[1024];
  __shared__ float fp[64];
  const int tid = threadIdx.x;
  const int M = N / Nl;
  if (tid < 64) { hist[tid] = 0; tm[tid] = 0; }
  __syncthreads();
  if (mode == MIXLORA_AUX_TOP1) {
    for (int t = tid; t < T; t += 1024) atomicAdd(&hist[idx[(int64_t)t * k]], 1);
  } else {
    for (int64_t p = tid; p < (int64_t)T * k; p += 1024) atomicAdd(&hist[idx[p]], 1);
  }
  if (token_model) {
    for (int t = tid; t < T; t += 1024) atomicAdd(&tm[token_model[t]], 1);
  } else if (tid == 0) {
    tm[0] = T;
  }
  const int G = 1024 / N;
  const int e = tid % N, g = tid / N;
  float s = 0.f;
  if (g < G) {
#pragma unroll 8
    for (int t = g; t < T; t += G) s += probs[(int64_t)t * N + e];
  }
  part[tid] = s;
  __syncthreads();
  if (tid < N) {
    float ps = 0.f;
    for (int gg = 0; gg < G; gg++) ps += part[gg * N + tid];
    const int Tm = tm[tid / Nl];
    const float denom = mode == MIXLORA_AUX_TOP1 ? (float)Tm : (float)Tm * (float)k;
    const float P = Tm > 0 ? ps / (float)Tm : 0.f;
    const float F = Tm > 0 ? (float)hist[tid] / denom : 0.f;
    if (P_out) P_out[tid] = P;
    if (F_out) F_out[tid] = F;
    fp[tid] = F * P;
  }
  __syncthreads();
  if (tid < M) {
    float acc = 0.f;
    for (int n = 0; n < Nl; n++) acc += fp[tid * Nl + n];
    loss[tid] = coeff * (float)Nl * acc;
    if (model_tokens) model_tokens[tid] = tm[tid];
  }
}

__global__ __launch_bounds__(1024) void aux_loss_kernel(const float *__restrict__ probs,
                                                        const int32_t *__restrict__ idx, int T,
                                                        int N, int k, float coeff, int mode,
                                                        float *__restrict__ loss,
                                                        float *__restrict__ F_out,
                                                        float *__restrict__ P_out, int Nl,
                                                        const int32_t *__restrict__ token_model,
                                                        int32_t *__restrict__ model_tokens) {
  aux_loss_block(probs, idx, T, N, k, coeff, mode, loss, F_out, P_out, Nl, token_model, model_tokens);
}

constexpr int PG_GROUPS = PG_MAX_EXPERTS * PG_MAX_EXPERTS;   // group id a * N + b, a < b
constexpr int PG_GWAVES = 16;

// ---- tokens grouped by unordered expert pair (stable counting sort, one workgroup) -------------
// tok_of_pos[pos] = token at position pos of the grouped order; tile_info[tile] = {group id,
// first position, rows (<= 32), 0}; ntiles[0] = number of tiles.
__device__ __forceinline__ void group_token_pairs_block(
    const int32_t *__restrict__ idx, int T, int N, int32_t *__restrict__ tok_of_pos,
    int32_t *__restrict__ tile_info, int32_t *__restrict__ ntiles) {
  __shared__ int cnt[PG_GWAVES][PG_GROUPS];   // per wavefront: count, then next free position
  __shared__ int gtot[PG_GROUPS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int G = N * N;
  for (int i = tid; i < PG_GWAVES * PG_GROUPS; i += PG_GWAVES * 64) (&cnt[0][0])[i] = 0;
  __syncthreads();
  const int per = (((T + PG_GWAVES - 1) / PG_GWAVES) + 63) & ~63;
  const int lo = wave * per;
  const int hi = lo + per < T ? lo + per : T;
  auto group_of = [&](int t) {
    const int e0 = idx[(int64_t)t * 2], e1 = idx[(int64_t)t * 2 + 1];
    return e0 < e1 ? e0 * N + e1 : e1 * N + e0;
  };
  for (int t0 = lo; t0 < hi; t0 += 64) {
    const int t = t0 + lane;
    if (t < hi) atomicAdd(&cnt[wave][group_of(t)], 1);   // integer counts: order does not matter
  }
  __syncthreads();
  if (tid < PG_GROUPS) {
    int tot = 0;
    if (tid < G)
      for (int w = 0; w < PG_GWAVES; w++) tot += cnt[w][tid];
    gtot[tid] = tot;
  }
  __syncthreads();
  if (tid < G) {
    int off = 0, tb = 0;
    for (int g = 0; g < tid; g++) {
      off += gtot[g];
      tb += (gtot[g] + PG_TILE_ROWS - 1) / PG_TILE_ROWS;
    }
    const int tot = gtot[tid], nt = (tot + PG_TILE_ROWS - 1) / PG_TILE_ROWS;
    int run = off;
    for (int w = 0; w < PG_GWAVES; w++) {
      const int c = cnt[w][tid];
      cnt[w][tid] = run;
      run += c;
    }
    for (int i = 0; i < nt; i++) {
      int32_t *ti = tile_info + (int64_t)(tb + i) * 4;
      ti[0] = tid;
      ti[1] = off + i * PG_TILE_ROWS;
      ti[2] = tot - i * PG_TILE_ROWS < PG_TILE_ROWS ? tot - i * PG_TILE_ROWS : PG_TILE_ROWS;
      ti[3] = 0;
    }
    if (tid == G - 1) ntiles[0] = tb + nt;
  }
  __syncthreads();
  const unsigned long long lt = lane == 0 ? 0ull : (~0ull >> (64 - lane));
  for (int t0 = lo; t0 < hi; t0 += 64) {
    const int t = t0 + lane;
    const bool valid = t < hi;
    const int gid = valid ? group_of(t) : -1;
    // m = the lanes whose token is in this lane's group: one ballot per bit of the group id
    // (ids are below PG_GROUPS = 256), no loop over the groups present
    unsigned long long m = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; b++) {
      const unsigned long long has = __ballot(valid && ((gid >> b) & 1));
      m &= ((gid >> b) & 1) ? has : ~has;
    }
    if (valid) {
      // every lane of the group reads the group's next free position (one LDS instruction for
      // the whole wavefront), then the group's first lane moves it on
      const int start = cnt[wave][gid];
      const int pos = start + __popcll(m & lt);
      if ((m & lt) == 0) cnt[wave][gid] = start + __popcll(m);
      tok_of_pos[pos] = t;
    }
  }
}

__global__ __launch_bounds__(PG_GWAVES * 64) void group_token_pairs_kernel(
    const int32_t *__restrict__ idx, int T, int N, int32_t *__restrict__ tok_of_pos,
    int32_t *__restrict__ tile_info, int32_t *__restrict__ ntiles) {
  group_token_pairs_block(idx, T, N, tok_of_pos, tile_info, ntiles);
}

hipError_t launch_group_token_pairs(const PairCtx &pc, int32_t *tok_of_pos, int32_t *tile_info,
                                    int32_t *ntiles, hipStream_t st) {
  hipLaunchKernelGGL(group_token_pairs_kernel, dim3(1), dim3(PG_GWAVES * 64), 0, st, pc.idx, pc.T,
                     pc.N, tok_of_pos, tile_info, ntiles);
  return hipGetLastError();
}

// Grouping and auxiliary loss of one forward pass in one launch of a few workgroups, each bound
// by its own latency and independent of the others: the grouping of the pairs by expert (which
// also writes the two-entry offsets {0, T} that let the grouped outer-product kernel treat all
// tokens as one group), Eq. 8-9, and with pg_tok != NULL the grouping of the tokens by expert pair.
__global__ __launch_bounds__(GP_WAVES * 64) void group_pairs_aux_kernel(
    const int32_t *__restrict__ idx, int T, int N, int k, int32_t *__restrict__ counts,
    int32_t *__restrict__ counts_out, int32_t *__restrict__ first_counts,
    int32_t *__restrict__ offs, int32_t *__restrict__ row_of_pair,
    int32_t *__restrict__ pair_of_row, int32_t *__restrict__ tok_offs,
    const float *__restrict__ probs, float coeff, int mode, float *__restrict__ loss,
    float *__restrict__ F_out, float *__restrict__ P_out, int Nl,
    const int32_t *__restrict__ token_model, int32_t *__restrict__ model_tokens,
    int32_t *__restrict__ pg_tok, int32_t *__restrict__ pg_tiles, int32_t *__restrict__ pg_ntiles) {
  static_assert(GP_WAVES * 64 == 1024, "the auxiliary-loss block code assumes 1024 threads");
  static_assert(PG_GWAVES == GP_WAVES, "both block routines run with the same workgroup size");
  // independent pieces of work, one workgroup each (all workgroup-uniform branches)
  if (blockIdx.x == 0) {
    group_pairs_block(idx, T * k, N, k, counts, counts_out, first_counts, offs, row_of_pair, pair_of_row);
    if (threadIdx.x == 0) { tok_offs[0] = 0; tok_offs[1] = T; }
  } else if (blockIdx.x == 1) {
    aux_loss_block(probs, idx, T, N, k, coeff, mode, loss, F_out, P_out, Nl, token_model, model_tokens);
  } else if (pg_tok) {
    group_token_pairs_block(idx, T, N, pg_tok, pg_tiles, pg_ntiles);
  }
}

hipError_t launch_group_pairs_aux(const int32_t *idx, int T, int N, int k, int32_t *counts,
                                  int32_t *counts_out, int32_t *first_counts, int32_t *offs,
                                  int32_t *row_of_pair, int32_t *pair_of_row, int32_t *tok_offs,
                                  const float *probs, float coeff, int mode, float *loss, float *F,
                                  float *P, int Nl, const int32_t *token_model,
                                  int32_t *model_tokens, int32_t *pg_tok, int32_t *pg_tiles,
                                  int32_t *pg_ntiles, hipStream_t st) {
  hipLaunchKernelGGL(group_pairs_aux_kernel, dim3(pg_tok ? 3 : 2), dim3(GP_WAVES * 64), 0, st, idx,
                     T, N, k, counts, counts_out, first_counts, offs, row_of_pair, pair_of_row,
                     tok_offs, probs, coeff, mode, loss, F, P, Nl, token_model, model_tokens,
                     pg_tok, pg_tiles, pg_ntiles);
  return hipGetLastError();
}

// ---- grouping and auxiliary loss over many workgroups (long token batches) --------------------
// The pairs are cut into chunks of GPM_CHUNK; one wavefront owns a chunk.  Pass 1 counts the
// chunk's pairs per expert (all slots and first slots) and sums its share of the tokens' router
// probabilities and adapter ids; pass 2 (one workgroup) turns the counts into every chunk's
// first row per expert - chunks in ascending order inside an expert, so the row order is the
// same stable order the single-workgroup kernel produces - and finishes Eq. 8-9; pass 3 places
// the pairs.  All sums run in a fixed order.  scratch: 4 arrays of [chunks][64] 4-byte words.
constexpr int GPM_CHUNK = 256;

size_t group_pairs_scratch_bytes(int T, int k) {
  const size_t chunks = ((size_t)T * k + GPM_CHUNK - 1) / GPM_CHUNK;
  return chunks * 64 * 4 * 4;
}

__global__ __launch_bounds__(256) void gpm_count_kernel(
    const int32_t *__restrict__ idx, int T, int N, int k, int chunks,
    const float *__restrict__ probs, const int32_t *__restrict__ token_model, int M,
    int32_t *__restrict__ tot, int32_t *__restrict__ first, float *__restrict__ psum,
    int32_t *__restrict__ tmc) {
  const int lane = threadIdx.x & 63;
  const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (c >= chunks) return;
  const int nP = T * k;
  int cnt = 0, fcnt = 0;
#pragma unroll
  for (int st = 0; st < GPM_CHUNK / 64; st++) {
    const int p = c * GPM_CHUNK + st * 64 + lane;
    const int e = p < nP ? idx[p] : -1;
    const bool is_first = (p % k) == 0;
    for (int n = 0; n < N; n++) {
      const unsigned long long b = __ballot(e == n);
      const unsigned long long bf = __ballot(e == n && is_first);
      if (lane == n) { cnt += __popcll(b); fcnt += __popcll(bf); }
    }
  }
  tot[(int64_t)c * 64 + lane] = cnt;
  first[(int64_t)c * 64 + lane] = fcnt;
  // this chunk's share of the tokens
  const int tw = (T + chunks - 1) / chunks;
  const int t0 = c * tw, t1 = t0 + tw < T ? t0 + tw : T;
  const int G = 64 / N, e = lane % N, g = lane / N;
  float s = 0.f;
  if (g < G)
    for (int t = t0 + g; t < t1; t += G) s += probs[(int64_t)t * N + e];
  float acc = 0.f;
  for (int gg = 0; gg < G; gg++) acc += __shfl(s, (e + gg * N) & 63, 64);   // ascending gg
  psum[(int64_t)c * 64 + lane] = lane < N ? acc : 0.f;
  int tmcnt = 0;
  if (token_model) {
    for (int tb = t0; tb < t1; tb += 64) {
      const int t = tb + lane;
      const int m = t < t1 ? token_model[t] : -1;
      for (int n = 0; n < M; n++) {
        const unsigned long long b = __ballot(m == n);
        if (lane == n) tmcnt += __popcll(b);
      }
    }
  } else if (lane == 0) {
    tmcnt = t1 > t0 ? t1 - t0 : 0;
  }
  tmc[(int64_t)c * 64 + lane] = tmcnt;
}

__global__ __launch_bounds__(1024) void gpm_scan_kernel(
    int T, int N, int k, int chunks, int32_t *__restrict__ tot, const int32_t *__restrict__ first,
    const float *__restrict__ psum, const int32_t *__restrict__ tmc, int32_t *__restrict__ counts,
    int32_t *__restrict__ counts_out, int32_t *__restrict__ first_counts,
    int32_t *__restrict__ offs, int32_t *__restrict__ tok_offs, float coeff, int mode,
    float *__restrict__ loss, float *__restrict__ F_out, float *__restrict__ P_out, int Nl,
    int32_t *__restrict__ model_tokens) {
  __shared__ int seg_tot[16][64], seg_first[16][64], seg_tm[16][64];
  __shared__ float seg_p[16][64];
  __shared__ int eoffs[64], tmtot[64];
  __shared__ float fp[64];
  const int n = threadIdx.x & 63, seg = threadIdx.x >> 6;
  const int cs = (chunks + 15) / 16;
  const int c0 = seg * cs, c1 = c0 + cs < chunks ? c0 + cs : chunks;
  int st = 0, sf = 0, sm = 0;
  float sp = 0.f;
  for (int c = c0; c < c1; c++) {
    st += tot[(int64_t)c * 64 + n];
    sf += first[(int64_t)c * 64 + n];
    sm += tmc[(int64_t)c * 64 + n];
    sp += psum[(int64_t)c * 64 + n];
  }
  seg_tot[seg][n] = st;
  seg_first[seg][n] = sf;
  seg_tm[seg][n] = sm;
  seg_p[seg][n] = sp;
  __syncthreads();
  const int M = N / Nl;
  int c = 0, fc = 0;
  float ps = 0.f;
  if (threadIdx.x < 64) {
    int tmv = 0;
    for (int s2 = 0; s2 < 16; s2++) {
      c += seg_tot[s2][n];
      fc += seg_first[s2][n];
      tmv += seg_tm[s2][n];
      ps += seg_p[s2][n];
    }
    if (n >= N) c = 0;
    int incl = c;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int v = __shfl_up(incl, o, 64);
      if (n >= o) incl += v;
    }
    eoffs[n] = incl - c;
    tmtot[n] = tmv;
    if (n < N) {
      counts[n] = c;
      if (counts_out) counts_out[n] = c;
      first_counts[n] = fc;
      offs[n] = incl - c;
      if (n == N - 1) offs[N] = incl;
    }
    if (n == 0) { tok_offs[0] = 0; tok_offs[1] = T; }
  }
  __syncthreads();
  if (threadIdx.x < N) {
    const int Tm = tmtot[n / Nl];
    const float denom = mode == MIXLORA_AUX_TOP1 ? (float)Tm : (float)Tm * (float)k;
    const float P = Tm > 0 ? ps / (float)Tm : 0.f;
    const float F = Tm > 0 ? (float)(mode == MIXLORA_AUX_TOP1 ? fc : c) / denom : 0.f;
    if (P_out) P_out[n] = P;
    if (F_out) F_out[n] = F;
    fp[n] = F * P;
  }
  __syncthreads();
  if (threadIdx.x < M) {
    float acc = 0.f;
    for (int q = 0; q < Nl; q++) acc += fp[n * Nl + q];
    loss[n] = coeff * (float)Nl * acc;
    if (model_tokens) model_tokens[n] = tmtot[n];
  }
  // first row of every chunk per expert, written over the chunk's count
  int run = eoffs[n];
  for (int s2 = 0; s2 < seg; s2++) run += seg_tot[s2][n];
  for (int c = c0; c < c1; c++) {
    const int v = tot[(int64_t)c * 64 + n];
    tot[(int64_t)c * 64 + n] = run;
    run += v;
  }
}

__global__ __launch_bounds__(256) void gpm_place_kernel(const int32_t *__restrict__ idx, int nP,
                                                        int N, int chunks,
                                                        const int32_t *__restrict__ base,
                                                        int32_t *__restrict__ row_of_pair,
                                                        int32_t *__restrict__ pair_of_row) {
  const int lane = threadIdx.x & 63;
  const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (c >= chunks) return;
  int running = base[(int64_t)c * 64 + lane];
  const unsigned long long lt = lane == 0 ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
  for (int st = 0; st < GPM_CHUNK / 64; st++) {
    const int p = c * GPM_CHUNK + st * 64 + lane;
    const int e = p < nP ? idx[p] : -1;
    unsigned long long mine = 0;
    int add = 0;
    for (int n = 0; n < N; n++) {
      const unsigned long long b = __ballot(e == n);
      if (e == n) mine = b;
      if (lane == n) add = __popcll(b);
    }
    const int start = __shfl(running, e < 0 ? 0 : e, 64);
    if (e >= 0) {
      const int row = start + __popcll(mine & lt);
      row_of_pair[p] = row;
      pair_of_row[row] = p;
    }
    running += add;
  }
}

hipError_t launch_group_pairs_aux_multi(const int32_t *idx, int T, int N, int k, int32_t *counts,
                                        int32_t *counts_out, int32_t *first_counts, int32_t *offs,
                                        int32_t *row_of_pair, int32_t *pair_of_row,
                                        int32_t *tok_offs, const float *probs, float coeff, int mode,
                                        float *loss, float *F, float *P, int Nl,
                                        const int32_t *token_model, int32_t *model_tokens,
                                        void *scratch, hipStream_t st) {
  const int nP = T * k;
  const int chunks = (nP + GPM_CHUNK - 1) / GPM_CHUNK;
  int32_t *tot = (int32_t *)scratch, *first = tot + (size_t)chunks * 64;
  float *psum = (float *)(first + (size_t)chunks * 64);
  int32_t *tmc = (int32_t *)(psum + (size_t)chunks * 64);
  const dim3 grid((chunks + 3) / 4), block(256);
  hipLaunchKernelGGL(gpm_count_kernel, grid, block, 0, st, idx, T, N, k, chunks, probs, token_model,
                     N / Nl, tot, first, psum, tmc);
  hipLaunchKernelGGL(gpm_scan_kernel, dim3(1), dim3(1024), 0, st, T, N, k, chunks, tot, first, psum,
                     tmc, counts, counts_out, first_counts, offs, tok_offs, coeff, mode, loss, F, P,
                     Nl, model_tokens);
  hipLaunchKernelGGL(gpm_place_kernel, grid, block, 0, st, idx, nP, N, chunks, tot, row_of_pair,
                     pair_of_row);
  return hipGetLastError();
}

// d loss / d probs[t, e] = coeff * N * F_e / T   (F is piecewise constant)
__global__ void aux_dprobs_kernel(const int32_t *__restrict__ idx, int T, int N, int k,
                                  float coeff, int mode, float *__restrict__ dprobs) {
  __shared__ int hist[64];
  if (threadIdx.x < 64) hist[threadIdx.x] = 0;
  __syncthreads();
  // every block rebuilds the (tiny) histogram: integer counts, identical in every block
  if (mode == MIXLORA_AUX_TOP1) {
    for (int t = threadIdx.x; t < T; t += blockDim.x) atomicAdd(&hist[idx[(int64_t)t * k]], 1);
  } else {
    for (int64_t p = threadIdx.x; p < (int64_t)T * k; p += blockDim.x) atomicAdd(&hist[idx[p]], 1);
  }
  __syncthreads();
  const float denom = mode == MIXLORA_AUX_TOP1 ? (float)T : (float)T * (float)k;
  const int64_t total = (int64_t)T * N;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * blockDim.x) {
    const int e = (int)(i % N);
    dprobs[i] = coeff * (float)N * ((float)hist[e] / denom) / (float)T;
  }
}

hipError_t launch_aux_loss(const float *probs, const int32_t *idx, int T, int N, int k,
                           float coeff, int mode, float *loss, float *F, float *P,
                           float *dprobs, int Nl, const int32_t *token_model,
                           int32_t *model_tokens, hipStream_t st) {
  hipLaunchKernelGGL(aux_loss_kernel, dim3(1), dim3(1024), 0, st, probs, idx, T, N, k, coeff,
                     mode, loss, F, P, Nl, token_model, model_tokens);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (dprobs) {
    hipLaunchKernelGGL(aux_dprobs_kernel, dim3(8), dim3(1024), 0, st, idx, T, N, k, coeff, mode,
                       dprobs);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace mixlora
