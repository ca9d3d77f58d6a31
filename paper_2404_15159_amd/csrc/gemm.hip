// GEMM engine of libmixlora:  C[M,N] = sum_s A_s[M,K_s] * B_s[N,K_s]^T  ("NT", K contiguous).
//
// bf16 storage: MFMA 32x32x16 bf16 -> fp32 tiles, 64-wide wavefronts, operands staged through
// padded LDS tiles with register prefetch of the next K tile (double-buffered LDS, one barrier
// per K tile), XCD-aware + grouped tile order so that the tiles resident on one XCD share
// operand rows in that XCD's L2.
// fp32 storage: plain FMA tiles (the fp32 configuration is a small parity case).
//
// Every frozen projection of the block (shared gate/up: Algorithm 1 lines 7-8; down: line 14)
// and their transposes in the backward go through here; LoRA terms enter either as extra
// K segments (low-rank K-extension) or through the element-wise kernels.
#include "common.h"

#include <type_traits>

namespace mixlora {

struct GemmBatch {
  GemmProblem p[GEMM_MAX_PROBLEMS];
};

constexpr int GEMM_LONG_K = 8192;   // summed K of a problem from which the half-slot ring is used

// Map the hardware block id to a tile so that (a) blocks that land on the same XCD (id % 8)
// get consecutive logical ids and (b) consecutive logical ids walk GROUP tile-rows at a time.
__device__ __forceinline__ void tile_of_block(int bid, int tiles_m, int tiles_n, int &tm, int &tn) {
  const int nb = tiles_m * tiles_n;
  const int q = nb >> 3, rem = nb & 7;
  const int xcd = bid & 7, local = bid >> 3;
  const int lid = xcd * q + (xcd < rem ? xcd : rem) + local;
  constexpr int GROUP = 4;   // measured: 4 slightly ahead of 2, 8, 16 (all within 3 %)
  const int width = GROUP * tiles_n;
  const int group_id = lid / width;
  const int first_m = group_id * GROUP;
  const int gsz = (tiles_m - first_m) < GROUP ? (tiles_m - first_m) : GROUP;
  const int in_group = lid - group_id * width;
  tm = first_m + in_group % gsz;
  tn = in_group / gsz;
}

template <typename OutT> __device__ __forceinline__ void store_c(OutT *p, float v);
template <> __device__ __forceinline__ void store_c<float>(float *p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_c<bf16_t>(bf16_t *p, float v) { *p = (bf16_t)v; }

template <typename OutT>
__device__ __forceinline__ void store_c4(OutT *p, float a, float b, float c, float d);
template <> __device__ __forceinline__ void store_c4<float>(float *p, float a, float b, float c, float d) {
  *reinterpret_cast<float4 *>(p) = make_float4(a, b, c, d);
}
template <> __device__ __forceinline__ void store_c4<bf16_t>(bf16_t *p, float a, float b, float c, float d) {
  typedef bf16_t bf16x4v_t __attribute__((ext_vector_type(4)));
  bf16x4v_t v;
  v[0] = (bf16_t)a; v[1] = (bf16_t)b; v[2] = (bf16_t)c; v[3] = (bf16_t)d;
  *reinterpret_cast<bf16x4v_t *>(p) = v;
}

template <int BM, int BN, int BK, int WGM, int WGN, typename OutT>
__global__ __launch_bounds__(WGM *WGN * 64) void gemm_bf16_kernel(GemmBatch args) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int LD = BK + 8;        // LDS row pitch in elements: 16 bytes of padding per row
  constexpr int CPR = BK / 8;       // 16-byte chunks per tile row
  constexpr int RPP = NT / CPR;     // tile rows covered by one pass of all threads
  constexpr int A_IT = BM / RPP, B_IT = BN / RPP;
  constexpr int TM = BM / WGM, TN = BN / WGN, MI = TM / 32, NI = TN / 32;
  static_assert(BM % RPP == 0 && BN % RPP == 0, "tile/threads mismatch");
  static_assert(TM % 32 == 0 && TN % 32 == 0 && BK % 16 == 0, "wave tile");

  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t *As = reinterpret_cast<bf16_t *>(smem);   // [2][BM][LD]
  bf16_t *Bs = As + 2 * BM * LD;                   // [2][BN][LD]

  const GemmProblem &P = args.p[blockIdx.z];
  const int M = P.M, N = P.N;
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  int tm, tn;
  tile_of_block(blockIdx.x, tiles_m, tiles_n, tm, tn);
  const int row0 = tm * BM, col0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int kc = tid % CPR;         // this thread's 16-byte chunk within a tile row
  const int r_in = tid / CPR;       // first tile row this thread loads

  f32x16_t acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; i++)
#pragma unroll
    for (int j = 0; j < NI; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

  // Global -> register prefetch.  Rows/columns past the matrix edge are clamped to the last
  // valid one: their products land in C rows/columns that are never stored.  K chunks past
  // the segment's end are loaded from a valid address and replaced by zeros.
  uint4 ra[A_IT], rb[B_IT];
  const bf16_t *pa[A_IT], *pb[B_IT];
  int Kcur = 0;
  auto setup = [&](int s) {
    const GemmSeg &S = P.seg[s];
    const bf16_t *Ab = reinterpret_cast<const bf16_t *>(S.A) + kc * 8;
    const bf16_t *Bb = reinterpret_cast<const bf16_t *>(S.B) + kc * 8;
#pragma unroll
    for (int i = 0; i < A_IT; i++) {
      int r = row0 + r_in + i * RPP;
      r = r < M ? r : M - 1;
      pa[i] = Ab + (int64_t)r * S.lda;
    }
#pragma unroll
    for (int i = 0; i < B_IT; i++) {
      int c = col0 + r_in + i * RPP;
      c = c < N ? c : N - 1;
      pb[i] = Bb + (int64_t)c * S.ldb;
    }
    Kcur = S.K;
  };
  auto gload = [&](int k0) {
    const bool kok = k0 + kc * 8 < Kcur;
    const int ko = kok ? k0 : 0;
#pragma unroll
    for (int i = 0; i < A_IT; i++) {
      const uint4 v = *reinterpret_cast<const uint4 *>(pa[i] + ko);
      ra[i] = kok ? v : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < B_IT; i++) {
      const uint4 v = *reinterpret_cast<const uint4 *>(pb[i] + ko);
      rb[i] = kok ? v : make_uint4(0, 0, 0, 0);
    }
  };
  auto lstore = [&](int buf) {
    bf16_t *a = As + buf * BM * LD, *b = Bs + buf * BN * LD;
#pragma unroll
    for (int i = 0; i < A_IT; i++)
      *reinterpret_cast<uint4 *>(a + (r_in + i * RPP) * LD + kc * 8) = ra[i];
#pragma unroll
    for (int i = 0; i < B_IT; i++)
      *reinterpret_cast<uint4 *>(b + (r_in + i * RPP) * LD + kc * 8) = rb[i];
  };

  const int nseg_total = P.nseg;
  int total_tiles = 0;
  for (int s = 0; s < nseg_total; s++) total_tiles += (P.seg[s].K + BK - 1) / BK;

  int seg = 0, k0 = 0;   // position of the tile being prefetched
  setup(0);
  gload(0);
  lstore(0);
  __syncthreads();
  int buf = 0;
  const bf16_t *a_rd = As + (wm * TM + (lane & 31)) * LD + (lane >> 5) * 8;
  const bf16_t *b_rd = Bs + (wn * TN + (lane & 31)) * LD + (lane >> 5) * 8;
  for (int it = 0; it < total_tiles; it++) {
    const bool more = it + 1 < total_tiles;
    if (more) {
      k0 += BK;
      if (k0 >= Kcur) {   // next segment (rare)
        seg++;
        setup(seg);
        k0 = 0;
      }
      gload(k0);
    }
    const bf16_t *a = a_rd + buf * BM * LD;
    const bf16_t *b = b_rd + buf * BN * LD;
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      bf16x8_t af[MI], bfr[NI];
#pragma unroll
      for (int i = 0; i < MI; i++) af[i] = *reinterpret_cast<const bf16x8_t *>(a + i * 32 * LD + kk);
#pragma unroll
      for (int j = 0; j < NI; j++) bfr[j] = *reinterpret_cast<const bf16x8_t *>(b + j * 32 * LD + kk);
#pragma unroll
      for (int i = 0; i < MI; i++)
#pragma unroll
        for (int j = 0; j < NI; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (more) {
      lstore(buf ^ 1);
      __syncthreads();
      buf ^= 1;
    }
  }

  // C fragment of a 32x32 block: column = lane % 32, row = 8*(e/4) + 4*(lane/32) + e%4
  OutT *C = reinterpret_cast<OutT *>(P.C);
  const int cbase = col0 + wn * TN + (lane & 31);
  const int rbase = row0 + wm * TM + (lane >> 5) * 4;
#pragma unroll
  for (int i = 0; i < MI; i++)
#pragma unroll
    for (int j = 0; j < NI; j++) {
      const int c = cbase + j * 32;
      if (c < N) {
#pragma unroll
        for (int e = 0; e < 16; e++) {
          const int r = rbase + i * 32 + (e >> 2) * 8 + (e & 3);
          if (r < M) store_c<OutT>(C + (int64_t)r * P.ldc + c, acc[i][j][e]);
        }
      }
    }
}

// ---- bf16, direct-to-LDS variant ---------------------------------------------------------------
// Same tiling and MFMA fragments as above, but the operand tiles go from global memory straight
// into LDS (global_load_lds_dwordx4: lane i's 16 bytes land at M0 + 16*i, no VGPR round trip)
// through a ring of STAGES tiles, so that STAGES-1 K tiles are in flight while one is consumed:
// HBM latency under load is longer than one K tile's worth of MFMA work.  LDS rows are unpadded
// (the DMA writes 1 KiB contiguous per wave instruction); bank conflicts of the 128-bit
// fragment reads are avoided by an XOR swizzle of the 16-byte chunk index with the row's
// 256-byte bank-row number, applied on the global-address side of the copy.
// The loads and their s_waitcnt are inline asm: the compiler's own bookkeeping would wait for
// all outstanding LDS DMA before every LDS read and collapse the ring to depth one.
// Requires every K_s % BK == 0 and operands below 4 GiB (32-bit lane offsets).
// PW > 0 makes only the first PW waves issue the copies (all of them, IA + IB instructions each).
// A compute unit's vector-memory front end takes one 1 KiB copy instruction per ~16 cycles, so
// the 64 instructions of a 256x256x64 tile keep their issuing waves stalled for ~1000 cycles
// right after the barrier.  If every wave issues its share, both waves of each SIMD stall
// together and the matrix pipe runs dry; with one issuing wave per SIMD (PW = 4 of 8 waves)
// the other wave works through its MFMAs meanwhile, and the issuing wave follows with its own.
// H5 replaces the two whole stages by five half-slots of one operand's K tile each (all 160 KB
// of LDS).  A and B tiles rotate through them separately, so the A tile of step t+3 is requested
// together with the B tile of step t+2: a barrier still frees and refills 64 KB, but the half
// needed at the next barrier is first in the burst and the other half has one tile longer to
// arrive.  That pays where the copies come from HBM rather than from L2 (one round of tiles over
// a long K, operands last touched by other kernels); over short K it costs a few percent.
__device__ __forceinline__ void dma16(uint32_t voff, const void *sbase, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(voff), "s"(sbase), "s"(lds_addr)
               : "memory", "m0");
}
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}
__device__ __forceinline__ const void *uniform_ptr(const void *p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return reinterpret_cast<const void *>(((uint64_t)hi << 32) | lo);
}

template <int BM, int BN, int BK, int STAGES, int WGM, int WGN, bool PIPE = false, int PW = 0, bool H5 = false>
__global__ __launch_bounds__(WGM *WGN * 64) void gemm_bf16_dl_kernel(GemmBatch args) {
  constexpr int NW = WGM * WGN;
  constexpr int NPW = PW > 0 ? PW : NW;   // waves that issue the copies
  constexpr int ROWB = BK * 2;            // bytes per tile row in LDS
  constexpr int CPR = BK / 8;             // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;           // rows covered by one wave-wide DMA instruction
  constexpr int RPB = 256 / ROWB;         // rows per 256-byte bank row
  constexpr int IA = BM / RPI / NPW, IB = BN / RPI / NPW;   // DMA instructions per issuing wave per tile
  constexpr int IPW = IA + IB;
  constexpr int STAGE_BYTES = (BM + BN) * ROWB;
  constexpr int TM = BM / WGM, TN = BN / WGN, MI = TM / 32, NI = TN / 32, KS = BK / 16;
  static_assert(NPW <= NW && BM % (RPI * NPW) == 0 && BN % (RPI * NPW) == 0, "tile/waves mismatch");
  static_assert((STAGES - 2) * IPW < 64 && STAGES >= 2, "ring depth");

  extern __shared__ __align__(16) unsigned char smem[];
  const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) unsigned char *)smem;

  const GemmProblem &P = args.p[blockIdx.z];
  const int M = P.M, N = P.N;
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  if ((int)blockIdx.x >= tiles_m * tiles_n) return;   // problems of one launch may differ in N
  int tm, tn;
  tile_of_block(blockIdx.x, tiles_m, tiles_n, tm, tn);
  const int row0 = tm * BM, col0 = tn * BN;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WGN, wn = wave % WGN;

  f32x16_t acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; i++)
#pragma unroll
    for (int j = 0; j < NI; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

  // --- producer side: per-lane byte offsets of this wave's DMA instructions -----------------
  const int lrow = lane / CPR, lpos = lane % CPR;
  uint32_t offA[IA], offB[IB];
  const unsigned char *baseA = nullptr, *baseB = nullptr;
  int Kcur = 0;
  auto setup = [&](int sgi) {
    const GemmSeg &S = P.seg[sgi];
#pragma unroll
    for (int j = 0; j < IA; j++) {
      const int rt = (wave * IA + j) * RPI + lrow;        // row within the tile
      const int kc = lpos ^ ((rt / RPB) % CPR);
      int r = row0 + rt;
      r = r < M ? r : M - 1;
      offA[j] = (uint32_t)r * (uint32_t)S.lda * 2u + kc * 16;
    }
#pragma unroll
    for (int j = 0; j < IB; j++) {
      const int rt = (wave * IB + j) * RPI + lrow;
      const int kc = lpos ^ ((rt / RPB) % CPR);
      int c = col0 + rt;
      c = c < N ? c : N - 1;
      offB[j] = (uint32_t)c * (uint32_t)S.ldb * 2u + kc * 16;
    }
    baseA = reinterpret_cast<const unsigned char *>(S.A);
    baseB = reinterpret_cast<const unsigned char *>(S.B);
    Kcur = S.K;
  };
  auto issue = [&](int k0, int stage) {
    const void *ga = uniform_ptr(baseA + (size_t)k0 * 2);
    const void *gb = uniform_ptr(baseB + (size_t)k0 * 2);
    const uint32_t la = lds0 + stage * STAGE_BYTES + wave * IA * 1024;
    const uint32_t lb = lds0 + stage * STAGE_BYTES + BM * ROWB + wave * IB * 1024;
    if (NPW == NW || wave < NPW) {   // the other waves' offsets point past the tile and are never used
#pragma unroll
      for (int j = 0; j < IA; j++) dma16(offA[j], ga, la + j * 1024);
#pragma unroll
      for (int j = 0; j < IB; j++) dma16(offB[j], gb, lb + j * 1024);
    }
  };

  int total_tiles = 0;
  for (int sgi = 0; sgi < P.nseg; sgi++) total_tiles += P.seg[sgi].K / BK;

  int seg = 0, k0 = 0, issued = 0;
  setup(0);
  auto issue_next = [&]() {   // issue tile number `issued` (if any) into its ring slot
    if (issued < total_tiles) {
      if (k0 >= Kcur) {
        seg++;
        setup(seg);
        k0 = 0;
      }
      issue(k0, issued % STAGES);
      k0 += BK;
    }
    issued++;
  };
  if constexpr (!H5) {
#pragma unroll
    for (int s0 = 0; s0 < STAGES - 1; s0++) issue_next();
  }

  // --- consumer side: swizzled fragment addresses -------------------------------------------
  const int l31 = lane & 31, hi = lane >> 5;
  const int swz = (l31 / RPB) % CPR;
  int koff[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ks++) koff[ks] = ((ks * 2 + hi) ^ swz) * 16;
  const unsigned char *a_rd = smem + (wm * TM + l31) * ROWB;
  const unsigned char *b_rd = smem + BM * ROWB + (wn * TN + l31) * ROWB;

  auto wait_tile = [&](int it) {
    // tiles it+1 .. min(it+STAGES-2, last) may stay in flight; tile `it` must have landed
    // (a wave that issues no copies has nothing outstanding: it learns of the tile at the barrier)
    const int newer = total_tiles - 1 - it;
    if (newer >= STAGES - 2) wait_vmcnt<(STAGES - 2) * IPW>();
    else if (STAGES > 3 && newer == 1) wait_vmcnt<IPW>();
    else if (STAGES > 4 && newer == 2) wait_vmcnt<2 * IPW>();
    else wait_vmcnt<0>();
  };
  if constexpr (H5) {
    static_assert(BM == BN && IA == IB && KS == 4 && PIPE, "half-slot ring shape");
    constexpr int HS = BM * ROWB, NSLOT = 5;
    // the two operands advance through the K segments separately
    int segA = 0, segB = 0, k0A = 0, k0B = 0, KA = Kcur, KB = Kcur, nA = 0, nB = 0;
    const unsigned char *bA = baseA, *bB = baseB;
    const void *gA = uniform_ptr(bA), *gB = uniform_ptr(bB);   // also the source of copies issued past the end
    auto setupA = [&](int sgi) {
      const GemmSeg &S = P.seg[sgi];
#pragma unroll
      for (int j = 0; j < IA; j++) {
        const int rt = (wave * IA + j) * RPI + lrow;
        const int kc = lpos ^ ((rt / RPB) % CPR);
        int r = row0 + rt;
        r = r < M ? r : M - 1;
        offA[j] = (uint32_t)r * (uint32_t)S.lda * 2u + kc * 16;
      }
      bA = reinterpret_cast<const unsigned char *>(S.A);
      KA = S.K;
    };
    auto setupB = [&](int sgi) {
      const GemmSeg &S = P.seg[sgi];
#pragma unroll
      for (int j = 0; j < IB; j++) {
        const int rt = (wave * IB + j) * RPI + lrow;
        const int kc = lpos ^ ((rt / RPB) % CPR);
        int c = col0 + rt;
        c = c < N ? c : N - 1;
        offB[j] = (uint32_t)c * (uint32_t)S.ldb * 2u + kc * 16;
      }
      bB = reinterpret_cast<const unsigned char *>(S.B);
      KB = S.K;
    };
    // Past the last tile the previous address is copied again into the slot that is free anyway,
    // so that the number of copies in flight at every wait is the same constant.
    auto issueA = [&]() {
      if (nA < total_tiles) {
        if (k0A >= KA) {
          segA++;
          setupA(segA);
          k0A = 0;
        }
        gA = uniform_ptr(bA + (size_t)k0A * 2);
        k0A += BK;
      }
      const uint32_t l = lds0 + ((2 * nA) % NSLOT) * HS + wave * IA * 1024;
      if (NPW == NW || wave < NPW) {
#pragma unroll
        for (int j = 0; j < IA; j++) dma16(offA[j], gA, l + j * 1024);
      }
      nA++;
    };
    auto issueB = [&]() {
      if (nB < total_tiles) {
        if (k0B >= KB) {
          segB++;
          setupB(segB);
          k0B = 0;
        }
        gB = uniform_ptr(bB + (size_t)k0B * 2);
        k0B += BK;
      }
      const uint32_t l = lds0 + ((2 * nB + 1) % NSLOT) * HS + wave * IB * 1024;
      if (NPW == NW || wave < NPW) {
#pragma unroll
        for (int j = 0; j < IB; j++) dma16(offB[j], gB, l + j * 1024);
      }
      nB++;
    };
    bf16x8_t af[2][MI], bfr[2][NI];
    const unsigned char *a5 = smem + (wm * TM + l31) * ROWB, *b5 = smem + (wn * TN + l31) * ROWB;
    auto load_frags = [&](int buf, int sa, int sb, int ks) {
      const unsigned char *a = a5 + sa * HS + koff[ks];
      const unsigned char *b = b5 + sb * HS + koff[ks];
#pragma unroll
      for (int i = 0; i < MI; i++) af[buf][i] = *reinterpret_cast<const bf16x8_t *>(a + i * 32 * ROWB);
#pragma unroll
      for (int j = 0; j < NI; j++) bfr[buf][j] = *reinterpret_cast<const bf16x8_t *>(b + j * 32 * ROWB);
    };
    auto mfma_step = [&](int cur) {
#pragma unroll
      for (int i = 0; i < MI; i++)
#pragma unroll
        for (int j = 0; j < NI; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cur][j], af[cur][i], acc[i][j], 0, 0, 0);
    };
    issueA(); issueB(); issueA(); issueB(); issueA();    // A0 B0 A1 B1 A2
    wait_vmcnt<3 * IA>();                                // A0 and B0 have landed
    __syncthreads();
    int sa = 0, sb = 1;                                  // half-slots of the tile being consumed
    load_frags(0, sa, sb, 0);
    for (int t = 0; t + 1 < total_tiles; t++) {
      const int sa1 = sa + 2 >= NSLOT ? sa + 2 - NSLOT : sa + 2;
      const int sb1 = sb + 2 >= NSLOT ? sb + 2 - NSLOT : sb + 2;
#pragma unroll
      for (int ks = 0; ks < KS; ks++) {
        const int cur = ks & 1, nxt = cur ^ 1;
        if (ks + 1 < KS) {
          load_frags(nxt, sa, sb, ks + 1);
        } else {
          wait_vmcnt<IA>();     // A(t+2) may be in flight; A(t+1) and B(t+1) have landed
          __syncthreads();      // ... for every wave, and the half-slots of A(t) and B(t) are free
          issueB();             // B(t+2) into A(t)'s half-slot: needed at the next barrier
          issueA();             // A(t+3) into B(t)'s: needed one barrier later
          load_frags(nxt, sa1, sb1, 0);
        }
        mfma_step(cur);
#pragma unroll
        for (int q = 0; q < MI + NI; q++) {
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read ...
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // ... then one MFMA
        }
        __builtin_amdgcn_sched_group_barrier(0x008, MI * NI - MI - NI, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      sa = sa1;
      sb = sb1;
    }
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      const int cur = ks & 1;
      if (ks + 1 < KS) load_frags(cur ^ 1, sa, sb, ks + 1);
      __builtin_amdgcn_sched_barrier(0);
      mfma_step(cur);
      __builtin_amdgcn_sched_barrier(0);
    }
    wait_vmcnt<0>();            // the copies issued past the end have to be out of the ring
  } else if constexpr (!PIPE) {
    for (int it = 0; it < total_tiles; it++) {
      wait_tile(it);
      __syncthreads();
      issue_next();   // refills the slot that tile it-1 occupied: every wave is past reading it
      const int st = it % STAGES;
      const unsigned char *a = a_rd + st * STAGE_BYTES;
      const unsigned char *b = b_rd + st * STAGE_BYTES;
#pragma unroll
      for (int ks = 0; ks < KS; ks++) {
        bf16x8_t af[MI], bfr[NI];
#pragma unroll
        for (int i = 0; i < MI; i++)
          af[i] = *reinterpret_cast<const bf16x8_t *>(a + i * 32 * ROWB + koff[ks]);
#pragma unroll
        for (int j = 0; j < NI; j++)
          bfr[j] = *reinterpret_cast<const bf16x8_t *>(b + j * 32 * ROWB + koff[ks]);
#pragma unroll
        for (int i = 0; i < MI; i++)
#pragma unroll
          for (int j = 0; j < NI; j++)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
      }
    }
  } else {
    // Register double-buffered fragments: the LDS reads of K step s+1 (or of the next tile's
    // first step, right after its barrier) are issued before the MFMAs of step s.
    bf16x8_t af[2][MI], bfr[2][NI];
    auto load_frags = [&](int buf, int st, int ks) {
      const unsigned char *a = a_rd + st * STAGE_BYTES + koff[ks];
      const unsigned char *b = b_rd + st * STAGE_BYTES + koff[ks];
#pragma unroll
      for (int i = 0; i < MI; i++) af[buf][i] = *reinterpret_cast<const bf16x8_t *>(a + i * 32 * ROWB);
#pragma unroll
      for (int j = 0; j < NI; j++) bfr[buf][j] = *reinterpret_cast<const bf16x8_t *>(b + j * 32 * ROWB);
    };
    auto mfma_step = [&](int cur) {
#pragma unroll
      for (int i = 0; i < MI; i++)
#pragma unroll
        for (int j = 0; j < NI; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cur][j], af[cur][i], acc[i][j], 0, 0, 0);
    };
    wait_tile(0);
    __syncthreads();
    issue_next();
    load_frags(0, 0, 0);
    // All tiles but the last: no data-dependent branch inside, so that the wait counts the
    // compiler derives for the fragment reads are exact (a merge with a path that skips the
    // tile switch would make every post-barrier MFMA wait for the reads just issued).
    for (int it = 0; it + 1 < total_tiles; it++) {
      const int st = it % STAGES;
#pragma unroll
      for (int ks = 0; ks < KS; ks++) {
        const int cur = ks & 1, nxt = cur ^ 1;   // KS is even, so step 0 always uses buffer 0
        if (ks + 1 < KS) {
          load_frags(nxt, st, ks + 1);
        } else {
          wait_tile(it + 1);
          __syncthreads();
          issue_next();
          load_frags(nxt, (it + 1) % STAGES, 0);
        }
        // issue order within the step: one LDS read between consecutive MFMAs, so the reads of
        // the next step trickle out while the matrix pipe is busy
        mfma_step(cur);
#pragma unroll
        for (int q = 0; q < MI + NI; q++) {
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read ...
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // ... then one MFMA
        }
        __builtin_amdgcn_sched_group_barrier(0x008, MI * NI - MI - NI, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    {
      const int st = (total_tiles - 1) % STAGES;
#pragma unroll
      for (int ks = 0; ks < KS; ks++) {
        const int cur = ks & 1;
        if (ks + 1 < KS) load_frags(cur ^ 1, st, ks + 1);
        __builtin_amdgcn_sched_barrier(0);
        mfma_step(cur);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }

  const int cbase = col0 + wn * TN + hi * 4;
  const int rbase = row0 + wm * TM + l31;
  auto store_all = [&](auto *C) {
    typedef typename std::remove_pointer<decltype(C)>::type OutT;
#pragma unroll
    for (int i = 0; i < MI; i++) {
      const int r = rbase + i * 32;
      if (r < M) {
#pragma unroll
        for (int j = 0; j < NI; j++)
#pragma unroll
          for (int g = 0; g < 4; g++) {
            const int c = cbase + j * 32 + g * 8;
            OutT *o = C + (int64_t)r * P.ldc + c;
            if (c + 3 < N && (P.ldc & 3) == 0) {
              store_c4<OutT>(o, acc[i][j][g * 4], acc[i][j][g * 4 + 1], acc[i][j][g * 4 + 2],
                             acc[i][j][g * 4 + 3]);
            } else {
#pragma unroll
              for (int m = 0; m < 4; m++)
                if (c + m < N) store_c<OutT>(o + m, acc[i][j][g * 4 + m]);
            }
          }
      }
    }
  };
  // Outputs whose rows are whole 16-byte pieces: the accumulators go through a per-wave LDS tile
  // (32 rows x TN columns, padded pitch; the ring is free by now) so that every global store is
  // 16 bytes per lane and a whole row segment of the wave tile per group of lanes, instead of
  // short pieces of 32 different rows.  LDS operations of one wave execute in order, so the
  // tile needs no workgroup barrier after the first one.
  auto store_rows = [&](auto *C) {
    typedef typename std::remove_pointer<decltype(C)>::type OutT;
    constexpr int PER = 16 / (int)sizeof(OutT);     // elements per 16-byte piece
    constexpr int EP = TN + PER;                    // tile pitch in elements
    constexpr int CPW = TN / PER, RPW = 64 / CPW;   // pieces per row, rows per instruction
    static_assert(NW * 32 * EP * (int)sizeof(OutT) <= STAGES * STAGE_BYTES, "epilogue tiles fit in the ring");
    static_assert(CPW <= 64 && 32 % RPW == 0, "lane mapping of the row-major stores");
    typedef OutT out4_t __attribute__((ext_vector_type(4)));
    typedef OutT outp_t __attribute__((ext_vector_type(PER)));
    __syncthreads();   // every wave has finished reading the last ring slot
    OutT *tile = reinterpret_cast<OutT *>(smem) + wave * 32 * EP;
    const int rr = lane / CPW, cc = lane % CPW;
    const int c = col0 + wn * TN + cc * PER;
#pragma unroll
    for (int i = 0; i < MI; i++) {
#pragma unroll
      for (int j = 0; j < NI; j++)
#pragma unroll
        for (int g = 0; g < 4; g++) {
          out4_t v;
#pragma unroll
          for (int m = 0; m < 4; m++) v[m] = (OutT)acc[i][j][g * 4 + m];
          *reinterpret_cast<out4_t *>(tile + l31 * EP + j * 32 + g * 8 + hi * 4) = v;
        }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int p = 0; p < 32 / RPW; p++) {
        const int rl = p * RPW + rr;
        const int r = row0 + wm * TM + i * 32 + rl;
        const outp_t v = *reinterpret_cast<const outp_t *>(tile + rl * EP + cc * PER);
        // streaming (non-temporal) stores: an output tile is never read again by this launch,
        // so it should not displace the operand tiles that other workgroups re-read from L2
        if (r < M && c < N) __builtin_nontemporal_store(v, reinterpret_cast<outp_t *>(C + (int64_t)r * P.ldc + c));
      }
      __builtin_amdgcn_wave_barrier();
    }
  };
  const int per = P.c_f32 ? 4 : 8;
  if ((N % per) == 0 && (P.ldc % per) == 0 && (reinterpret_cast<uintptr_t>(P.C) & 15) == 0) {
    if (P.c_f32) store_rows(reinterpret_cast<float *>(P.C));
    else store_rows(reinterpret_cast<bf16_t *>(P.C));
    return;
  }
  if (P.c_f32) store_all(reinterpret_cast<float *>(P.C));
  else store_all(reinterpret_cast<bf16_t *>(P.C));
}

// ---- fp32 storage: 64x64 tile, 256 threads, 4x4 outputs per thread ----------------------
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmBatch args) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const GemmProblem &P = args.p[blockIdx.z];
  const int M = P.M, N = P.N;
  const int tiles_n = (N + BN - 1) / BN;
  const int tm = blockIdx.x / tiles_n, tn = blockIdx.x % tiles_n;
  const int row0 = tm * BM, col0 = tn * BN;
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  float acc[4][4] = {};
  const int lr = tid >> 2, lk = (tid & 3) * 4;   // 64 rows x 4 float4 chunks
  for (int s = 0; s < P.nseg; s++) {
    const GemmSeg &S = P.seg[s];
    const float *A = reinterpret_cast<const float *>(S.A);
    const float *B = reinterpret_cast<const float *>(S.B);
    for (int k0 = 0; k0 < S.K; k0 += BK) {
      float4 va = make_float4(0, 0, 0, 0), vb = va;
      if (k0 + lk < S.K) {   // K % 8 == 0, so a float4 chunk is entirely in or out
        if (row0 + lr < M) va = *reinterpret_cast<const float4 *>(A + (int64_t)(row0 + lr) * S.lda + k0 + lk);
        if (col0 + lr < N) vb = *reinterpret_cast<const float4 *>(B + (int64_t)(col0 + lr) * S.ldb + k0 + lk);
      }
      __syncthreads();
      As[lk + 0][lr] = va.x; As[lk + 1][lr] = va.y; As[lk + 2][lr] = va.z; As[lk + 3][lr] = va.w;
      Bs[lk + 0][lr] = vb.x; Bs[lk + 1][lr] = vb.y; Bs[lk + 2][lr] = vb.z; Bs[lk + 3][lr] = vb.w;
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < BK; kk++) {
        float a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; i++) a[i] = As[kk][ty * 4 + i];
#pragma unroll
        for (int j = 0; j < 4; j++) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
          for (int j = 0; j < 4; j++) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
      }
    }
  }
  float *C = reinterpret_cast<float *>(P.C);
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int r = row0 + ty * 4 + i;
    if (r >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const int c = col0 + tx * 4 + j;
      if (c < N) C[(int64_t)r * P.ldc + c] = acc[i][j];
    }
  }
}

// floating-point operations a launch executes (2 M N K over its problems' K segments)
static double batch_flops(const GemmBatch &b, int nprob) {
  double fl = 0.0;
  for (int i = 0; i < nprob; i++)
    for (int sgi = 0; sgi < b.p[i].nseg; sgi++)
      fl += 2.0 * b.p[i].M * (double)b.p[i].N * b.p[i].seg[sgi].K;
  return fl;
}

template <int BM, int BN, int BK, int WGM, int WGN, typename OutT>
static hipError_t launch_bf16(const GemmBatch &b, int nprob, hipStream_t st) {
  constexpr size_t smem = (size_t)2 * (BM + BN) * (BK + 8) * sizeof(bf16_t);
  auto kern = gemm_bf16_kernel<BM, BN, BK, WGM, WGN, OutT>;
  static bool attr_set = false;   // per template instance; the attribute is per function
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int tiles = ((b.p[0].M + BM - 1) / BM) * ((b.p[0].N + BN - 1) / BN);
  // launches that carry a frozen projection (more than 128 output columns) count as GEMM
  // launches for the measurement hook; a launch of narrow rank-r or router problems does not
  const int slot = prof_on() ? prof_mark_begin(b.p[0].N > 128 ? PROF_GEMM : PROF_OTHER, st) : -1;
  hipLaunchKernelGGL(kern, dim3(tiles, 1, nprob), dim3(WGM * WGN * 64), smem, st, b);
  if (slot >= 0) prof_mark_end(slot, st, b.p[0].N > 128 ? batch_flops(b, nprob) : 0.0);
  return hipGetLastError();
}

template <int BM, int BN, int BK, int STAGES, int WGM, int WGN, bool PIPE = false, int PW = 0, bool H5 = false>
static hipError_t launch_bf16_dl(const GemmBatch &b, int nprob, hipStream_t st) {
  constexpr size_t smem = H5 ? (size_t)5 * BM * BK * sizeof(bf16_t) : (size_t)STAGES * (BM + BN) * BK * sizeof(bf16_t);
  auto kern = gemm_bf16_dl_kernel<BM, BN, BK, STAGES, WGM, WGN, PIPE, PW, H5>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  int tiles = 0;
  for (int i = 0; i < nprob; i++) {
    const int t = ((b.p[i].M + BM - 1) / BM) * ((b.p[i].N + BN - 1) / BN);
    tiles = t > tiles ? t : tiles;
  }
  // every launch of this kernel family is a frozen-projection launch (large tiles at training
  // shapes, the narrow weight-streaming tiles at decode shapes): all count as GEMM launches
  const int slot = prof_on() ? prof_mark_begin(PROF_GEMM, st) : -1;
  hipLaunchKernelGGL(kern, dim3(tiles, 1, nprob), dim3(WGM * WGN * 64), smem, st, b);
  if (slot >= 0) prof_mark_end(slot, st, batch_flops(b, nprob));
  return hipGetLastError();
}

// The direct-to-LDS kernel needs whole K tiles and 32-bit operand offsets.
static bool dl_eligible(const GemmBatch &b, int nprob, int BK) {
  for (int i = 0; i < nprob; i++) {
    const GemmProblem &p = b.p[i];
    for (int sgi = 0; sgi < p.nseg; sgi++) {
      const GemmSeg &sg = p.seg[sgi];
      if (sg.K <= 0 || sg.K % BK) return false;
      if ((uint64_t)p.M * (uint64_t)sg.lda * 2 >= (1ull << 32)) return false;
      if ((uint64_t)p.N * (uint64_t)sg.ldb * 2 >= (1ull << 32)) return false;
    }
  }
  return true;
}

bool gemm_mixed_rows_ok(int dtype, const GemmProblem *probs, int nprob) {
  if (dtype != MIXLORA_BF16 || nprob < 1 || nprob > GEMM_MAX_PROBLEMS) return false;
  GemmBatch b;
  bool any_big = false;
  for (int i = 0; i < GEMM_MAX_PROBLEMS; i++) b.p[i] = probs[i < nprob ? i : 0];
  for (int i = 0; i < nprob; i++) {
    if (probs[i].M <= 128 || probs[i].N <= 0) return false;
    if (probs[i].N > 128) any_big = true;
  }
  return any_big && dl_eligible(b, nprob, 64);
}

hipError_t launch_gemm(int dtype, const GemmProblem *probs, int nprob, hipStream_t st) {
  if (nprob < 1 || nprob > GEMM_MAX_PROBLEMS) return hipErrorInvalidValue;
  GemmBatch b;
  for (int i = 0; i < GEMM_MAX_PROBLEMS; i++) b.p[i] = probs[i < nprob ? i : 0];
  const int M = probs[0].M, N = probs[0].N;
  bool uniform = true, any_big = false, same_m = true;
  for (int i = 0; i < nprob; i++) {
    if (probs[i].M != M) same_m = false;
    if (probs[i].N != N || probs[i].c_f32 != probs[0].c_f32) uniform = false;
    if (probs[i].N > 128) any_big = true;
    if (probs[i].N <= 0) return hipErrorInvalidValue;
  }
  if (!same_m) {
    // problems of different row counts (per-token and per-pair operands) can share a launch of
    // the large-tile kernel only: every tile takes M from its own problem
    if (!gemm_mixed_rows_ok(dtype, probs, nprob)) return hipErrorInvalidValue;
    return launch_bf16_dl<256, 256, 64, 2, 2, 4, true, 4>(b, nprob, st);
  }
  if (M <= 0) return hipSuccess;
  if (dtype == MIXLORA_BF16 && M > 128 && any_big) {
    // large tiles: direct-to-LDS ring; BK = 64 needs whole 64-wide K tiles, else BK = 32.
    // Problems of one launch may differ in N and output type (narrow ones ride in the slack
    // of the last, partially filled round of workgroups).
    if (dl_eligible(b, nprob, 64)) {
      // long K (the down projection and the input-gradient products): the half-slot ring
      bool long_k = true;
      for (int i = 0; i < nprob; i++) {
        int64_t kt = 0;
        for (int sgi = 0; sgi < probs[i].nseg; sgi++) kt += probs[i].seg[sgi].K;
        if (kt < GEMM_LONG_K) long_k = false;
      }
      if (long_k) return launch_bf16_dl<256, 256, 64, 2, 2, 4, true, 4, true>(b, nprob, st);
      return launch_bf16_dl<256, 256, 64, 2, 2, 4, true, 4>(b, nprob, st);
    }
    if (dl_eligible(b, nprob, 32)) return launch_bf16_dl<256, 256, 32, 4, 2, 4, false>(b, nprob, st);
  }
  if (dtype == MIXLORA_BF16 && M <= 128 && any_big && dl_eligible(b, nprob, 64)) {
    // few rows (decode-shaped calls): the launch is bound by streaming the weights once, so the
    // tiles are narrow (64 output columns: enough workgroups to cover the chip) and the ring is
    // deep (4 K tiles in flight per workgroup, 2 workgroups per CU)
    if (M <= 64) return launch_bf16_dl<64, 64, 64, 4, 1, 2, false>(b, nprob, st);
    return launch_bf16_dl<128, 64, 64, 4, 2, 2, false>(b, nprob, st);
  }
  if (!uniform || nprob > 2) {   // the generic kernels take uniform batches of at most two
    for (int i = 0; i < nprob; i++) {
      const hipError_t e = launch_gemm(dtype, probs + i, 1, st);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  if (dtype == MIXLORA_F32) {
    const int tiles = ((M + 63) / 64) * ((N + 63) / 64);
    hipLaunchKernelGGL(gemm_f32_kernel, dim3(tiles, 1, nprob), dim3(256), 0, st, b);
    return hipGetLastError();
  }
  const bool f32out = probs[0].c_f32 != 0;
  if (N <= 128 || M <= 128) {
    return f32out ? launch_bf16<128, 128, 64, 2, 2, float>(b, nprob, st)
                  : launch_bf16<128, 128, 64, 2, 2, bf16_t>(b, nprob, st);
  }
  return f32out ? launch_bf16<256, 256, 64, 2, 4, float>(b, nprob, st)
                : launch_bf16<256, 256, 64, 2, 4, bf16_t>(b, nprob, st);
}

}  // namespace mixlora
