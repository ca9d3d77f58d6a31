// Body of the batched weight re-layout (see csrc/elementwise.hip), shared with the launch that
// runs it beside the routing of a forward pass (csrc/router.hip).
#pragma once
#include "common.h"

namespace mixlora {

struct RelayoutBatch {
  RelayoutJob job[RELAYOUT_MAX_JOBS];
};

// One job, as block bx of gx blocks (any workgroup size; every thread of the workgroup calls it).
template <typename E>
__device__ __forceinline__ void relayout_body(const RelayoutJob &J, int bx, int gx) {
  const E *__restrict__ src = reinterpret_cast<const E *>(J.src);
  E *__restrict__ dst = reinterpret_cast<E *>(J.dst);
  if (J.zero_bytes) {   // plain zero fill, 16 bytes per store (dst is 16-byte aligned)
    uint4 *z = reinterpret_cast<uint4 *>(J.dst);
    const size_t nv = J.zero_bytes / 16;
    for (size_t i = (size_t)bx * blockDim.x + threadIdx.x; i < nv; i += (size_t)gx * blockDim.x)
      z[i] = make_uint4(0u, 0u, 0u, 0u);
    return;
  }
  if (J.batched_transpose) {
    // dst[dst0 + b*d0 + q*d1 + p] = scale * src[b*s0 + p*n2 + q] for b < n0, p < n1, q < n2
    // (zeros where p >= valid2): 64x64 tiles through LDS so that both the reads and the writes
    // run along a contiguous dimension (long thin tiles for the rank-wide banks were measured
    // slower)
    constexpr int TP = 64, TQ = 64, pitch = TQ + 1;
    __shared__ float tile[TP * pitch];
    const int P = J.n1, Q = J.n2, PV = J.valid2;
    const int tp = (P + TP - 1) / TP, tq = (Q + TQ - 1) / TQ;
    const int ntiles = J.n0 * tp * tq;
    for (int tid = bx; tid < ntiles; tid += gx) {
      const int b = tid / (tp * tq), rem = tid % (tp * tq);
      const int p0 = (rem / tq) * TP, q0 = (rem % tq) * TQ;
      const int hp = P - p0 < TP ? P - p0 : TP, hq = Q - q0 < TQ ? Q - q0 : TQ;
      // reads walk the source rows (hq contiguous elements each; one contiguous block when the
      // whole row fits), writes walk the destination rows (hp contiguous elements each)
      for (int x = threadIdx.x; x < hp * hq; x += (int)blockDim.x) {
        const int i = x / hq, j = x - i * hq;
        tile[i * pitch + j] =
            p0 + i < PV ? J.scale * to_f32(src[b * J.s0 + (int64_t)(p0 + i) * Q + q0 + j]) : 0.f;
      }
      __syncthreads();
      for (int x = threadIdx.x; x < hp * hq; x += (int)blockDim.x) {
        const int j = x / hp, i = x - j * hp;
        dst[J.dst0 + b * J.d0 + (q0 + j) * J.d1 + p0 + i] = from_f32<E>(tile[i * pitch + j]);
      }
      __syncthreads();
    }
    return;
  }
  // element counts are below 2^31 (checked by the launcher): 32-bit index arithmetic
  const unsigned n2 = J.n2, n1 = J.n1, total = (unsigned)J.n0 * n1 * n2;
  for (unsigned o = (unsigned)bx * blockDim.x + threadIdx.x; o < total; o += (unsigned)gx * blockDim.x) {
    const unsigned i2 = o % n2, t = o / n2;
    const unsigned i1 = t % n1, i0 = t / n1;
    const float v = (int)i2 < J.valid2 ? J.scale * to_f32(src[i0 * J.s0 + i1 * J.s1 + i2 * J.s2]) : 0.f;
    dst[J.dst0 + i0 * J.d0 + i1 * J.d1 + i2 * J.d2] = from_f32<E>(v);
  }
}

// blocks per job for a launch of these jobs (one per 256 elements or per 64x64 tile, capped:
// grid-stride beyond that); 0 if a job is too large for 32-bit indexing
inline int64_t relayout_blocks(const RelayoutJob *jobs, int njobs) {
  int64_t most = 1;
  for (int i = 0; i < njobs; i++) {
    const RelayoutJob &j = jobs[i];
    const int64_t n = (int64_t)j.n0 * j.n1 * j.n2;
    if (n >= ((int64_t)1 << 31)) return 0;
    const int64_t want = j.batched_transpose ? (int64_t)j.n0 * ((j.n1 + 63) / 64) * ((j.n2 + 63) / 64)
                         : j.zero_bytes      ? (int64_t)(j.zero_bytes / 16 + 255) / 256
                                             : (n + 255) / 256;
    most = want > most ? want : most;
  }
  return most > 8192 ? 8192 : most;
}

}  // namespace mixlora
