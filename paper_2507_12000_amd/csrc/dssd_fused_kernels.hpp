// Single-launch verification step for small batches with uniform gamma (the paper's own
// scenario is one session per device; Algorithm 1 with everything at the edge).  When a batch
// has only a few thousand chunks the step is bound by launch latency, not by HBM, so the five
// kernels of the streaming path are chained inside one launch:
//
//   every workgroup   : softmax statistics of up to sixteen chunks of its session's rows, published
//                       with device-coherent stores; then it bumps the session's arrival counter;
//   the workgroup that arrives last for a session goes on alone (no workgroup ever waits):
//                       merges the rows, runs the accept / first-reject scan, and either
//                       - computes the residual chunk masses of the rejected row with its
//                         waves and draws the token, or
//                       - draws the bonus token from the chunk statistics.
// Results are bit-identical to the three-call path: the same device functions in the same order.
#pragma once
#include "dssd_kernels.hpp"

namespace dssd {

// Workgroups of kFusedWaves waves: the lone workgroup that finishes a session streams the
// rejected row with all of them, which is what bounds the step (16 waves cover a row of 16
// chunks in one round trip; with 4 the same row took four).
constexpr int kFusedWaves = 16;
constexpr int kFusedMassSlots = 64;   // chunk masses kept in LDS when a row has at most this many chunks

// TAIL_RESID = false leaves the redraw of rejected sessions to a following resid_mass launch
// (rows too long for one workgroup to stream alone): two launches instead of four.
template <bool BF16, bool ALIGNED, bool TAIL_RESID>
__global__ __launch_bounds__(kFusedWaves * kWave) void fused_small_step(const BatchView a, int32_t groups,
                                                                        int32_t* arrive_stats) {
  __shared__ int32_t sh_last;
  __shared__ float sh_mass[kFusedMassSlots];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int32_t b = blockIdx.x / groups;
  const int32_t j = blockIdx.x - b * groups;
  const int32_t g = a.gamma;                         // uniform gamma only
  const int64_t lrow0 = (int64_t)b * (g + 1);
  const int32_t ntask = (g + 1) * a.C;               // chunk tasks of this session
  const int32_t t = j * kFusedWaves + wave;
  if (t < ntask) {
    const int32_t i = t / a.C, c = t - i * a.C;
    auto c1_of = [&]() { return (a.inv_temp ? a.inv_temp[b] : 1.f) * kLog2e; };
    const float2 st = chunk_stats_of<BF16, ALIGNED>(logits_row<BF16>(a, lrow0 + i), c, a.V, c1_of, lane);
    if (lane == 0) {
      publish2(a.chunk_stats + (lrow0 + i) * a.C + c, st);
      stores_done();   // acknowledged before the barrier that precedes the arrival
    }
  }
  __syncthreads();
  if (threadIdx.x == 0)
    sh_last = __hip_atomic_fetch_add(arrive_stats + b, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == groups - 1;
  __syncthreads();
  if (!sh_last) return;
  if (threadIdx.x == 0) __hip_atomic_store(arrive_stats + b, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

  // ---- the last workgroup of session b carries the session to its token
  Job job;
  const int32_t kind = accept_session<BF16>(a, b, &job);
  if (kind == 1) {
    if constexpr (!TAIL_RESID) return;
    const bool in_lds = a.C <= kFusedMassSlots;
    for (int32_t c = wave; c < a.C; c += kFusedWaves) {
      const float m = resid_chunk_mass<BF16, ALIGNED, kUnroll>(a, b, job, c, lane);
      if (lane == 0) {
        if (in_lds) sh_mass[c] = m;
        else publish(a.resid_mass + (int64_t)b * a.C + c, m);
      }
    }
    if (!in_lds && lane == 0) stores_done();
    __syncthreads();
    if (wave == 0) pick_for_session<BF16, ALIGNED, true>(a, b, job, lane, in_lds ? sh_mass : nullptr);
  } else if (kind == 2) {
    if (wave == 0) pick_for_session<BF16, ALIGNED, false>(a, b, job, lane);
  }
}

}  // namespace dssd
