// Small kernels that are not part of the step: they expose pieces of it for checking.
#pragma once
#include "dssd_device.hpp"

namespace dssd {

// The random block of every (session, position) in a rectangle, exactly as the step's kernels
// form it: counter = (session, position, step_lo, step_hi), key = (seed_lo, seed_hi).
// words[(s * n_positions + p) * 4 + k] = word k of session_first + s, position_first + p
// (32-bit wrap-around in both).
__global__ __launch_bounds__(256) void random_words(uint32_t session_first, uint32_t position_first,
                                                    int32_t n_sessions, int32_t n_positions, uint32_t step_lo,
                                                    uint32_t step_hi, uint32_t seed_lo, uint32_t seed_hi,
                                                    uint32_t* words) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= (int64_t)n_sessions * n_positions) return;
  const uint32_t s = (uint32_t)(t / n_positions), p = (uint32_t)(t - (int64_t)s * n_positions);
  const Philox rnd(session_first + s, position_first + p, step_lo, step_hi, seed_lo, seed_hi);
#pragma unroll
  for (int k = 0; k < 4; ++k) words[t * 4 + k] = rnd.w[k];
}

}  // namespace dssd
