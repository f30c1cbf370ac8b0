// Device-side building blocks of the DSSD verification kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dssd {

constexpr int kWave = 64;
constexpr int kUnroll = 8;                    // 16-byte vectors per lane per chunk
constexpr int kChunkVecs = kWave * kUnroll;   // 512 vectors = 8 KiB of logits per chunk
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <bool BF16> struct Elems { static constexpr int per_vec = BF16 ? 8 : 4; };
template <bool BF16> constexpr int chunk_elems() { return kChunkVecs * Elems<BF16>::per_vec; }

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float as_float(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }
__device__ __forceinline__ float neg_inf() { return as_float(0xFF800000u); }
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
// largest float below a positive finite x; 0 for x <= 0
__device__ __forceinline__ float next_below(float x) { return x > 0.f ? as_float(as_u32(x) - 1u) : 0.f; }

// ------------------------------------------------------------------ Philox4x32-10
// Counter-based generator of Salmon, Moraes, Dror and Shaw (SC'11): ten rounds, each
// replacing (c0,c1,c2,c3) by (hi(B*c2)^c1^k0, lo(B*c2), hi(A*c0)^c3^k1, lo(A*c0)) and then
// advancing the key by two Weyl constants.
struct Philox {
  uint32_t w[4];
  __device__ __forceinline__ Philox(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                    uint32_t k1) {
    constexpr uint32_t A = 0xD2511F53u, Bm = 0xCD9E8D57u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
      const uint32_t hiA = __umulhi(A, c0), loA = A * c0;
      const uint32_t hiB = __umulhi(Bm, c2), loB = Bm * c2;
      const uint32_t n0 = hiB ^ c1 ^ k0, n2 = hiA ^ c3 ^ k1;
      c0 = n0; c1 = loB; c2 = n2; c3 = loA;
      k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    w[0] = c0; w[1] = c1; w[2] = c2; w[3] = c3;
  }
};
// The block of (session, position) at the launch's step.  The step is the host's value plus,
// when step_dev is given, a 64-bit counter in device memory read at run time: a captured graph
// then draws fresh numbers on every replay if the caller bumps the counter between replays.
__device__ __forceinline__ Philox step_block(uint32_t session, uint32_t position, uint32_t step_lo,
                                             uint32_t step_hi, const uint64_t* step_dev, uint32_t seed_lo,
                                             uint32_t seed_hi) {
  uint64_t step = ((uint64_t)step_hi << 32) | step_lo;
  if (step_dev) step += *step_dev;
  return Philox(session, position, (uint32_t)step, (uint32_t)(step >> 32), seed_lo, seed_hi);
}
// top 24 bits -> [0,1), exact in fp32
__device__ __forceinline__ float u01(uint32_t word) { return (float)(word >> 8) * 5.9604644775390625e-8f; }

// ------------------------------------------------------------------ wave64 reductions (DPP)
template <int CTRL> __device__ __forceinline__ float dpp(float x) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float lane_value(float x, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), lane));
}
// Every lane receives the result.  Fixed pairing order: xor 1, xor 2, mirror within 8, mirror
// within 16, then the four rows of 16 lanes.
__device__ __forceinline__ float wave_max(float x) {
  x = fmaxf(x, dpp<0xB1>(x));    // quad_perm [1,0,3,2]
  x = fmaxf(x, dpp<0x4E>(x));    // quad_perm [2,3,0,1]
  x = fmaxf(x, dpp<0x141>(x));   // row_half_mirror
  x = fmaxf(x, dpp<0x140>(x));   // row_mirror
  return fmaxf(fmaxf(lane_value(x, 0), lane_value(x, 16)), fmaxf(lane_value(x, 32), lane_value(x, 48)));
}
__device__ __forceinline__ float wave_sum(float x) {
  x += dpp<0xB1>(x);
  x += dpp<0x4E>(x);
  x += dpp<0x141>(x);
  x += dpp<0x140>(x);
  return (lane_value(x, 0) + lane_value(x, 16)) + (lane_value(x, 32) + lane_value(x, 48));
}
// Inclusive prefix sum over the 64 lanes, in lane order, on the DPP path (no LDS traffic): four
// shifted adds inside each row of 16 lanes (a lane whose source falls outside its row adds 0),
// then lane 15 of rows 0 and 2 is broadcast into rows 1 and 3, then lane 31 into the upper half.
// Each lane sums its own tree, so with rounding the result need not be monotone across lanes:
// callers that search it for a threshold must also ask for a positive weight.
template <int CTRL, int ROW_MASK> __device__ __forceinline__ float dpp_or_zero(float x) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, ROW_MASK, 0xF, false));
}
__device__ __forceinline__ float wave_scan(float x, int /*lane*/) {
  x += dpp_or_zero<0x111, 0xF>(x);   // row_shr:1
  x += dpp_or_zero<0x112, 0xF>(x);   // row_shr:2
  x += dpp_or_zero<0x114, 0xF>(x);   // row_shr:4
  x += dpp_or_zero<0x118, 0xF>(x);   // row_shr:8
  x += dpp_or_zero<0x142, 0xA>(x);   // row_bcast:15 into rows 1 and 3
  x += dpp_or_zero<0x143, 0xC>(x);   // row_bcast:31 into rows 2 and 3
  return x;
}

// ------------------------------------------------------------------ row access
// Loads the `vec`-th group of per_vec consecutive logits of a row as floats.  Entries at or
// beyond V read as -inf.  ALIGNED: the row starts on a 16-byte boundary and V is a multiple of
// per_vec, so the group is one 128-bit load; it is issued non-temporal (the rows are streamed
// once and far exceed the caches) and without a branch (the address is clamped into the row,
// the value replaced afterwards).
// INSIDE (rows that are not ALIGNED): the caller knows that the whole group lies within the row;
// it is then one 128-bit load at the row's element alignment, which the hardware serves at any
// alignment (a load that straddles cache lines costs a second access), instead of per_vec scalar
// loads.
typedef u32x4 u32x4_at2 __attribute__((aligned(2)));
typedef u32x4 u32x4_at4 __attribute__((aligned(4)));
typedef f32x4 f32x4_at4 __attribute__((aligned(4)));
template <bool BF16, bool ALIGNED, bool INSIDE = false>
__device__ __forceinline__ void load_logits(const void* row, int64_t vec, int32_t V, float* z) {
  constexpr int E = Elems<BF16>::per_vec;
  const int64_t e0 = vec * E;
  if constexpr (!ALIGNED && INSIDE) {
    u32x4 v;
    if constexpr (BF16)
      v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_at2*>(static_cast<const uint16_t*>(row) + e0));
    else
      v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_at4*>(static_cast<const float*>(row) + e0));
    if constexpr (BF16) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        z[2 * i] = as_float(v[i] << 16);
        z[2 * i + 1] = as_float(v[i] & 0xFFFF0000u);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) z[i] = as_float(v[i]);
    }
  } else if constexpr (ALIGNED) {
    const int64_t last = V / E - 1;
    const bool inside = vec <= last;
    const u32x4* p = reinterpret_cast<const u32x4*>(row) + (inside ? vec : last);
    u32x4 v = __builtin_nontemporal_load(p);
    if (!inside) {
      const uint32_t ninf = BF16 ? 0xFF80FF80u : 0xFF800000u;
      v = (u32x4){ninf, ninf, ninf, ninf};
    }
    if constexpr (BF16) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        z[2 * i] = as_float(v[i] << 16);
        z[2 * i + 1] = as_float(v[i] & 0xFFFF0000u);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) z[i] = as_float(v[i]);
    }
  } else {
#pragma unroll
    for (int i = 0; i < E; ++i) {
      const int64_t e = e0 + i;
      float x = neg_inf();
      if (e < V) {
        if constexpr (BF16) x = as_float((uint32_t) static_cast<const uint16_t*>(row)[e] << 16);
        else x = static_cast<const float*>(row)[e];
      }
      z[i] = x;
    }
  }
}
__device__ __forceinline__ float load_logit(const void* row, int64_t e, bool bf16) {
  return bf16 ? as_float((uint32_t) static_cast<const uint16_t*>(row)[e] << 16)
              : static_cast<const float*>(row)[e];
}
// Loads draft probabilities [e0, e0+N) of a row (N = 4 or 8, e0 a multiple of N); entries at
// or beyond V read as 0.  ALIGNED as above: non-temporal 128-bit loads, clamped, no branch.
template <int N, bool ALIGNED, bool INSIDE = false>
__device__ __forceinline__ void load_probs(const float* row, int64_t e0, int32_t V, float* q) {
  if constexpr (!ALIGNED && INSIDE) {
    const f32x4_at4* p = reinterpret_cast<const f32x4_at4*>(row + e0);
#pragma unroll
    for (int i = 0; i < N / 4; ++i) {
      const f32x4 v = __builtin_nontemporal_load(p + i);
      q[4 * i] = v[0]; q[4 * i + 1] = v[1]; q[4 * i + 2] = v[2]; q[4 * i + 3] = v[3];
    }
  } else if constexpr (ALIGNED) {
    const bool inside = e0 < V;
    const f32x4* p = reinterpret_cast<const f32x4*>(row + (inside ? e0 : (int64_t)V - N));
#pragma unroll
    for (int i = 0; i < N / 4; ++i) {
      const f32x4 v = __builtin_nontemporal_load(p + i);
      q[4 * i] = inside ? v[0] : 0.f; q[4 * i + 1] = inside ? v[1] : 0.f;
      q[4 * i + 2] = inside ? v[2] : 0.f; q[4 * i + 3] = inside ? v[3] : 0.f;
    }
  } else {
#pragma unroll
    for (int i = 0; i < N; ++i) q[i] = (e0 + i < V) ? row[e0 + i] : 0.f;
  }
}

// ------------------------------------------------------------------ cross-workgroup hand-over
// A value written by one workgroup and read by another inside the same launch.  publish()
// writes it through to the device-coherent level, stores_done() holds the wave until every
// store it has issued is acknowledged there, arrive() does that and then bumps a counter,
// observe() reads at the device-coherent level.  A reader that saw the counter complete
// therefore finds every value published before the matching arrive().  No cache-wide
// write-back or invalidate is involved, so streaming waves are not disturbed.
__device__ __forceinline__ void publish(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float observe(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void publish2(float2* p, float2 v) {
  const uint64_t bits = (uint64_t)as_u32(v.x) | ((uint64_t)as_u32(v.y) << 32);
  __hip_atomic_store(reinterpret_cast<uint64_t*>(p), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 observe2(const float2* p) {
  const uint64_t bits =
      __hip_atomic_load(reinterpret_cast<const uint64_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(as_float((uint32_t)bits), as_float((uint32_t)(bits >> 32)));
}
// A workgroup-scope release fence orders the compiler but emits no wait on this target (the
// waves of a workgroup share one vector cache), and the counter usually lives in another
// memory channel than the published values: without the explicit wait the increment could be
// performed before a published store has landed.
__device__ __forceinline__ void stores_done() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}
__device__ __forceinline__ int32_t arrive(int32_t* counter) {
  stores_done();
  return __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Consecutive workgroup ids are dealt round-robin to the chip's XCDs (8 on MI355X; the host reads
// the count from the device).  This maps a hardware workgroup id to a logical one so that each
// XCD walks one contiguous share of the work (and of the address range) instead of every n-th
// block of it.  Workgroups beyond the last full round keep their id.
__device__ __forceinline__ int64_t xcd_contiguous(uint32_t block, uint32_t blocks, uint32_t xcds) {
  const uint32_t per = blocks / xcds;
  return block < per * xcds ? (int64_t)(block % xcds) * per + block / xcds : (int64_t)block;
}

}  // namespace dssd
