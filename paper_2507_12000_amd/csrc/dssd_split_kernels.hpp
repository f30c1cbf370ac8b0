// Kernels of the DSSD split proper (arXiv 2507.12000, Sec. 3, Algorithm 2): what crosses the
// link.  The edge materialises the one distribution P_j it has to send down after a rejection
// ("Downlink Transmission": P_j(x) and j), in b_prob = 32 or 16 bit; the device redraws from the
// received P_j and its own Q_j ("Resample") without ever seeing logits.
#pragma once
#include "dssd_kernels.hpp"

namespace dssd {

// ---------------------------------------------------------------------------------------
// Edge: write P_n(v) = 2^(z_v*c1 - M2)/Z of every rejected session's row n to p_rows[b, :].
// One wave per chunk of the row, as in resid_mass.  Streaming read + streaming write.
// ---------------------------------------------------------------------------------------
template <bool BF16, bool ALIGNED, bool F16OUT>
__global__ __launch_bounds__(256) void export_p_rows(const BatchView a, int32_t groups, void* p_rows) {
  constexpr int E = Elems<BF16>::per_vec;
  const int lane = threadIdx.x & 63;
  const int32_t b = (int32_t)(blockIdx.x / groups);
  const int32_t c = (int32_t)(blockIdx.x - (int64_t)b * groups) * 4 + (threadIdx.x >> 6);
  if (c >= a.C) return;
  const Job job = a.resid_job[b];
  if (job.lrow < 0) return;
  const float c1 = (a.inv_temp ? a.inv_temp[b] : 1.f) * kLog2e;
  const float invZ = 1.f / job.Z;
  const char* lp = logits_row<BF16>(a, job.lrow);
  const int64_t v0 = (int64_t)c * kChunkVecs + lane;
  char* out_row = static_cast<char*>(p_rows) + (int64_t)b * a.V * (F16OUT ? 2 : 4);
  // Rows that are not 16-byte aligned: a chunk that lies entirely inside the row (wave-uniform)
  // is read and written with vector accesses at the rows' own alignment, the last chunk scalar.
  const bool inside = !ALIGNED && (int64_t)(c + 1) * kChunkVecs * E <= a.V;
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  typedef u32x2 u32x2_at2 __attribute__((aligned(2)));
  using Store16 = typename std::conditional<ALIGNED, u32x4, u32x4_at2>::type;
  using Store8 = typename std::conditional<ALIGNED, u32x2, u32x2_at2>::type;
  using StoreF4 = typename std::conditional<ALIGNED, f32x4, f32x4_at4>::type;
#pragma unroll
  for (int k0 = 0; k0 < kUnroll; k0 += 4) {
    float z[4][E];
    if (inside) {
#pragma unroll
      for (int k = 0; k < 4; ++k) load_logits<BF16, ALIGNED, true>(lp, v0 + (k0 + k) * kWave, a.V, z[k]);
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) load_logits<BF16, ALIGNED>(lp, v0 + (k0 + k) * kWave, a.V, z[k]);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int64_t e0 = (v0 + (k0 + k) * kWave) * E;
      float p[E];
#pragma unroll
      for (int e = 0; e < E; ++e) p[e] = fast_exp2(fmaf(z[k][e], c1, -job.M2)) * invZ;
      // aligned rows: V is a multiple of E, so a group that starts inside the row lies inside it
      const bool whole = ALIGNED ? e0 < a.V : inside;
      if (whole) {
        if constexpr (F16OUT) {
          uint32_t packed[E / 2];
#pragma unroll
          for (int e = 0; e < E; e += 2) {
            const _Float16 lo = (_Float16)p[e], hi = (_Float16)p[e + 1];
            packed[e / 2] = (uint32_t)__builtin_bit_cast(uint16_t, lo) |
                            ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
          }
          if constexpr (E == 8) {
            const u32x4 v = {packed[0], packed[1], packed[2], packed[3]};
            __builtin_nontemporal_store(v, reinterpret_cast<Store16*>(out_row + e0 * 2));
          } else {
            const u32x2 v = {packed[0], packed[1]};
            __builtin_nontemporal_store(v, reinterpret_cast<Store8*>(out_row + e0 * 2));
          }
        } else {
#pragma unroll
          for (int i = 0; i < E / 4; ++i) {
            const f32x4 v = {p[4 * i], p[4 * i + 1], p[4 * i + 2], p[4 * i + 3]};
            __builtin_nontemporal_store(v, reinterpret_cast<StoreF4*>(out_row + (e0 + 4 * i) * 4));
          }
        }
      } else if constexpr (!ALIGNED) {
#pragma unroll
        for (int e = 0; e < E; ++e) {
          if (e0 + e < a.V) {
            if constexpr (F16OUT) reinterpret_cast<_Float16*>(out_row)[e0 + e] = (_Float16)p[e];
            else reinterpret_cast<float*>(out_row)[e0 + e] = p[e];
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// Device: everything it knows -- its Q rows, the received P_j rows and j.
// ---------------------------------------------------------------------------------------
struct DeviceView {
  int32_t B, V, gamma, C;            // C = chunks of 4096 entries per row
  int64_t R_Q;
  const int32_t* offsets;            // may be null
  const float* draft_probs;          // [R_Q, V]
  const void* p_rows;                // [B, V] fp16 or fp32
  const int32_t* accepted_len;       // [B] received j - 1
  const int32_t* rejected;           // [B]
  uint32_t seed_lo, seed_hi, step_lo, step_hi, session_base;
  const uint64_t* step_dev;          // may be null: device-resident counter added to the step
  int32_t* out_token;                // [B]
  int32_t* status;                   // may be null
  float* resid_mass;                 // workspace [B, C]
};

// Groups of 8 entries of a probability row (16 bytes of fp16, 32 bytes of fp32).
// INSIDE (rows that are not ALIGNED): the group is known to lie within the row and is read with
// vector loads at the row's element alignment.
template <bool PF16, bool ALIGNED, bool INSIDE = false>
__device__ __forceinline__ void load_p8(const void* row, int64_t g, int32_t V, float* p) {
  const int64_t e0 = g * 8;
  if constexpr (!ALIGNED && INSIDE) {
    if constexpr (PF16) {
      const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_at2*>(static_cast<const uint16_t*>(row) + e0));
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        p[2 * i] = (float)__builtin_bit_cast(_Float16, (uint16_t)(v[i] & 0xFFFFu));
        p[2 * i + 1] = (float)__builtin_bit_cast(_Float16, (uint16_t)(v[i] >> 16));
      }
    } else {
      const f32x4_at4* q = reinterpret_cast<const f32x4_at4*>(static_cast<const float*>(row) + e0);
      const f32x4 lo = __builtin_nontemporal_load(q), hi = __builtin_nontemporal_load(q + 1);
      p[0] = lo[0]; p[1] = lo[1]; p[2] = lo[2]; p[3] = lo[3];
      p[4] = hi[0]; p[5] = hi[1]; p[6] = hi[2]; p[7] = hi[3];
    }
  } else if constexpr (ALIGNED) {
    const int64_t last = V / 8 - 1;
    const bool inside = g <= last;
    const int64_t gg = inside ? g : last;
    if constexpr (PF16) {
      const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(row) + gg);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        p[2 * i] = (float)__builtin_bit_cast(_Float16, (uint16_t)(v[i] & 0xFFFFu));
        p[2 * i + 1] = (float)__builtin_bit_cast(_Float16, (uint16_t)(v[i] >> 16));
      }
    } else {
      const f32x4 lo = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(row) + 2 * gg);
      const f32x4 hi = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(row) + 2 * gg + 1);
      p[0] = lo[0]; p[1] = lo[1]; p[2] = lo[2]; p[3] = lo[3];
      p[4] = hi[0]; p[5] = hi[1]; p[6] = hi[2]; p[7] = hi[3];
    }
    if (!inside) {
#pragma unroll
      for (int i = 0; i < 8; ++i) p[i] = 0.f;
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float x = 0.f;
      if (e0 + i < V) {
        if constexpr (PF16) x = (float)static_cast<const _Float16*>(row)[e0 + i];
        else x = static_cast<const float*>(row)[e0 + i];
      }
      p[i] = x;
    }
  }
}

// w = max(0, P~ - Q) (RESID) or w = P~ (fallback when the residual has no mass).
template <bool PF16, bool ALIGNED, bool RESID, bool INSIDE = false>
struct ProbWeights {
  static constexpr int E = 8;
  static constexpr bool kAligned = ALIGNED;
  const void* pp; const float* qp; int32_t V;
  __device__ __forceinline__ ProbWeights<PF16, ALIGNED, RESID, true> inside() const { return {pp, qp, V}; }
  __device__ __forceinline__ float group(int64_t g, float* w) const {
    float p[8];
    load_p8<PF16, ALIGNED, INSIDE>(pp, g, V, p);
    float sum = 0.f;
    if constexpr (RESID) {
      float q[8];
      load_probs<8, ALIGNED, INSIDE>(qp, g * 8, V, q);
#pragma unroll
      for (int e = 0; e < 8; ++e) { w[e] = fmaxf(0.f, p[e] - q[e]); sum += w[e]; }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) { w[e] = p[e]; sum += w[e]; }
    }
    return sum;
  }
};

// Session b's record as the device received it; false if it has nothing to redraw or the
// record is inconsistent (then status gets DSSD_SESSION_BAD_OFFSETS = 4 and out_token = -1).
__device__ __forceinline__ bool device_session(const DeviceView& d, int32_t b, int64_t* qrow, int32_t* n_out,
                                               bool report) {
  if (!d.rejected[b]) return false;
  const int64_t off0 = d.offsets ? (int64_t)d.offsets[b] : (int64_t)b * d.gamma;
  const int64_t off1 = d.offsets ? (int64_t)d.offsets[b + 1] : off0 + d.gamma;
  const int32_t n = d.accepted_len[b];
  if (off0 < 0 || off1 < off0 || off1 > d.R_Q || n < 0 || n >= off1 - off0) {
    if (report) {
      d.out_token[b] = -1;
      if (d.status) d.status[b] = 4;
    }
    return false;
  }
  *qrow = off0 + n;
  *n_out = n;
  return true;
}

template <bool PF16, bool ALIGNED>
__global__ __launch_bounds__(256) void device_resid_mass(const DeviceView d, int32_t groups) {
  const int lane = threadIdx.x & 63;
  const int32_t b = (int32_t)(blockIdx.x / groups);
  const int32_t c = (int32_t)(blockIdx.x - (int64_t)b * groups) * 4 + (threadIdx.x >> 6);
  if (c >= d.C) return;
  int64_t qrow; int32_t n;
  if (!device_session(d, b, &qrow, &n, false)) return;
  const char* pp = static_cast<const char*>(d.p_rows) + (int64_t)b * d.V * (PF16 ? 2 : 4);
  const float* qp = d.draft_probs + qrow * (int64_t)d.V;
  float acc = 0.f;
  if constexpr (ALIGNED) {
    // Lane l takes entries [4l, 4l+4) of every 256-entry half-block: one 8-byte (fp16) or 16-byte
    // (fp32) load of P~ and one 16-byte load of Q, so every wave instruction reads one contiguous
    // stretch of its row (8 entries per lane would leave the 32-byte-per-lane loads touching half
    // of each cache line they visit).  All loads of the chunk are in flight at once.
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    constexpr int kHalves = 4096 / 256;
    const int64_t e_chunk = (int64_t)c * 4096 + lane * 4;
    f32x4 p[kHalves], q[kHalves];
#pragma unroll
    for (int h = 0; h < kHalves; ++h) {
      const int64_t e0 = e_chunk + h * 256;
      const bool inside = e0 < d.V;                       // V is a multiple of 8: inside means entirely inside
      const int64_t ec = inside ? e0 : (int64_t)d.V - 4;
      if constexpr (PF16) {
        const u32x2 raw = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(pp + ec * 2));
        p[h] = (f32x4){(float)__builtin_bit_cast(_Float16, (uint16_t)(raw[0] & 0xFFFFu)),
                       (float)__builtin_bit_cast(_Float16, (uint16_t)(raw[0] >> 16)),
                       (float)__builtin_bit_cast(_Float16, (uint16_t)(raw[1] & 0xFFFFu)),
                       (float)__builtin_bit_cast(_Float16, (uint16_t)(raw[1] >> 16))};
      } else {
        p[h] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(pp + ec * 4));
      }
      q[h] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(qp + ec));
      if (!inside) {
        p[h] = (f32x4){0.f, 0.f, 0.f, 0.f};
        q[h] = (f32x4){0.f, 0.f, 0.f, 0.f};
      }
    }
#pragma unroll
    for (int h = 0; h < kHalves; ++h)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc += fmaxf(0.f, p[h][i] - q[h][i]);
  } else {
    const int64_t g0 = (int64_t)c * kChunkVecs + lane;
    if ((int64_t)(c + 1) * 4096 <= d.V) {   // wave-uniform: the chunk lies inside the row
      const ProbWeights<PF16, ALIGNED, true, true> wf{pp, qp, d.V};
#pragma unroll
      for (int k = 0; k < kUnroll; ++k) {
        float w[8];
        acc += wf.group(g0 + k * kWave, w);
      }
    } else {
      const ProbWeights<PF16, ALIGNED, true> wf{pp, qp, d.V};
#pragma unroll
      for (int k = 0; k < kUnroll; ++k) {
        float w[8];
        acc += wf.group(g0 + k * kWave, w);
      }
    }
  }
  acc = wave_sum(acc);
  if (lane == 0) d.resid_mass[(int64_t)b * d.C + c] = acc;
}

// One wave per session: x' ~ norm(max(0, P~_n - Q_n)) with r = word 1 of the position-n block.
template <bool PF16, bool ALIGNED>
__global__ __launch_bounds__(256) void device_pick(const DeviceView d) {
  const int lane = threadIdx.x & 63;
  const int32_t b = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (b >= d.B) return;
  int64_t qrow; int32_t n;
  if (!device_session(d, b, &qrow, &n, lane == 0)) return;
  const char* pp = static_cast<const char*>(d.p_rows) + (int64_t)b * d.V * (PF16 ? 2 : 4);
  const float* qp = d.draft_probs + qrow * (int64_t)d.V;
  const Philox rnd = step_block(d.session_base + (uint32_t)b, (uint32_t)n, d.step_lo, d.step_hi, d.step_dev,
                                d.seed_lo, d.seed_hi);
  const float r = u01(rnd.w[1]);
  float* rm = d.resid_mass + (int64_t)b * d.C;
  float target = 0.f, total = 0.f;
  int32_t token = -1;
  int32_t c = pick_chunk([&](int32_t cc) { return rm[cc]; }, d.C, r, lane, &target, &total);
  if (c >= 0) token = pick_in_chunk_of_row(ProbWeights<PF16, ALIGNED, true>{pp, qp, d.V}, c, target, lane);
  bool from_p = false;
  if (token < 0) {
    // No residual mass (P~ <= Q everywhere after rounding): draw from the received P~ itself.
    from_p = true;
    const ProbWeights<PF16, ALIGNED, false> wf{pp, nullptr, d.V};
    for (int32_t cc = 0; cc < d.C; ++cc) {
      float acc = 0.f;
#pragma unroll
      for (int k = 0; k < kUnroll; ++k) {
        float w[8];
        acc += wf.group((int64_t)cc * kChunkVecs + lane + k * kWave, w);
      }
      acc = wave_sum(acc);
      if (lane == 0) rm[cc] = acc;
    }
    __threadfence();   // lane 0's stores are visible to the other lanes' loads (and stale cached lines dropped)
    c = pick_chunk([&](int32_t cc) { return rm[cc]; }, d.C, r, lane, &target, &total);
    if (c >= 0) token = pick_in_chunk_of_row(wf, c, target, lane);
  }
  if (lane == 0) {
    d.out_token[b] = token;
    if (d.status) d.status[b] = (from_p ? 2 : 0) | (token < 0 ? 8 : 0);
  }
}

}  // namespace dssd
