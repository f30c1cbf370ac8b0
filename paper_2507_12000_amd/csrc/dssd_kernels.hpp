// Kernels of the DSSD verification step (arXiv 2507.12000, Sec. 2.1 / Sec. 3, Algorithms 1-2)
// for gfx950.  Everything here is a streaming reduction or scan over the vocabulary, so the
// kernels are organised around one unit of work: a *chunk* of 512 16-byte vectors (8 KiB) of
// one logits row, owned by one 64-lane wave, which keeps the chunk in registers.
//
//   row_chunk_stats : per chunk, m2_c = max(z) * c1 and s_c = sum 2^(z*c1 - m2_c), with
//                     c1 = log2(e)/T.  One exp per element, no cross-wave traffic.
//   accept_scan     : per session (one workgroup), merges the chunk pairs into row (M2, Z), gathers
//                     p_i(x_i) and q_i(x_i), draws r_i, finds the first rejected draft with a ballot.
//   resid_mass      : per chunk of the rejected row, the mass of max(0, P - Q); for small
//                     batches the last wave of a session also draws the token.
//   pick_token      : scan the chunk masses, then re-read the one chunk that holds r * total
//                     and locate the token by a wave prefix sum (residual or bonus draw).
#pragma once
#include "dssd_device.hpp"

namespace dssd {

// What verify leaves for the samplers, per session: the logits row to draw from and its
// softmax statistics.  lrow < 0: nothing to do (other branch taken, or a device-side error).
struct __attribute__((aligned(16))) Job {
  int64_t lrow;
  float M2, Z;
};

struct BatchView {
  int32_t B, V, gamma, C;            // C = chunks per row
  int32_t xcds;                      // XCDs of the device (round-robin targets of consecutive workgroups)
  int32_t xcd_shift;                 // log2(xcds) when that is a power of two, else -1
  int64_t R_L, R_Q;
  const int32_t* offsets;            // may be null
  const void* logits;
  const float* draft_probs;          // may be null when q_scalars is given (verify only)
  const float* q_scalars;            // [R_Q] q_i(x_i) as uploaded by the device, or null
  const int32_t* tokens;
  const float* inv_temp;             // may be null
  uint32_t seed_lo, seed_hi, step_lo, step_hi, session_base;
  const uint64_t* step_dev;          // may be null: device-resident counter added to the step
  // outputs
  int32_t* accepted_len;
  int32_t* rejected;
  int32_t* out_token;
  float* row_stats;                  // may be null
  float* p_tok;                      // may be null
  float* q_tok;                      // may be null
  int32_t* status;                   // may be null
  // workspace
  float2* chunk_stats;               // [R_L, C]  (m2_c, s_c)
  float2* row_tab;                   // [R_L]     (M2, Z) in the log2 domain
  float* resid_mass;                 // [B, C]
  Job* resid_job;                    // [B] rejected sessions: row n
  Job* bonus_job;                    // [B] all-accepted sessions: row gamma_b
  int32_t* arrive_resid;             // [B] chunk masses finished per session; zero between calls
  int32_t* support_count;            // [R_L] sparse-support mode: finite entries per row
  int32_t* support_idx;              // [R_L, kMaxSupport]
  float* support_z;                  // [R_L, kMaxSupport]
};

// xcd_contiguous for grids below 2^31 workgroups, without a division when the XCD count is a
// power of two.
__device__ __forceinline__ uint32_t xcd_contiguous32(uint32_t block, uint32_t blocks, const BatchView& a) {
  if (a.xcd_shift >= 0) {
    const uint32_t per = blocks >> a.xcd_shift;
    return block < (per << a.xcd_shift) ? (block & ((1u << a.xcd_shift) - 1u)) * per + (block >> a.xcd_shift) : block;
  }
  return (uint32_t)xcd_contiguous(block, blocks, (uint32_t)a.xcds);
}

__device__ __forceinline__ int64_t session_first_draft(const BatchView& a, int32_t b) {
  return a.offsets ? (int64_t)a.offsets[b] : (int64_t)b * a.gamma;
}
// Session that owns logits row `row`: the largest b with first_draft(b) + b <= row.
__device__ __forceinline__ int32_t session_of_row(const BatchView& a, int64_t row) {
  if (!a.offsets) return (int32_t)((uint32_t)row / (uint32_t)(a.gamma + 1));   // rows < 2^31
  int32_t lo = 0, hi = a.B - 1;
  while (lo < hi) {
    const int32_t mid = (lo + hi + 1) >> 1;
    if ((int64_t)a.offsets[mid] + mid <= row) lo = mid; else hi = mid - 1;
  }
  return lo;
}
template <bool BF16> __device__ __forceinline__ const char* logits_row(const BatchView& a, int64_t row) {
  return static_cast<const char*>(a.logits) + row * (int64_t)a.V * (BF16 ? 2 : 4);
}

// ---------------------------------------------------------------------------------------
// Softmax statistics, one wave per chunk.  Step "LLM gets the gamma+1 distributions" of the
// verification process: P(v) = 2^(z_v*c1 - M2)/Z.  This kernel reads every logit exactly once.
// ---------------------------------------------------------------------------------------
// (m2_c, s_c) of chunk c of the row at `src`, computed by one wave; every lane gets the result.
// A row's support: its entries above -inf, at most kMaxSupport of them, in arrival order.
constexpr int kMaxSupport = 64;
struct SupportRow {
  int32_t* count;   // entries seen so far (may exceed kMaxSupport: overflow)
  int32_t* idx;     // [kMaxSupport] vocabulary indices
  float* z;         // [kMaxSupport] their logits
};

// SUPPORT: the wave also appends the chunk's finite entries to the row's support list (rows
// are expected to be almost entirely -inf, e.g. after top-k filtering, so nearly every chunk
// skips this at the cost of one wave-uniform branch).
// c1_of() yields log2(e)/T of the row; it is called after the chunk's loads have been issued, so
// whatever it costs (a session lookup, a dependent load) runs under their latency.
template <bool BF16, bool ALIGNED, bool SUPPORT = false, class C1Fn>
__device__ __forceinline__ float2 chunk_stats_of(const char* src, int32_t c, int32_t V, C1Fn c1_of, int lane,
                                                 SupportRow sup = SupportRow{}) {
  constexpr int E = Elems<BF16>::per_vec;
  const int64_t v0 = (int64_t)c * kChunkVecs + lane;
  float z[kUnroll][E];
  // Rows that are not 16-byte aligned: every chunk but a row's last lies entirely inside the row
  // (a wave-uniform test) and is read with 128-bit loads at the row's own alignment; the last
  // chunk takes scalar loads, which stop at the row's end.
  if (!ALIGNED && (int64_t)(c + 1) * kChunkVecs * E <= V) {
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) load_logits<BF16, ALIGNED, true>(src, v0 + k * kWave, V, z[k]);
  } else {
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) load_logits<BF16, ALIGNED>(src, v0 + k * kWave, V, z[k]);
  }
  const float c1 = c1_of();

  float mx = neg_inf();
#pragma unroll
  for (int k = 0; k < kUnroll; ++k)
#pragma unroll
    for (int e = 0; e < E; ++e) mx = fmaxf(mx, z[k][e]);
  const float lane_mx = mx;
  mx = wave_max(mx);
  if constexpr (SUPPORT) {
    if (mx > neg_inf() && lane_mx > neg_inf()) {
#pragma unroll
      for (int k = 0; k < kUnroll; ++k)
#pragma unroll
        for (int e = 0; e < E; ++e)
          if (z[k][e] > neg_inf()) {
            const int32_t pos = atomicAdd(sup.count, 1);
            if (pos < kMaxSupport) {
              sup.idx[pos] = (int32_t)((v0 + k * kWave) * E + e);
              sup.z[pos] = z[k][e];
            }
          }
    }
  }

  float m2 = neg_inf(), s = 0.f;
  if (mx > neg_inf()) {
    m2 = mx * c1;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < kUnroll; ++k)
#pragma unroll
      for (int e = 0; e < E; ++e) acc[e & 3] += fast_exp2(fmaf(z[k][e], c1, -m2));
    s = wave_sum((acc[0] + acc[1]) + (acc[2] + acc[3]));
  }
  return make_float2(m2, s);
}

// Workgroups of kStatsWaves waves, one chunk each.  How many of them share a compute unit is
// capped by the host at launch (see occupancy_cap_lds).  Two-wave workgroups let the cap move in
// steps of two waves and measured 1-3 % faster than four-wave ones at their respective best caps
// (12 waves per unit for bf16 logits, 10 for fp32), at every batch size from 160 MB to 5 GB.
constexpr int kStatsWaves = 2;
template <bool BF16, bool ALIGNED, bool SUPPORT>
__global__ __launch_bounds__(kStatsWaves * kWave) void row_chunk_stats(const BatchView a) {
  // Everything before the loads is wave-uniform 32-bit arithmetic (the host refuses batches with
  // 2^31 chunks or more), so a wave has its loads in flight a few dozen scalar instructions
  // after it starts.
  const int lane = threadIdx.x & 63;
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const uint32_t C = (uint32_t)a.C;
  const uint32_t tasks = (uint32_t)a.R_L * C;
  const uint32_t task = xcd_contiguous32(blockIdx.x, gridDim.x, a) * kStatsWaves + wave;
  if (task >= tasks) return;
  const uint32_t row = task / C;
  const int32_t c = (int32_t)(task - row * C);
  SupportRow sup{};
  if constexpr (SUPPORT)
    sup = SupportRow{a.support_count + row, a.support_idx + (int64_t)row * kMaxSupport,
                     a.support_z + (int64_t)row * kMaxSupport};
  auto c1_of = [&]() { return a.inv_temp ? kLog2e * a.inv_temp[session_of_row(a, row)] : kLog2e; };
  const float2 st = chunk_stats_of<BF16, ALIGNED, SUPPORT>(logits_row<BF16>(a, row), c, a.V, c1_of, lane, sup);
  if (lane == 0) a.chunk_stats[task] = st;
}

__global__ __launch_bounds__(256) void zero_i32(int32_t* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0;
}

// Measurement aid: a pure read of the statistics kernel's kind (one wave per LOADS KiB, LOADS
// non-temporal 128-bit loads per lane all in flight, XCD-contiguous block order) with no
// arithmetic but an OR.  Swept over LOADS and over the waves resident per compute unit, its best
// rate is the read ceiling the statistics kernel can be held against on a given chip.
template <int LOADS>
__global__ __launch_bounds__(256) void read_probe(const u32x4* src, int64_t units, uint32_t* sink, int32_t xcds) {
  const int lane = threadIdx.x & 63;
  const int64_t unit = xcd_contiguous(blockIdx.x, gridDim.x, xcds) * 4 + (threadIdx.x >> 6);
  if (unit >= units) return;
  const u32x4* p = src + unit * (kWave * LOADS) + lane;
  uint32_t acc = 0;
  u32x4 v[LOADS];
#pragma unroll
  for (int k = 0; k < LOADS; ++k) v[k] = __builtin_nontemporal_load(p + k * kWave);
#pragma unroll
  for (int k = 0; k < LOADS; ++k) acc |= v[k][0] | v[k][1] | v[k][2] | v[k][3];
  if (acc == 0x5EEDF00Du) sink[0] = acc;   // keeps the loads alive; practically never taken
}

// ---------------------------------------------------------------------------------------
// Accept / reject and first-reject scan, one workgroup per session.
// Algorithm 2, "Verification Process" loop: accept x_i iff r_i < min(1, p_i(x_i)/q_i(x_i)),
// evaluated as r_i*q < p; stop at the first failure.
// ---------------------------------------------------------------------------------------
// Row (M2, Z) from its chunk pairs, computed by one wave: lane = chunk (batches of 64), fixed
// butterfly order.  `first` holds the pair of chunk `lane` (already loaded by the caller).
__device__ __forceinline__ float2 merge_row_wave(const float2* cs, int32_t C, int lane, float2 first) {
  float M2 = wave_max(lane < C ? first.x : neg_inf());
  for (int32_t base = kWave; base < C; base += kWave)
    M2 = fmaxf(M2, wave_max(base + lane < C ? observe2(cs + base + lane).x : neg_inf()));
  if (!(M2 > neg_inf())) return make_float2(M2, 0.f);
  float Z = wave_sum(lane < C ? first.y * fast_exp2(first.x - M2) : 0.f);
  for (int32_t base = kWave; base < C; base += kWave) {
    const int32_t c = base + lane;
    const float2 v = c < C ? observe2(cs + c) : make_float2(neg_inf(), 0.f);
    Z += wave_sum(v.y * fast_exp2(v.x - M2));
  }
  return make_float2(M2, Z);
}

// One workgroup per session.  Its waves merge the session's rows (four rows per wave in flight
// at a time); wave 0 then takes lane i = draft position i.
// Returns (to every thread of the workgroup) what the session has to draw next: kind 1 = redraw
// from the residual at job.lrow, kind 2 = bonus token from job.lrow, 0 = nothing (device-side
// error).  Chunk pairs are read with device-coherent loads, so the caller may be the launch that
// produced them.
//
// [row_begin, row_end) restricts the call to those rows of the session (positions before
// row_begin are known to be accepted; statistics exist for the rows in the range only).  If the
// range holds neither a rejection nor the bonus row the session is left open: nothing is
// written and kind 3 is returned.  With partial = true a session that is closed here gets NaN
// in the row_stats / p_tok / q_tok entries of the rows and positions from row_end on.
template <bool BF16>
__device__ int32_t accept_session(const BatchView& a, int32_t b, Job* job_out, int32_t row_begin = 0,
                                  int32_t row_end = 0x7FFFFFFF, bool partial = false) {
  __shared__ float2 row_st[kWave + 1];
  __shared__ Job sh_job;
  __shared__ int32_t sh_kind;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int32_t nwaves = (int32_t)(blockDim.x >> 6);   // each row is merged by one wave, whatever their number
  const int64_t off0 = session_first_draft(a, b);
  const int64_t off1 = a.offsets ? (int64_t)a.offsets[b + 1] : off0 + a.gamma;
  int32_t bad = 0;
  if (off0 < 0 || off1 < off0 || off1 > a.R_Q) bad = 4;
  float tau = 1.f;
  if (a.inv_temp) {
    tau = a.inv_temp[b];
    if (!(tau > 0.f) || !(tau < 3.0e38f)) bad |= 8;
  }
  const int32_t g = bad & 4 ? 0 : (int32_t)(off1 - off0);
  const int64_t lrow0 = off0 + b;
  const float c1 = tau * kLog2e;
  int32_t first_reject = g;
  float2 sel_st = make_float2(0.f, 0.f);   // statistics of the row the session will draw from
  const int32_t hi = min(row_end, g + 1);   // rows [row_begin, hi) are examined here
  if (!(bad & 4)) {
    for (int32_t base = row_begin; base < hi; base += kWave) {
      // rows base .. base+nrows-1 of the session (the last pass includes the bonus row)
      const int32_t nrows = min(kWave, hi - base);
      // what the accept test gathers does not depend on the statistics: asked for first, so the
      // latency runs under the row merges (wave 0, lane = position base + lane)
      int32_t x = 0;
      float zx = 0.f, q = 0.f;
      if (wave == 0 && lane < nrows && base + lane < g) {
        const int64_t qrow = off0 + base + lane;
        x = a.tokens[qrow];
        if (x >= 0 && x < a.V) {
          zx = load_logit(logits_row<BF16>(a, lrow0 + base + lane), x, BF16);
          q = a.q_scalars ? a.q_scalars[qrow] : a.draft_probs[qrow * (int64_t)a.V + x];
        }
      }
      for (int32_t r0 = wave; r0 < nrows; r0 += 4 * nwaves) {
        float2 first[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int32_t r = r0 + nwaves * j;
          first[j] = (r < nrows && lane < a.C) ? observe2(a.chunk_stats + (lrow0 + base + r) * a.C + lane)
                                               : make_float2(neg_inf(), 0.f);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int32_t r = r0 + nwaves * j;
          if (r < nrows) {
            const int64_t lrow = lrow0 + base + r;
            const float2 st = merge_row_wave(a.chunk_stats + lrow * a.C, a.C, lane, first[j]);
            if (lane == 0) {
              row_st[r] = st;
              a.row_tab[lrow] = st;
              if (a.row_stats) {
                a.row_stats[2 * lrow] = st.x * kLn2;
                a.row_stats[2 * lrow + 1] = st.y;
              }
            }
          }
        }
      }
      __syncthreads();
      if (wave == 0) {
        const int32_t i = base + lane;
        bool reject = false;
        int32_t lane_bad = 0;
        if (lane < nrows) {
          const float2 st = row_st[lane];
          if (!(st.y > 0.f) || !(st.y < 3.0e38f) || !(fabsf(st.x) < 3.0e38f)) lane_bad |= 8;
          if (i < g) {
            const int64_t qrow = off0 + i;
            float p = 0.f;
            if (x < 0 || x >= a.V) {
              lane_bad |= 1;
            } else {
              p = fast_exp2(fmaf(zx, c1, -st.x)) / st.y;
              const Philox rnd = step_block(a.session_base + (uint32_t)b, (uint32_t)i, a.step_lo, a.step_hi, a.step_dev,
                                      a.seed_lo, a.seed_hi);
              const float r = u01(rnd.w[0]);
              reject = !(__fmul_rn(r, q) < p);
            }
            if (a.p_tok) a.p_tok[qrow] = p;
            if (a.q_tok) a.q_tok[qrow] = q;
          }
        }
        // Faults count where Algorithm 2's loop looks: positions and rows up to the first
        // rejection (its row feeds the redraw), or all of them and the bonus row when every
        // draft is accepted.  A fault stops the loop where it stands, like a rejection would.
        const bool was_open = first_reject == g && !(bad & 9);
        const uint64_t rej_mask = __ballot(reject);
        const uint64_t b1 = __ballot(lane_bad & 1), b8 = __ballot(lane_bad & 8);
        const int idx = rej_mask ? __ffsll((long long)rej_mask) - 1 : kWave;   // first rejection of this pass
        const uint64_t upto = idx >= kWave - 1 ? ~0ull : (2ull << idx) - 1ull;  // lanes 0..idx
        if (was_open) {
          bad |= ((b1 & upto) ? 1 : 0) | ((b8 & upto) ? 8 : 0);
          if (rej_mask) {
            first_reject = base + idx;
            sel_st = row_st[idx];
          } else if (base + nrows - 1 == g) {
            sel_st = row_st[nrows - 1];        // all accepted: the bonus row
          }
        }
      }
      __syncthreads();
    }
  }
  if (wave == 0) {
    const bool open = !bad && first_reject == g && hi <= g;   // no rejection yet, bonus row not reached
    if (partial && !open && !(bad & 4)) {
      const float nan = __builtin_nanf("");
      if (a.row_stats)
        for (int32_t j = hi + lane; j <= g; j += kWave) {
          a.row_stats[2 * (lrow0 + j)] = nan;
          a.row_stats[2 * (lrow0 + j) + 1] = nan;
        }
      for (int32_t j = hi + lane; j < g; j += kWave) {
        if (a.p_tok) a.p_tok[off0 + j] = nan;
        if (a.q_tok) a.q_tok[off0 + j] = nan;
      }
    }
    if (lane == 0) {
      // (records are built field by field: choosing between two whole structs made the compiler
      // park both in scratch memory and pick one by address, at the end of a latency-bound chain)
      Job job;
      job.lrow = lrow0 + first_reject; job.M2 = sel_st.x; job.Z = sel_st.y;
      const auto job_if = [&](bool wanted) {
        Job j;
        j.lrow = wanted ? job.lrow : -1; j.M2 = wanted ? job.M2 : 0.f; j.Z = wanted ? job.Z : 0.f;
        return j;
      };
      if (!open) {
        if (bad) {
          a.accepted_len[b] = 0;
          a.rejected[b] = 1;
          a.out_token[b] = -1;
        } else {
          a.accepted_len[b] = first_reject;
          a.rejected[b] = first_reject < g ? 1 : 0;
        }
        a.resid_job[b] = job_if(!bad && first_reject < g);
        a.bonus_job[b] = job_if(!bad && first_reject == g);
        if (a.status) a.status[b] = bad;
      }
      sh_job = job;
      sh_kind = open ? 3 : (bad ? 0 : (first_reject < g ? 1 : 2));
    }
  }
  __syncthreads();
  *job_out = sh_job;
  return sh_kind;
}

// One 256-thread workgroup per session.
template <bool BF16>
__global__ __launch_bounds__(256) void accept_scan(const BatchView a) {
  Job job;
  accept_session<BF16>(a, blockIdx.x, &job);
}

// ---------------------------------------------------------------------------------------
// Weights of one 16-byte group of a row, shared by the mass and pick kernels so that both
// see bit-identical values: w = max(0, 2^(z*c1 - M2)*invZ - q) (residual, Algorithm 2
// "Resample") or w = 2^(z*c1 - M2) (bonus draw from P).
// ---------------------------------------------------------------------------------------
template <bool BF16, bool ALIGNED, bool RESID, bool INSIDE = false>
__device__ __forceinline__ float group_weights(const char* lrow, const float* qrow, int64_t vec, int32_t V,
                                               float c1, float M2, float invZ, float* w) {
  constexpr int E = Elems<BF16>::per_vec;
  float z[E];
  load_logits<BF16, ALIGNED, INSIDE>(lrow, vec, V, z);
  float sum = 0.f;
  if constexpr (RESID) {
    float q[E];
    load_probs<E, ALIGNED, INSIDE>(qrow, vec * E, V, q);
#pragma unroll
    for (int e = 0; e < E; ++e) {
      w[e] = fmaxf(0.f, fmaf(fast_exp2(fmaf(z[e], c1, -M2)), invZ, -q[e]));
      sum += w[e];
    }
  } else {
#pragma unroll
    for (int e = 0; e < E; ++e) {
      w[e] = fast_exp2(fmaf(z[e], c1, -M2));
      sum += w[e];
    }
  }
  return sum;
}

// INSIDE: every group asked for lies within the row (see load_logits); inside() is the same
// functor with that promise made.
template <bool BF16, bool ALIGNED, bool RESID, bool INSIDE = false>
struct LogitWeights {
  static constexpr int E = Elems<BF16>::per_vec;
  static constexpr bool kAligned = ALIGNED;
  const char* lp; const float* qp; int32_t V; float c1, M2, invZ;
  __device__ __forceinline__ float group(int64_t vec, float* w) const {
    return group_weights<BF16, ALIGNED, RESID, INSIDE>(lp, qp, vec, V, c1, M2, invZ, w);
  }
  __device__ __forceinline__ LogitWeights<BF16, ALIGNED, RESID, true> inside() const {
    return {lp, qp, V, c1, M2, invZ};
  }
};

template <bool BF16, bool ALIGNED, bool RESID>
__device__ void pick_for_session(const BatchView& a, int32_t b, const Job& job, int lane,
                                 const float* lds_mass = nullptr);

// Residual resample (Algorithm 2 "Resample"): mass of max(0, P - Q) per chunk of the rejected
// row, one wave per chunk.  Sessions that were not rejected exit at once.  FUSE_PICK: the last
// workgroup of a session to finish also draws the token, which saves the second launch.
// GROUPS_IN_FLIGHT (4 or 8) only sets how many of a lane's 8 groups are loaded before the sums
// start on the path that loads 16-byte groups; the order of the sums, and so every bit of the
// result, is the same.
template <bool BF16, bool ALIGNED, int GROUPS_IN_FLIGHT = 4>
__device__ __forceinline__ float resid_chunk_mass(const BatchView& a, int32_t b, const Job& job, int32_t c,
                                                  int lane) {
  constexpr int E = Elems<BF16>::per_vec;
  const float2 st = make_float2(job.M2, job.Z);
  const float c1 = (a.inv_temp ? a.inv_temp[b] : 1.f) * kLog2e;
  const float invZ = 1.f / st.y;
  const char* lp = logits_row<BF16>(a, job.lrow);
  const float* qp = a.draft_probs + (job.lrow - b) * (int64_t)a.V;   // draft row = logits row - session
  float acc = 0.f;
  if constexpr (BF16 && ALIGNED) {
    // Lane l takes elements [4l, 4l+4) of every 256-entry half-block: an 8-byte load of logits and
    // a 16-byte load of Q, so that every wave instruction reads one contiguous stretch of its row
    // (with 8 elements per lane the Q loads would touch only half of each cache line they visit:
    // measured 6 % slower).  All 32 loads of the chunk are in flight at once.
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    constexpr int kHalves = chunk_elems<true>() / 256;
    const int64_t e_chunk = (int64_t)c * chunk_elems<true>() + lane * 4;
    u32x2 z[kHalves];
    f32x4 q[kHalves];
#pragma unroll
    for (int h = 0; h < kHalves; ++h) {
      const int64_t e0 = e_chunk + h * 256;
      const bool inside = e0 < a.V;                     // V is a multiple of 8: inside means entirely inside
      const int64_t ec = inside ? e0 : (int64_t)a.V - 4;
      z[h] = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(lp + ec * 2));
      q[h] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(qp + ec));
      if (!inside) {
        z[h] = (u32x2){0xFF80FF80u, 0xFF80FF80u};
        q[h] = (f32x4){0.f, 0.f, 0.f, 0.f};
      }
    }
#pragma unroll
    for (int h = 0; h < kHalves; ++h) {
      const float z0 = as_float(z[h][0] << 16), z1 = as_float(z[h][0] & 0xFFFF0000u);
      const float z2 = as_float(z[h][1] << 16), z3 = as_float(z[h][1] & 0xFFFF0000u);
      acc += fmaxf(0.f, fmaf(fast_exp2(fmaf(z0, c1, -st.x)), invZ, -q[h][0]));
      acc += fmaxf(0.f, fmaf(fast_exp2(fmaf(z1, c1, -st.x)), invZ, -q[h][1]));
      acc += fmaxf(0.f, fmaf(fast_exp2(fmaf(z2, c1, -st.x)), invZ, -q[h][2]));
      acc += fmaxf(0.f, fmaf(fast_exp2(fmaf(z3, c1, -st.x)), invZ, -q[h][3]));
    }
  } else {
    // fp32 logits are 4 per 16-byte group, like Q: already one contiguous stretch per instruction.
    // Streaming launches take two half-chunks of 4 groups each (measured faster than all 8 at
    // once there); a lone workgroup finishing a session takes all 8 (one round trip fewer).
    // Unaligned rows: vector loads at the row's alignment inside the row, scalar loads in its last chunk.
    constexpr int G = GROUPS_IN_FLIGHT;
    const int64_t v0 = (int64_t)c * kChunkVecs + lane;
    const bool inside = !ALIGNED && (int64_t)(c + 1) * kChunkVecs * E <= a.V;   // wave-uniform, as in chunk_stats_of
#pragma unroll
    for (int k0 = 0; k0 < kUnroll; k0 += G) {
      float z[G][E], q[G][E];
      if (inside) {
#pragma unroll
        for (int k = 0; k < G; ++k) {
          load_logits<BF16, ALIGNED, true>(lp, v0 + (k0 + k) * kWave, a.V, z[k]);
          load_probs<E, ALIGNED, true>(qp, (v0 + (k0 + k) * kWave) * E, a.V, q[k]);
        }
      } else {
#pragma unroll
        for (int k = 0; k < G; ++k) {
          load_logits<BF16, ALIGNED>(lp, v0 + (k0 + k) * kWave, a.V, z[k]);
          load_probs<E, ALIGNED>(qp, (v0 + (k0 + k) * kWave) * E, a.V, q[k]);
        }
      }
#pragma unroll
      for (int k = 0; k < G; ++k)
#pragma unroll
        for (int e = 0; e < E; ++e)
          acc += fmaxf(0.f, fmaf(fast_exp2(fmaf(z[k][e], c1, -st.x)), invZ, -q[k][e]));
    }
  }
  return wave_sum(acc);
}

template <bool BF16, bool ALIGNED, bool FUSE_PICK>
__global__ __launch_bounds__(256) void resid_mass(const BatchView a, int32_t groups) {
  __shared__ int32_t sh_last;
  const int lane = threadIdx.x & 63;
  const int64_t blk = blockIdx.x;   // plain order: measured faster here than the XCD-contiguous map
  const int32_t b = (int32_t)(blk / groups);
  const int32_t c = (int32_t)(blk - (int64_t)b * groups) * 4 + (threadIdx.x >> 6);
  const Job job = a.resid_job[b];
  if (job.lrow < 0) return;          // the whole workgroup: the job belongs to the session
  if (c < a.C) {
    const float acc = resid_chunk_mass<BF16, ALIGNED>(a, b, job, c, lane);
    if constexpr (!FUSE_PICK) {
      if (lane == 0) a.resid_mass[(int64_t)b * a.C + c] = acc;
    } else if (lane == 0) {
      publish(a.resid_mass + (int64_t)b * a.C + c, acc);
      stores_done();   // acknowledged before the barrier that precedes the arrival
    }
  }
  if constexpr (!FUSE_PICK) return;
  // The workgroup that completes the session's chunk masses draws the token (one arrival per
  // workgroup, nobody waits).  The masses are published with device-coherent stores and read
  // back with device-coherent loads, so the arrival counter needs no cache-wide fence.  The
  // counter is left at zero for the next call.
  __syncthreads();
  if (threadIdx.x == 0) {
    const bool last =
        __hip_atomic_fetch_add(a.arrive_resid + b, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == groups - 1;
    if (last) __hip_atomic_store(a.arrive_resid + b, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sh_last = last;
  }
  __syncthreads();
  if (sh_last && threadIdx.x < kWave) pick_for_session<BF16, ALIGNED, true>(a, b, job, lane);
}

// Inverse-CDF draw inside one chunk: target in [0, chunk mass) -> vocabulary index.
// The wave scans the chunk's 8 sub-blocks of 64 groups; at each level (sub-block, lane, element)
// the local target is clamped into [0, local total) so that a token is always found and a
// zero-weight token never is.
// `wf.group(g, w)` fills the W::E weights of group g of the row and returns their sum (summed in
// element order).  The chunk masses the target came from may have been summed in another order:
// the clamps absorb the difference.
template <typename W>
__device__ __forceinline__ int32_t pick_in_chunk(const W& wf, int32_t c, float target, int lane) {
  constexpr int E = W::E;
  const int64_t v0 = (int64_t)c * kChunkVecs + lane;
  float lsum[kUnroll], scan[kUnroll], S[kUnroll];
#pragma unroll
  for (int k = 0; k < kUnroll; ++k) {
    float w[E];
    lsum[k] = wf.group(v0 + k * kWave, w);
    scan[k] = wave_scan(lsum[k], lane);
    S[k] = lane_value(scan[k], 63);
  }
  float total = 0.f;
#pragma unroll
  for (int k = 0; k < kUnroll; ++k) total += S[k];
  if (!(total > 0.f)) return -1;
  float t = fminf(fmaxf(target, 0.f), next_below(total));
  // sub-block
  int ksel = kUnroll - 1;
  float before = 0.f, run = 0.f;
  bool found = false;
#pragma unroll
  for (int k = 0; k < kUnroll; ++k) {
    const float upto = run + S[k];
    if (!found && upto > t && S[k] > 0.f) { found = true; ksel = k; before = run; }
    run = upto;
  }
  float my_sum = 0.f, my_scan = 0.f, Ssel = 0.f;
#pragma unroll
  for (int k = 0; k < kUnroll; ++k)
    if (k == ksel) { my_sum = lsum[k]; my_scan = scan[k]; Ssel = S[k]; }
  // lane
  // (a lane of zero weight can sit one rounding above its predecessor in the scan: never taken)
  float t2 = fminf(fmaxf(t - before, 0.f), next_below(Ssel));
  const uint64_t weighty = __ballot(my_sum > 0.f);
  const uint64_t over = __ballot(my_scan > t2 && my_sum > 0.f);
  if (!weighty) return -1;
  const int lsel = over ? __ffsll((long long)over) - 1 : 63 - __clzll((long long)weighty);
  const float excl = lsel > 0 ? lane_value(my_scan, lsel - 1) : 0.f;
  const float sum_sel = lane_value(my_sum, lsel);
  const float t3 = fminf(fmaxf(t2 - excl, 0.f), next_below(sum_sel));
  // element: the selected lane recomputes its group
  int32_t token = -1;
  if (lane == lsel) {
    float w[E];
    const int64_t vec = v0 + (int64_t)ksel * kWave;
    wf.group(vec, w);
    float pre = 0.f;
    int esel = E - 1;
    bool hit = false;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      pre += w[e];
      if (!hit && pre > t3) { hit = true; esel = e; }
    }
    token = (int32_t)(vec * E + esel);
  }
  return __builtin_amdgcn_readlane(token, lsel);   // lsel is wave-uniform
}

// pick_in_chunk for a chunk of any row: on rows that are not 16-byte aligned, a chunk that lies
// entirely inside its row (wave-uniform) is read with vector loads at the row's alignment.
template <typename W>
__device__ __forceinline__ int32_t pick_in_chunk_of_row(const W& wf, int32_t c, float target, int lane) {
  if constexpr (!W::kAligned) {
    if ((int64_t)(c + 1) * kChunkVecs * W::E <= wf.V) return pick_in_chunk(wf.inside(), c, target, lane);
  }
  return pick_in_chunk(wf, c, target, lane);
}

// Scans per-chunk masses (lane = chunk, batches of 64) and returns the chunk that holds
// r * total; *target_in_chunk is what is left of r * total once the chunks before it are
// taken away.  mass(c) must be a pure function of c.  Returns -1 when total is not positive.
template <typename MassFn>
__device__ __forceinline__ int32_t pick_chunk(MassFn mass, int32_t C, float r, int lane, float* target_in_chunk,
                                              float* total_out) {
  float run = 0.f;
  float m_first = 0.f, sc_first = 0.f;   // the first batch (the only one when C <= 64) is kept for the second pass
  for (int32_t base = 0; base < C; base += kWave) {
    const int32_t c = base + lane;
    const float m = c < C ? mass(c) : 0.f;
    const float sc = wave_scan(m, lane);
    if (base == 0) { m_first = m; sc_first = sc; }
    run = run + lane_value(sc, 63);
  }
  *total_out = run;
  if (!(run > 0.f) || !(run < 3.0e38f)) return -1;
  const float t = fminf(__fmul_rn(r, run), next_below(run));
  run = 0.f;
  int32_t last_weighty = -1;
  float before_last = 0.f;
  for (int32_t base = 0; base < C; base += kWave) {
    const int32_t c = base + lane;
    const float m = base == 0 ? m_first : (c < C ? mass(c) : 0.f);
    const float sc = base == 0 ? sc_first : wave_scan(m, lane);
    // a chunk of zero mass can sit one rounding above its predecessor in the scan: never taken
    const uint64_t weighty = __ballot(m > 0.f);
    const uint64_t over = __ballot((run + sc) > t && m > 0.f);
    if (over) {
      const int lsel = __ffsll((long long)over) - 1;
      const float before = lsel > 0 ? run + lane_value(sc, lsel - 1) : run;
      *target_in_chunk = t - before;
      return base + lsel;
    }
    if (weighty) {
      const int l = 63 - __clzll((long long)weighty);
      last_weighty = base + l;
      before_last = l > 0 ? run + lane_value(sc, l - 1) : run;
    }
    run = run + lane_value(sc, 63);
  }
  // rounding left no prefix above t: the last chunk that has mass (pick_in_chunk clamps the target)
  *target_in_chunk = t - before_last;
  return last_weighty;
}

// One wave per session.  RESID: rejected sessions, row n, weights max(0, P - Q), r = word 1 of
// the position-n block.  Otherwise: all-accepted sessions, row gamma_b, weights P, r = word 2 of
// the position-gamma_b block (Algorithm 2: "Sample x_{gamma+1} ~ P_{gamma+1}").
// lds_mass: the session's residual chunk masses in LDS when the calling workgroup has just
// computed them itself (same values as in a.resid_mass, two round trips to memory fewer).
template <bool BF16, bool ALIGNED, bool RESID>
__device__ void pick_for_session(const BatchView& a, int32_t b, const Job& job, int lane, const float* lds_mass) {
  const int64_t lrow = job.lrow;
  const int32_t n = (int32_t)(lrow - b - session_first_draft(a, b));   // position inside the session
  const float2 st = make_float2(job.M2, job.Z);
  const float c1 = (a.inv_temp ? a.inv_temp[b] : 1.f) * kLog2e;
  const float invZ = 1.f / st.y;
  const char* lp = logits_row<BF16>(a, lrow);
  const float* qp = RESID ? a.draft_probs + (lrow - b) * (int64_t)a.V : nullptr;
  const Philox rnd = step_block(a.session_base + (uint32_t)b, (uint32_t)n, a.step_lo, a.step_hi, a.step_dev,
                                      a.seed_lo, a.seed_hi);
  const float r = u01(rnd.w[RESID ? 1 : 2]);

  const float2* cs = a.chunk_stats + lrow * a.C;
  auto p_mass = [&](int32_t c) { const float2 v = observe2(cs + c); return v.y * fast_exp2(v.x - st.x); };
  float target = 0.f, total = 0.f;
  int32_t token = -1;
  bool from_p = !RESID;
  if constexpr (RESID) {
    const float* rm = a.resid_mass + (int64_t)b * a.C;
    const int32_t c = pick_chunk([&](int32_t cc) { return lds_mass ? lds_mass[cc] : observe(rm + cc); }, a.C, r,
                                 lane, &target, &total);
    if (c >= 0) token = pick_in_chunk_of_row(LogitWeights<BF16, ALIGNED, true>{lp, qp, a.V, c1, st.x, invZ}, c, target, lane);
    if (token < 0) from_p = true;   // residual mass rounded to zero: draw from P_n instead
  }
  if (from_p) {
    const int32_t c = pick_chunk(p_mass, a.C, r, lane, &target, &total);
    if (c >= 0) token = pick_in_chunk_of_row(LogitWeights<BF16, ALIGNED, false>{lp, nullptr, a.V, c1, st.x, invZ}, c, target, lane);
  }
  if (lane == 0) {
    a.out_token[b] = token;
    if (a.status) {
      if (RESID && from_p) a.status[b] |= 2;
      if (token < 0) a.status[b] |= 8;
    }
  }
}

// Token draw as a launch of its own, one wave per session: the bonus token of all-accepted
// sessions (RESID = false) or the redrawn token of rejected ones after resid_mass (RESID = true).
template <bool BF16, bool ALIGNED, bool RESID>
__global__ __launch_bounds__(256) void pick_token(const BatchView a) {
  const int lane = threadIdx.x & 63;
  const int32_t b = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (b >= a.B) return;
  const Job job = RESID ? a.resid_job[b] : a.bonus_job[b];
  if (job.lrow < 0) return;
  pick_for_session<BF16, ALIGNED, RESID>(a, b, job, lane);
}

// accept_scan that also draws the bonus token of an all-accepted session (Algorithm 1 runs the
// two back to back at the edge): the session's workgroup already holds the last row's merged
// statistics, so the draw costs one chunk re-read and saves a launch.
template <bool BF16, bool ALIGNED>
__global__ __launch_bounds__(256) void accept_scan_bonus(const BatchView a) {
  Job job;
  const int32_t kind = accept_session<BF16>(a, blockIdx.x, &job);
  if (kind == 2 && threadIdx.x < kWave) pick_for_session<BF16, ALIGNED, false>(a, blockIdx.x, job, threadIdx.x);
}

// ---------------------------------------------------------------------------------------
// Sparse-support draw, one wave per session, lane = one entry of the row's support (at most
// 64 entries above -inf, recorded by row_chunk_stats<..., SUPPORT>).  The same weights and the
// same inverse-CDF rule in vocabulary order as the dense kernels, on up to 64 entries instead
// of V: entries are ranked by vocabulary index, moved into rank order with a lane permute, and
// prefix-summed across the wave.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ int32_t draw_from_ranked(float w_ranked, int32_t idx_ranked, float r, int lane) {
  const float scan = wave_scan(w_ranked, lane);
  const float total = lane_value(scan, 63);
  if (!(total > 0.f) || !(total < 3.0e38f)) return -1;
  const float t = fminf(__fmul_rn(r, total), next_below(total));
  // an entry of zero weight (padding included) can sit one rounding above its predecessor in
  // the scan: never taken
  const uint64_t weighty = __ballot(w_ranked > 0.f);
  const uint64_t over = __ballot(scan > t && w_ranked > 0.f);
  const int sel = over ? __ffsll((long long)over) - 1 : 63 - __clzll((long long)weighty);
  return __builtin_amdgcn_readlane(idx_ranked, sel);   // sel is wave-uniform
}

template <bool BF16, bool RESID>
__global__ __launch_bounds__(256) void pick_sparse(const BatchView a) {
  const int lane = threadIdx.x & 63;
  const int32_t b = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (b >= a.B) return;
  const Job job = RESID ? a.resid_job[b] : a.bonus_job[b];
  if (job.lrow < 0) return;
  const int64_t row = job.lrow;
  const int32_t cnt = a.support_count[row];
  if (cnt < 1 || cnt > kMaxSupport) {   // the promise of at most 64 finite logits does not hold
    if (lane == 0) {
      a.out_token[b] = -1;
      if (a.status) a.status[b] |= 16;
    }
    return;
  }
  const int32_t n = (int32_t)(row - b - session_first_draft(a, b));
  const float c1 = (a.inv_temp ? a.inv_temp[b] : 1.f) * kLog2e;
  const float invZ = 1.f / job.Z;
  const bool live = lane < cnt;
  const int32_t idx = live ? a.support_idx[row * kMaxSupport + lane] : 0x7FFFFFFF;
  const float z = live ? a.support_z[row * kMaxSupport + lane] : neg_inf();
  const float e = fast_exp2(fmaf(z, c1, -job.M2));                 // 0 for the padding lanes
  float w = e;
  if constexpr (RESID) {
    const float q = live ? a.draft_probs[(row - b) * (int64_t)a.V + idx] : 0.f;
    w = fmaxf(0.f, fmaf(e, invZ, -q));
  }
  // rank = number of entries with a smaller vocabulary index (indices are distinct; padding
  // lanes carry the largest index and rank after every live entry, among themselves by lane)
  int32_t rank = 0;
  for (int32_t m = 0; m < kWave; ++m) {
    const int32_t im = __builtin_amdgcn_readlane(idx, m);
    rank += (im < idx || (im == idx && m < lane)) ? 1 : 0;
  }
  const int32_t idx_r = __builtin_amdgcn_ds_permute(rank * 4, idx);
  const float w_r = __builtin_bit_cast(float, __builtin_amdgcn_ds_permute(rank * 4, __builtin_bit_cast(int, w)));
  const Philox rnd = step_block(a.session_base + (uint32_t)b, (uint32_t)n, a.step_lo, a.step_hi, a.step_dev,
                                      a.seed_lo, a.seed_hi);
  const float r = u01(rnd.w[RESID ? 1 : 2]);
  int32_t token = draw_from_ranked(w_r, idx_r, r, lane);
  bool from_p = false;
  if (RESID && token < 0) {   // residual mass rounded to zero: draw from P_n instead
    from_p = true;
    const float e_r = __builtin_bit_cast(float, __builtin_amdgcn_ds_permute(rank * 4, __builtin_bit_cast(int, e)));
    token = draw_from_ranked(e_r, idx_r, r, lane);
  }
  if (lane == 0) {
    a.out_token[b] = token;
    if (a.status) {
      if (from_p) a.status[b] |= 2;
      if (token < 0) a.status[b] |= 8;
    }
  }
}

}  // namespace dssd
