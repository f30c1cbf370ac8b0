// The verification step on top-k lists (Sec. 4 of the paper samples with top-k = 10): when both
// models' rows arrive as k (token id, value) pairs there is nothing of size V left to stream.
// The step is what the dense kernels compute on rows that are -inf (target logits) or 0 (draft
// probabilities) outside the lists:
//   P_i = softmax over the k listed logits (times 1/T), p_i(x) = 0 for x outside the list;
//   q_i(x) from the draft's list, 0 outside;
//   accept iff r*q < p, stop at the first failure (Algorithm 2, the while loop);
//   redraw from norm(max(0, P_n - Q_n)): its support lies inside the target's list, since p = 0
//   elsewhere; inverse CDF in vocabulary order, as everywhere in this library;
//   bonus token from P_gamma if every draft was accepted.
// One wave per session, lane = list entry, the whole step in one launch; a session's rows are
// read only as far as its first rejection (plus up to four rows fetched ahead).
#pragma once
#include "dssd_kernels.hpp"

namespace dssd {

struct TopkView {
  int32_t B, k, gamma, V;            // V = 0: token ids are not range-checked
  int64_t R_Q;
  const int32_t* offsets;            // may be null
  const int32_t* p_idx;              // [R_L, k] ids of the target's list, -1 = unused entry
  const float* p_logit;              // [R_L, k]
  const int32_t* q_idx;              // [R_Q, k] ids of the draft's list, -1 = unused entry
  const float* q_prob;               // [R_Q, k]
  const int32_t* tokens;             // [R_Q]
  const float* inv_temp;             // may be null
  uint32_t seed_lo, seed_hi, step_lo, step_hi, session_base;
  const uint64_t* step_dev;          // may be null
  int32_t* accepted_len;
  int32_t* rejected;
  int32_t* out_token;
  float* row_stats;                  // may be null
  float* p_tok;                      // may be null
  float* q_tok;                      // may be null
  int32_t* status;                   // may be null
};

// Inverse-CDF draw in vocabulary order from up to 64 (id, weight) pairs, one per lane; unused
// lanes carry weight 0 and id -1.  Entries are ranked by id and moved into rank order with a lane
// permute, then draw_from_ranked prefix-sums them.
__device__ __forceinline__ int32_t draw_from_list(int32_t idx, float w, float r, int lane) {
  const int32_t key = idx >= 0 ? idx : 0x7FFFFFFF;   // unused entries rank last
  int32_t rank = 0;
  for (int32_t m = 0; m < kWave; ++m) {
    const int32_t km = __builtin_amdgcn_readlane(key, m);
    rank += (km < key || (km == key && m < lane)) ? 1 : 0;
  }
  const int32_t idx_r = __builtin_amdgcn_ds_permute(rank * 4, idx);
  const float w_r = __builtin_bit_cast(float, __builtin_amdgcn_ds_permute(rank * 4, __builtin_bit_cast(int, w)));
  return draw_from_ranked(w_r, idx_r, r, lane);
}

__global__ __launch_bounds__(256) void topk_step(const TopkView t) {
  const int lane = threadIdx.x & 63;
  const int32_t b = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (b >= t.B) return;
  const int64_t off0 = t.offsets ? (int64_t)t.offsets[b] : (int64_t)b * t.gamma;
  const int64_t off1 = t.offsets ? (int64_t)t.offsets[b + 1] : off0 + t.gamma;
  int32_t bad = 0;
  if (off0 < 0 || off1 < off0 || off1 > t.R_Q) bad = 4;
  float tau = 1.f;
  if (t.inv_temp) {
    tau = t.inv_temp[b];
    if (!(tau > 0.f) || !(tau < 3.0e38f)) bad |= 8;
  }
  const int32_t g = bad & 4 ? 0 : (int32_t)(off1 - off0);
  const int64_t lrow0 = off0 + b;
  const float c1 = tau * kLog2e;
  const bool in_list = lane < t.k;
  int32_t first_reject = g, token = -1, last = -1;
  if (!bad) {
    // What position i reads: entry `lane` of the target's list of row i, the draft token and entry
    // `lane` of the draft's list of position i.  Always the same five loads, from addresses
    // clamped into the session (row min(i, g), position min(i, g-1), entry min(lane, k-1); a
    // session without drafts reads its target row twice), and nothing is done with the values
    // here: the number of loads in flight is then a constant the compiler can count on, and a
    // wave never waits for lists it asked for ahead of time.  visit() masks what is not real.
    struct Lists { int32_t idx; float z; int32_t x, qi; float qp; };
    const int32_t lk = min(lane, t.k - 1);
    auto fetch = [&](int32_t i) {
      Lists L;
      const int64_t at_p = (lrow0 + min(i, g)) * t.k + lk;
      const int64_t qrow = off0 + min(i, max(g - 1, 0));
      const int32_t* x_at = g > 0 ? t.tokens + qrow : t.p_idx + at_p;
      const int32_t* qi_at = g > 0 ? t.q_idx + qrow * t.k + lk : t.p_idx + at_p;
      const float* qp_at = g > 0 ? t.q_prob + qrow * t.k + lk : t.p_logit + at_p;
      L.idx = t.p_idx[at_p]; L.z = t.p_logit[at_p];
      L.x = *x_at; L.qi = *qi_at; L.qp = *qp_at;
      return L;
    };
    // The random blocks of 64 positions at a time, lane = position: one Philox evaluation per wave
    // and batch instead of one per position inside the walk (ten rounds of quarter-rate multiplies
    // are a third of a microsecond in a chain that is all latency).
    uint32_t w_accept = 0, w_redraw = 0, w_bonus = 0;
    const auto draw_blocks = [&](int32_t first) {
      const Philox rnd = step_block(t.session_base + (uint32_t)b, (uint32_t)(first + lane), t.step_lo, t.step_hi,
                                    t.step_dev, t.seed_lo, t.seed_hi);
      w_accept = rnd.w[0]; w_redraw = rnd.w[1]; w_bonus = rnd.w[2];
    };
    draw_blocks(0);
    // One position of the loop; false = the session is decided (or faulty) and the walk ends.
    const auto visit = [&](int32_t i, const Lists& cur) -> bool {
      last = i;
      if (i > 0 && (i & 63) == 0) draw_blocks(i);
      const int64_t row = lrow0 + i;
      const int32_t idx = in_list ? cur.idx : -1;
      const bool live = idx >= 0;
      const float z = live ? cur.z : neg_inf();
      const float M2 = wave_max(live ? z * c1 : neg_inf());
      const float e = (M2 > neg_inf()) ? fast_exp2(fmaf(z, c1, -M2)) : 0.f;   // 0 for unused entries
      const float Z = wave_sum(live ? e : 0.f);
      if (lane == 0 && t.row_stats) {
        t.row_stats[2 * row] = M2 * kLn2;
        t.row_stats[2 * row + 1] = Z;
      }
      if (!(Z > 0.f) || !(Z < 3.0e38f) || !(fabsf(M2) < 3.0e38f)) { bad |= 8; return false; }
      if (i == g) {   // every draft accepted: the bonus token, from P_gamma
        token = draw_from_list(idx, live ? e : 0.f, u01((uint32_t)__builtin_amdgcn_readlane((int)w_bonus, i & 63)), lane);
        return false;
      }
      const int64_t qrow = off0 + i;
      const int32_t x = cur.x;
      const int32_t qi = in_list ? cur.qi : -1;   // (i < g here: the draft's list of this position is real)
      const float qp = qi >= 0 ? cur.qp : 0.f;
      if (x < 0 || (t.V > 0 && x >= t.V)) {
        bad |= 1;
        if (lane == 0) {
          if (t.p_tok) t.p_tok[qrow] = 0.f;
          if (t.q_tok) t.q_tok[qrow] = 0.f;
        }
        return false;
      }
      const uint64_t hit_p = __ballot(live && idx == x), hit_q = __ballot(qi == x);
      // (the lanes read here are wave-uniform: a register read, not a trip through the LDS crossbar)
      const float p = hit_p ? lane_value(e, __ffsll((long long)hit_p) - 1) / Z : 0.f;
      const float q = hit_q ? lane_value(qp, __ffsll((long long)hit_q) - 1) : 0.f;
      const uint32_t r_accept = (uint32_t)__builtin_amdgcn_readlane((int)w_accept, i & 63);
      if (lane == 0) {
        if (t.p_tok) t.p_tok[qrow] = p;
        if (t.q_tok) t.q_tok[qrow] = q;
      }
      if (__fmul_rn(u01(r_accept), q) < p) return true;   // accepted
      // rejected at i: x' ~ norm(max(0, P_i - Q_i)); q at each listed target id, 0 if the draft
      // does not list it
      first_reject = i;
      float q_here = 0.f;
      for (int32_t j = 0; j < t.k; ++j) {
        const int32_t qj = __builtin_amdgcn_readlane(qi, j);
        const float pj = lane_value(qp, j);
        if (live && qj == idx) q_here = pj;
      }
      const float invZ = 1.f / Z;
      const float w = live ? fmaxf(0.f, fmaf(e, invZ, -q_here)) : 0.f;
      const float r = u01((uint32_t)__builtin_amdgcn_readlane((int)w_redraw, i & 63));
      token = draw_from_list(idx, w, r, lane);
      if (token < 0) {   // residual mass rounded to zero: draw from P_i instead
        bad |= 2;        // reported through status only; the session stays valid
        token = draw_from_list(idx, live ? e : 0.f, r, lane);
      }
      return false;
    };
    // Four positions ahead: the lists of positions i+1 .. i+4 are in flight while position i is
    // decided, so a long run of accepted drafts costs arithmetic per position, not a round trip to
    // memory (at most four rows are fetched in vain per session; a row is a few dozen bytes).
    Lists l0 = fetch(0), l1 = fetch(1), l2 = fetch(2), l3 = fetch(3);
    for (int32_t i = 0; i <= g; i += 4) {
      if (!visit(i, l0)) break;
      l0 = fetch(i + 4);
      if (i + 1 > g || !visit(i + 1, l1)) break;
      l1 = fetch(i + 5);
      if (i + 2 > g || !visit(i + 2, l2)) break;
      l2 = fetch(i + 6);
      if (i + 3 > g || !visit(i + 3, l3)) break;
      l3 = fetch(i + 7);
    }
  }
  const int32_t fatal = bad & ~2;
  if (!(bad & 4)) {   // rows and positions never visited: say so
    const float nan = __builtin_nanf("");
    if (t.row_stats)
      for (int32_t j = last + 1 + lane; j <= g; j += kWave) {
        t.row_stats[2 * (lrow0 + j)] = nan;
        t.row_stats[2 * (lrow0 + j) + 1] = nan;
      }
    for (int32_t j = last + 1 + lane; j < g; j += kWave) {
      if (t.p_tok) t.p_tok[off0 + j] = nan;
      if (t.q_tok) t.q_tok[off0 + j] = nan;
    }
  }
  if (lane == 0) {
    if (fatal || token < 0) {
      t.accepted_len[b] = 0;
      t.rejected[b] = 1;
      t.out_token[b] = -1;
      if (t.status) t.status[b] = bad | (fatal ? 0 : 8);
    } else {
      t.accepted_len[b] = first_reject;
      t.rejected[b] = first_reject < g ? 1 : 0;
      t.out_token[b] = token;
      if (t.status) t.status[b] = bad;
    }
  }
}

}  // namespace dssd
