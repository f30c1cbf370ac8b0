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
// read only as far as its first rejection (plus one row fetched ahead).
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
    const int32_t km = __shfl(key, m, kWave);
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
    // one position ahead: the lists of position i + 1 are asked for before position i is decided,
    // so that their latency runs under the arithmetic (at most one row is fetched in vain)
    struct Lists { int32_t idx; float z; int32_t x, qi; float qp; };
    auto fetch = [&](int32_t i) {
      Lists L{-1, 0.f, 0, -1, 0.f};
      if (i > g) return L;
      const int64_t row = lrow0 + i;
      if (in_list) { L.idx = t.p_idx[row * t.k + lane]; L.z = t.p_logit[row * t.k + lane]; }
      if (i < g) {
        const int64_t qrow = off0 + i;
        L.x = t.tokens[qrow];
        if (in_list) { L.qi = t.q_idx[qrow * t.k + lane]; L.qp = t.q_prob[qrow * t.k + lane]; }
      }
      return L;
    };
    Lists next = fetch(0);
    for (int32_t i = 0; i <= g; ++i) {
      last = i;
      const Lists cur = next;
      next = fetch(i + 1);
      const int64_t row = lrow0 + i;
      const int32_t idx = cur.idx;
      const bool live = idx >= 0;
      const float z = live ? cur.z : neg_inf();
      const float M2 = wave_max(live ? z * c1 : neg_inf());
      const float e = (M2 > neg_inf()) ? fast_exp2(fmaf(z, c1, -M2)) : 0.f;   // 0 for unused entries
      const float Z = wave_sum(live ? e : 0.f);
      if (lane == 0 && t.row_stats) {
        t.row_stats[2 * row] = M2 * kLn2;
        t.row_stats[2 * row + 1] = Z;
      }
      if (!(Z > 0.f) || !(Z < 3.0e38f) || !(fabsf(M2) < 3.0e38f)) { bad |= 8; break; }
      if (i == g) {   // every draft accepted: the bonus token, from P_gamma
        const Philox rnd = step_block(t.session_base + (uint32_t)b, (uint32_t)i, t.step_lo, t.step_hi, t.step_dev,
                                      t.seed_lo, t.seed_hi);
        token = draw_from_list(idx, live ? e : 0.f, u01(rnd.w[2]), lane);
        break;
      }
      const int64_t qrow = off0 + i;
      const int32_t x = cur.x;
      const int32_t qi = cur.qi;
      const float qp = qi >= 0 ? cur.qp : 0.f;
      if (x < 0 || (t.V > 0 && x >= t.V)) {
        bad |= 1;
        if (lane == 0) {
          if (t.p_tok) t.p_tok[qrow] = 0.f;
          if (t.q_tok) t.q_tok[qrow] = 0.f;
        }
        break;
      }
      const uint64_t hit_p = __ballot(live && idx == x), hit_q = __ballot(qi == x);
      const float p = hit_p ? __shfl(e, __ffsll((long long)hit_p) - 1, kWave) / Z : 0.f;
      const float q = hit_q ? __shfl(qp, __ffsll((long long)hit_q) - 1, kWave) : 0.f;
      const Philox rnd = step_block(t.session_base + (uint32_t)b, (uint32_t)i, t.step_lo, t.step_hi, t.step_dev,
                                    t.seed_lo, t.seed_hi);
      if (lane == 0) {
        if (t.p_tok) t.p_tok[qrow] = p;
        if (t.q_tok) t.q_tok[qrow] = q;
      }
      if (__fmul_rn(u01(rnd.w[0]), q) < p) continue;   // accepted
      // rejected at i: x' ~ norm(max(0, P_i - Q_i)); q at each listed target id, 0 if the draft
      // does not list it
      first_reject = i;
      float q_here = 0.f;
      for (int32_t j = 0; j < t.k; ++j) {
        const int32_t qj = __shfl(qi, j, kWave);
        const float pj = __shfl(qp, j, kWave);
        if (live && qj == idx) q_here = pj;
      }
      const float invZ = 1.f / Z;
      const float w = live ? fmaxf(0.f, fmaf(e, invZ, -q_here)) : 0.f;
      const float r = u01(rnd.w[1]);
      token = draw_from_list(idx, w, r, lane);
      if (token < 0) {   // residual mass rounded to zero: draw from P_i instead
        bad |= 2;        // reported through status only; the session stays valid
        token = draw_from_list(idx, live ? e : 0.f, r, lane);
      }
      break;
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
