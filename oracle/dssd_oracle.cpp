// CPU oracle for the speculative-decoding verification step of DSSD
// (arXiv 2507.12000: Sec. 2.1 "Verification Process", Sec. 3, Algorithms 1 and 2).
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, single-threaded fp64
// statement of what the verification step computes.  It exists so that the GPU
// library can be checked against it; nothing in the product path may call it.
// It shares no code, header, table or constant generator with the GPU library.
//
// What it follows, in the paper's order (Algorithm 2, "Verification Process" at the
// edge and "Resample" on the device; Algorithm 1 is the same arithmetic in one place):
//   1. P_1..P_{gamma+1}: softmax over the vocabulary of the target model's logits.
//   2. for j = 1..gamma while Flag = 1: draw r_j ~ U[0,1); accept x_j iff
//      r_j < min(1, p_j(x_j)/q_j(x_j)); otherwise Flag = 0.
//   3. Flag = 0: x'_j ~ norm(max(0, P_j - Q_j)).
//   4. all accepted: x_{gamma+1} ~ P_{gamma+1}.
//   5. result (x_j, j).
//
// Readings of points the paper leaves open or prints inconsistently:
//   * The paper's algorithms print the acceptance ratio as q/p.  Only p/q, together
//     with the residual norm(max(0, P - Q)) printed in the same algorithms, keeps the
//     emitted token distributed as P (the "no loss of inference quality" property the
//     paper claims and the two works its footnote cites define); p/q is used.
//   * The test is evaluated without a division, as r*q < p, so q = 0 is defined:
//     q = 0 and p > 0 accepts, q = 0 and p = 0 rejects.
//   * r ~ U[0,1): r = (w >> 8) * 2^-24 from one 32-bit random word w, so r < 1 always
//     and p >= q always accepts.
//   * Random words come from Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) with
//     key = (seed_lo, seed_hi) and counter = (session, position, step_lo, step_hi):
//     word 0 feeds the accept test of that position, word 1 the residual draw at that
//     position, word 2 the bonus draw (position gamma), word 3 is unused.
//   * x ~ w/sum(w) is the inverse CDF: the smallest k whose inclusive prefix sum
//     exceeds t = r * sum(w).  Tokens of zero weight are never drawn.
//   * A residual of zero total mass cannot follow a genuine rejection; if rounding
//     produces one the draw falls back to P_j with the same r and a status bit is set.
//   * Indices are 0-based here: n = j - 1 is the number of accepted drafts.
//
// Pins (tests/ with -m "not gpu"): Philox known-answer vectors; softmax against an
// independent library routine and closed forms; brute force over all 2^24 values of r
// for the accept test and the inverse CDF; exact enumeration of the emitted-token law
// on tiny vocabularies; chi-square Monte Carlo on whole sample paths; the paper's
// Table 1 column 1 - alpha^gamma; invariants.
//
// The second half of the file states the same step as the paper's split (Sec. 3): an edge
// function that sees only tokens and the scalars q_j(x_j) and emits either the bonus token
// or the b_prob-bit distribution P_j, and a device function that redraws from the received
// P_j and its own Q_j.  Pins: with an exact downlink the split equals the unsplit step bit
// for bit; the binary16 rounding agrees with numpy's converter on every half value's
// neighbourhood; the device draw agrees with a numpy restatement.
//
// Build: g++ -O2 -std=c++17 -shared -fPIC (no -ffast-math: summation order is part
// of the definition).

#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <vector>

extern "C" {

// ---------------------------------------------------------------------------
// Philox4x32-10 (SC'11, Sec. 3.3 and Table 2 of that paper): a 4-word counter is
// passed through ten rounds; each round multiplies words 0 and 2 by two fixed odd
// constants, keeps high and low halves of the 64-bit products, and xors the high
// halves with the other counter words and the round key; the key is advanced by
// two Weyl constants between rounds.
// ---------------------------------------------------------------------------
void dssd_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  const uint64_t mult_a = 0xD2511F53ull;  // multiplier applied to word 0
  const uint64_t mult_b = 0xCD9E8D57ull;  // multiplier applied to word 2
  const uint32_t weyl_a = 0x9E3779B9u;    // key word 0 increment (golden ratio)
  const uint32_t weyl_b = 0xBB67AE85u;    // key word 1 increment (sqrt(3) - 1)
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) {
      k0 += weyl_a;
      k1 += weyl_b;
    }
    const uint64_t prod_a = mult_a * (uint64_t)c0;
    const uint64_t prod_b = mult_b * (uint64_t)c2;
    const uint32_t n0 = (uint32_t)(prod_b >> 32) ^ c1 ^ k0;
    const uint32_t n1 = (uint32_t)prod_b;
    const uint32_t n2 = (uint32_t)(prod_a >> 32) ^ c3 ^ k1;
    const uint32_t n3 = (uint32_t)prod_a;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// r in [0,1): the top 24 bits of a random word, scaled by 2^-24.
double dssd_oracle_u01(uint32_t w) { return (double)(w >> 8) * (1.0 / 16777216.0); }

// The four words of the block that belongs to (session, position, step) under seed.
void dssd_oracle_random_block(uint64_t seed, uint64_t step, uint32_t session, uint32_t position,
                              uint32_t out[4]) {
  const uint32_t ctr[4] = {session, position, (uint32_t)step, (uint32_t)(step >> 32)};
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  dssd_oracle_philox4x32_10(ctr, key, out);
}

// ---------------------------------------------------------------------------
// Widening of stored logits.  dtype 0: IEEE fp32.  dtype 1: bfloat16 (the upper 16
// bits of an fp32), widened exactly.
// ---------------------------------------------------------------------------
static double logit_at(const void* row, int dtype, int64_t v) {
  if (dtype == 0) return (double)((const float*)row)[v];
  const uint32_t bits = (uint32_t)((const uint16_t*)row)[v] << 16;
  float f;
  std::memcpy(&f, &bits, sizeof f);
  return (double)f;
}

// Step 1: P = softmax(logits * inv_temperature) over one row.
// m = max_v y_v, Z = sum_v exp(y_v - m) in index order, P_v = exp(y_v - m)/Z.
void dssd_oracle_softmax_row(const void* logits_row, int dtype, int32_t V, double inv_temperature,
                             double* P, double* m_out, double* Z_out) {
  double m = -std::numeric_limits<double>::infinity();
  for (int32_t v = 0; v < V; ++v) {
    const double y = logit_at(logits_row, dtype, v) * inv_temperature;
    if (y > m) m = y;
  }
  double Z = 0.0;
  for (int32_t v = 0; v < V; ++v) {
    const double e = std::exp(logit_at(logits_row, dtype, v) * inv_temperature - m);
    P[v] = e;
    Z += e;
  }
  for (int32_t v = 0; v < V; ++v) P[v] /= Z;
  *m_out = m;
  *Z_out = Z;
}

// Step 2, one position: accept iff r < min(1, p/q), evaluated as r*q < p.
int dssd_oracle_accept(double r, double p, double q) { return (r * q < p) ? 1 : 0; }

// How far r is from the boundary of that test, in the units of r: |r - p/q| for q > 0, written
// as |r*q - p| / q.  With q = 0 the test does not depend on r (p > 0 accepts, p = 0 rejects):
// infinitely far, except that a p below 1e-30 counts as on the boundary, because a 32-bit
// float evaluation may flush such a p to zero.  Used only to tell the comparison with another
// implementation which decisions are near-ties; it takes no part in the decision.
double dssd_oracle_accept_margin(double r, double p, double q) {
  const double gap = std::fabs(r * q - p);
  return q > 0.0 ? gap / q : (p > 1e-30 ? std::numeric_limits<double>::infinity() : 0.0);
}

// Probability that step 2 accepts a token whose probabilities are (p, q).
double dssd_oracle_accept_prob(double p, double q) {
  if (q <= 0.0) return p > 0.0 ? 1.0 : 0.0;
  return p >= q ? 1.0 : p / q;
}

// Step 3, the distribution: w_v = max(0, P_v - Q_v) (unnormalised) and its mass R.
double dssd_oracle_residual(const double* P, const float* Q, int32_t V, double* w) {
  double R = 0.0;
  for (int32_t v = 0; v < V; ++v) {
    const double d = P[v] - (double)Q[v];
    w[v] = d > 0.0 ? d : 0.0;
    R += w[v];
  }
  return R;
}

// x ~ w / sum(w) by inverse CDF with the uniform r: smallest k with
// w_0 + .. + w_k > r * sum(w).  Returns -1 if sum(w) <= 0.  *margin (if not NULL)
// receives min(t - C_{k-1}, C_k - t) / sum(w): how far t is from the two CDF
// boundaries of the chosen token, as a fraction of the total mass.
int32_t dssd_oracle_inverse_cdf(const double* w, int32_t V, double r, double* margin) {
  double total = 0.0;
  for (int32_t v = 0; v < V; ++v) total += w[v];
  if (margin) *margin = 0.0;
  if (!(total > 0.0)) return -1;
  const double t = r * total;
  double below = 0.0;
  int32_t last_positive = -1;
  for (int32_t v = 0; v < V; ++v) {
    if (w[v] > 0.0) last_positive = v;
    const double upto = below + w[v];
    if (upto > t) {
      if (margin) {
        const double lo = t - below, hi = upto - t;
        *margin = (lo < hi ? lo : hi) / total;
      }
      return v;
    }
    below = upto;
  }
  return last_positive;
}

// The same draw for an array of uniforms (used by the brute-force pins).
void dssd_oracle_inverse_cdf_many(const double* w, int32_t V, const double* r, int64_t count,
                                  int32_t* token) {
  for (int64_t i = 0; i < count; ++i) token[i] = dssd_oracle_inverse_cdf(w, V, r[i], nullptr);
}

// The same accept test for an array of uniforms (used by the brute-force pins).
int64_t dssd_oracle_accept_count(const double* r, int64_t count, double p, double q) {
  int64_t accepted = 0;
  for (int64_t i = 0; i < count; ++i) accepted += dssd_oracle_accept(r[i], p, q);
  return accepted;
}

// ---------------------------------------------------------------------------
// One session, steps 1-5.
// ---------------------------------------------------------------------------
typedef struct {
  int32_t n;          // accepted drafts, 0..gamma  (the paper's j - 1)
  int32_t rejected;   // 1 iff n < gamma            (the paper's Flag = 0, a = 1)
  int32_t token;      // resampled token (rejected) or bonus token (all accepted)
  int32_t status;     // bit 0: a draft token outside [0,V); bit 1: zero residual mass, drew from P_n
  double  resid_mass; // R = sum_v max(0, P_n - Q_n); 0 when not rejected
  double  cdf_margin; // distance of the draw from a CDF boundary, fraction of total mass
  double  accept_margin;  // min over tested positions of |r - p/q| (see near-tie rule)
} dssd_oracle_result;

// logits: (gamma+1) rows of V; draft_probs: gamma rows of V fp32; tokens: gamma.
// Per-position outputs (may be NULL): p_tok, q_tok, r_acc [gamma] for EVERY position
// (also those after the first rejection, which the decision loop never looks at);
// row_m, row_Z [gamma+1]; beta [gamma] = sum_v min(P_i, Q_i) (costly, optional).
void dssd_oracle_verify_session(const void* logits, int dtype, const float* draft_probs,
                                const int32_t* tokens, int32_t gamma, int32_t V,
                                double inv_temperature, uint64_t seed, uint64_t step,
                                uint32_t session, dssd_oracle_result* res, double* p_tok,
                                double* q_tok, double* r_acc, double* row_m, double* row_Z,
                                double* beta) {
  const size_t elem = dtype == 0 ? 4 : 2;
  const char* base = (const char*)logits;
  std::vector<double> P((size_t)V), w((size_t)V);
  res->n = gamma; res->rejected = 0; res->token = -1; res->status = 0;
  res->resid_mass = 0.0; res->cdf_margin = 0.0;
  res->accept_margin = std::numeric_limits<double>::infinity();

  // Step 1 for every row, then the per-position scalars of step 2.  A draft token outside the
  // vocabulary is malformed input: it counts where the loop of Algorithm 2 meets it (while
  // Flag = 1), and then the session is reported and emits nothing; one that lies after the
  // first rejection is never looked at, like everything else there.
  bool open = true;  // Flag = 1
  for (int32_t i = 0; i <= gamma; ++i) {
    double m, Z;
    dssd_oracle_softmax_row(base + (size_t)i * (size_t)V * elem, dtype, V, inv_temperature,
                            P.data(), &m, &Z);
    if (row_m) row_m[i] = m;
    if (row_Z) row_Z[i] = Z;
    if (i == gamma) break;
    const float* Q = draft_probs + (size_t)i * (size_t)V;
    const bool in_vocabulary = tokens[i] >= 0 && tokens[i] < V;
    const double p = in_vocabulary ? P[tokens[i]] : 0.0;
    const double q = in_vocabulary ? (double)Q[tokens[i]] : 0.0;
    uint32_t words[4];
    dssd_oracle_random_block(seed, step, session, (uint32_t)i, words);
    const double r = dssd_oracle_u01(words[0]);
    if (p_tok) p_tok[i] = p;
    if (q_tok) q_tok[i] = q;
    if (r_acc) r_acc[i] = r;
    if (beta) {
      double b = 0.0;
      for (int32_t v = 0; v < V; ++v) b += P[v] < (double)Q[v] ? P[v] : (double)Q[v];
      beta[i] = b;
    }
    if (!open) continue;
    if (!in_vocabulary) {  // malformed input met by the loop: report, emit nothing
      open = false;
      res->status |= 1;
      res->n = 0; res->rejected = 1; res->token = -1;
      res->accept_margin = std::numeric_limits<double>::infinity();
      continue;
    }
    // Step 2, and how close r came to its boundary.
    const double margin = dssd_oracle_accept_margin(r, p, q);
    if (margin < res->accept_margin) res->accept_margin = margin;
    if (!dssd_oracle_accept(r, p, q)) {
      open = false;  // Flag = 0
      res->n = i;
      res->rejected = 1;
      // Step 3 on this row, with word 1 of this position's block.
      const double R = dssd_oracle_residual(P.data(), Q, V, w.data());
      const double r2 = dssd_oracle_u01(words[1]);
      res->resid_mass = R;
      if (R > 0.0) {
        res->token = dssd_oracle_inverse_cdf(w.data(), V, r2, &res->cdf_margin);
      } else {
        res->status |= 2;
        res->token = dssd_oracle_inverse_cdf(P.data(), V, r2, &res->cdf_margin);
      }
    }
  }
  if (open) {
    // Step 4: P currently holds row gamma (the (gamma+1)-th distribution).
    uint32_t words[4];
    dssd_oracle_random_block(seed, step, session, (uint32_t)gamma, words);
    res->token = dssd_oracle_inverse_cdf(P.data(), V, dssd_oracle_u01(words[2]), &res->cdf_margin);
  }
}

// A batch of sessions laid out as the GPU library takes them: session b owns drafts
// [off_b, off_{b+1}) with off_b = draft_offsets[b] (or b*gamma when draft_offsets is
// NULL); its logits rows are off_b + b .. off_{b+1} + b.  Per-position outputs are
// indexed by draft row, row_m/row_Z by logits row.  Sessions are taken one after the
// other, in order.
void dssd_oracle_verify_batch(int32_t B, int32_t V, int32_t gamma, const int32_t* draft_offsets,
                              const void* logits, int dtype, const float* draft_probs,
                              const int32_t* draft_tokens, const float* inv_temperature,
                              uint64_t seed, uint64_t step, uint32_t session_base,
                              dssd_oracle_result* res, double* p_tok, double* q_tok, double* r_acc,
                              double* row_m, double* row_Z, double* beta) {
  const size_t elem = dtype == 0 ? 4 : 2;
  for (int32_t b = 0; b < B; ++b) {
    const int64_t off = draft_offsets ? draft_offsets[b] : (int64_t)b * gamma;
    const int32_t g = draft_offsets ? draft_offsets[b + 1] - draft_offsets[b] : gamma;
    const int64_t lrow = off + b;
    dssd_oracle_verify_session(
        (const char*)logits + (size_t)lrow * (size_t)V * elem, dtype,
        draft_probs + (size_t)off * (size_t)V, draft_tokens + off, g, V,
        inv_temperature ? (double)inv_temperature[b] : 1.0, seed, step, session_base + (uint32_t)b,
        res + b, p_tok ? p_tok + off : nullptr, q_tok ? q_tok + off : nullptr,
        r_acc ? r_acc + off : nullptr, row_m ? row_m + lrow : nullptr,
        row_Z ? row_Z + lrow : nullptr, beta ? beta + off : nullptr);
  }
}

// ---------------------------------------------------------------------------
// The split of Algorithm 2 (Sec. 3): what the edge and the device each compute
// when only DSSD's payloads cross the link.
//   uplink   : tokens x_i and the scalars q_i(x_i)            (no Q rows at the edge)
//   downlink : if Flag = 0, the distribution P_j(x) in b_prob-bit values, and j;
//              else the bonus token and gamma+1
//   device   : x'_j ~ norm(max(0, P_j - Q_j)) from the received P_j and its own Q_j
// b_prob = 32 is IEEE fp32, b_prob = 16 is IEEE fp16 (Sec. 2.2: "32 bits for full
// precision or 16 bits for half precision"); both are rounded to nearest-even from
// the fp32 value of P, the precision the GPU library computes P in.  p_dtype 3
// (fp64, no rounding) exists only to pin the split against the unsplit path.
// ---------------------------------------------------------------------------
enum { ORACLE_P_F32 = 0, ORACLE_P_F16 = 2, ORACLE_P_F64 = 3 };

// fp32 -> IEEE binary16, round to nearest, ties to even; subnormals kept.
uint16_t dssd_oracle_f32_to_f16(float f) {
  uint32_t bits;
  std::memcpy(&bits, &f, sizeof bits);
  const uint32_t sign = (bits >> 16) & 0x8000u;
  const int32_t exp32 = (int32_t)((bits >> 23) & 0xFFu);
  uint32_t man = bits & 0x7FFFFFu;
  if (exp32 == 255) return (uint16_t)(sign | 0x7C00u | (man ? 0x200u : 0u));
  const int32_t e = exp32 - 127 + 15;
  if (e >= 31) return (uint16_t)(sign | 0x7C00u);
  if (e <= 0) {
    if (e < -10) return (uint16_t)sign;          // below half of the smallest subnormal
    man |= 0x800000u;                            // implicit one
    const int shift = 14 - e;                    // 14 .. 24
    uint32_t half = man >> shift;
    const uint32_t rem = man & ((1u << shift) - 1u), mid = 1u << (shift - 1);
    if (rem > mid || (rem == mid && (half & 1u))) ++half;
    return (uint16_t)(sign | half);
  }
  uint32_t half = ((uint32_t)e << 10) | (man >> 13);
  const uint32_t rem = man & 0x1FFFu;
  if (rem > 0x1000u || (rem == 0x1000u && (half & 1u))) ++half;   // may carry into the exponent
  return (uint16_t)(sign | half);
}

double dssd_oracle_f16_to_f64(uint16_t h) {
  const int sign = (h >> 15) & 1, e = (h >> 10) & 0x1F, man = h & 0x3FF;
  double v;
  if (e == 0) v = std::ldexp((double)man, -24);
  else if (e == 31) v = man ? std::numeric_limits<double>::quiet_NaN() : std::numeric_limits<double>::infinity();
  else v = std::ldexp((double)(man | 0x400), e - 25);
  return sign ? -v : v;
}

static size_t p_elem_size(int p_dtype) { return p_dtype == ORACLE_P_F16 ? 2 : p_dtype == ORACLE_P_F32 ? 4 : 8; }

// The downlink payload: P in b_prob-bit values.
void dssd_oracle_quantize_p_row(const double* P, int32_t V, int p_dtype, void* out) {
  for (int32_t v = 0; v < V; ++v) {
    if (p_dtype == ORACLE_P_F64) ((double*)out)[v] = P[v];
    else if (p_dtype == ORACLE_P_F32) ((float*)out)[v] = (float)P[v];
    else ((uint16_t*)out)[v] = dssd_oracle_f32_to_f16((float)P[v]);
  }
}

static double p_at(const void* row, int p_dtype, int32_t v) {
  if (p_dtype == ORACLE_P_F64) return ((const double*)row)[v];
  if (p_dtype == ORACLE_P_F32) return (double)((const float*)row)[v];
  return dssd_oracle_f16_to_f64(((const uint16_t*)row)[v]);
}

// Edge side of one session.  q_scalars[i] = q_i(x_i) as uploaded.  On a rejection the
// P row of the rejected position is written to p_row_out in p_dtype; otherwise the bonus
// token is drawn.  res->token is -1 for rejected sessions: the edge does not redraw.
void dssd_oracle_edge_session(const void* logits, int dtype, const float* q_scalars,
                              const int32_t* tokens, int32_t gamma, int32_t V, double inv_temperature,
                              uint64_t seed, uint64_t step, uint32_t session, int p_dtype,
                              dssd_oracle_result* res, void* p_row_out, double* p_tok) {
  const size_t elem = dtype == 0 ? 4 : 2;
  std::vector<double> P((size_t)V);
  res->n = gamma; res->rejected = 0; res->token = -1; res->status = 0;
  res->resid_mass = 0.0; res->cdf_margin = 0.0;
  res->accept_margin = std::numeric_limits<double>::infinity();
  for (int32_t i = 0; i <= gamma; ++i) {
    double m, Z;
    dssd_oracle_softmax_row((const char*)logits + (size_t)i * (size_t)V * elem, dtype, V,
                            inv_temperature, P.data(), &m, &Z);
    uint32_t words[4];
    dssd_oracle_random_block(seed, step, session, (uint32_t)i, words);
    if (i == gamma) {   // all accepted: bonus token, word 2 of the position-gamma block
      res->token = dssd_oracle_inverse_cdf(P.data(), V, dssd_oracle_u01(words[2]), &res->cdf_margin);
      return;
    }
    if (tokens[i] < 0 || tokens[i] >= V) {  // malformed input met by the loop: report, emit nothing
      res->status |= 1; res->n = 0; res->rejected = 1;
      res->accept_margin = std::numeric_limits<double>::infinity();
      return;
    }
    const double p = P[tokens[i]], q = (double)q_scalars[i], r = dssd_oracle_u01(words[0]);
    if (p_tok) p_tok[i] = p;
    const double margin = dssd_oracle_accept_margin(r, p, q);
    if (margin < res->accept_margin) res->accept_margin = margin;
    if (!dssd_oracle_accept(r, p, q)) {
      res->n = i;
      res->rejected = 1;
      dssd_oracle_quantize_p_row(P.data(), V, p_dtype, p_row_out);
      return;
    }
  }
}

// Device side of one session: it knows j (n = j - 1), received P_j, and owns Q_j.
// Draws with word 1 of the position-n block.  Returns the token; fills R, the margin and
// status bit 1 (zero residual: drew from the received P_j).
int32_t dssd_oracle_device_session(const void* p_row, int p_dtype, const float* Q_row, int32_t V,
                                   int32_t n, uint64_t seed, uint64_t step, uint32_t session,
                                   double* resid_mass, double* cdf_margin, int32_t* status) {
  std::vector<double> P((size_t)V), w((size_t)V);
  for (int32_t v = 0; v < V; ++v) P[v] = p_at(p_row, p_dtype, v);
  const double R = dssd_oracle_residual(P.data(), Q_row, V, w.data());
  uint32_t words[4];
  dssd_oracle_random_block(seed, step, session, (uint32_t)n, words);
  const double r = dssd_oracle_u01(words[1]);
  if (resid_mass) *resid_mass = R;
  if (status) *status = 0;
  if (R > 0.0) return dssd_oracle_inverse_cdf(w.data(), V, r, cdf_margin);
  if (status) *status = 2;
  return dssd_oracle_inverse_cdf(P.data(), V, r, cdf_margin);
}

// Batch forms.  p_rows is [B, V] in p_dtype, row b written (edge) / read (device) only for
// rejected sessions.  Layout of everything else as in dssd_oracle_verify_batch.
void dssd_oracle_edge_batch(int32_t B, int32_t V, int32_t gamma, const int32_t* draft_offsets,
                            const void* logits, int dtype, const float* q_scalars,
                            const int32_t* draft_tokens, const float* inv_temperature, uint64_t seed,
                            uint64_t step, uint32_t session_base, int p_dtype,
                            dssd_oracle_result* res, void* p_rows, double* p_tok) {
  const size_t elem = dtype == 0 ? 4 : 2;
  for (int32_t b = 0; b < B; ++b) {
    const int64_t off = draft_offsets ? draft_offsets[b] : (int64_t)b * gamma;
    const int32_t g = draft_offsets ? draft_offsets[b + 1] - draft_offsets[b] : gamma;
    dssd_oracle_edge_session((const char*)logits + (size_t)(off + b) * (size_t)V * elem, dtype,
                             q_scalars + off, draft_tokens + off, g, V,
                             inv_temperature ? (double)inv_temperature[b] : 1.0, seed, step,
                             session_base + (uint32_t)b, p_dtype, res + b,
                             (char*)p_rows + (size_t)b * (size_t)V * p_elem_size(p_dtype),
                             p_tok ? p_tok + off : nullptr);
  }
}

void dssd_oracle_device_batch(int32_t B, int32_t V, int32_t gamma, const int32_t* draft_offsets,
                              const float* draft_probs, const void* p_rows, int p_dtype,
                              const int32_t* accepted_len, const int32_t* rejected, uint64_t seed,
                              uint64_t step, uint32_t session_base, int32_t* token,
                              double* resid_mass, double* cdf_margin, int32_t* status) {
  for (int32_t b = 0; b < B; ++b) {
    token[b] = -1;
    if (status) status[b] = 0;
    if (!rejected[b]) continue;
    const int64_t off = draft_offsets ? draft_offsets[b] : (int64_t)b * gamma;
    const int32_t g = draft_offsets ? draft_offsets[b + 1] - draft_offsets[b] : gamma;
    const int32_t n = accepted_len[b];
    if (n < 0 || n >= g) { if (status) status[b] = 4; continue; }
    token[b] = dssd_oracle_device_session(
        (const char*)p_rows + (size_t)b * (size_t)V * p_elem_size(p_dtype), p_dtype,
        draft_probs + (size_t)(off + n) * (size_t)V, V, n, seed, step, session_base + (uint32_t)b,
        resid_mass ? resid_mass + b : nullptr, cdf_margin ? cdf_margin + b : nullptr,
        status ? status + b : nullptr);
  }
}

}  // extern "C"
