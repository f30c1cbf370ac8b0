// Host-side sanitizer run of the oracle (test infrastructure): built by
// tests/test_oracle_sanitizers.py with -fsanitize=address,undefined and executed on the CPU.
// Drives every exported function over seeded inputs, including the degenerate ones.
#include "../oracle/dssd_oracle.cpp"

#include <cstdio>
#include <cstdlib>

static uint32_t lcg_state = 12345u;
static double unif() { lcg_state = lcg_state * 1664525u + 1013904223u; return (lcg_state >> 8) / 16777216.0; }

static void make_batch(int B, int V, int gmax, int dtype, std::vector<int32_t>& off, std::vector<char>& logits,
                       std::vector<float>& Q, std::vector<int32_t>& tok, std::vector<float>& tau) {
  off.assign(B + 1, 0);
  for (int b = 0; b < B; ++b) off[b + 1] = off[b] + (gmax ? (int)(unif() * (gmax + 1)) : 0);
  const int R_Q = off[B], R_L = R_Q + B;
  logits.assign((size_t)R_L * V * (dtype == 0 ? 4 : 2), 0);
  for (size_t i = 0; i < (size_t)R_L * V; ++i) {
    const float z = (float)(unif() * 8.0 - 4.0);
    if (dtype == 0) std::memcpy(&logits[i * 4], &z, 4);
    else { uint32_t bits; std::memcpy(&bits, &z, 4); const uint16_t h = (uint16_t)(bits >> 16); std::memcpy(&logits[i * 2], &h, 2); }
  }
  Q.assign((size_t)R_Q * V, 0.f);
  tok.assign(R_Q, 0);
  for (int r = 0; r < R_Q; ++r) {
    double s = 0;
    for (int v = 0; v < V; ++v) { Q[(size_t)r * V + v] = (float)unif(); s += Q[(size_t)r * V + v]; }
    for (int v = 0; v < V; ++v) Q[(size_t)r * V + v] = (float)(Q[(size_t)r * V + v] / s);
    tok[r] = (int)(unif() * V);
  }
  tau.assign(B, 1.f);
  for (int b = 0; b < B; ++b) tau[b] = (float)(0.5 + unif());
}

int main() {
  long checks = 0;
  for (int dtype = 0; dtype < 2; ++dtype)
    for (int V : {1, 2, 7, 300})
      for (int gmax : {0, 1, 5}) {
        const int B = 9;
        std::vector<int32_t> off, tok; std::vector<char> logits; std::vector<float> Q, tau;
        make_batch(B, V, gmax, dtype, off, logits, Q, tok, tau);
        if (!tok.empty() && V > 1) tok[0] = V;                      // one malformed token id
        const int R_Q = off[B], R_L = R_Q + B;
        std::vector<dssd_oracle_result> res(B);
        std::vector<double> p(R_Q + 1), q(R_Q + 1), r(R_Q + 1), m(R_L), Z(R_L), beta(R_Q + 1);
        dssd_oracle_verify_batch(B, V, 0, off.data(), logits.data(), dtype, Q.data(), tok.data(), tau.data(), 7, 3, 100,
                                 res.data(), p.data(), q.data(), r.data(), m.data(), Z.data(), beta.data());
        dssd_oracle_verify_batch(B, V, 0, off.data(), logits.data(), dtype, Q.data(), tok.data(), nullptr, 7, 4, 0,
                                 res.data(), nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
        for (int b = 0; b < B; ++b) {
          const int g = off[b + 1] - off[b];
          if (res[b].status & 1) continue;
          if (res[b].n < 0 || res[b].n > g || res[b].token < 0 || res[b].token >= V) { std::printf("bad record\n"); return 1; }
          ++checks;
        }
        // the split, all three downlink types
        std::vector<float> qs(R_Q + 1);
        for (int i = 0; i < R_Q; ++i) qs[i] = (tok[i] >= 0 && tok[i] < V) ? Q[(size_t)i * V + tok[i]] : 0.f;
        for (int p_dtype : {0, 2, 3}) {
          std::vector<char> rows((size_t)B * V * 8);
          dssd_oracle_edge_batch(B, V, 0, off.data(), logits.data(), dtype, qs.data(), tok.data(), tau.data(), 7, 3, 100,
                                 p_dtype, res.data(), rows.data(), p.data());
          std::vector<int32_t> n(B), rj(B), out(B), st(B);
          for (int b = 0; b < B; ++b) { n[b] = res[b].n; rj[b] = res[b].rejected && !(res[b].status & 1); }
          std::vector<double> R(B), mg(B);
          dssd_oracle_device_batch(B, V, 0, off.data(), Q.data(), rows.data(), p_dtype, n.data(), rj.data(), 7, 3, 100,
                                   out.data(), R.data(), mg.data(), st.data());
          for (int b = 0; b < B; ++b)
            if (rj[b] && (out[b] < 0 || out[b] >= V)) { std::printf("bad device token\n"); return 1; }
          ++checks;
        }
      }
  // every binary16 code survives a round trip through fp32
  for (uint32_t h = 0; h < 0x7C00u; ++h) {
    const double v = dssd_oracle_f16_to_f64((uint16_t)h);
    if (dssd_oracle_f32_to_f16((float)v) != h) { std::printf("f16 round trip %u\n", h); return 1; }
    ++checks;
  }
  const double w[4] = {0.0, 0.5, 0.0, 0.5};
  double margin;
  if (dssd_oracle_inverse_cdf(w, 4, 0.75, &margin) != 3 || dssd_oracle_inverse_cdf(w, 0, 0.5, nullptr) != -1) return 1;
  std::printf("sanitized oracle run ok: %ld checks\n", checks);
  return 0;
}
