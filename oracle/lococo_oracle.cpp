// CPU oracle for the LoCoCo segment step  --  TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, double-precision implementation of what the paper's
// Algorithm 2 ("LoCoCo attention") computes for already-projected Q/K/V:
//   step 3  block-vs-(cache+block) causal attention        (Eq. 1, Alg. 2 step 3)
//   IF      fill the cache while everything still fits      (Alg. 2, the IF branch)
//   step 4  1-D convolution over [cache; block] -> logits,  (Eq. 5)
//           normalised per slot over the positions          (Eq. 6)
//   step 5  weighted fusion of K and V with shared weights  (Eq. 4a / 4b, Eq. 3)
// and the scan of that step over a sequence (Alg. 2 loop), plus the backward
// pass of one step (chain rule on the same definitions; the fine-tuning of the
// convolution heads needs it).
//
// Only the tests, the smoke check and the benchmark's cpu_baseline leg may
// call this file.  It shares no code, header, table or helper with the HIP
// library, and the HIP library never calls it.
//
// Every function follows the definition directly: no tiling, no fusion, no
// online softmax.  The only liberties are (a) a transposed copy of the filter
// bank so the innermost channel loop is contiguous (layout, not arithmetic)
// and (b) optional threads over independent chains / output rows.
//
// Readings of the paper taken here (the paper is silent or inconsistent):
//   * segments are 0-based, [n*B, min((n+1)*B, L)); the last may be shorter;
//   * the mask is additive: cache slots are visible to every block query and
//     block key j' is visible to block query r iff j' <= r;
//   * concatenation order is cache first, then block, for attention (Alg. 2
//     step 3), for the convolution input and for the fusion (Eq. 3);
//   * the convolution is a cross-correlation with zero "same" padding of
//     (k-1)/2 on both sides, stride 1, odd width (output length = input length);
//   * Eq. 6 is read as a softmax over the positions (norm = 0).  The literal
//     form relu(W) / (sum relu(W) + eps) is norm = 1 (the rectifier of the
//     convolution head read as acting on the convolution OUTPUT, so that the
//     weights are convex).  norm = 2 is the other reading of "a ReLU is
//     prepended": the rectifier acts on the convolution's INPUT (the stacked
//     keys / values that Eq. 5 convolves; the entries that Eq. 4 fuses stay as
//     they are) and Eq. 6 is taken exactly as printed, W / sum(W); a row sum
//     of magnitude below eps is replaced by +-eps (such a sum is signed and can
//     vanish: the reason the other two forms exist).  Forward only;
//   * conv_in = 0 feeds the keys only (C = d); conv_in = 1 feeds keys stacked
//     on values along channels (C = 2d, Eq. 5 as printed), K channels first;
//   * when the cache is partly full and cache + block exceeds M, the entries
//     present (m + B_n of them) are compressed to M;
//   * combination with an eviction policy (the ablation that adds attention
//     sinks or heavy hitters): the paper only says that such tokens are stored
//     in addition.  Read here as a per-slot "protected" mark: a live protected
//     slot is kept as it is by every compression step and its position
//     carries no weight in the mixing of the other slots; attention sees all
//     slots as before.  Which slots to protect (the first few tokens, the
//     tokens with the largest accumulated attention) is the caller's policy.
//
// Pins (tests/test_oracle_*.py): brute-force full causal attention when the
// sequence fits, sliding-window attention under one-hot logits, closed-form
// mean recursion under zero filters, library conv1d / matmul / SDPA, row sums,
// convexity, shift invariance, chain independence, resumability, plan vs.
// simulation; for protected slots: a numpy recursion with given logits, rows
// that never change, all-protected = frozen cache; for the backward pass:
// central finite differences of the forward pass, every input, every branch
// and variant.  Fidelity to the authors'
// trained heads (normalisation variant, ReLU placement, padding convention)
// and to their way of combining with eviction policies is parity unpinned:
// their code and weights are not available.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <thread>
#include <vector>

namespace {

struct Cfg {
  int32_t group;        // query heads per kv head
  int32_t head_dim;     // d
  int32_t M;            // cache slots
  int32_t conv_width;   // k, odd
  int32_t conv_in;      // 0: keys only; 1: [K;V] stacked on channels
  int32_t norm;         // 0: softmax over positions; 1: relu(W) / (sum + eps); 2: relu on the conv input, W / sum(W)
  int32_t state_round;  // 0: keep double; 1: fp32; 2: bf16 (on every cache write and on O)
  int32_t reserved;
  double attn_scale;    // <= 0 means 1/sqrt(d)
  double norm_eps;      // only for norm = 1
};

// Round-to-nearest-even of a double to the bf16 grid (8 significant bits,
// exponent range of fp32), done directly from the double so there is no
// double rounding through fp32.
double round_bf16(double x) {
  if (x == 0.0 || !std::isfinite(x)) return x;
  int e;
  std::frexp(x, &e);                    // |x| = f * 2^e, f in [0.5, 1)
  int qe = std::max(e - 8, -133);       // exponent of the quantum; -133 = smallest bf16 subnormal
  return std::ldexp(std::nearbyint(std::ldexp(x, -qe)), qe);
}

double round_store(double x, int mode) {
  if (mode == 1) return (double)(float)x;
  if (mode == 2) return round_bf16(x);
  return x;
}

template <class F>
void parallel_for(int64_t n, int nthreads, F f) {
  if (nthreads <= 1 || n <= 1) {
    for (int64_t i = 0; i < n; ++i) f(i);
    return;
  }
  int nt = (int)std::min<int64_t>(nthreads, n);
  std::vector<std::thread> th;
  for (int t = 0; t < nt; ++t)
    th.emplace_back([=] { for (int64_t i = t; i < n; i += nt) f(i); });
  for (auto& x : th) x.join();
}

// Alg. 2 step 3 with Eq. 1 for one query head: rows r < Bn of q against
// the m cache slots (all visible) followed by block keys j' <= r.
// colsum (or null): [m] accumulators; the probability each query row puts on cache slot j is added
// to colsum[j] (the accumulated attention scores a heavy-hitter policy ranks slots by).
void attention_block(const double* q, const double* kb, const double* vb,
                     const double* ck, const double* cv, int m, int Bn, int d,
                     double scale, double* o, double* colsum = nullptr) {
  std::vector<double> s((size_t)m + Bn);
  for (int r = 0; r < Bn; ++r) {
    const double* qr = q + (size_t)r * d;
    int n_vis = m + r + 1;
    double mx = -std::numeric_limits<double>::infinity();
    for (int j = 0; j < n_vis; ++j) {
      const double* kj = j < m ? ck + (size_t)j * d : kb + (size_t)(j - m) * d;
      double acc = 0.0;
      for (int c = 0; c < d; ++c) acc += qr[c] * kj[c];
      s[j] = acc * scale;
      mx = std::max(mx, s[j]);
    }
    double z = 0.0;
    for (int j = 0; j < n_vis; ++j) { s[j] = std::exp(s[j] - mx); z += s[j]; }
    double* orow = o + (size_t)r * d;
    for (int c = 0; c < d; ++c) orow[c] = 0.0;
    for (int j = 0; j < n_vis; ++j) {
      const double* vj = j < m ? cv + (size_t)j * d : vb + (size_t)(j - m) * d;
      double p = s[j] / z;
      if (colsum && j < m) colsum[j] += p;
      for (int c = 0; c < d; ++c) orow[c] += p * vj[c];
    }
  }
}

// Eq. 5: W[i, j] = bias[i] + sum_c sum_tau Wc[i, c, tau] * X[j + tau - (k-1)/2, c],
// X zero outside [0, T).  X is [T, C], Wc is [M, C, k], W is [M, T].
// relu_input: the input entries pass through max(., 0) first (the rectifier in front of the
// convolution layer, norm = 2).
void conv_logits(const double* X, int T, int C, const double* Wc, const double* bias,
                 int M, int k, double* W, int nthreads, bool relu_input = false) {
  const int pad = (k - 1) / 2;
  std::vector<double> Xr;
  if (relu_input) {
    Xr.assign(X, X + (size_t)T * C);
    for (double& x : Xr) x = x > 0.0 ? x : 0.0;
    X = Xr.data();
  }
  // layout-only copy: Wt[i][tau][c] = Wc[i][c][tau]
  std::vector<double> Wt((size_t)M * k * C);
  for (int i = 0; i < M; ++i)
    for (int c = 0; c < C; ++c)
      for (int t = 0; t < k; ++t)
        Wt[((size_t)i * k + t) * C + c] = Wc[((size_t)i * C + c) * k + t];
  parallel_for(M, nthreads, [&](int64_t i) {
    for (int j = 0; j < T; ++j) {
      double acc = bias ? bias[i] : 0.0;
      for (int t = 0; t < k; ++t) {
        int jj = j + t - pad;
        if (jj < 0 || jj >= T) continue;
        const double* w = &Wt[((size_t)i * k + t) * C];
        const double* x = X + (size_t)jj * C;
        double a = 0.0;
        for (int c = 0; c < C; ++c) a += w[c] * x[c];
        acc += a;
      }
      W[(size_t)i * T + j] = acc;
    }
  });
}

// Eq. 6: each row of W normalised over the T positions.
void normalise_rows(const double* W, int M, int T, int norm, double eps, double* w) {
  for (int i = 0; i < M; ++i) {
    const double* r = W + (size_t)i * T;
    double* out = w + (size_t)i * T;
    if (norm == 0) {
      double mx = r[0];
      for (int j = 1; j < T; ++j) mx = std::max(mx, r[j]);
      double z = 0.0;
      for (int j = 0; j < T; ++j) { out[j] = std::exp(r[j] - mx); z += out[j]; }
      for (int j = 0; j < T; ++j) out[j] /= z;
    } else if (norm == 1) {
      double z = 0.0;
      for (int j = 0; j < T; ++j) { out[j] = r[j] > 0.0 ? r[j] : 0.0; z += out[j]; }
      for (int j = 0; j < T; ++j) out[j] /= (z + eps);
    } else {
      // Eq. 6 as printed: W[i, j] / sum_k W[i, k].  Positions excluded from the mixing (-inf:
      // protected slots) carry no weight and do not enter the sum.
      double z = 0.0;
      for (int j = 0; j < T; ++j) { out[j] = std::isfinite(r[j]) ? r[j] : 0.0; z += out[j]; }
      if (std::fabs(z) < eps) z = z < 0.0 ? -eps : eps;
      for (int j = 0; j < T; ++j) out[j] /= z;
    }
  }
}

// Eq. 4a / 4b: out[i, :] = sum_j w[i, j] * Y[j, :], Y = [cache; block] of K or of V.
void mix(const double* w, const double* Y, int M, int T, int d, double* out) {
  for (int i = 0; i < M; ++i) {
    double* o = out + (size_t)i * d;
    for (int c = 0; c < d; ++c) o[c] = 0.0;
    for (int j = 0; j < T; ++j) {
      double wij = w[(size_t)i * T + j];
      const double* y = Y + (size_t)j * d;
      for (int c = 0; c < d; ++c) o[c] += wij * y[c];
    }
  }
}

// One pass of the Alg. 2 loop body for one (batch, kv-head) chain.
// q [g, Bn, d] (row stride q_ld between heads), kb/vb [Bn, d], cache ck/cv [M, d]
// with *len live rows, o [g, Bn, d].  logits_override (or null) is [M, T].
void segment_step_chain(const Cfg& cf, const double* q, int64_t q_head_stride,
                        const double* kb, const double* vb, int Bn, double* o,
                        int64_t o_head_stride, double* ck, double* cv, int* len,
                        const double* conv_w, const double* conv_b,
                        const double* logits_override, const uint8_t* protect, double* colsum,
                        int nthreads) {
  const int d = cf.head_dim, M = cf.M, m = *len;
  const double scale = cf.attn_scale > 0.0 ? cf.attn_scale : 1.0 / std::sqrt((double)d);
  for (int h = 0; h < cf.group; ++h) {
    double* oh = o + h * o_head_stride;
    attention_block(q + h * q_head_stride, kb, vb, ck, cv, m, Bn, d, scale, oh, colsum);
    for (size_t e = 0; e < (size_t)Bn * d; ++e) oh[e] = round_store(oh[e], cf.state_round);
  }
  if (m + Bn <= M) {                       // fill branch
    for (size_t e = 0; e < (size_t)Bn * d; ++e) {
      ck[(size_t)m * d + e] = round_store(kb[e], cf.state_round);
      cv[(size_t)m * d + e] = round_store(vb[e], cf.state_round);
    }
    *len = m + Bn;
    return;
  }
  const int T = m + Bn;
  const int C = cf.conv_in ? 2 * d : d;
  std::vector<double> YK((size_t)T * d), YV((size_t)T * d), X((size_t)T * C);
  std::memcpy(YK.data(), ck, sizeof(double) * (size_t)m * d);
  std::memcpy(YV.data(), cv, sizeof(double) * (size_t)m * d);
  std::memcpy(YK.data() + (size_t)m * d, kb, sizeof(double) * (size_t)Bn * d);
  std::memcpy(YV.data() + (size_t)m * d, vb, sizeof(double) * (size_t)Bn * d);
  for (int j = 0; j < T; ++j) {
    for (int c = 0; c < d; ++c) X[(size_t)j * C + c] = YK[(size_t)j * d + c];
    if (cf.conv_in)
      for (int c = 0; c < d; ++c) X[(size_t)j * C + d + c] = YV[(size_t)j * d + c];
  }
  std::vector<double> W((size_t)M * T), w((size_t)M * T);
  if (logits_override)
    std::memcpy(W.data(), logits_override, sizeof(double) * (size_t)M * T);
  else
    conv_logits(X.data(), T, C, conv_w, conv_b, M, cf.conv_width, W.data(), nthreads, cf.norm == 2);
  // Protected slots (combination with an eviction policy that keeps some tokens as they are:
  // attention sinks, heavy hitters): a live protected slot is no input of the mixing -- its
  // position carries no weight in any row -- and is not rewritten (below).
  if (protect)
    for (int j = 0; j < m; ++j)
      if (protect[j])
        for (int i = 0; i < M; ++i) W[(size_t)i * T + j] = -INFINITY;
  normalise_rows(W.data(), M, T, cf.norm, cf.norm_eps, w.data());
  std::vector<double> nk((size_t)M * d), nv((size_t)M * d);
  mix(w.data(), YK.data(), M, T, d, nk.data());
  mix(w.data(), YV.data(), M, T, d, nv.data());
  for (int i = 0; i < M; ++i) {
    if (protect && i < m && protect[i]) continue;        // kept as it is
    for (int c = 0; c < d; ++c) {
      ck[(size_t)i * d + c] = round_store(nk[(size_t)i * d + c], cf.state_round);
      cv[(size_t)i * d + c] = round_store(nv[(size_t)i * d + c], cf.state_round);
    }
  }
  *len = M;
}


// ---------------------------------------------------------------------------------------------
// Backward of one pass of the Alg. 2 loop body for one chain (training the convolution heads
// through the scan: the fine-tuning the paper runs on the heads).  Plain chain rule on the
// definitions above, storage rounding treated as the identity.
//   given   dO [g, Bn, d], dNewK, dNewV [M, d]   (gradients of a scalar loss)
//   returns dq [g, Bn, d], dkb, dvb [Bn, d], dck, dcv [M, d] (rows >= m zero unless the step fills),
//           and adds into dWc [M, C, k], db [M].
void segment_step_backward_chain(const Cfg& cf, const double* q, int64_t q_head_stride,
                                 const double* kb, const double* vb, int Bn, const double* ck,
                                 const double* cv, int m, const double* conv_w, const double* conv_b,
                                 const uint8_t* protect, const double* dO, int64_t do_head_stride,
                                 const double* dNewK, const double* dNewV, double* dq,
                                 int64_t dq_head_stride, double* dkb, double* dvb, double* dck,
                                 double* dcv, double* dWc, double* db) {
  const int d = cf.head_dim, M = cf.M, T = m + Bn;
  const double scale = cf.attn_scale > 0.0 ? cf.attn_scale : 1.0 / std::sqrt((double)d);
  std::vector<double> YK((size_t)T * d), YV((size_t)T * d), dYK((size_t)T * d, 0.0), dYV((size_t)T * d, 0.0);
  std::memcpy(YK.data(), ck, sizeof(double) * (size_t)m * d);
  std::memcpy(YV.data(), cv, sizeof(double) * (size_t)m * d);
  std::memcpy(YK.data() + (size_t)m * d, kb, sizeof(double) * (size_t)Bn * d);
  std::memcpy(YV.data() + (size_t)m * d, vb, sizeof(double) * (size_t)Bn * d);

  // ---- attention (Alg. 2 step 3): O[r] = sum_j P[r, j] Yv[j], P = softmax over the visible j
  std::vector<double> p(T), dp(T);
  for (int h = 0; h < cf.group; ++h)
    for (int r = 0; r < Bn; ++r) {
      const double* qr = q + h * q_head_stride + (size_t)r * d;
      const double* dor = dO + h * do_head_stride + (size_t)r * d;
      double* dqr = dq + h * dq_head_stride + (size_t)r * d;
      const int n_vis = m + r + 1;
      double mx = -std::numeric_limits<double>::infinity(), z = 0.0;
      for (int j = 0; j < n_vis; ++j) {
        double acc = 0.0;
        for (int c = 0; c < d; ++c) acc += qr[c] * YK[(size_t)j * d + c];
        p[j] = acc * scale;
        mx = std::max(mx, p[j]);
      }
      for (int j = 0; j < n_vis; ++j) { p[j] = std::exp(p[j] - mx); z += p[j]; }
      double dot = 0.0;                               // sum_j P_j dP_j
      for (int j = 0; j < n_vis; ++j) {
        p[j] /= z;
        double acc = 0.0;
        for (int c = 0; c < d; ++c) acc += dor[c] * YV[(size_t)j * d + c];
        dp[j] = acc;
        dot += p[j] * acc;
      }
      for (int c = 0; c < d; ++c) dqr[c] = 0.0;
      for (int j = 0; j < n_vis; ++j) {
        const double ds = p[j] * (dp[j] - dot) * scale;     // d loss / d (q . k_j)
        for (int c = 0; c < d; ++c) {
          dqr[c] += ds * YK[(size_t)j * d + c];
          dYK[(size_t)j * d + c] += ds * qr[c];
          dYV[(size_t)j * d + c] += p[j] * dor[c];
        }
      }
    }

  if (m + Bn <= M) {
    // ---- fill branch: the new cache is [cache ; block]
    for (int j = 0; j < T; ++j)
      for (int c = 0; c < d; ++c) {
        dYK[(size_t)j * d + c] += dNewK[(size_t)j * d + c];
        dYV[(size_t)j * d + c] += dNewV[(size_t)j * d + c];
      }
  } else {
    // ---- steps 4-5: W = conv(X) (Eq. 5), w = normalise(W) (Eq. 6), new = w Y (Eq. 4a / 4b)
    const int C = cf.conv_in ? 2 * d : d, k = cf.conv_width, pad = (k - 1) / 2;
    std::vector<double> X((size_t)T * C), W((size_t)M * T), w((size_t)M * T), dW((size_t)M * T);
    for (int j = 0; j < T; ++j) {
      for (int c = 0; c < d; ++c) X[(size_t)j * C + c] = YK[(size_t)j * d + c];
      if (cf.conv_in)
        for (int c = 0; c < d; ++c) X[(size_t)j * C + d + c] = YV[(size_t)j * d + c];
    }
    conv_logits(X.data(), T, C, conv_w, conv_b, M, k, W.data(), 1);
    if (protect)
      for (int j = 0; j < m; ++j)
        if (protect[j])
          for (int i = 0; i < M; ++i) W[(size_t)i * T + j] = -INFINITY;
    normalise_rows(W.data(), M, T, cf.norm, cf.norm_eps, w.data());
    for (int i = 0; i < M; ++i) {
      const double* gk = dNewK + (size_t)i * d;
      const double* gv = dNewV + (size_t)i * d;
      double* dWi = dW.data() + (size_t)i * T;
      if (protect && i < m && protect[i]) {           // the row was carried over
        for (int c = 0; c < d; ++c) {
          dYK[(size_t)i * d + c] += gk[c];
          dYV[(size_t)i * d + c] += gv[c];
        }
        for (int j = 0; j < T; ++j) dWi[j] = 0.0;
        continue;
      }
      const double* wi = w.data() + (size_t)i * T;
      double dot = 0.0, zsum = 0.0;
      std::vector<double> dwv(T);
      for (int j = 0; j < T; ++j) {
        double acc = 0.0;
        for (int c = 0; c < d; ++c)
          acc += gk[c] * YK[(size_t)j * d + c] + gv[c] * YV[(size_t)j * d + c];
        dwv[j] = acc;                                 // d loss / d w[i, j]
        dot += wi[j] * acc;
        for (int c = 0; c < d; ++c) {
          dYK[(size_t)j * d + c] += wi[j] * gk[c];
          dYV[(size_t)j * d + c] += wi[j] * gv[c];
        }
      }
      if (cf.norm == 0) {
        for (int j = 0; j < T; ++j) dWi[j] = wi[j] * (dwv[j] - dot);
      } else {
        // w = r / (z + eps), r = relu(W), z = sum r
        for (int j = 0; j < T; ++j) zsum += std::isfinite(W[(size_t)i * T + j]) && W[(size_t)i * T + j] > 0.0 ? W[(size_t)i * T + j] : 0.0;
        for (int j = 0; j < T; ++j)
          dWi[j] = W[(size_t)i * T + j] > 0.0 ? (dwv[j] - dot) / (zsum + cf.norm_eps) : 0.0;
      }
    }
    // Eq. 5 backwards: bias, filters, input
    for (int i = 0; i < M; ++i) {
      const double* dWi = dW.data() + (size_t)i * T;
      for (int j = 0; j < T; ++j) {
        const double g = dWi[j];
        if (g == 0.0) continue;
        if (db) db[i] += g;
        for (int t = 0; t < k; ++t) {
          const int jj = j + t - pad;
          if (jj < 0 || jj >= T) continue;
          for (int c = 0; c < C; ++c) {
            dWc[((size_t)i * C + c) * k + t] += g * X[(size_t)jj * C + c];
            const double gx = g * conv_w[((size_t)i * C + c) * k + t];
            if (c < d) dYK[(size_t)jj * d + c] += gx;
            else dYV[(size_t)jj * d + (c - d)] += gx;
          }
        }
      }
    }
  }
  for (size_t e = 0; e < (size_t)M * d; ++e) dck[e] = dcv[e] = 0.0;
  std::memcpy(dck, dYK.data(), sizeof(double) * (size_t)m * d);
  std::memcpy(dcv, dYV.data(), sizeof(double) * (size_t)m * d);
  std::memcpy(dkb, dYK.data() + (size_t)m * d, sizeof(double) * (size_t)Bn * d);
  std::memcpy(dvb, dYV.data() + (size_t)m * d, sizeof(double) * (size_t)Bn * d);
}

}  // namespace

extern "C" {

typedef Cfg lococo_oracle_cfg;

// Integer plan of the scan (Alg. 2 loop bounds and its IF), six int64 per
// segment: start, len, branch (0 fill / 1 compress), len_before, len_after,
// buf_after (ping-pong index, flips on every compress).  Returns the number
// of segments; writes at most cap of them.
int64_t lococo_oracle_plan(int64_t L, int32_t B, int32_t M, int32_t len0, int32_t cur0,
                           int64_t* out, int64_t cap) {
  int64_t n = 0;
  int32_t m = len0, cur = cur0;
  for (int64_t s = 0; s < L; s += B, ++n) {
    int32_t Bn = (int32_t)std::min<int64_t>(B, L - s);
    int32_t branch = (m + Bn <= M) ? 0 : 1;
    int32_t after = branch ? M : m + Bn;
    if (branch) cur ^= 1;
    if (n < cap) {
      int64_t* r = out + 6 * n;
      r[0] = s; r[1] = Bn; r[2] = branch; r[3] = m; r[4] = after; r[5] = cur;
    }
    m = after;
  }
  return n;
}

double lococo_oracle_round(double x, int32_t mode) { return round_store(x, mode); }

// The single operations, for the pins.  Each returns 0, or 1 on null pointers / sizes that make no sense.
int32_t lococo_oracle_attention_block(const double* q, const double* kb, const double* vb,
                                      const double* ck, const double* cv, int32_t m, int32_t Bn,
                                      int32_t d, double scale, double* o) {
  if (!q || !kb || !vb || !o || m < 0 || Bn <= 0 || d <= 0 || (m > 0 && (!ck || !cv))) return 1;
  attention_block(q, kb, vb, ck, cv, m, Bn, d, scale, o);
  return 0;
}

int32_t lococo_oracle_conv_logits(const double* X, int32_t T, int32_t C, const double* Wc,
                                  const double* bias, int32_t M, int32_t k, int32_t relu_input, double* W) {
  if (!X || !Wc || !W || T <= 0 || C <= 0 || M <= 0 || k < 1 || k % 2 == 0) return 1;
  conv_logits(X, T, C, Wc, bias, M, k, W, 1, relu_input != 0);
  return 0;
}

int32_t lococo_oracle_normalise(const double* W, int32_t M, int32_t T, int32_t norm, double eps,
                                double* w) {
  if (!W || !w || M <= 0 || T <= 0 || norm < 0 || norm > 2 || !(eps >= 0.0)) return 1;
  normalise_rows(W, M, T, norm, eps, w);
  return 0;
}

int32_t lococo_oracle_mix(const double* w, const double* Y, int32_t M, int32_t T, int32_t d,
                          double* out) {
  if (!w || !Y || !out || M <= 0 || T <= 0 || d <= 0) return 1;
  mix(w, Y, M, T, d, out);
  return 0;
}

// Whole scan (Alg. 2) over all chains.  Contiguous layouts:
//   q, o [batch, Hkv*group, L, d];  k, v [batch, Hkv, L, d];
//   cache_k, cache_v [batch, Hkv, M, d] in-out, *len in-out (shared by chains);
//   conv_w [M, C, k] (+ w_head_stride elements per kv head, 0 = shared bank);
//   conv_b [M] or null (+ b_head_stride per kv head);
//   logits_override null, or [n_compress_steps, batch, Hkv, M, M+B] (row
//   stride M+B even when T is smaller) replacing Eq. 5's output.
// Returns 0, or 1 on bad arguments.
//   protect null, or one byte per slot ([M], + protect_chain_stride bytes per chain, 0 = one
//   mask for all chains): non-zero = the slot, once live, is kept as it is by every
//   compression step and carries no weight in the mixing of the other slots.
//   attn_colsum null, or [batch, Hkv, M] accumulators: every attention (step 3) adds, for each
//   live cache slot, the probabilities the block's queries (all heads of the group) put on it.
int32_t lococo_oracle_sequence_forward_protected(
    const lococo_oracle_cfg* cfg, int32_t batch, int32_t Hkv, int64_t L, int32_t B, const double* q,
    const double* k, const double* v, double* o, double* cache_k, double* cache_v, int32_t* len,
    const double* conv_w, int64_t w_head_stride, const double* conv_b, int64_t b_head_stride,
    const double* logits_override, const uint8_t* protect, int64_t protect_chain_stride,
    double* attn_colsum, int32_t nthreads) {
  const Cfg cf = *cfg;
  const int d = cf.head_dim, M = cf.M, g = cf.group;
  if (!cfg || !len) return 1;
  if (d <= 0 || M <= 0 || g <= 0 || B <= 0 || L < 0 || batch <= 0 || Hkv <= 0 || cf.conv_width < 1 ||
      cf.conv_width % 2 == 0 || *len < 0 || *len > M || cf.norm < 0 || cf.norm > 2 ||
      cf.conv_in < 0 || cf.conv_in > 1 || cf.state_round < 0 || cf.state_round > 2 ||
      !(cf.norm_eps >= 0.0) || nthreads < 1 || w_head_stride < 0 || b_head_stride < 0 || protect_chain_stride < 0)
    return 1;
  if (L > 0 && (!q || !k || !v || !o || !cache_k || !cache_v)) return 1;
  {
    // a step that compresses needs filters (or given logits): decided by the same test the scan applies
    int m = *len;
    for (int64_t s = 0; s < L; s += B) {
      const int Bn = (int)std::min<int64_t>(B, L - s);
      if (m + Bn <= M) { m += Bn; continue; }
      if (!conv_w && !logits_override) return 1;
      m = M;
    }
  }
  const int64_t chains = (int64_t)batch * Hkv;
  const int len0 = *len;
  const int inner = chains >= nthreads ? 1 : nthreads;  // few chains: thread the conv rows instead
  parallel_for(chains, chains >= nthreads ? nthreads : 1, [&](int64_t ch) {
    const int64_t b = ch / Hkv, h = ch % Hkv;
    const double* qc = q + ((b * Hkv + h) * g) * L * d;
    double* oc = o + ((b * Hkv + h) * g) * L * d;
    const double* kc = k + ch * L * d;
    const double* vc = v + ch * L * d;
    double* ck = cache_k + ch * (int64_t)M * d;
    double* cv = cache_v + ch * (int64_t)M * d;
    const double* cw = conv_w ? conv_w + h * w_head_stride : nullptr;
    const double* cb = conv_b ? conv_b + h * b_head_stride : nullptr;
    int m = len0;
    int64_t step = 0;
    for (int64_t s = 0; s < L; s += B) {
      int Bn = (int)std::min<int64_t>(B, L - s);
      const double* ov = nullptr;
      bool compress = m + Bn > M;
      std::vector<double> packed;
      if (compress && logits_override) {
        // repack the [M, M+B]-strided rows to the dense [M, T] the step expects
        const int T = m + Bn;
        const double* src = logits_override + ((step * chains + ch) * M) * (int64_t)(M + B);
        packed.resize((size_t)M * T);
        for (int i = 0; i < M; ++i)
          std::memcpy(&packed[(size_t)i * T], src + (int64_t)i * (M + B), sizeof(double) * T);
        ov = packed.data();
      }
      segment_step_chain(cf, qc + s * d, L * d, kc + s * d, vc + s * d, Bn, oc + s * d, L * d,
                         ck, cv, &m, cw, cb, ov, protect ? protect + ch * protect_chain_stride : nullptr,
                         attn_colsum ? attn_colsum + ch * (int64_t)M : nullptr, inner);
      if (compress) ++step;
    }
  });
  int m = len0;                             // occupancy after the scan (same for every chain)
  for (int64_t s = 0; s < L; s += B) {
    int Bn = (int)std::min<int64_t>(B, L - s);
    m = (m + Bn <= M) ? m + Bn : M;
  }
  *len = m;
  return 0;
}

int32_t lococo_oracle_sequence_forward(const lococo_oracle_cfg* cfg, int32_t batch, int32_t Hkv,
                                       int64_t L, int32_t B, const double* q, const double* k,
                                       const double* v, double* o, double* cache_k,
                                       double* cache_v, int32_t* len, const double* conv_w,
                                       int64_t w_head_stride, const double* conv_b,
                                       int64_t b_head_stride, const double* logits_override,
                                       int32_t nthreads) {
  return lococo_oracle_sequence_forward_protected(cfg, batch, Hkv, L, B, q, k, v, o, cache_k, cache_v,
                                                  len, conv_w, w_head_stride, conv_b, b_head_stride,
                                                  logits_override, nullptr, 0, nullptr, nthreads);
}

// Backward of ONE block step over all chains (the caller walks the scan in reverse with the cache
// states it kept).  Layouts as in the forward; q, dO, dq [batch, Hkv*group, Bn, d]; kb, vb, dkb,
// dvb [batch, Hkv, Bn, d]; cache_k/v (state BEFORE the step), d_new_k/v, d_cache_k/v
// [batch, Hkv, M, d]; d_conv_w [M, C, k] (+ w_head_stride per kv head) and d_conv_b are ADDED to
// (d_conv_b may be null).  len = live slots before the step.  Returns 0, or 1 on bad arguments.
int32_t lococo_oracle_step_backward(const lococo_oracle_cfg* cfg, int32_t batch, int32_t Hkv, int32_t Bn,
                                    const double* q, const double* kb, const double* vb,
                                    const double* cache_k, const double* cache_v, int32_t len,
                                    const double* conv_w, int64_t w_head_stride, const double* conv_b,
                                    int64_t b_head_stride, const uint8_t* protect,
                                    int64_t protect_chain_stride, const double* dO, const double* d_new_k,
                                    const double* d_new_v, double* dq, double* dkb, double* dvb,
                                    double* d_cache_k, double* d_cache_v, double* d_conv_w,
                                    double* d_conv_b) {
  if (!cfg) return 1;
  const Cfg cf = *cfg;
  const int d = cf.head_dim, M = cf.M, g = cf.group;
  if (d <= 0 || M <= 0 || g <= 0 || Bn <= 0 || len < 0 || len > M || batch <= 0 || Hkv <= 0) return 1;
  if (cf.norm != 0 && cf.norm != 1) return 1;            // the input-side rectifier (norm = 2) is forward only
  if (!q || !kb || !vb || !cache_k || !cache_v || !dO || !d_new_k || !d_new_v || !dq || !dkb || !dvb ||
      !d_cache_k || !d_cache_v)
    return 1;
  if (len + Bn > M && (!conv_w || !d_conv_w || cf.conv_width < 1 || cf.conv_width % 2 == 0)) return 1;
  for (int64_t ch = 0; ch < (int64_t)batch * Hkv; ++ch) {     // serial: chains add into shared filter gradients
    const int64_t h = ch % Hkv;
    segment_step_backward_chain(
        cf, q + ch * g * Bn * d, (int64_t)Bn * d, kb + ch * Bn * d, vb + ch * Bn * d, Bn,
        cache_k + ch * (int64_t)M * d, cache_v + ch * (int64_t)M * d, len,
        conv_w ? conv_w + h * w_head_stride : nullptr, conv_b ? conv_b + h * b_head_stride : nullptr,
        protect ? protect + ch * protect_chain_stride : nullptr, dO + ch * g * Bn * d, (int64_t)Bn * d,
        d_new_k + ch * (int64_t)M * d, d_new_v + ch * (int64_t)M * d, dq + ch * g * Bn * d, (int64_t)Bn * d,
        dkb + ch * Bn * d, dvb + ch * Bn * d, d_cache_k + ch * (int64_t)M * d, d_cache_v + ch * (int64_t)M * d,
        d_conv_w ? d_conv_w + h * w_head_stride : nullptr, d_conv_b ? d_conv_b + h * b_head_stride : nullptr);
  }
  return 0;
}

}  // extern "C"
