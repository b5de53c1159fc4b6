// CPU oracle for the attentive knowledge-graph aggregation layer whose saved
// activations TinyKG compresses.  TEST INFRASTRUCTURE ONLY: nothing in the
// product path may include, link or call this file, and it shares no code with
// the GPU sources.
//
// What it follows:
//   * The layer has the three-stage shape of Sec. 3.2, Eq. (2): a sparse
//     neighbour aggregation H = spmm(A, E), a dense map J = mm(H, Theta), and
//     E' = sigma(J); the backward pass consumes the saved context of each stage
//     (grad_Theta = H^T grad_J, grad_H = grad_J Theta^T, grad_E = A^T grad_H).
//   * The aggregation weights are KGAT's attention (the paper names the model in
//     Sec. 4.1.2 but prints no formula; the formula is the benchmark's):
//       a_j = W_r e_t,  b_j = W_r e_h + e_r,  s_j = a_j . tanh(b_j)
//       pi_j = softmax of s_j over the out-edges j of head h
//       H_h = e_h + sum_j pi_j e_t,   J_h = W H_h,   E'_h = LeakyReLU(J_h).
//   * Sec. 3.3 / Fig. 1: the forward pass is exact; the backward pass is the
//     vector-Jacobian product of the layer evaluated at the *saved* tensors
//     (E_hat, H_hat, sign mask of J), whatever they hold.  ReLU-type stages keep
//     one bit per element (Sec. 4.1.4).
// Readings: the backward differentiates through the attention weights; nothing
// per-edge is saved (projections, scores and softmax are recomputed from
// E_hat); a head with no out-edge has H_h = e_h; repeated triplets and
// self-loops are separate edges.
//
// Everything is evaluated in double, edge by edge, in the order of the formulas
// above.  The float entry points convert inputs to double and round each output
// to float once.  `threads` > 1 only splits the loop over heads into contiguous
// ranges (backward: one private set of accumulators per range, summed in range
// order afterwards); it changes no formula.
//
// Parity pins for this file live in tests/test_oracle_agg.py.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <thread>
#include <vector>

namespace {

struct Graph {
  int64_t N = 0, T = 0;
  int R = 0;
  std::vector<int64_t> rowptr;   // N+1, out-edges of each head
  std::vector<int64_t> eid;      // T, original triplet index, grouped by head
};

bool build_graph(int64_t N, int R, int64_t T, const int32_t* head, const int32_t* rel,
                 const int32_t* tail, Graph& g) {
  if (N < 0 || R < 0 || T < 0) return false;
  for (int64_t e = 0; e < T; ++e) {
    if (head[e] < 0 || head[e] >= N || tail[e] < 0 || tail[e] >= N) return false;
    if (rel[e] < 0 || rel[e] >= R) return false;
  }
  g.N = N; g.T = T; g.R = R;
  g.rowptr.assign((size_t)N + 1, 0);
  for (int64_t e = 0; e < T; ++e) g.rowptr[(size_t)head[e] + 1]++;
  for (int64_t i = 0; i < N; ++i) g.rowptr[(size_t)i + 1] += g.rowptr[(size_t)i];
  g.eid.resize((size_t)T);
  std::vector<int64_t> fill(g.rowptr.begin(), g.rowptr.end() - 1);
  for (int64_t e = 0; e < T; ++e) g.eid[(size_t)fill[(size_t)head[e]]++] = e;
  return true;
}

struct Params {
  const double* Wr;   // [R, k, d]
  const double* er;   // [R, k]
  const double* W;    // [dout, d]
  int d, k, dout;
  double slope;
};

// Attention of one head h on embeddings E: fills a (deg x k), v (deg x k) and
// pi (deg) for its out-edges, in the head's edge order.
void head_attention(const Graph& g, const int32_t* rel, const int32_t* tail, const Params& P,
                    const double* E, int64_t h, std::vector<double>& a, std::vector<double>& v,
                    std::vector<double>& pi) {
  const int d = P.d, k = P.k;
  const int64_t lo = g.rowptr[(size_t)h], hi = g.rowptr[(size_t)h + 1];
  const int64_t deg = hi - lo;
  a.assign((size_t)(deg * k), 0.0);
  v.assign((size_t)(deg * k), 0.0);
  pi.assign((size_t)deg, 0.0);
  if (deg == 0) return;
  const double* eh = E + h * d;
  double smax = -INFINITY;
  for (int64_t q = 0; q < deg; ++q) {
    const int64_t e = g.eid[(size_t)(lo + q)];
    const double* Wr = P.Wr + (int64_t)rel[e] * k * d;
    const double* err = P.er + (int64_t)rel[e] * k;
    const double* et = E + (int64_t)tail[e] * d;
    double s = 0.0;
    for (int c = 0; c < k; ++c) {
      double ac = 0.0, bc = err[c];
      for (int i = 0; i < d; ++i) {
        ac += Wr[c * d + i] * et[i];
        bc += Wr[c * d + i] * eh[i];
      }
      const double vc = std::tanh(bc);
      a[(size_t)(q * k + c)] = ac;
      v[(size_t)(q * k + c)] = vc;
      s += ac * vc;
    }
    pi[(size_t)q] = s;
    smax = std::max(smax, s);
  }
  double z = 0.0;
  for (int64_t q = 0; q < deg; ++q) {
    pi[(size_t)q] = std::exp(pi[(size_t)q] - smax);
    z += pi[(size_t)q];
  }
  for (int64_t q = 0; q < deg; ++q) pi[(size_t)q] /= z;
}

void fwd_range(const Graph& g, const int32_t* rel, const int32_t* tail, const Params& P,
               const double* E, int64_t h0, int64_t h1, double* Eout, double* H, double* J,
               double* pi_out) {
  const int d = P.d, dout = P.dout;
  std::vector<double> a, v, pi, Hh((size_t)d);
  for (int64_t h = h0; h < h1; ++h) {
    head_attention(g, rel, tail, P, E, h, a, v, pi);
    const int64_t lo = g.rowptr[(size_t)h], deg = g.rowptr[(size_t)h + 1] - lo;
    for (int i = 0; i < d; ++i) Hh[(size_t)i] = E[h * d + i];
    for (int64_t q = 0; q < deg; ++q) {
      const int64_t e = g.eid[(size_t)(lo + q)];
      const double* et = E + (int64_t)tail[e] * d;
      for (int i = 0; i < d; ++i) Hh[(size_t)i] += pi[(size_t)q] * et[i];
      if (pi_out) pi_out[e] = pi[(size_t)q];
    }
    for (int i = 0; i < d; ++i) H[h * d + i] = Hh[(size_t)i];
    for (int o = 0; o < dout; ++o) {
      double j = 0.0;
      for (int i = 0; i < d; ++i) j += P.W[o * d + i] * Hh[(size_t)i];
      if (J) J[h * dout + o] = j;
      Eout[h * dout + o] = j > 0.0 ? j : P.slope * j;
    }
  }
}

struct Grads {
  std::vector<double> gE, gWr, ger;
};

void bwd_range(const Graph& g, const int32_t* rel, const int32_t* tail, const Params& P,
               const double* Ehat, const double* gH, int64_t h0, int64_t h1, Grads& G) {
  const int d = P.d, k = P.k;
  std::vector<double> a, v, pi, gq, ga((size_t)k), gb((size_t)k);
  for (int64_t h = h0; h < h1; ++h) {
    const int64_t lo = g.rowptr[(size_t)h], deg = g.rowptr[(size_t)h + 1] - lo;
    if (deg == 0) continue;
    head_attention(g, rel, tail, P, Ehat, h, a, v, pi);
    const double* gHh = gH + h * d;
    const double* eh = Ehat + h * d;
    // g_j = grad_H_h . e_t ;  c = sum_j pi_j g_j
    gq.assign((size_t)deg, 0.0);
    double c = 0.0;
    for (int64_t q = 0; q < deg; ++q) {
      const int64_t e = g.eid[(size_t)(lo + q)];
      const double* et = Ehat + (int64_t)tail[e] * d;
      double dot = 0.0;
      for (int i = 0; i < d; ++i) dot += gHh[i] * et[i];
      gq[(size_t)q] = dot;
      c += pi[(size_t)q] * dot;
    }
    for (int64_t q = 0; q < deg; ++q) {
      const int64_t e = g.eid[(size_t)(lo + q)];
      const int r = rel[e];
      const int64_t t = tail[e];
      const double* Wr = P.Wr + (int64_t)r * k * d;
      const double* et = Ehat + t * d;
      const double gs = pi[(size_t)q] * (gq[(size_t)q] - c);   // grad of the score s_j
      for (int cc = 0; cc < k; ++cc) {
        const double ac = a[(size_t)(q * k + cc)], vc = v[(size_t)(q * k + cc)];
        ga[(size_t)cc] = gs * vc;                       // grad a_j
        gb[(size_t)cc] = gs * ac * (1.0 - vc * vc);     // grad b_j (through tanh)
      }
      double* gEt = G.gE.data() + t * d;
      double* gEh = G.gE.data() + h * d;
      double* gWr = G.gWr.data() + (int64_t)r * k * d;
      double* ger = G.ger.data() + (int64_t)r * k;
      for (int i = 0; i < d; ++i) gEt[i] += pi[(size_t)q] * gHh[i];   // through n_h = sum pi e_t
      for (int cc = 0; cc < k; ++cc) {
        for (int i = 0; i < d; ++i) {
          gEt[i] += Wr[cc * d + i] * ga[(size_t)cc];     // a_j = W_r e_t
          gEh[i] += Wr[cc * d + i] * gb[(size_t)cc];     // b_j = W_r e_h + e_r
          gWr[cc * d + i] += ga[(size_t)cc] * et[i] + gb[(size_t)cc] * eh[i];
        }
        ger[cc] += gb[(size_t)cc];
      }
    }
  }
}

int core_fwd(int64_t N, int R, int64_t T, const int32_t* head, const int32_t* rel,
             const int32_t* tail, const Params& P, const double* E, int threads, double* Eout,
             double* H, double* J, double* pi_out) {
  Graph g;
  if (P.d <= 0 || P.k <= 0 || P.dout <= 0) return 1;
  if (!build_graph(N, R, T, head, rel, tail, g)) return 1;
  threads = (int)std::max<int64_t>(1, std::min<int64_t>(threads, N));
  if (threads == 1) {
    fwd_range(g, rel, tail, P, E, 0, N, Eout, H, J, pi_out);
  } else {
    std::vector<std::thread> pool;
    for (int w = 0; w < threads; ++w) {
      const int64_t h0 = N * w / threads, h1 = N * (w + 1) / threads;
      pool.emplace_back(fwd_range, std::cref(g), rel, tail, std::cref(P), E, h0, h1, Eout, H, J,
                        pi_out);
    }
    for (auto& t : pool) t.join();
  }
  return 0;
}

// mask[n*dout+o] != 0  <=>  J[n][o] > 0 in the forward pass.
int core_bwd(int64_t N, int R, int64_t T, const int32_t* head, const int32_t* rel,
             const int32_t* tail, const Params& P, const double* Ehat, const double* Hhat,
             const uint8_t* mask, const double* gEout, int threads, double* gE, double* gWr,
             double* ger, double* gW) {
  Graph g;
  if (P.d <= 0 || P.k <= 0 || P.dout <= 0) return 1;
  if (!build_graph(N, R, T, head, rel, tail, g)) return 1;
  const int d = P.d, k = P.k, dout = P.dout;
  // sigma stage: grad_J = grad_E' * (J > 0 ? 1 : slope)
  std::vector<double> gJ((size_t)(N * dout)), gH((size_t)(N * d), 0.0);
  for (int64_t i = 0; i < N * dout; ++i) gJ[(size_t)i] = gEout[i] * (mask[i] ? 1.0 : P.slope);
  // dense stage: grad_W = grad_J^T H_hat ; grad_H = grad_J W
  for (int64_t i = 0; i < (int64_t)dout * d; ++i) gW[i] = 0.0;
  for (int64_t n = 0; n < N; ++n) {
    for (int o = 0; o < dout; ++o) {
      const double gj = gJ[(size_t)(n * dout + o)];
      for (int i = 0; i < d; ++i) {
        gW[o * d + i] += gj * Hhat[n * d + i];
        gH[(size_t)(n * d + i)] += gj * P.W[o * d + i];
      }
    }
  }
  // aggregation stage: H_h = e_h + sum_j pi_j e_t  (grad_E starts as grad_H)
  threads = (int)std::max<int64_t>(1, std::min<int64_t>(threads, std::max<int64_t>(N, 1)));
  std::vector<Grads> parts((size_t)threads);
  for (auto& G : parts) {
    G.gE.assign((size_t)(N * d), 0.0);
    G.gWr.assign((size_t)((int64_t)R * k * d), 0.0);
    G.ger.assign((size_t)((int64_t)R * k), 0.0);
  }
  if (threads == 1) {
    bwd_range(g, rel, tail, P, Ehat, gH.data(), 0, N, parts[0]);
  } else {
    std::vector<std::thread> pool;
    for (int w = 0; w < threads; ++w) {
      const int64_t h0 = N * w / threads, h1 = N * (w + 1) / threads;
      pool.emplace_back(bwd_range, std::cref(g), rel, tail, std::cref(P), Ehat, gH.data(), h0, h1,
                        std::ref(parts[(size_t)w]));
    }
    for (auto& t : pool) t.join();
  }
  for (int64_t i = 0; i < N * d; ++i) {
    double s = gH[(size_t)i];
    for (auto& G : parts) s += G.gE[(size_t)i];
    gE[i] = s;
  }
  for (int64_t i = 0; i < (int64_t)R * k * d; ++i) {
    double s = 0.0;
    for (auto& G : parts) s += G.gWr[(size_t)i];
    gWr[i] = s;
  }
  for (int64_t i = 0; i < (int64_t)R * k; ++i) {
    double s = 0.0;
    for (auto& G : parts) s += G.ger[(size_t)i];
    ger[i] = s;
  }
  return 0;
}

std::vector<double> widen(const float* x, int64_t n) {
  std::vector<double> y((size_t)n);
  for (int64_t i = 0; i < n; ++i) y[(size_t)i] = (double)x[i];
  return y;
}

void narrow(const std::vector<double>& x, float* y) {
  for (size_t i = 0; i < x.size(); ++i) y[i] = (float)x[i];
}

}  // namespace

extern "C" {

// Double-precision forward.  Outputs: Eout [N,dout], H [N,d]; optional J
// [N,dout] and pi [T] (attention weight of each input triplet), may be null.
int tinykg_ref_kg_aggregate_fwd_f64(int64_t N, int R, int64_t T, const int32_t* head,
                                    const int32_t* rel, const int32_t* tail, const double* E,
                                    const double* Wr, const double* er, const double* W, int d,
                                    int k, int dout, double slope, int threads, double* Eout,
                                    double* H, double* J, double* pi) {
  Params P{Wr, er, W, d, k, dout, slope};
  return core_fwd(N, R, T, head, rel, tail, P, E, threads, Eout, H, J, pi);
}

int tinykg_ref_kg_aggregate_bwd_f64(int64_t N, int R, int64_t T, const int32_t* head,
                                    const int32_t* rel, const int32_t* tail, const double* Ehat,
                                    const double* Hhat, const uint8_t* mask, const double* Wr,
                                    const double* er, const double* W, int d, int k, int dout,
                                    double slope, const double* gEout, int threads, double* gE,
                                    double* gWr, double* ger, double* gW) {
  Params P{Wr, er, W, d, k, dout, slope};
  return core_bwd(N, R, T, head, rel, tail, P, Ehat, Hhat, mask, gEout, threads, gE, gWr, ger, gW);
}

// Float forward: inputs widened to double, outputs rounded to float once.
// mask_out [N*dout] receives 1 where J > 0 (decided in double), else 0.
int tinykg_ref_kg_aggregate_fwd(int64_t N, int R, int64_t T, const int32_t* head,
                                const int32_t* rel, const int32_t* tail, const float* E,
                                const float* Wr, const float* er, const float* W, int d, int k,
                                int dout, float slope, int threads, float* Eout, float* H,
                                uint8_t* mask_out) {
  if (N < 0 || d <= 0 || k <= 0 || dout <= 0) return 1;
  auto Ed = widen(E, N * d), Wrd = widen(Wr, (int64_t)R * k * d), erd = widen(er, (int64_t)R * k),
       Wd = widen(W, (int64_t)dout * d);
  std::vector<double> Eo((size_t)(N * dout)), Hd((size_t)(N * d)), Jd((size_t)(N * dout));
  Params P{Wrd.data(), erd.data(), Wd.data(), d, k, dout, (double)slope};
  int rc = core_fwd(N, R, T, head, rel, tail, P, Ed.data(), threads, Eo.data(), Hd.data(),
                    Jd.data(), nullptr);
  if (rc) return rc;
  narrow(Eo, Eout);
  narrow(Hd, H);
  if (mask_out)
    for (int64_t i = 0; i < N * dout; ++i) mask_out[i] = Jd[(size_t)i] > 0.0 ? 1 : 0;
  return 0;
}

int tinykg_ref_kg_aggregate_bwd(int64_t N, int R, int64_t T, const int32_t* head,
                                const int32_t* rel, const int32_t* tail, const float* Ehat,
                                const float* Hhat, const uint8_t* mask, const float* Wr,
                                const float* er, const float* W, int d, int k, int dout,
                                float slope, const float* gEout, int threads, float* gE,
                                float* gWr, float* ger, float* gW) {
  if (N < 0 || d <= 0 || k <= 0 || dout <= 0) return 1;
  auto Ed = widen(Ehat, N * d), Hd = widen(Hhat, N * d), Wrd = widen(Wr, (int64_t)R * k * d),
       erd = widen(er, (int64_t)R * k), Wd = widen(W, (int64_t)dout * d),
       gd = widen(gEout, N * dout);
  std::vector<double> gEd((size_t)(N * d)), gWrd((size_t)((int64_t)R * k * d)),
      gerd((size_t)((int64_t)R * k)), gWd((size_t)((int64_t)dout * d));
  Params P{Wrd.data(), erd.data(), Wd.data(), d, k, dout, (double)slope};
  int rc = core_bwd(N, R, T, head, rel, tail, P, Ed.data(), Hd.data(), mask, gd.data(), threads,
                    gEd.data(), gWrd.data(), gerd.data(), gWd.data());
  if (rc) return rc;
  narrow(gEd, gE);
  narrow(gWrd, gWr);
  narrow(gerd, ger);
  narrow(gWd, gW);
  return 0;
}

}  // extern "C"
