// CPU oracle for SLA (sparse-linear attention).  TEST INFRASTRUCTURE ONLY.
//
// A slow, plain, obviously-correct implementation of the forward pass (Algorithm 1)
// and the backward pass (Algorithm 2) of the paper, written from its equations.
// Nothing here is shared with the HIP library: no headers, no helpers, no tables.
// Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
//
// Conventions
//   * tensors are [BH, N, d] row-major (batch and heads flattened: they are independent),
//     blocks are runs of bq (queries) / bkv (keys) consecutive tokens, the last one may be
//     short (T = ceil(N / b));
//   * the block mask is [BH, Tm, Tn] int8 with 1 = critical, 0 = marginal, -1 = negligible
//     (Eq. 3);
//   * every floating-point routine exists in float and in double (suffix _f32 / _f64);
//     the mask routines exist in float only, in one fixed evaluation order, because the
//     mask is an integer result that the GPU has to reproduce bit for bit;
//   * loops are written so that each output element is accumulated in ascending index
//     order of the contraction; build with -ffp-contract=off.
//
// Readings of points the paper leaves open (each is pinned by a CPU test):
//   - ranking uses the pre-softmax pooled score; the row softmax of Eq. 2 is monotone, so
//     the top/bottom sets are the same;
//   - counts: n_h = floor(k_h*Tn + 1/2), n_l = min(floor(k_l*Tn + 1/2), Tn - n_h);
//   - top-k is taken per query-block row (Alg. 1, the TopK over P_c[i,:]);
//   - ties: critical = first n_h under (score descending, index ascending); negligible =
//     first n_l of the remaining entries under (score ascending, index ascending);
//   - bottom-k entries are labelled -1 (Eq. 3), the "=0" of Alg. 1's mask line is a typo;
//   - the backward pass multiplies dQ, dK by 1/sqrt(d) (S = QK^T/sqrt(d) in Alg. 2);
//   - dP_ij = dO^s_i V_j^T; the last line of Alg. 2 accumulates into dV_j and uses the
//     column sums of dH_i, dZ_i;
//   - Z_i sums over marginal blocks only (Eq. 5);
//   - phi = softmax over the d features of a token, or elu+1;
//   - Proj is one bias-free d x d matrix W shared by all heads, O = O^s + O^l W;
//   - a row with no critical block has O^s = 0, L = -inf; a row with no marginal block has
//     O^l = 0 and H_i = Z_i = 0;
//   - the mask is a constant in the backward pass; gradients do flow through phi.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <vector>

namespace {

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// ---------------------------------------------------------------- mask (float only)

// Eq. 2, pool(): mean over the valid tokens of each block.  Sequential float sum in
// ascending token order from +0, then one IEEE division by the token count.
void pool_f32(const float* X, int N, int d, int b, float* out) {
  const int T = ceil_div(N, b);
  for (int i = 0; i < T; ++i) {
    const int cnt = std::min(b, N - i * b);
    for (int c = 0; c < d; ++c) {
      float s = 0.0f;
      for (int r = 0; r < cnt; ++r) s = s + X[(size_t)(i * b + r) * d + c];
      out[(size_t)i * d + c] = s / (float)cnt;
    }
  }
}

// Eq. 2 before the softmax: s_ij = (pool(Q)_i . pool(K)_j) / sqrt(d), as a fused
// multiply-add chain over the feature index from +0, times the float constant 1/sqrt(d).
void scores_f32(const float* qbar, const float* kbar, int Tm, int Tn, int d, float* s) {
  const float scale = 1.0f / sqrtf((float)d);
  for (int i = 0; i < Tm; ++i)
    for (int j = 0; j < Tn; ++j) {
      float acc = 0.0f;
      for (int c = 0; c < d; ++c) acc = fmaf(qbar[(size_t)i * d + c], kbar[(size_t)j * d + c], acc);
      s[(size_t)i * Tn + j] = acc * scale;
    }
}

// Eq. 3 / Alg. 1 mask line, one row.
void classify_row(const float* s, int Tn, int n_h, int n_l, int8_t* m) {
  std::vector<int> idx(Tn);
  for (int j = 0; j < Tn; ++j) { idx[j] = j; m[j] = 0; }
  std::stable_sort(idx.begin(), idx.end(), [&](int a, int b) { return s[a] > s[b]; });
  for (int k = 0; k < n_h; ++k) m[idx[k]] = 1;
  std::vector<int> rest;
  for (int j = 0; j < Tn; ++j) if (m[j] == 0) rest.push_back(j);      // ascending index
  std::stable_sort(rest.begin(), rest.end(), [&](int a, int b) { return s[a] < s[b]; });
  for (int k = 0; k < n_l && k < (int)rest.size(); ++k) m[rest[k]] = -1;
}

// ---------------------------------------------------------------- feature map phi

template <typename R>
void phi_row(const R* x, int d, int phi, R* y) {
  if (phi == 0) {                       // softmax over the feature dimension
    R mx = x[0];
    for (int c = 1; c < d; ++c) mx = std::max(mx, x[c]);
    R sum = 0;
    for (int c = 0; c < d; ++c) { y[c] = std::exp(x[c] - mx); sum += y[c]; }
    for (int c = 0; c < d; ++c) y[c] = y[c] / sum;
  } else {                              // elu + 1
    for (int c = 0; c < d; ++c) y[c] = x[c] > 0 ? x[c] + 1 : std::exp(x[c]);
  }
}

// dx += J_phi(x)^T dy
template <typename R>
void phi_row_backward(const R* x, const R* y, const R* dy, int d, int phi, R* dx) {
  if (phi == 0) {
    R dot = 0;
    for (int c = 0; c < d; ++c) dot += dy[c] * y[c];
    for (int c = 0; c < d; ++c) dx[c] += y[c] * (dy[c] - dot);
  } else {
    for (int c = 0; c < d; ++c) dx[c] += dy[c] * (x[c] > 0 ? (R)1 : std::exp(x[c]));
  }
}

// ---------------------------------------------------------------- forward (Algorithm 1)

template <typename R>
void forward_head(int N, int d, int bq, int bkv, int phi,
                  const R* Q, const R* K, const R* V, const R* W, const int8_t* Mc,
                  R* O, R* Os, R* Ol, R* L, R* Hi, R* Zi) {
  const int Tm = ceil_div(N, bq), Tn = ceil_div(N, bkv);
  const R sqrt_d = std::sqrt((R)d);
  std::vector<R> Qphi((size_t)N * d), Kphi((size_t)N * d);
  for (int n = 0; n < N; ++n) {
    phi_row(Q + (size_t)n * d, d, phi, Qphi.data() + (size_t)n * d);
    phi_row(K + (size_t)n * d, d, phi, Kphi.data() + (size_t)n * d);
  }
  // Alg. 1, precompute line: h_j = phi(K_j)^T V_j  [d x d],  z_j = rowsum(phi(K_j)^T)  [d]
  std::vector<R> h((size_t)Tn * d * d, 0), z((size_t)Tn * d, 0);
  for (int j = 0; j < Tn; ++j) {
    const int n0 = j * bkv, cnt = std::min(bkv, N - n0);
    R* hj = h.data() + (size_t)j * d * d;
    R* zj = z.data() + (size_t)j * d;
    for (int r = 0; r < cnt; ++r) {
      const R* kp = Kphi.data() + (size_t)(n0 + r) * d;
      const R* v = V + (size_t)(n0 + r) * d;
      for (int c = 0; c < d; ++c) {
        const R kc = kp[c];
        zj[c] += kc;
        for (int e = 0; e < d; ++e) hj[(size_t)c * d + e] += kc * v[e];
      }
    }
  }
  std::vector<R> S((size_t)bq * bkv), P((size_t)bq * bkv), acc((size_t)bq * d);
  std::vector<R> m(bq), l(bq), H((size_t)d * d), Z(d);
  for (int i = 0; i < Tm; ++i) {
    const int q0 = i * bq, rows = std::min(bq, N - q0);
    std::fill(acc.begin(), acc.end(), (R)0);
    std::fill(H.begin(), H.end(), (R)0);
    std::fill(Z.begin(), Z.end(), (R)0);
    for (int r = 0; r < rows; ++r) { m[r] = -std::numeric_limits<R>::infinity(); l[r] = 0; }
    int n_crit = 0, n_marg = 0;
    for (int j = 0; j < Tn; ++j) {
      const int8_t mc = Mc[(size_t)i * Tn + j];
      const int k0 = j * bkv, cols = std::min(bkv, N - k0);
      if (mc == 1) {
        ++n_crit;
        // S_ij = Q_i K_j^T / sqrt(d)
        for (int r = 0; r < rows; ++r) {
          R* Sr = S.data() + (size_t)r * bkv;
          for (int cc = 0; cc < cols; ++cc) Sr[cc] = 0;
          for (int c = 0; c < d; ++c) {
            const R q = Q[(size_t)(q0 + r) * d + c];
            for (int cc = 0; cc < cols; ++cc) Sr[cc] += q * K[(size_t)(k0 + cc) * d + c];
          }
          for (int cc = 0; cc < cols; ++cc) Sr[cc] = Sr[cc] / sqrt_d;
        }
        // online softmax: m, P, l, O^s
        for (int r = 0; r < rows; ++r) {
          const R* Sr = S.data() + (size_t)r * bkv;
          R* Pr = P.data() + (size_t)r * bkv;
          R mnew = m[r];
          for (int cc = 0; cc < cols; ++cc) mnew = std::max(mnew, Sr[cc]);
          R rowsum = 0;
          for (int cc = 0; cc < cols; ++cc) { Pr[cc] = std::exp(Sr[cc] - mnew); rowsum += Pr[cc]; }
          const R alpha = std::exp(m[r] - mnew);     // exp(-inf) = 0 on the first block
          l[r] = alpha * l[r] + rowsum;
          R* a = acc.data() + (size_t)r * d;
          for (int e = 0; e < d; ++e) a[e] = alpha * a[e];
          for (int cc = 0; cc < cols; ++cc) {
            const R p = Pr[cc];
            const R* v = V + (size_t)(k0 + cc) * d;
            for (int e = 0; e < d; ++e) a[e] += p * v[e];
          }
          m[r] = mnew;
        }
      } else if (mc == 0) {
        ++n_marg;
        const R* hj = h.data() + (size_t)j * d * d;
        const R* zj = z.data() + (size_t)j * d;
        for (size_t t = 0; t < (size_t)d * d; ++t) H[t] += hj[t];
        for (int c = 0; c < d; ++c) Z[c] += zj[c];
      }
    }
    // closing line of Alg. 1: O^s_i = diag(l)^-1 O^s, L_i = m + log l, O^l_i = Q^phi H / (Q^phi Z)
    for (int r = 0; r < rows; ++r) {
      const size_t n = (size_t)(q0 + r);
      if (n_crit > 0) {
        for (int e = 0; e < d; ++e) Os[n * d + e] = acc[(size_t)r * d + e] / l[r];
        L[n] = m[r] + std::log(l[r]);
      } else {
        for (int e = 0; e < d; ++e) Os[n * d + e] = 0;
        L[n] = -std::numeric_limits<R>::infinity();
      }
      if (n_marg > 0) {
        const R* qp = Qphi.data() + n * d;
        R den = 0;
        for (int c = 0; c < d; ++c) den += qp[c] * Z[c];
        for (int e = 0; e < d; ++e) Ol[n * d + e] = 0;
        for (int c = 0; c < d; ++c)
          for (int e = 0; e < d; ++e) Ol[n * d + e] += qp[c] * H[(size_t)c * d + e];
        for (int e = 0; e < d; ++e) Ol[n * d + e] = Ol[n * d + e] / den;
      } else {
        for (int e = 0; e < d; ++e) Ol[n * d + e] = 0;
      }
      // Eq. 6: O = O^s + Proj(O^l),  Proj(x) = x W
      for (int e = 0; e < d; ++e) O[n * d + e] = Os[n * d + e];
      for (int c = 0; c < d; ++c) {
        const R o = Ol[n * d + c];
        for (int e = 0; e < d; ++e) O[n * d + e] += o * W[(size_t)c * d + e];
      }
    }
    if (Hi) std::memcpy(Hi + (size_t)i * d * d, H.data(), sizeof(R) * d * d);
    if (Zi) std::memcpy(Zi + (size_t)i * d, Z.data(), sizeof(R) * d);
  }
}

// ---------------------------------------------------------------- backward (Algorithm 2)

template <typename R>
void backward_head(int N, int d, int bq, int bkv, int phi,
                   const R* Q, const R* K, const R* V, const R* W, const int8_t* Mc,
                   const R* L, const R* Hi, const R* Zi, const R* Os, const R* Ol, const R* dO,
                   R* dQ, R* dK, R* dV, R* dW /* += */, R* dQphi_out, R* dKphi_out) {
  const int Tm = ceil_div(N, bq), Tn = ceil_div(N, bkv);
  const R sqrt_d = std::sqrt((R)d);
  const size_t nd = (size_t)N * d;
  std::vector<R> Qphi(nd), Kphi(nd), dOl(nd, 0), dQphi(nd, 0), dKphi(nd, 0), Ds(N), Dl(N);
  for (int n = 0; n < N; ++n) {
    phi_row(Q + (size_t)n * d, d, phi, Qphi.data() + (size_t)n * d);
    phi_row(K + (size_t)n * d, d, phi, Kphi.data() + (size_t)n * d);
  }
  std::fill(dQ, dQ + nd, (R)0);
  std::fill(dK, dK + nd, (R)0);
  std::fill(dV, dV + nd, (R)0);
  // chain rule of Eq. 6: dO^s = dO, dO^l = dO W^T, dW += (O^l)^T dO; then the D line of Alg. 2
  for (int n = 0; n < N; ++n) {
    const R* g = dO + (size_t)n * d;
    for (int c = 0; c < d; ++c) {
      R s = 0;
      for (int e = 0; e < d; ++e) s += g[e] * W[(size_t)c * d + e];
      dOl[(size_t)n * d + c] = s;
      const R o = Ol[(size_t)n * d + c];
      for (int e = 0; e < d; ++e) dW[(size_t)c * d + e] += o * g[e];
    }
    R a = 0, b = 0;
    for (int e = 0; e < d; ++e) {
      a += g[e] * Os[(size_t)n * d + e];
      b += dOl[(size_t)n * d + e] * Ol[(size_t)n * d + e];
    }
    Ds[n] = a;
    Dl[n] = b;
  }
  // first loop of Alg. 2: dH_i, dZ_i, dQ^phi_i
  std::vector<R> dHi((size_t)Tm * d * d, 0), dZi((size_t)Tm * d, 0);
  for (int i = 0; i < Tm; ++i) {
    int n_marg = 0;
    for (int j = 0; j < Tn; ++j) n_marg += (Mc[(size_t)i * Tn + j] == 0);
    if (n_marg == 0) continue;            // O^l_i is identically 0: no gradient
    const int q0 = i * bq, rows = std::min(bq, N - q0);
    const R* H = Hi + (size_t)i * d * d;
    const R* Z = Zi + (size_t)i * d;
    R* dH = dHi.data() + (size_t)i * d * d;
    R* dZ = dZi.data() + (size_t)i * d;
    for (int r = 0; r < rows; ++r) {
      const size_t n = (size_t)(q0 + r);
      const R* qp = Qphi.data() + n * d;
      const R* g = dOl.data() + n * d;
      R den = 0;
      for (int c = 0; c < d; ++c) den += qp[c] * Z[c];
      for (int c = 0; c < d; ++c) {
        const R a = qp[c] / den;
        for (int e = 0; e < d; ++e) dH[(size_t)c * d + e] += a * g[e];
        dZ[c] += -(a * Dl[n]);
        R t = 0;
        for (int e = 0; e < d; ++e) t += g[e] * H[(size_t)c * d + e];
        dQphi[n * d + c] = (t - Dl[n] * Z[c]) / den;
      }
    }
  }
  // second loop of Alg. 2
  std::vector<R> S((size_t)bq * bkv), P((size_t)bq * bkv), dS((size_t)bq * bkv);
  std::vector<R> dH((size_t)d * d), dZ(d);
  for (int j = 0; j < Tn; ++j) {
    const int k0 = j * bkv, cols = std::min(bkv, N - k0);
    std::fill(dH.begin(), dH.end(), (R)0);
    std::fill(dZ.begin(), dZ.end(), (R)0);
    for (int i = 0; i < Tm; ++i) {
      const int8_t mc = Mc[(size_t)i * Tn + j];
      const int q0 = i * bq, rows = std::min(bq, N - q0);
      if (mc == 1) {
        for (int r = 0; r < rows; ++r) {
          const size_t n = (size_t)(q0 + r);
          R* Sr = S.data() + (size_t)r * bkv;
          R* Pr = P.data() + (size_t)r * bkv;
          R* dSr = dS.data() + (size_t)r * bkv;
          for (int cc = 0; cc < cols; ++cc) { Sr[cc] = 0; dSr[cc] = 0; }
          for (int c = 0; c < d; ++c) {
            const R q = Q[n * d + c], g = dO[n * d + c];
            for (int cc = 0; cc < cols; ++cc) {
              Sr[cc] += q * K[(size_t)(k0 + cc) * d + c];          // Q_i K_j^T
              dSr[cc] += g * V[(size_t)(k0 + cc) * d + c];         // dP = dO^s_i V_j^T
            }
          }
          for (int cc = 0; cc < cols; ++cc) {
            Pr[cc] = std::exp(Sr[cc] / sqrt_d - L[n]);             // P = exp(S - L)
            dSr[cc] = Pr[cc] * (dSr[cc] - Ds[n]);                  // dS = P (dP - D^s)
          }
          for (int cc = 0; cc < cols; ++cc) {
            const size_t kn = (size_t)(k0 + cc);
            const R p = Pr[cc], ds = dSr[cc] / sqrt_d;
            for (int e = 0; e < d; ++e) {
              dV[kn * d + e] += p * dO[n * d + e];                 // dV_j += P^T dO^s_i
              dQ[n * d + e] += ds * K[kn * d + e];                 // dQ_i += dS K_j / sqrt(d)
              dK[kn * d + e] += ds * Q[n * d + e];                 // dK_j += dS^T Q_i / sqrt(d)
            }
          }
        }
      } else if (mc == 0) {
        const R* a = dHi.data() + (size_t)i * d * d;
        const R* b = dZi.data() + (size_t)i * d;
        for (size_t t = 0; t < (size_t)d * d; ++t) dH[t] += a[t];
        for (int c = 0; c < d; ++c) dZ[c] += b[c];
      }
    }
    // dK^phi_j = V_j dH^T + 1 dZ^T,  dV_j += K^phi_j dH
    for (int r = 0; r < cols; ++r) {
      const size_t n = (size_t)(k0 + r);
      for (int c = 0; c < d; ++c) {
        R t = 0;
        for (int e = 0; e < d; ++e) t += V[n * d + e] * dH[(size_t)c * d + e];
        dKphi[n * d + c] = t + dZ[c];
        const R kc = Kphi[n * d + c];
        for (int e = 0; e < d; ++e) dV[n * d + e] += kc * dH[(size_t)c * d + e];
      }
    }
  }
  // through phi (the paper returns dQ^phi, dK^phi; the chain rule is the standard Jacobian)
  for (int n = 0; n < N; ++n) {
    phi_row_backward(Q + (size_t)n * d, Qphi.data() + (size_t)n * d, dQphi.data() + (size_t)n * d,
                     d, phi, dQ + (size_t)n * d);
    phi_row_backward(K + (size_t)n * d, Kphi.data() + (size_t)n * d, dKphi.data() + (size_t)n * d,
                     d, phi, dK + (size_t)n * d);
  }
  if (dQphi_out) std::memcpy(dQphi_out, dQphi.data(), sizeof(R) * nd);
  if (dKphi_out) std::memcpy(dKphi_out, dKphi.data(), sizeof(R) * nd);
}

template <typename R>
int forward_all(int BH, int N, int d, int bq, int bkv, int phi, const R* Q, const R* K, const R* V,
                const R* W, const int8_t* Mc, R* O, R* Os, R* Ol, R* L, R* Hi, R* Zi) {
  if (BH <= 0 || N <= 0 || d <= 0 || bq <= 0 || bkv <= 0 || (phi != 0 && phi != 1)) return -1;
  const int Tm = ceil_div(N, bq), Tn = ceil_div(N, bkv);
  const size_t nd = (size_t)N * d;
#pragma omp parallel for schedule(dynamic)
  for (int g = 0; g < BH; ++g)
    forward_head<R>(N, d, bq, bkv, phi, Q + g * nd, K + g * nd, V + g * nd, W,
                    Mc + (size_t)g * Tm * Tn, O + g * nd, Os + g * nd, Ol + g * nd,
                    L + (size_t)g * N, Hi ? Hi + (size_t)g * Tm * d * d : nullptr,
                    Zi ? Zi + (size_t)g * Tm * d : nullptr);
  return 0;
}

template <typename R>
int backward_all(int BH, int N, int d, int bq, int bkv, int phi, const R* Q, const R* K,
                 const R* V, const R* W, const int8_t* Mc, const R* L, const R* Hi, const R* Zi,
                 const R* Os, const R* Ol, const R* dO, R* dQ, R* dK, R* dV, R* dW, R* dQphi,
                 R* dKphi) {
  if (BH <= 0 || N <= 0 || d <= 0 || bq <= 0 || bkv <= 0 || (phi != 0 && phi != 1)) return -1;
  const int Tm = ceil_div(N, bq), Tn = ceil_div(N, bkv);
  const size_t nd = (size_t)N * d;
  std::vector<R> dW_part((size_t)BH * d * d, 0);
#pragma omp parallel for schedule(dynamic)
  for (int g = 0; g < BH; ++g)
    backward_head<R>(N, d, bq, bkv, phi, Q + g * nd, K + g * nd, V + g * nd, W,
                     Mc + (size_t)g * Tm * Tn, L + (size_t)g * N, Hi + (size_t)g * Tm * d * d,
                     Zi + (size_t)g * Tm * d, Os + g * nd, Ol + g * nd, dO + g * nd, dQ + g * nd,
                     dK + g * nd, dV + g * nd, dW_part.data() + (size_t)g * d * d,
                     dQphi ? dQphi + g * nd : nullptr, dKphi ? dKphi + g * nd : nullptr);
  // Proj is shared: dW sums over batch and heads, in ascending order
  for (size_t t = 0; t < (size_t)d * d; ++t) {
    R s = 0;
    for (int g = 0; g < BH; ++g) s += dW_part[(size_t)g * d * d + t];
    dW[t] = s;
  }
  return 0;
}

}  // namespace

extern "C" {

// Block counts for fractions k_h, k_l of Tn key blocks.
void sla_oracle_counts(int Tn, double k_h, double k_l, int* n_h, int* n_l) {
  long a = (long)std::floor(k_h * (double)Tn + 0.5);
  a = std::max(0L, std::min((long)Tn, a));
  long b = (long)std::floor(k_l * (double)Tn + 0.5);
  b = std::max(0L, std::min((long)Tn - a, b));
  *n_h = (int)a;
  *n_l = (int)b;
}

// pool(X) for one head: X [N,d] -> out [ceil(N/b), d].
void sla_oracle_pool(const float* X, int N, int d, int b, float* out) { pool_f32(X, N, d, b, out); }

// Pre-softmax block scores for one head.
void sla_oracle_scores(const float* qbar, const float* kbar, int Tm, int Tn, int d, float* s) {
  scores_f32(qbar, kbar, Tm, Tn, d, s);
}

// Three-way classification of a score matrix [rows, Tn].
void sla_oracle_classify(const float* s, int rows, int Tn, int n_h, int n_l, int8_t* Mc) {
#pragma omp parallel for schedule(static)
  for (int i = 0; i < rows; ++i) classify_row(s + (size_t)i * Tn, Tn, n_h, n_l, Mc + (size_t)i * Tn);
}

// Whole mask step: Q,K [BH,N,d] float -> Mc [BH,Tm,Tn]; s_out [BH,Tm,Tn] optional.
int sla_oracle_build_mask(int BH, int N, int d, int bq, int bkv, double k_h, double k_l,
                          const float* Q, const float* K, int8_t* Mc, float* s_out) {
  if (BH <= 0 || N <= 0 || d <= 0 || bq <= 0 || bkv <= 0) return -1;
  const int Tm = ceil_div(N, bq), Tn = ceil_div(N, bkv);
  int n_h, n_l;
  sla_oracle_counts(Tn, k_h, k_l, &n_h, &n_l);
#pragma omp parallel for schedule(dynamic)
  for (int g = 0; g < BH; ++g) {
    std::vector<float> qb((size_t)Tm * d), kb((size_t)Tn * d), s((size_t)Tm * Tn);
    pool_f32(Q + (size_t)g * N * d, N, d, bq, qb.data());
    pool_f32(K + (size_t)g * N * d, N, d, bkv, kb.data());
    scores_f32(qb.data(), kb.data(), Tm, Tn, d, s.data());
    for (int i = 0; i < Tm; ++i)
      classify_row(s.data() + (size_t)i * Tn, Tn, n_h, n_l, Mc + ((size_t)g * Tm + i) * Tn);
    if (s_out) std::memcpy(s_out + (size_t)g * Tm * Tn, s.data(), sizeof(float) * Tm * Tn);
  }
  return 0;
}

// Row softmax of the block scores (P_c of Eq. 2); only a debugging aid, never ranked.
void sla_oracle_pc(const float* s, int rows, int Tn, float* Pc) {
  for (int i = 0; i < rows; ++i) {
    const float* r = s + (size_t)i * Tn;
    float mx = r[0];
    for (int j = 1; j < Tn; ++j) mx = std::max(mx, r[j]);
    double sum = 0;
    for (int j = 0; j < Tn; ++j) sum += std::exp((double)r[j] - mx);
    for (int j = 0; j < Tn; ++j) Pc[(size_t)i * Tn + j] = (float)(std::exp((double)r[j] - mx) / sum);
  }
}

// Alg. 1 accumulation line on its own: out[i][:] = sum, in ascending j, of the rows h[j][:] with
// Mc[i][j] == 0 (marginal), for given rows h [BH, Tn, len] (double) and masks Mc [BH, Tm, Tn].
void sla_oracle_accumulate(int BH, int Tm, int Tn, int len, const double* h, const int8_t* Mc, double* out) {
  for (int g = 0; g < BH; ++g)
    for (int i = 0; i < Tm; ++i) {
      double* o = out + ((size_t)g * Tm + i) * len;
      for (int c = 0; c < len; ++c) o[c] = 0.0;
      for (int j = 0; j < Tn; ++j) {
        if (Mc[((size_t)g * Tm + i) * Tn + j] != 0) continue;
        const double* r = h + ((size_t)g * Tn + j) * len;
        for (int c = 0; c < len; ++c) o[c] += r[c];
      }
    }
}

#define SLA_ORACLE_API(SUF, R)                                                                     \
  int sla_oracle_forward_##SUF(int BH, int N, int d, int bq, int bkv, int phi, const R* Q,          \
                               const R* K, const R* V, const R* W, const int8_t* Mc, R* O, R* Os,  \
                               R* Ol, R* L, R* Hi, R* Zi) {                                        \
    return forward_all<R>(BH, N, d, bq, bkv, phi, Q, K, V, W, Mc, O, Os, Ol, L, Hi, Zi);           \
  }                                                                                                \
  int sla_oracle_backward_##SUF(int BH, int N, int d, int bq, int bkv, int phi, const R* Q,         \
                                const R* K, const R* V, const R* W, const int8_t* Mc, const R* L,  \
                                const R* Hi, const R* Zi, const R* Os, const R* Ol, const R* dO,   \
                                R* dQ, R* dK, R* dV, R* dW, R* dQphi, R* dKphi) {                  \
    return backward_all<R>(BH, N, d, bq, bkv, phi, Q, K, V, W, Mc, L, Hi, Zi, Os, Ol, dO, dQ, dK,  \
                           dV, dW, dQphi, dKphi);                                                  \
  }

SLA_ORACLE_API(f32, float)
SLA_ORACLE_API(f64, double)

}  // extern "C"
