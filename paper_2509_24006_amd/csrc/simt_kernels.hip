// Float-arithmetic SLA path for gfx950: every contraction of Algorithm 1 and Algorithm 2 is
// carried out with fp32 fused multiply-adds on LDS-staged 64-row tiles.  This is the path
// for float tensors (1e-5 agreement with the definition needs float products, which the
// bf16 matrix cores cannot give).
//
// Thread layout of every kernel: 256 threads, ty = tid / 16, tx = tid % 16.  A thread owns
// rows ty + 16a and columns tx + 16b of whatever 64-row tile product is being formed, so
// that LDS reads are broadcasts (same ty) or unit-stride (consecutive tx).
#include "sla_internal.h"

namespace sla {
namespace {

constexpr int kThreads = 256;

// ------------------------------------------------------------------ tile helpers
template <typename T>
__device__ __forceinline__ void load_tile(float* dst, int ld, const T* src, int rows_valid, int d, int src_ld) {
  for (int idx = threadIdx.x; idx < kBlk * d; idx += kThreads) {
    const int r = idx / d, c = idx - r * d;
    dst[r * ld + c] = (r < rows_valid) ? to_f32(src[(size_t)r * src_ld + c]) : 0.0f;
  }
}

// reduce over the 16 threads that share ty (16 consecutive lanes)
__device__ __forceinline__ float tx_sum(float v) {
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float tx_max(float v) {
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// acc[a][b] += sum_k A[(ty+16a)*lda + k] * B[(tx+16b)*ldb + k]
template <int NC>
__device__ __forceinline__ void mm_abt(const float* A, int lda, const float* B, int ldb, int kdim,
                                       float (&acc)[4][NC]) {
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  for (int k = 0; k < kdim; ++k) {
    float av[4], bv[NC];
#pragma unroll
    for (int a = 0; a < 4; ++a) av[a] = A[(ty + 16 * a) * lda + k];
#pragma unroll
    for (int b = 0; b < NC; ++b) bv[b] = B[(tx + 16 * b) * ldb + k];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < NC; ++b) acc[a][b] = fmaf(av[a], bv[b], acc[a][b]);
  }
}

// acc[a][b] += sum_k A[(ty+16a)*lda + k] * B[k*ldb + tx+16b]
template <int NC>
__device__ __forceinline__ void mm_ab(const float* A, int lda, const float* B, int ldb, int kdim,
                                      float (&acc)[4][NC]) {
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  for (int k = 0; k < kdim; ++k) {
    float av[4], bv[NC];
#pragma unroll
    for (int a = 0; a < 4; ++a) av[a] = A[(ty + 16 * a) * lda + k];
#pragma unroll
    for (int b = 0; b < NC; ++b) bv[b] = B[k * ldb + tx + 16 * b];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < NC; ++b) acc[a][b] = fmaf(av[a], bv[b], acc[a][b]);
  }
}

// acc[a][b] += sum_k A[k*lda + ty+16a] * B[k*ldb + tx+16b]
template <int NR, int NC>
__device__ __forceinline__ void mm_atb(const float* A, int lda, const float* B, int ldb, int kdim,
                                       float (&acc)[NR][NC]) {
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  for (int k = 0; k < kdim; ++k) {
    float av[NR], bv[NC];
#pragma unroll
    for (int a = 0; a < NR; ++a) av[a] = A[k * lda + ty + 16 * a];
#pragma unroll
    for (int b = 0; b < NC; ++b) bv[b] = B[k * ldb + tx + 16 * b];
#pragma unroll
    for (int a = 0; a < NR; ++a)
#pragma unroll
      for (int b = 0; b < NC; ++b) acc[a][b] = fmaf(av[a], bv[b], acc[a][b]);
  }
}

template <int NR, int NC>
__device__ __forceinline__ void zero(float (&acc)[NR][NC]) {
#pragma unroll
  for (int a = 0; a < NR; ++a)
#pragma unroll
    for (int b = 0; b < NC; ++b) acc[a][b] = 0.0f;
}

// In-place feature map on a 64 x D tile in LDS (rows >= rows_valid become 0).
// phi = 0: softmax over the D features of each token; phi = 1: elu + 1.
template <int D>
__device__ __forceinline__ void phi_tile(const float* X, float* Y, int ld, int rows_valid, int phi) {
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  constexpr int NC = D / 16;
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int r = ty + 16 * a;
    float v[NC];
#pragma unroll
    for (int b = 0; b < NC; ++b) v[b] = X[r * ld + tx + 16 * b];
    if (phi == 0) {
      float mx = v[0];
#pragma unroll
      for (int b = 1; b < NC; ++b) mx = fmaxf(mx, v[b]);
      mx = tx_max(mx);
      float sum = 0.0f;
#pragma unroll
      for (int b = 0; b < NC; ++b) {
        v[b] = expf(v[b] - mx);
        sum += v[b];
      }
      sum = tx_sum(sum);
#pragma unroll
      for (int b = 0; b < NC; ++b) v[b] = v[b] / sum;
    } else {
#pragma unroll
      for (int b = 0; b < NC; ++b) v[b] = v[b] > 0.0f ? v[b] + 1.0f : expf(v[b]);
    }
#pragma unroll
    for (int b = 0; b < NC; ++b) Y[r * ld + tx + 16 * b] = (r < rows_valid) ? v[b] : 0.0f;
  }
}

// g[a][b] (gradient w.r.t. phi(x) at rows ty+16a, features tx+16b) -> gradient w.r.t. x.
template <int D>
__device__ __forceinline__ void phi_backward(const float* X, const float* Y, int ld, int phi,
                                             float (&g)[4][D / 16]) {
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  constexpr int NC = D / 16;
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int r = ty + 16 * a;
    if (phi == 0) {
      float dot = 0.0f;
#pragma unroll
      for (int b = 0; b < NC; ++b) dot = fmaf(g[a][b], Y[r * ld + tx + 16 * b], dot);
      dot = tx_sum(dot);
#pragma unroll
      for (int b = 0; b < NC; ++b) g[a][b] = Y[r * ld + tx + 16 * b] * (g[a][b] - dot);
    } else {
#pragma unroll
      for (int b = 0; b < NC; ++b) {
        const float x = X[r * ld + tx + 16 * b];
        g[a][b] = g[a][b] * (x > 0.0f ? 1.0f : expf(x));
      }
    }
  }
}

// ------------------------------------------------------------------ key-block states
// Alg. 1 precompute line: h_j = phi(K_j)^T V_j, z_j = rowsum(phi(K_j)^T), one workgroup per key
// block; stored as a state row (h transposed, then z).
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void states_kernel(const T* __restrict__ K,
                                                          const T* __restrict__ V, int N, int Tn, Lay lay,
                                                          int phi, float* __restrict__ hz) {
  extern __shared__ float lds[];
  constexpr int LD = D + 1;
  float* Ks = lds;
  float* Vs = lds + kBlk * LD;
  const int j = blockIdx.x, bh = blockIdx.y;
  const int n0 = j * kBlk, cnt = min(kBlk, N - n0);
  const size_t ubase = lay.head(bh) + (size_t)n0 * lay.ts;   // in the caller's tensors
  load_tile(Ks, LD, K + ubase, cnt, D, lay.ts);
  load_tile(Vs, LD, V + ubase, cnt, D, lay.ts);
  __syncthreads();
  phi_tile<D>(Ks, Ks, LD, cnt, phi);
  __syncthreads();
  // hT[e][c] = sum_n V[n][e] Kphi[n][c]
  constexpr int NB = D / 16;
  float* out = hz + ((size_t)bh * Tn + j) * (D * D + D);
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  for (int e0 = 0; e0 < D; e0 += 64) {
    float acc[4][NB];
    zero(acc);
    mm_atb<4, NB>(Vs + e0, LD, Ks, LD, kBlk, acc);
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < NB; ++b) out[(size_t)(e0 + ty + 16 * a) * D + tx + 16 * b] = acc[a][b];
  }
  if (threadIdx.x < D) {
    float z = 0.0f;
    for (int n = 0; n < kBlk; ++n) z += Ks[n * LD + threadIdx.x];
    out[(size_t)D * D + threadIdx.x] = z;
  }
}

// Alg. 1 accumulation line (and its column-wise twin in Alg. 2): out_row[i] = sum of the
// state rows in[k] over the k with a marginal label, in ascending k.
// With m(q, j) = Mc[q / rq][j] the label of query tile q (64 tokens) and key block j:
//   by_column = 0: label(i, k) = m(i, k)  (H_i, Z_i of query tile i over key blocks)
//   by_column = 1: label(i, k) = m(k, i)  (dH, dZ of key block i over query tiles)
__global__ __launch_bounds__(kThreads) void aggregate_kernel(const float* __restrict__ in,
                                                             const int8_t* __restrict__ Mc, int Tq, int rq, int T,
                                                             int row_len, int by_column,
                                                             float* __restrict__ out) {
  const int col = blockIdx.x * kThreads + threadIdx.x;
  const int i = blockIdx.y, bh = blockIdx.z;
  if (col >= row_len) return;
  const int8_t* m = Mc + (size_t)bh * Tq * T;
  const float* src = in + (size_t)bh * T * row_len + col;
  float s = 0.0f;
  for (int k = 0; k < T; ++k) {
    const int8_t lab = by_column ? m[(size_t)(k / rq) * T + i] : m[(size_t)(i / rq) * T + k];
    if (lab == 0) s += src[(size_t)k * row_len];
  }
  out[((size_t)bh * T + i) * row_len + col] = s;
}

// ------------------------------------------------------------------ forward
// One workgroup per query block: critical-block loop (Alg. 1 inner loop, M_c = 1 branch),
// then the closing line and Eq. 6.
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void forward_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const T* __restrict__ W, const int32_t* __restrict__ row_idx, const float* __restrict__ HZ,
    int N, int Tn, Lay lay, int n_h, int n_0, int phi, float scale, T* __restrict__ O, T* __restrict__ Os,
    T* __restrict__ Ol, float* __restrict__ L) {
  extern __shared__ float lds[];
  constexpr int LD = D + 1, NB = D / 16;
  float* Qs = lds;                 // 64 x LD
  float* Xs = lds + kBlk * LD;     // 64 x LD   K_j, then V_j, later phi(Q_i)
  float* Ps = lds + 2 * kBlk * LD; // 64 x 65   P, later 32-row chunks of H_i^T / W
  const int i = blockIdx.x, bh = blockIdx.y;
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  const int q0 = i * kBlk, rows = min(kBlk, N - q0);
  const size_t qbase = ((size_t)bh * N + q0) * D;                  // in the library's packed tensors
  const size_t uq = lay.head(bh) + (size_t)q0 * lay.ts;            // in the caller's tensors
  load_tile(Qs, LD, Q + uq, rows, D, lay.ts);
  float m[4], l[4], acc[4][NB];
#pragma unroll
  for (int a = 0; a < 4; ++a) { m[a] = -INFINITY; l[a] = 0.0f; }
  zero(acc);
  const int32_t* lut = row_idx + ((size_t)bh * Tn + i) * n_h;
  for (int t = 0; t < n_h; ++t) {
    const int j = lut[t];
    const int k0 = j * kBlk, cols = min(kBlk, N - k0);
    const size_t kbase = lay.head(bh) + (size_t)k0 * lay.ts;
    __syncthreads();
    load_tile(Xs, LD, K + kbase, cols, D, lay.ts);
    __syncthreads();
    float s[4][4];
    zero(s);
    mm_abt<4>(Qs, LD, Xs, LD, D, s);
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      float mx = -INFINITY;
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        s[a][b] = (tx + 16 * b < cols) ? s[a][b] * scale : -INFINITY;
        mx = fmaxf(mx, s[a][b]);
      }
      const float mnew = fmaxf(m[a], tx_max(mx));
      float sum = 0.0f;
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        s[a][b] = expf(s[a][b] - mnew);
        sum += s[a][b];
        Ps[(ty + 16 * a) * 65 + tx + 16 * b] = s[a][b];
      }
      const float alpha = expf(m[a] - mnew);
      l[a] = alpha * l[a] + tx_sum(sum);
      m[a] = mnew;
#pragma unroll
      for (int b = 0; b < NB; ++b) acc[a][b] *= alpha;
    }
    __syncthreads();
    load_tile(Xs, LD, V + kbase, cols, D, lay.ts);
    __syncthreads();
    mm_ab<NB>(Ps, 65, Xs, LD, kBlk, acc);
  }
  // closing line of Alg. 1, sparse part
  float os[4][NB];
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int r = ty + 16 * a;
    const float inv = n_h > 0 ? 1.0f / l[a] : 0.0f;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      os[a][b] = acc[a][b] * inv;
      if (Os && r < rows) from_f32(Os[qbase + (size_t)r * D + tx + 16 * b], os[a][b]);
    }
    if (L && tx == 0 && r < rows) L[(size_t)bh * N + q0 + r] = n_h > 0 ? m[a] + logf(l[a]) : -INFINITY;
  }
  float ol[4][NB];
  zero(ol);
  __syncthreads();
  if (n_0 > 0) {
    // O^l_i = phi(Q_i) H_i / (phi(Q_i) Z_i)
    phi_tile<D>(Qs, Xs, LD, kBlk, phi);
    __syncthreads();
    const float* Hrow = HZ + ((size_t)bh * Tn + i) * (D * D + D);
    const float* Z = Hrow + D * D;
    float den[4];
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      float p = 0.0f;
#pragma unroll
      for (int b = 0; b < NB; ++b) p = fmaf(Xs[(ty + 16 * a) * LD + tx + 16 * b], Z[tx + 16 * b], p);
      den[a] = tx_sum(p);
    }
    for (int c0 = 0; c0 < D; c0 += 32) {
      // chunk[cc][e] = H_i[c0+cc][e] = Hrow[e*D + c0 + cc]
      for (int idx = threadIdx.x; idx < 32 * D; idx += kThreads) {
        const int e = idx >> 5, cc = idx & 31;
        Ps[cc * LD + e] = Hrow[(size_t)e * D + c0 + cc];
      }
      __syncthreads();
      mm_ab<NB>(Xs + c0, LD, Ps, LD, 32, ol);
      __syncthreads();
    }
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < NB; ++b) ol[a][b] = ol[a][b] / den[a];
  }
  // Eq. 6: O = O^s + O^l W
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < NB; ++b) Qs[(ty + 16 * a) * LD + tx + 16 * b] = ol[a][b];
  __syncthreads();
  if (n_0 > 0) {
    for (int c0 = 0; c0 < D; c0 += 32) {
      for (int idx = threadIdx.x; idx < 32 * D; idx += kThreads) {
        const int cc = idx / D, e = idx - cc * D;
        Ps[cc * LD + e] = to_f32(W[(size_t)(c0 + cc) * D + e]);
      }
      __syncthreads();
      mm_ab<NB>(Qs + c0, LD, Ps, LD, 32, os);   // os now accumulates O
      __syncthreads();
    }
  }
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int r = ty + 16 * a;
    if (r >= rows) continue;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const size_t o = qbase + (size_t)r * D + tx + 16 * b;
      from_f32(O[uq + (size_t)r * lay.ts + tx + 16 * b], os[a][b]);
      if (Ol) from_f32(Ol[o], ol[a][b]);
    }
  }
}

// ------------------------------------------------------------------ backward, prologue
// dO^l = dO W^T, D^s = rowsum(dO * O^s), D^l = rowsum(dO^l * O^l)   (Alg. 2, D line)
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void bwd_prologue_kernel(
    const T* __restrict__ dO, const T* __restrict__ W, const T* __restrict__ Os,
    const T* __restrict__ Ol, int N, Lay lay, float* __restrict__ dOl, float* __restrict__ Ds,
    float* __restrict__ Dl) {
  extern __shared__ float lds[];
  constexpr int LD = D + 1, NB = D / 16;
  float* Gs = lds;              // dO_i
  float* Ws = lds + kBlk * LD;  // 64 rows of W
  const int i = blockIdx.x, bh = blockIdx.y;
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  const int q0 = i * kBlk, rows = min(kBlk, N - q0);
  const size_t base = ((size_t)bh * N + q0) * D;
  load_tile(Gs, LD, dO + lay.head(bh) + (size_t)q0 * lay.ts, rows, D, lay.ts);
  __syncthreads();
  float ds[4], dl[4];
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int r = ty + 16 * a;
    float p = 0.0f;
    if (r < rows)
#pragma unroll
      for (int b = 0; b < NB; ++b)
        p = fmaf(Gs[r * LD + tx + 16 * b], to_f32(Os[base + (size_t)r * D + tx + 16 * b]), p);
    ds[a] = tx_sum(p);
    dl[a] = 0.0f;
  }
  for (int c0 = 0; c0 < D; c0 += 64) {
    __syncthreads();
    load_tile(Ws, LD, W + (size_t)c0 * D, kBlk, D, D);
    __syncthreads();
    float g[4][4];
    zero(g);
    mm_abt<4>(Gs, LD, Ws, LD, D, g);  // g[r][c] = sum_e dO[r][e] W[c][e]
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const int r = ty + 16 * a;
      if (r >= rows) continue;
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const size_t o = base + (size_t)r * D + c0 + tx + 16 * b;
        dOl[o] = g[a][b];
        dl[a] = fmaf(g[a][b], to_f32(Ol[o]), dl[a]);
      }
    }
  }
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int r = ty + 16 * a;
    const float t = tx_sum(dl[a]);
    if (tx == 0 && r < rows) {
      Ds[(size_t)bh * N + q0 + r] = ds[a];
      Dl[(size_t)bh * N + q0 + r] = t;
    }
  }
}

// dW = sum over tokens of (O^l)^T dO: each workgroup sums a strided set of 64-token tiles
// into its own partial, a second kernel adds the partials in order.
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void dw_partial_kernel(const T* __restrict__ Ol,
                                                              const T* __restrict__ dO, int BH,
                                                              int N, int Tn, Lay lay,
                                                              float* __restrict__ part) {
  extern __shared__ float lds[];
  constexpr int LD = D + 1, NB = D / 16;
  float* As = lds;
  float* Bs = lds + kBlk * LD;
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  float acc[NB][NB];
  zero(acc);
  for (int t = blockIdx.x; t < BH * Tn; t += gridDim.x) {
    const int bh = t / Tn, i = t - bh * Tn;
    const int q0 = i * kBlk, rows = min(kBlk, N - q0);
    const size_t base = ((size_t)bh * N + q0) * D;
    __syncthreads();
    load_tile(As, LD, Ol + base, rows, D, D);
    load_tile(Bs, LD, dO + lay.head(bh) + (size_t)q0 * lay.ts, rows, D, lay.ts);
    __syncthreads();
    mm_atb<NB, NB>(As, LD, Bs, LD, kBlk, acc);
  }
  float* out = part + (size_t)blockIdx.x * D * D;
#pragma unroll
  for (int a = 0; a < NB; ++a)
#pragma unroll
    for (int b = 0; b < NB; ++b) out[(size_t)(ty + 16 * a) * D + tx + 16 * b] = acc[a][b];
}

__global__ void fill_zero_kernel(float* __restrict__ p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    p[i] = 0.0f;
}

// dW = sum of the partial d x d sums.  A workgroup owns 64 consecutive elements; its four waves
// take every fourth partial each (one element per lane, 256 contiguous bytes per load) and meet
// in LDS.
__global__ __launch_bounds__(256) void dw_reduce_kernel(const float* __restrict__ part, int nparts, int dd,
                                                        float* __restrict__ dW) {
  __shared__ float red[4][64];
  const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
  const int idx = blockIdx.x * 64 + l;
  float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
  if (idx < dd) {
    int p = w;
    for (; p + 12 < nparts; p += 16) {
      s0 += part[(size_t)p * dd + idx];
      s1 += part[(size_t)(p + 4) * dd + idx];
      s2 += part[(size_t)(p + 8) * dd + idx];
      s3 += part[(size_t)(p + 12) * dd + idx];
    }
    for (; p < nparts; p += 4) s0 += part[(size_t)p * dd + idx];
  }
  red[w][l] = (s0 + s1) + (s2 + s3);
  __syncthreads();
  if (w == 0 && idx < dd) dW[idx] = (red[0][l] + red[1][l]) + (red[2][l] + red[3][l]);
}

// ------------------------------------------------------------------ backward, linear, query side
// First loop of Alg. 2: dH_i, dZ_i, dQ^phi_i; then dQ^phi is taken through phi.
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void bwd_linear_q_kernel(
    const T* __restrict__ Q, const float* __restrict__ dOl, const float* __restrict__ Dl,
    const float* __restrict__ HZ, int N, int Tn, Lay lay, int phi, float* __restrict__ dHZ,
    float* __restrict__ dQlin) {
  extern __shared__ float lds[];
  constexpr int LD = D + 1, NB = D / 16;
  float* Qs = lds;                  // Q_i
  float* Ys = lds + kBlk * LD;      // phi(Q_i)
  float* Gs = lds + 2 * kBlk * LD;  // dO^l_i / (phi(Q_i) Z_i)
  float* Cs = lds + 3 * kBlk * LD;  // 32 x LD chunk of H_i^T
  float* dls = Cs + 32 * LD;        // 64: D^l / den
  const int i = blockIdx.x, bh = blockIdx.y;
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  const int q0 = i * kBlk, rows = min(kBlk, N - q0);
  const size_t base = ((size_t)bh * N + q0) * D;
  const float* Hrow = HZ + ((size_t)bh * Tn + i) * (D * D + D);
  const float* Z = Hrow + D * D;
  load_tile(Qs, LD, Q + lay.head(bh) + (size_t)q0 * lay.ts, rows, D, lay.ts);
  load_tile(Gs, LD, dOl + base, rows, D, D);
  __syncthreads();
  phi_tile<D>(Qs, Ys, LD, rows, phi);
  __syncthreads();
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int r = ty + 16 * a;
    float p = 0.0f;
#pragma unroll
    for (int b = 0; b < NB; ++b) p = fmaf(Ys[r * LD + tx + 16 * b], Z[tx + 16 * b], p);
    const float den = tx_sum(p);
    const float inv = r < rows ? 1.0f / den : 0.0f;
#pragma unroll
    for (int b = 0; b < NB; ++b) Gs[r * LD + tx + 16 * b] *= inv;
    if (tx == 0) dls[r] = r < rows ? Dl[(size_t)bh * N + q0 + r] * inv : 0.0f;
  }
  __syncthreads();
  float* out = dHZ + ((size_t)bh * Tn + i) * (D * D + D);
  // dH_i^T[e][c] = sum_r (dO^l[r][e] / den_r) phi(Q)[r][c]
  for (int e0 = 0; e0 < D; e0 += 64) {
    float acc[4][NB];
    zero(acc);
    mm_atb<4, NB>(Gs + e0, LD, Ys, LD, kBlk, acc);
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < NB; ++b) out[(size_t)(e0 + ty + 16 * a) * D + tx + 16 * b] = acc[a][b];
  }
  // dZ_i[c] = - sum_r phi(Q)[r][c] D^l_r / den_r
  if (threadIdx.x < D) {
    float z = 0.0f;
    for (int r = 0; r < kBlk; ++r) z = fmaf(Ys[r * LD + threadIdx.x], dls[r], z);
    out[(size_t)D * D + threadIdx.x] = -z;
  }
  // dQ^phi[r][c] = sum_e (dO^l[r][e]/den_r) H_i[c][e] - (D^l_r/den_r) Z[c]
  float g[4][NB];
  zero(g);
  for (int e0 = 0; e0 < D; e0 += 32) {
    __syncthreads();
    for (int idx = threadIdx.x; idx < 32 * D; idx += kThreads) {
      const int ee = idx / D, c = idx - ee * D;
      Cs[ee * LD + c] = Hrow[(size_t)(e0 + ee) * D + c];
    }
    __syncthreads();
    mm_ab<NB>(Gs + e0, LD, Cs, LD, 32, g);
  }
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < NB; ++b) g[a][b] = fmaf(-dls[ty + 16 * a], Z[tx + 16 * b], g[a][b]);
  phi_backward<D>(Qs, Ys, LD, phi, g);
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int r = ty + 16 * a;
    if (r >= rows) continue;
#pragma unroll
    for (int b = 0; b < NB; ++b) dQlin[base + (size_t)r * D + tx + 16 * b] = g[a][b];
  }
}

// ------------------------------------------------------------------ backward, linear, key side
// Last line of Alg. 2 for key block j: dK^phi_j = V_j dH^T + 1 dZ^T (then through phi),
// linear part of dV_j = K^phi_j dH, with dH, dZ the column sums over marginal query blocks.
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void bwd_linear_k_kernel(
    const T* __restrict__ K, const T* __restrict__ V, const float* __restrict__ dHZcol, int N,
    int Tn, Lay lay, int phi, float* __restrict__ dKlin, float* __restrict__ dVlin) {
  extern __shared__ float lds[];
  constexpr int LD = D + 1, NB = D / 16;
  float* Ks = lds;
  float* Ys = lds + kBlk * LD;      // phi(K_j)
  float* Vs = lds + 2 * kBlk * LD;
  float* Cs = lds + 3 * kBlk * LD;  // 64 x LD chunk of dH^T
  const int j = blockIdx.x, bh = blockIdx.y;
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  const int n0 = j * kBlk, cnt = min(kBlk, N - n0);
  const size_t base = ((size_t)bh * N + n0) * D;
  const float* Hrow = dHZcol + ((size_t)bh * Tn + j) * (D * D + D);
  const float* dZ = Hrow + D * D;
  load_tile(Ks, LD, K + lay.head(bh) + (size_t)n0 * lay.ts, cnt, D, lay.ts);
  load_tile(Vs, LD, V + lay.head(bh) + (size_t)n0 * lay.ts, cnt, D, lay.ts);
  __syncthreads();
  phi_tile<D>(Ks, Ys, LD, cnt, phi);
  float gk[4][NB];
  zero(gk);
  for (int e0 = 0; e0 < D; e0 += 64) {
    __syncthreads();
    for (int idx = threadIdx.x; idx < 64 * D; idx += kThreads) {
      const int ee = idx / D, c = idx - ee * D;
      Cs[ee * LD + c] = Hrow[(size_t)(e0 + ee) * D + c];   // dH[c][e0+ee]
    }
    __syncthreads();
    // dK^phi[n][c] += sum_{e in chunk} V[n][e] dH[c][e]
    mm_ab<NB>(Vs + e0, LD, Cs, LD, 64, gk);
    // dV_lin[n][e0+ee] = sum_c K^phi[n][c] dH[c][e0+ee]
    float gv[4][4];
    zero(gv);
    mm_abt<4>(Ys, LD, Cs, LD, D, gv);
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const int r = ty + 16 * a;
      if (r >= cnt) continue;
#pragma unroll
      for (int b = 0; b < 4; ++b) dVlin[base + (size_t)r * D + e0 + tx + 16 * b] = gv[a][b];
    }
  }
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < NB; ++b) gk[a][b] += dZ[tx + 16 * b];
  phi_backward<D>(Ks, Ys, LD, phi, gk);
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int r = ty + 16 * a;
    if (r >= cnt) continue;
#pragma unroll
    for (int b = 0; b < NB; ++b) dKlin[base + (size_t)r * D + tx + 16 * b] = gk[a][b];
  }
}

// ------------------------------------------------------------------ backward, sparse, dK / dV
// Second loop of Alg. 2 for key block j (M_c = 1 branch), walking the column table.
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void bwd_sparse_kv_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const T* __restrict__ dO, const float* __restrict__ L, const float* __restrict__ Ds,
    const int32_t* __restrict__ col_ptr, const int32_t* __restrict__ col_rows,
    const float* __restrict__ dKlin, const float* __restrict__ dVlin, int N, int Tn, Lay lay, int n_h,
    float scale, T* __restrict__ dK, T* __restrict__ dV) {
  extern __shared__ float lds[];
  constexpr int LD = D + 1, NB = D / 16;
  float* Ks = lds;
  float* Vs = lds + kBlk * LD;
  float* Xs = lds + 2 * kBlk * LD;    // Q_i, then dO_i, then Q_i again
  float* Ps = lds + 3 * kBlk * LD;    // 64 x 65
  float* dSs = Ps + kBlk * 65;        // 64 x 65
  const int j = blockIdx.x, bh = blockIdx.y;
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  const int k0 = j * kBlk, cols = min(kBlk, N - k0);
  const size_t kbase = ((size_t)bh * N + k0) * D;              // in the library's packed tensors
  const size_t uk = lay.head(bh) + (size_t)k0 * lay.ts;        // in the caller's tensors
  load_tile(Ks, LD, K + uk, cols, D, lay.ts);
  load_tile(Vs, LD, V + uk, cols, D, lay.ts);
  float dk[4][NB], dv[4][NB];
  zero(dk);
  zero(dv);
  const int32_t* ptr = col_ptr + (size_t)bh * (Tn + 1);
  const int32_t* list = col_rows + (size_t)bh * Tn * n_h;
  for (int t = ptr[j]; t < ptr[j + 1]; ++t) {
    const int i = list[t];
    const int q0 = i * kBlk, rows = min(kBlk, N - q0);
    const size_t qbase = lay.head(bh) + (size_t)q0 * lay.ts;
    __syncthreads();
    load_tile(Xs, LD, Q + qbase, rows, D, lay.ts);
    __syncthreads();
    float p[4][4];
    zero(p);
    mm_abt<4>(Xs, LD, Ks, LD, D, p);
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const int r = ty + 16 * a;
      const float Lr = r < rows ? L[(size_t)bh * N + q0 + r] : 0.0f;
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        p[a][b] = (r < rows && tx + 16 * b < cols) ? expf(p[a][b] * scale - Lr) : 0.0f;
        Ps[r * 65 + tx + 16 * b] = p[a][b];
      }
    }
    __syncthreads();
    load_tile(Xs, LD, dO + qbase, rows, D, lay.ts);
    __syncthreads();
    float dp[4][4];
    zero(dp);
    mm_abt<4>(Xs, LD, Vs, LD, D, dp);
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const int r = ty + 16 * a;
      const float Dr = r < rows ? Ds[(size_t)bh * N + q0 + r] : 0.0f;
#pragma unroll
      for (int b = 0; b < 4; ++b) dSs[r * 65 + tx + 16 * b] = p[a][b] * (dp[a][b] - Dr);
    }
    mm_atb<4, NB>(Ps, 65, Xs, LD, kBlk, dv);   // dV_j += P^T dO_i
    __syncthreads();
    load_tile(Xs, LD, Q + qbase, rows, D, lay.ts);
    __syncthreads();
    mm_atb<4, NB>(dSs, 65, Xs, LD, kBlk, dk);  // dK_j += dS^T Q_i
  }
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int r = ty + 16 * a;
    if (r >= cols) continue;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const size_t o = kbase + (size_t)r * D + tx + 16 * b, uo = uk + (size_t)r * lay.ts + tx + 16 * b;
      from_f32(dK[uo], dk[a][b] * scale + (dKlin ? dKlin[o] : 0.0f));
      from_f32(dV[uo], dv[a][b] + (dVlin ? dVlin[o] : 0.0f));
    }
  }
}

// ------------------------------------------------------------------ backward, sparse, dQ
// The dQ_i accumulation of Alg. 2's second loop, regrouped by query block (row table) so
// that each dQ_i has one owner and no atomics are needed.
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void bwd_sparse_q_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const T* __restrict__ dO, const float* __restrict__ L, const float* __restrict__ Ds,
    const int32_t* __restrict__ row_idx, const float* __restrict__ dQlin, int N, int Tn, Lay lay, int n_h,
    float scale, T* __restrict__ dQ) {
  extern __shared__ float lds[];
  constexpr int LD = D + 1, NB = D / 16;
  float* Qs = lds;
  float* Gs = lds + kBlk * LD;        // dO_i
  float* Xs = lds + 2 * kBlk * LD;    // K_j, V_j, K_j
  float* dSs = lds + 3 * kBlk * LD;   // 64 x 65
  const int i = blockIdx.x, bh = blockIdx.y;
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  const int q0 = i * kBlk, rows = min(kBlk, N - q0);
  const size_t qbase = ((size_t)bh * N + q0) * D;              // in the library's packed tensors
  const size_t uq = lay.head(bh) + (size_t)q0 * lay.ts;        // in the caller's tensors
  load_tile(Qs, LD, Q + uq, rows, D, lay.ts);
  load_tile(Gs, LD, dO + uq, rows, D, lay.ts);
  float Lr[4], Dr[4];
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int r = ty + 16 * a;
    Lr[a] = r < rows ? L[(size_t)bh * N + q0 + r] : 0.0f;
    Dr[a] = r < rows ? Ds[(size_t)bh * N + q0 + r] : 0.0f;
  }
  float dq[4][NB];
  zero(dq);
  const int32_t* lut = row_idx + ((size_t)bh * Tn + i) * n_h;
  for (int t = 0; t < n_h; ++t) {
    const int j = lut[t];
    const int k0 = j * kBlk, cols = min(kBlk, N - k0);
    const size_t kbase = lay.head(bh) + (size_t)k0 * lay.ts;
    __syncthreads();
    load_tile(Xs, LD, K + kbase, cols, D, lay.ts);
    __syncthreads();
    float p[4][4];
    zero(p);
    mm_abt<4>(Qs, LD, Xs, LD, D, p);
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b)
        p[a][b] = (ty + 16 * a < rows && tx + 16 * b < cols) ? expf(p[a][b] * scale - Lr[a]) : 0.0f;
    __syncthreads();
    load_tile(Xs, LD, V + kbase, cols, D, lay.ts);
    __syncthreads();
    float dp[4][4];
    zero(dp);
    mm_abt<4>(Gs, LD, Xs, LD, D, dp);
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b) dSs[(ty + 16 * a) * 65 + tx + 16 * b] = p[a][b] * (dp[a][b] - Dr[a]);
    __syncthreads();
    load_tile(Xs, LD, K + kbase, cols, D, lay.ts);
    __syncthreads();
    mm_ab<NB>(dSs, 65, Xs, LD, kBlk, dq);  // dQ_i += dS K_j
  }
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int r = ty + 16 * a;
    if (r >= rows) continue;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const size_t o = qbase + (size_t)r * D + tx + 16 * b;
      from_f32(dQ[uq + (size_t)r * lay.ts + tx + 16 * b], dq[a][b] * scale + (dQlin ? dQlin[o] : 0.0f));
    }
  }
}

template <typename K>
hipError_t set_lds(K kernel, size_t bytes) {
  return ensure_dyn_lds(kernel, bytes);
}

#define SLA_TRY(x)                      \
  do {                                  \
    hipError_t e_ = (x);                \
    if (e_ != hipSuccess) return e_;    \
  } while (0)

template <typename T, int D>
hipError_t forward_impl(const Shape& s, const FwdArgs& a, hipStream_t st) {
  constexpr int LD = D + 1;
  const dim3 grid(s.T, s.BH);
  const int row_len = s.state_row();
  if (s.n_0 > 0) {
    const size_t lds1 = sizeof(float) * 2 * kBlk * LD;
    SLA_TRY(set_lds(states_kernel<T, D>, lds1));
    {
      KernelTimer kt("states", st);
      states_kernel<T, D><<<grid, kThreads, lds1, st>>>((const T*)a.K, (const T*)a.V, s.N, s.T, s.lay(), s.phi, a.hz);
    }
    {
      KernelTimer kt("aggregate", st);
      aggregate_kernel<<<dim3((row_len + kThreads - 1) / kThreads, s.T, s.BH), kThreads, 0, st>>>(
        a.hz, a.Mc, s.Tq, s.rq, s.T, row_len, 0, a.HZ);
    }
  } else {
    {
      KernelTimer kt("fill_zero", st);
      fill_zero_kernel<<<1024, 256, 0, st>>>(a.HZ, (size_t)s.BH * s.T * row_len);
    }
  }
  const size_t lds2 = sizeof(float) * (2 * kBlk * LD + kBlk * 65 + 64);
  SLA_TRY(set_lds(forward_kernel<T, D>, lds2));
  {
    KernelTimer kt("forward", st);
    forward_kernel<T, D><<<grid, kThreads, lds2, st>>>(
      (const T*)a.Q, (const T*)a.K, (const T*)a.V, (const T*)a.W, a.row_idx, a.HZ, s.N, s.T, s.lay(), s.n_h,
      s.n_0, s.phi, s.scale, (T*)a.O, (T*)a.Os, (T*)a.Ol, a.L);
  }
  return hipGetLastError();
}

struct BwdWs {
  float *dOl, *Ds, *Dl, *dHZ, *dHZcol, *dQlin, *dKlin, *dVlin, *dWpart;
  int nparts;
  size_t bytes;
};

BwdWs carve_bwd(const Shape& s, char* ws) {
  BwdWs w;
  size_t off = 0;
  auto take = [&](size_t n) {
    float* p = reinterpret_cast<float*>(ws + off);
    off += align_up(n * sizeof(float));
    return p;
  };
  const size_t nd = (size_t)s.BH * s.N * s.d, n = (size_t)s.BH * s.N;
  const size_t st = (size_t)s.BH * s.T * s.state_row();
  w.nparts = s.BH * s.T < 512 ? s.BH * s.T : 512;   // two workgroups per CU
  const bool simt = s.dtype == 0;   // the matrix-core path has no dO^l, D^l, dK, dV round trips
  w.dOl = take(simt ? nd : 0);
  w.Ds = take(n);
  w.Dl = take(simt ? n : 0);
  w.dHZ = take(st);
  w.dHZcol = take(st);
  w.dQlin = take(nd);
  w.dKlin = take(simt ? nd : 0);
  w.dVlin = take(simt ? nd : 0);
  w.dWpart = take((size_t)w.nparts * s.d * s.d);
  w.bytes = off;
  return w;
}

template <typename T, int D>
hipError_t backward_impl(const Shape& s, const BwdArgs& a, hipStream_t st) {
  constexpr int LD = D + 1;
  const BwdWs w = carve_bwd(s, a.ws);
  const dim3 grid(s.T, s.BH);
  const int row_len = s.state_row();
  const bool lin = s.n_0 > 0;
  {
    const size_t lds = sizeof(float) * 2 * kBlk * LD;
    SLA_TRY(set_lds(bwd_prologue_kernel<T, D>, lds));
    {
      KernelTimer kt("bwd_prologue", st);
      bwd_prologue_kernel<T, D><<<grid, kThreads, lds, st>>>((const T*)a.dO, (const T*)a.W, (const T*)a.Os,
                                                          (const T*)a.Ol, s.N, s.lay(), w.dOl, w.Ds, w.Dl);
    }
    SLA_TRY(set_lds(dw_partial_kernel<T, D>, lds));
    {
      KernelTimer kt("dw_partial", st);
      dw_partial_kernel<T, D><<<w.nparts, kThreads, lds, st>>>((const T*)a.Ol, (const T*)a.dO, s.BH, s.N,
                                                            s.T, s.lay(), w.dWpart);
    }
    {
      KernelTimer kt("dw_reduce", st);
      dw_reduce_kernel<<<(D * D + 63) / 64, 256, 0, st>>>(w.dWpart, w.nparts, D * D, a.dW);
    }
  }
  if (lin) {
    const size_t lds = sizeof(float) * (3 * kBlk * LD + 32 * LD + 64);
    SLA_TRY(set_lds(bwd_linear_q_kernel<T, D>, lds));
    {
      KernelTimer kt("bwd_linear_q", st);
      bwd_linear_q_kernel<T, D><<<grid, kThreads, lds, st>>>((const T*)a.Q, w.dOl, w.Dl, a.HZ, s.N, s.T,
                                                          s.lay(), s.phi, w.dHZ, w.dQlin);
    }
    {
      KernelTimer kt("aggregate", st);
      aggregate_kernel<<<dim3((row_len + kThreads - 1) / kThreads, s.T, s.BH), kThreads, 0, st>>>(
        w.dHZ, a.Mc, s.Tq, s.rq, s.T, row_len, 1, w.dHZcol);
    }
    const size_t lds2 = sizeof(float) * 4 * kBlk * LD;
    SLA_TRY(set_lds(bwd_linear_k_kernel<T, D>, lds2));
    {
      KernelTimer kt("bwd_linear_k", st);
      bwd_linear_k_kernel<T, D><<<grid, kThreads, lds2, st>>>((const T*)a.K, (const T*)a.V, w.dHZcol, s.N,
                                                           s.T, s.lay(), s.phi, w.dKlin, w.dVlin);
    }
  }
  {
    const size_t lds = sizeof(float) * (3 * kBlk * LD + 2 * kBlk * 65);
    SLA_TRY(set_lds(bwd_sparse_kv_kernel<T, D>, lds));
    {
      KernelTimer kt("bwd_sparse_kv", st);
      bwd_sparse_kv_kernel<T, D><<<grid, kThreads, lds, st>>>(
        (const T*)a.Q, (const T*)a.K, (const T*)a.V, (const T*)a.dO, a.L, w.Ds, a.col_ptr, a.col_rows,
        lin ? w.dKlin : nullptr, lin ? w.dVlin : nullptr, s.N, s.T, s.lay(), s.n_h, s.scale, (T*)a.dK, (T*)a.dV);
    }
    const size_t lds2 = sizeof(float) * (3 * kBlk * LD + kBlk * 65);
    SLA_TRY(set_lds(bwd_sparse_q_kernel<T, D>, lds2));
    {
      KernelTimer kt("bwd_sparse_q", st);
      bwd_sparse_q_kernel<T, D><<<grid, kThreads, lds2, st>>>(
        (const T*)a.Q, (const T*)a.K, (const T*)a.V, (const T*)a.dO, a.L, w.Ds, a.row_idx,
        lin ? w.dQlin : nullptr, s.N, s.T, s.lay(), s.n_h, s.scale, (T*)a.dQ);
    }
  }
  return hipGetLastError();
}

// bf16 tensors: every step on the matrix cores; this file only contributes the dW reduction
hipError_t backward_bf16(const Shape& s, const BwdArgs& a, hipStream_t st) {
  const BwdWs w = carve_bwd(s, a.ws);
  const bool lin = s.n_0 > 0;
  SLA_TRY(mfma_backward_query(s, a, w.Ds, w.dHZ, w.dQlin, st));   // dHZ holds bf16 rows
  SLA_TRY(mfma_backward_dw(s, a, w.dWpart, w.nparts, st));
  {
    KernelTimer kt("dw_reduce", st);
    dw_reduce_kernel<<<(s.d * s.d + 63) / 64, 256, 0, st>>>(w.dWpart, w.nparts, s.d * s.d, a.dW);
  }
  if (lin) {
    SLA_TRY(mfma_aggregate(w.dHZ, a.indT, s, w.dHZcol,
                           reinterpret_cast<float*>(reinterpret_cast<char*>(w.dHZcol) + state_z_offset(s)), st));
  }
  return mfma_backward_sparse(s, a, w.Ds, lin ? w.dHZcol : nullptr, st);
}

}  // namespace

hipError_t simt_forward(const Shape& s, const FwdArgs& a, hipStream_t st) {
  if (s.dtype == 0) return s.d == 64 ? forward_impl<float, 64>(s, a, st) : forward_impl<float, 128>(s, a, st);
  return s.d == 64 ? forward_impl<__hip_bfloat16, 64>(s, a, st)
                   : forward_impl<__hip_bfloat16, 128>(s, a, st);
}

size_t simt_backward_ws_bytes(const Shape& s) { return carve_bwd(s, nullptr).bytes; }

hipError_t simt_backward(const Shape& s, const BwdArgs& a, hipStream_t st) {
  if (s.dtype == 0) return s.d == 64 ? backward_impl<float, 64>(s, a, st) : backward_impl<float, 128>(s, a, st);
  return backward_bf16(s, a, st);
}

}  // namespace sla
