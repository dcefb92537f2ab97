// bf16 matrix-core backward kernels for the critical blocks (Algorithm 2, M_c = 1 branch;
// Eq. 7 with the 1/sqrt(d) factor on dQ and dK):
//   bwd_dkdv_mfma  one workgroup per key block j, walking the column table:
//                  dV_j += P^T dO_i, dK_j += dS^T Q_i / sqrt(d)
//   bwd_dq_mfma    one workgroup per query block i, walking the row table:
//                  dQ_i += dS K_j / sqrt(d)   (S, dP are recomputed; no atomics, one owner)
// P = exp(S - L) and dS = P (dP - D^s) are formed in float from MFMA accumulators.
#include "mfma_common.h"

namespace sla {
namespace {

constexpr int kRS(int D) { return D + 8; }   // row-major tile stride (elements)

// ------------------------------------------------------------------ dK, dV
// Wavefront (kh, par): kh = which 32 of the block's 64 keys, par = which of the two query
// tiles of a step.  S and dP are formed as [query][key] so that each lane owns one key; P
// and dS then feed the second products (contraction over queries) straight from registers.
template <int D>
struct KvLds {
  static constexpr int RS = kRS(D);
  static constexpr int ROW_ELEMS = kBlk * RS;       // one row-major tile
  static constexpr int T_ELEMS = D * kVS;           // one transposed tile
  static constexpr int TILE_ELEMS = 2 * ROW_ELEMS + 2 * T_ELEMS;   // Q, dO, Q^T, dO^T
  static constexpr int STAT_BYTES = 2 * 2 * kBlk * 4;              // L*log2e and D^s of both tiles
  static constexpr int BYTES = 2 * TILE_ELEMS * 2 + STAT_BYTES;
};

template <int D>
__global__ __launch_bounds__(256) void bwd_dkdv_mfma_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ K, const bf16* __restrict__ V,
    const bf16* __restrict__ dO, const float* __restrict__ L, const float* __restrict__ Ds,
    const int32_t* __restrict__ col_ptr, const int32_t* __restrict__ col_rows,
    const float* __restrict__ dKlin, const float* __restrict__ dVlin, int N, int Tn, int n_h,
    float scale, bf16* __restrict__ dK, bf16* __restrict__ dV) {
  using Lds = KvLds<D>;
  constexpr int RS = Lds::RS, NT = D / 32, KT = D / 16;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* tiles = reinterpret_cast<bf16*>(smem);
  float* stats = reinterpret_cast<float*>(smem + 2 * Lds::TILE_ELEMS * 2);   // [tile][2][64]
  float* xch = reinterpret_cast<float*>(smem);
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, g = l >> 5, ln = l & 31;
  const int kh = w & 1, par = w >> 1;
  const int j = blockIdx.x, bh = blockIdx.y;
  const int k0 = j * kBlk, cols = min(kBlk, N - k0);
  const int krow = kh * 32 + ln;
  const bool kok = krow < cols;
  const size_t koff = ((size_t)bh * N + k0 + krow) * D;
  bf16x8 kf[KT], vf[KT];
#pragma unroll
  for (int t = 0; t < KT; ++t) {
    kf[t] = kok ? *reinterpret_cast<const bf16x8*>(K + koff + 16 * t + 8 * g) : zero_bf16x8();
    vf[t] = kok ? *reinterpret_cast<const bf16x8*>(V + koff + 16 * t + 8 * g) : zero_bf16x8();
  }
  f32x16 dvT[NT], dkT[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    dvT[t] = zero_f32x16();
    dkT[t] = zero_f32x16();
  }
  const int32_t* ptr = col_ptr + (size_t)bh * (Tn + 1);
  const int32_t* list = col_rows + (size_t)bh * Tn * n_h;
  const int beg = ptr[j], cnt = ptr[j + 1] - beg;
  const float sl2 = scale * kLog2e;
  const bf16* Qb = Q + (size_t)bh * N * D;
  const bf16* dOb = dO + (size_t)bh * N * D;
  const float* Lb = L + (size_t)bh * N;
  const float* Dsb = Ds + (size_t)bh * N;
  const int steps = (cnt + 1) >> 1;
  constexpr int UPT = (16 * (D / 8) + 255) / 256;   // staging units per thread per tile
  for (int s = 0; s < steps; ++s) {
    const bool two = 2 * s + 1 < cnt;
    const int i0 = list[beg + 2 * s];
    const int i1 = two ? list[beg + 2 * s + 1] : i0;
    u32x4 qreg[2][UPT][4], greg[2][UPT][4];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const int ii = p ? i1 : i0;
      const int rows = (p == 0 || two) ? min(kBlk, N - ii * kBlk) : 0;
#pragma unroll
      for (int r = 0; r < UPT; ++r) {
        const int u = tid + 256 * r;
        const int fg = u % (D / 8), rg = u / (D / 8);
        if (rg < 16) {
          load_unit(Qb + (size_t)ii * kBlk * D, D, rg, fg, rows, qreg[p][r]);
          load_unit(dOb + (size_t)ii * kBlk * D, D, rg, fg, rows, greg[p][r]);
        }
      }
    }
    __syncthreads();   // every wave is done with the previous step's tiles
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      bf16* base = tiles + p * Lds::TILE_ELEMS;
#pragma unroll
      for (int r = 0; r < UPT; ++r) {
        const int u = tid + 256 * r;
        const int fg = u % (D / 8), rg = u / (D / 8);
        if (rg < 16) {
          store_unit_rows(base, RS, rg, fg, qreg[p][r]);
          store_unit_rows(base + Lds::ROW_ELEMS, RS, rg, fg, greg[p][r]);
          store_unit_t(base + 2 * Lds::ROW_ELEMS, rg, fg, qreg[p][r]);
          store_unit_t(base + 2 * Lds::ROW_ELEMS + Lds::T_ELEMS, rg, fg, greg[p][r]);
        }
      }
    }
    if (tid < 128) {   // per-query statistics of both tiles; rows past the end never contribute
      const int p = tid >> 6, q = tid & 63;
      const int ii = p ? i1 : i0;
      const bool ok = (p == 0 || two) && ii * kBlk + q < N;
      stats[(p * 2 + 0) * kBlk + q] = ok ? Lb[ii * kBlk + q] * kLog2e : INFINITY;
      stats[(p * 2 + 1) * kBlk + q] = ok ? Dsb[ii * kBlk + q] : 0.0f;
    }
    __syncthreads();
    if (par == 0 || two) {
      const bf16* Qs = tiles + par * Lds::TILE_ELEMS;
      const bf16* Gs = Qs + Lds::ROW_ELEMS;
      const bf16* Qt = Qs + 2 * Lds::ROW_ELEMS;
      const bf16* Gt = Qt + Lds::T_ELEMS;
      const float* Ls = stats + (par * 2 + 0) * kBlk;
      const float* Dq = stats + (par * 2 + 1) * kBlk;
      f32x16 sm[2], dp[2];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        sm[mt] = zero_f32x16();
        dp[mt] = zero_f32x16();
      }
#pragma unroll
      for (int t = 0; t < KT; ++t)
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
          const bf16x8 aq = *reinterpret_cast<const bf16x8*>(Qs + (32 * mt + ln) * RS + 16 * t + 8 * g);
          sm[mt] = mfma32(aq, kf[t], sm[mt]);
          const bf16x8 ag = *reinterpret_cast<const bf16x8*>(Gs + (32 * mt + ln) * RS + 16 * t + 8 * g);
          dp[mt] = mfma32(ag, vf[t], dp[mt]);
        }
      // P[q][key] = exp(S - L_q), dS = P (dP - D^s_q); rows q = 32 mt + c_row(r, g)
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const f32x4 lq = *reinterpret_cast<const f32x4*>(Ls + 32 * mt + 8 * r4 + 4 * g);
          const f32x4 dq = *reinterpret_cast<const f32x4*>(Dq + 32 * mt + 8 * r4 + 4 * g);
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const float pv = kok ? fast_exp2(sm[mt][4 * r4 + r] * sl2 - lq[r]) : 0.0f;
            sm[mt][4 * r4 + r] = pv;
            dp[mt][4 * r4 + r] = pv * (dp[mt][4 * r4 + r] - dq[r]);
          }
        }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const bf16x8 pb = c_to_operand(sm[u >> 1], u & 1);
        const bf16x8 sb = c_to_operand(dp[u >> 1], u & 1);
#pragma unroll
        for (int et = 0; et < NT; ++et) {
          const bf16x8 ag = *reinterpret_cast<const bf16x8*>(Gt + (32 * et + ln) * kVS + 16 * u + 8 * g);
          dvT[et] = mfma32(ag, pb, dvT[et]);
          const bf16x8 aq = *reinterpret_cast<const bf16x8*>(Qt + (32 * et + ln) * kVS + 16 * u + 8 * g);
          dkT[et] = mfma32(aq, sb, dkT[et]);
        }
      }
    }
  }
  // ---- add the two query-tile streams, then the linear-branch parts, and store
  __syncthreads();
  float* myx = xch + (size_t)kh * (2 * NT * 16) * 64;
  if (par == 1) {
#pragma unroll
    for (int et = 0; et < NT; ++et)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        myx[(et * 16 + r) * 64 + l] = dvT[et][r];
        myx[((NT + et) * 16 + r) * 64 + l] = dkT[et][r];
      }
  }
  __syncthreads();
  if (par == 0 && kok) {
#pragma unroll
    for (int et = 0; et < NT; ++et)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const size_t o = koff + 32 * et + 8 * r4 + 4 * g;
        f32x4 lv = {0.0f, 0.0f, 0.0f, 0.0f}, lk = {0.0f, 0.0f, 0.0f, 0.0f};
        if (dVlin) lv = *reinterpret_cast<const f32x4*>(dVlin + o);
        if (dKlin) lk = *reinterpret_cast<const f32x4*>(dKlin + o);
        bf16x4 pv, pk;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int rr = 4 * r4 + r;
          pv[r] = (__bf16)(dvT[et][rr] + myx[(et * 16 + rr) * 64 + l] + lv[r]);
          pk[r] = (__bf16)((dkT[et][rr] + myx[((NT + et) * 16 + rr) * 64 + l]) * scale + lk[r]);
        }
        *reinterpret_cast<bf16x4*>(dV + o) = pv;
        *reinterpret_cast<bf16x4*>(dK + o) = pk;
      }
  }
}

// ------------------------------------------------------------------ dQ
// Wavefront (qh, par) as in the forward kernel; S^T and dP^T are [key][query], one query per
// lane, so L and D^s are per-lane scalars and dS^T feeds dQ^T = K^T dS^T from registers.
template <int D>
struct QLds {
  static constexpr int RS = kRS(D);
  static constexpr int ROW_ELEMS = kBlk * RS;
  static constexpr int T_ELEMS = D * kVS;
  static constexpr int TILE_ELEMS = 2 * ROW_ELEMS + T_ELEMS;   // K, V, K^T
  static constexpr int BYTES = 2 * TILE_ELEMS * 2;
};

template <int D>
__global__ __launch_bounds__(256) void bwd_dq_mfma_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ K, const bf16* __restrict__ V,
    const bf16* __restrict__ dO, const float* __restrict__ L, const float* __restrict__ Ds,
    const int32_t* __restrict__ row_idx, const float* __restrict__ dQlin, int N, int Tn, int n_h,
    float scale, bf16* __restrict__ dQ) {
  using Lds = QLds<D>;
  constexpr int RS = Lds::RS, NT = D / 32, KT = D / 16;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* tiles = reinterpret_cast<bf16*>(smem);
  float* xch = reinterpret_cast<float*>(smem);
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, g = l >> 5, ln = l & 31;
  const int qh = w & 1, par = w >> 1;
  const int i = blockIdx.x, bh = blockIdx.y;
  const int q0 = i * kBlk, rows = min(kBlk, N - q0);
  const int qrow = qh * 32 + ln;
  const bool qok = qrow < rows;
  const size_t qoff = ((size_t)bh * N + q0 + qrow) * D;
  bf16x8 qf[KT], gf[KT];
#pragma unroll
  for (int t = 0; t < KT; ++t) {
    qf[t] = qok ? *reinterpret_cast<const bf16x8*>(Q + qoff + 16 * t + 8 * g) : zero_bf16x8();
    gf[t] = qok ? *reinterpret_cast<const bf16x8*>(dO + qoff + 16 * t + 8 * g) : zero_bf16x8();
  }
  const float Lq = qok ? L[(size_t)bh * N + q0 + qrow] * kLog2e : INFINITY;
  const float Dq = qok ? Ds[(size_t)bh * N + q0 + qrow] : 0.0f;
  f32x16 dqT[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) dqT[t] = zero_f32x16();
  const int32_t* lut = row_idx + ((size_t)bh * Tn + i) * n_h;
  const bf16* Kb = K + (size_t)bh * N * D;
  const bf16* Vb = V + (size_t)bh * N * D;
  const float sl2 = scale * kLog2e;
  const int steps = (n_h + 1) >> 1;
  constexpr int UPT = (16 * (D / 8) + 255) / 256;
  for (int s = 0; s < steps; ++s) {
    const bool two = 2 * s + 1 < n_h;
    const int j0 = lut[2 * s];
    const int j1 = two ? lut[2 * s + 1] : j0;
    u32x4 kreg[2][UPT][4], vreg[2][UPT][4];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const int jj = p ? j1 : j0;
      const int cols = (p == 0 || two) ? min(kBlk, N - jj * kBlk) : 0;
#pragma unroll
      for (int r = 0; r < UPT; ++r) {
        const int u = tid + 256 * r;
        const int fg = u % (D / 8), rg = u / (D / 8);
        if (rg < 16) {
          load_unit(Kb + (size_t)jj * kBlk * D, D, rg, fg, cols, kreg[p][r]);
          load_unit(Vb + (size_t)jj * kBlk * D, D, rg, fg, cols, vreg[p][r]);
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      bf16* base = tiles + p * Lds::TILE_ELEMS;
#pragma unroll
      for (int r = 0; r < UPT; ++r) {
        const int u = tid + 256 * r;
        const int fg = u % (D / 8), rg = u / (D / 8);
        if (rg < 16) {
          store_unit_rows(base, RS, rg, fg, kreg[p][r]);
          store_unit_rows(base + Lds::ROW_ELEMS, RS, rg, fg, vreg[p][r]);
          store_unit_t(base + 2 * Lds::ROW_ELEMS, rg, fg, kreg[p][r]);
        }
      }
    }
    __syncthreads();
    if (par == 0 || two) {
      const int jmine = par ? j1 : j0;
      const int cols = min(kBlk, N - jmine * kBlk);
      const bf16* Ks = tiles + par * Lds::TILE_ELEMS;
      const bf16* Vs = Ks + Lds::ROW_ELEMS;
      const bf16* Kt = Ks + 2 * Lds::ROW_ELEMS;
      f32x16 sT[2], dpT[2];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        sT[mt] = zero_f32x16();
        dpT[mt] = zero_f32x16();
      }
#pragma unroll
      for (int t = 0; t < KT; ++t)
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
          const bf16x8 ak = *reinterpret_cast<const bf16x8*>(Ks + (32 * mt + ln) * RS + 16 * t + 8 * g);
          sT[mt] = mfma32(ak, qf[t], sT[mt]);
          const bf16x8 av = *reinterpret_cast<const bf16x8*>(Vs + (32 * mt + ln) * RS + 16 * t + 8 * g);
          dpT[mt] = mfma32(av, gf[t], dpT[mt]);
        }
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = 32 * mt + c_row(r, g);
          const float pv = key < cols ? fast_exp2(sT[mt][r] * sl2 - Lq) : 0.0f;
          dpT[mt][r] = pv * (dpT[mt][r] - Dq);
        }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const bf16x8 sb = c_to_operand(dpT[u >> 1], u & 1);
#pragma unroll
        for (int dt = 0; dt < NT; ++dt) {
          const bf16x8 ak = *reinterpret_cast<const bf16x8*>(Kt + (32 * dt + ln) * kVS + 16 * u + 8 * g);
          dqT[dt] = mfma32(ak, sb, dqT[dt]);
        }
      }
    }
  }
  __syncthreads();
  float* myx = xch + (size_t)qh * (NT * 16) * 64;
  if (par == 1) {
#pragma unroll
    for (int dt = 0; dt < NT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) myx[(dt * 16 + r) * 64 + l] = dqT[dt][r];
  }
  __syncthreads();
  if (par == 0 && qok) {
#pragma unroll
    for (int dt = 0; dt < NT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const size_t o = qoff + 32 * dt + 8 * r4 + 4 * g;
        f32x4 lq = {0.0f, 0.0f, 0.0f, 0.0f};
        if (dQlin) lq = *reinterpret_cast<const f32x4*>(dQlin + o);
        bf16x4 pk;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int rr = 4 * r4 + r;
          pk[r] = (__bf16)((dqT[dt][rr] + myx[(dt * 16 + rr) * 64 + l]) * scale + lq[r]);
        }
        *reinterpret_cast<bf16x4*>(dQ + o) = pk;
      }
  }
}

#define SLA_TRY(x)                   \
  do {                               \
    hipError_t e_ = (x);             \
    if (e_ != hipSuccess) return e_; \
  } while (0)

template <int D>
hipError_t sparse_impl(const Shape& s, const BwdArgs& a, const float* Ds, const float* dQlin,
                       const float* dKlin, const float* dVlin, hipStream_t st) {
  const dim3 grid(s.T, s.BH);
  constexpr int lds_kv = KvLds<D>::BYTES, lds_q = QLds<D>::BYTES;
  SLA_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_dkdv_mfma_kernel<D>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, lds_kv));
  {
    KernelTimer kt("bwd_sparse_kv", st);
    bwd_dkdv_mfma_kernel<D><<<grid, 256, lds_kv, st>>>(
        (const bf16*)a.Q, (const bf16*)a.K, (const bf16*)a.V, (const bf16*)a.dO, a.L, Ds, a.col_ptr,
        a.col_rows, dKlin, dVlin, s.N, s.T, s.n_h, s.scale, (bf16*)a.dK, (bf16*)a.dV);
  }
  SLA_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_dq_mfma_kernel<D>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, lds_q));
  {
    KernelTimer kt("bwd_sparse_q", st);
    bwd_dq_mfma_kernel<D><<<grid, 256, lds_q, st>>>(
        (const bf16*)a.Q, (const bf16*)a.K, (const bf16*)a.V, (const bf16*)a.dO, a.L, Ds, a.row_idx,
        dQlin, s.N, s.T, s.n_h, s.scale, (bf16*)a.dQ);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t mfma_backward_sparse(const Shape& s, const BwdArgs& a, const float* Ds,
                                const float* dQlin, const float* dKlin, const float* dVlin,
                                hipStream_t st) {
  return s.d == 64 ? sparse_impl<64>(s, a, Ds, dQlin, dKlin, dVlin, st)
                   : sparse_impl<128>(s, a, Ds, dQlin, dKlin, dVlin, st);
}

}  // namespace sla
