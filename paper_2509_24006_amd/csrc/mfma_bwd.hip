// bf16 matrix-core backward kernels for the critical blocks (Algorithm 2, M_c = 1 branch;
// Eq. 7 with the 1/sqrt(d) factor on dQ and dK):
//   bwd_dkdv_mfma  one workgroup per key block j, walking the column table:
//                  dV_j += P^T dO_i, dK_j += dS^T Q_i / sqrt(d)
//   bwd_dq_mfma    one workgroup per query block i, walking the row table:
//                  dQ_i += dS K_j / sqrt(d)   (S, dP are recomputed; no atomics, one owner)
// P = exp(S - L) and dS = P (dP - D^s) are formed in float from MFMA accumulators.
//
// One critical pair per step.  The two streaming tiles of a pair go global -> LDS directly
// (no registers), row-major and chunk-swizzled, double-buffered: the loads of step s+1 are in
// flight during the arithmetic of step s and a step has a single barrier.  A product that
// needs a tile transposed (contraction over its rows) reads it with the transposing LDS read.
// The four waves split the 64 x 64 pair into 32 x 32 quarters; two workgroups share a CU so
// that one's matrix work overlaps the other's vector work.
#include "mfma_common.h"

namespace sla {
namespace {

template <int D>
struct PairLds {
  static constexpr int TILE = SwzTile<D>::BYTES;
  static constexpr int BUF = 2 * TILE;                   // the two tiles of a pair
  static constexpr int STAT_OFF = 2 * BUF;
  static constexpr int XCH = 2 * 2 * (D / 32) * 16 * 64 * 4;   // final exchange (dK/dV kernel)
  static constexpr int TILES = 2 * BUF > XCH ? 2 * BUF : XCH;
  static constexpr int BYTES = TILES + 2 * 2 * kBlk * 4; // + [buf][L, D^s][64]
};

// ------------------------------------------------------------------ dK, dV
// Wave (kh, qh): keys 32 kh .., queries 32 qh .. of the pair.  S and dP are [query][key] so
// that each lane owns one key; P and dS feed the second products from registers.  The two qh
// waves hold partial sums over their queries and are added at the end.
template <int D>
__global__ __launch_bounds__(256, 2) void bwd_dkdv_mfma_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ K, const bf16* __restrict__ V,
    const bf16* __restrict__ dO, const float* __restrict__ L, const float* __restrict__ Ds,
    const int32_t* __restrict__ col_ptr, const int32_t* __restrict__ col_rows,
    const int32_t* __restrict__ col_order, const float* __restrict__ dKlin,
    const float* __restrict__ dVlin, int N, int Tn, int n_h, float scale, bf16* __restrict__ dK,
    bf16* __restrict__ dV) {
  using Lds = PairLds<D>;
  constexpr int NT = D / 32, KT = D / 16;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* stats = reinterpret_cast<float*>(smem + Lds::TILES);   // [buf][2][64]
  float* xch = reinterpret_cast<float*>(smem);
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, g = l >> 5, ln = l & 31;
  const int kh = w & 1, qh = w >> 1;
  // longest column lists first, across all heads: the r-th heaviest key block of every head
  // precedes the (r+1)-th of any head, so the tail of the launch is made of short lists
  // (grouping an XCD's workgroups by head for L2 reuse was measured slower than this order)
  const int BH = gridDim.x / Tn;
  const int bh = blockIdx.x % BH;
  const int j = col_order[(size_t)bh * Tn + blockIdx.x / BH];
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
  float streg = 0.0f;
  // per-lane addresses, fixed for the whole kernel
  using T = SwzTile<D>;
  TileAddr<D> ad;
  ad.init(32 * qh, l);
  int ldv[T::IPW];   // byte offset inside a tile of the chunk this lane fetches with load k
#pragma unroll
  for (int k = 0; k < T::IPW; ++k) {
    const int row = T::RPI * (4 * k + w) + l / T::CPR;
    ldv[k] = swz_chunk_off<D>(row, l % T::CPR);
  }
  const int wlds = wave_uniform(w) * 1024;
  // (issue and step are inlined at call sites with a literal buffer index, which turns every
  // LDS offset below into register + constant)
  auto issue = [&](int s, const int bufi) __attribute__((always_inline)) {
    const int off = bufi * Lds::BUF;
    const int ii = list[beg + s];
    const int rows = min(kBlk, N - ii * kBlk);
    const __amdgpu_buffer_rsrc_t rq = tile_rsrc(Qb + (size_t)ii * kBlk * D, rows * T::ROW_BYTES);
    const __amdgpu_buffer_rsrc_t rg = tile_rsrc(dOb + (size_t)ii * kBlk * D, rows * T::ROW_BYTES);
#pragma unroll
    for (int k = 0; k < T::IPW; ++k) {
      load_to_lds16(rq, ldv[k], smem, off + 4096 * k + wlds);
      load_to_lds16(rg, ldv[k], smem, off + Lds::TILE + 4096 * k + wlds);
    }
    if (tid < 128) {   // per-query statistics; rows past the end give P = 0
      const int q = tid & 63;
      const bool ok = q < rows;
      if (tid < 64) streg = ok ? Lb[ii * kBlk + q] * kLog2e : INFINITY;
      else streg = ok ? Dsb[ii * kBlk + q] : 0.0f;
    }
  };
  auto step = [&](int s, const int buf) __attribute__((always_inline)) {
    const int QO = buf * Lds::BUF, GO = QO + Lds::TILE;
    wait_vm0();
    __syncthreads();   // tiles of step s have landed for every wave; step s-1 is fully consumed
    if (s + 1 < cnt) issue(s + 1, buf ^ 1);
    const float* Ls = stats + buf * 2 * kBlk;
    const float* Dq = Ls + kBlk;
    f32x16 sm = zero_f32x16(), dp = zero_f32x16();
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      sm = mfma32(lds_row(smem, ad.row[t] + QO), kf[t], sm);
      dp = mfma32(lds_row(smem, ad.row[t] + GO), vf[t], dp);
    }
    // P[q][key] = exp(S - L_q), dS = P (dP - D^s_q); rows q = 32 qh + c_row(r, g)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      const f32x4 lq = *reinterpret_cast<const f32x4*>(Ls + 32 * qh + 8 * r4 + 4 * g);
      const f32x4 dq = *reinterpret_cast<const f32x4*>(Dq + 32 * qh + 8 * r4 + 4 * g);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float pv = kok ? fast_exp2(fmaf(sm[4 * r4 + r], sl2, -lq[r])) : 0.0f;
        sm[4 * r4 + r] = pv;
        dp[4 * r4 + r] = pv * (dp[4 * r4 + r] - dq[r]);
      }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const bf16x8 pb = c_to_operand(sm, u);
      const bf16x8 sb = c_to_operand(dp, u);
      constexpr int RB = 16 * T::ROW_BYTES;
#pragma unroll
      for (int et = 0; et < NT; ++et) {
        const int o0 = ad.trb[0] + ad.trx[et], o1 = ad.trb[1] + ad.trx[et];
        dvT[et] = mfma32(lds_tr<D>(smem, o0 + GO + u * RB, o1 + GO + u * RB), pb, dvT[et]);   // dO_i^T P
        dkT[et] = mfma32(lds_tr<D>(smem, o0 + QO + u * RB, o1 + QO + u * RB), sb, dkT[et]);   // Q_i^T dS
      }
    }
    if (s + 1 < cnt && tid < 128) stats[(buf ^ 1) * 2 * kBlk + tid] = streg;
  };
  if (cnt > 0) {
    issue(0, 0);
    if (tid < 128) stats[tid] = streg;
  }
  for (int s = 0; s < cnt; s += 2) {
    step(s, 0);
    if (s + 1 < cnt) step(s + 1, 1);
  }
  // ---- add the two query halves, then the linear-branch parts, and store
  __syncthreads();
  float* myx = xch + (size_t)kh * (2 * NT * 16) * 64;
  if (qh == 1) {
#pragma unroll
    for (int et = 0; et < NT; ++et)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        myx[(et * 16 + r) * 64 + l] = dvT[et][r];
        myx[((NT + et) * 16 + r) * 64 + l] = dkT[et][r];
      }
  }
  __syncthreads();
  if (qh == 0 && kok) {
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
// Wave (qh, kh): S^T and dP^T are [key][query], one query per lane, so L and D^s are per-lane
// scalars and dS^T feeds dQ^T = K^T dS^T from registers.  The two kh waves hold partial sums
// over their keys and are added at the end.
template <int D>
__global__ __launch_bounds__(256, 2) void bwd_dq_mfma_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ K, const bf16* __restrict__ V,
    const bf16* __restrict__ dO, const float* __restrict__ L, const float* __restrict__ Ds,
    const int32_t* __restrict__ row_idx, const float* __restrict__ dQlin, int N, int Tn, int n_h,
    float scale, bf16* __restrict__ dQ) {
  using Lds = PairLds<D>;
  constexpr int NT = D / 32, KT = D / 16;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* xch = reinterpret_cast<float*>(smem);
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, g = l >> 5, ln = l & 31;
  const int qh = w & 1, kh = w >> 1;
  const int i = xcd_local_block(blockIdx.x, Tn), bh = blockIdx.y;
  if (i < 0) return;
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
  auto issue = [&](int s) {
    const int jj = lut[s];
    const int cols = min(kBlk, N - jj * kBlk);
    const int off = (s & 1) * Lds::BUF;
    issue_tile_load<D>(Kb + (size_t)jj * kBlk * D, cols, smem, off, w, l);
    issue_tile_load<D>(Vb + (size_t)jj * kBlk * D, cols, smem, off + Lds::TILE, w, l);
  };
  if (n_h > 0) issue(0);
  for (int s = 0; s < n_h; ++s) {
    const int buf = s & 1;
    const int cols = min(kBlk, N - lut[s] * kBlk);
    wait_vm0();
    __syncthreads();
    if (s + 1 < n_h) issue(s + 1);
    const unsigned char* Ks = smem + buf * Lds::BUF;
    const unsigned char* Vs = Ks + Lds::TILE;
    f32x16 sT = zero_f32x16(), dpT = zero_f32x16();
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      sT = mfma32(read_row_swz<D>(Ks, 32 * kh, t, l), qf[t], sT);
      dpT = mfma32(read_row_swz<D>(Vs, 32 * kh, t, l), gf[t], dpT);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float pv = fast_exp2(fmaf(sT[r], sl2, -Lq));
      if (cols < kBlk && 32 * kh + c_row(r, g) >= cols) pv = 0.0f;
      dpT[r] = pv * (dpT[r] - Dq);
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const bf16x8 sb = c_to_operand(dpT, u);
#pragma unroll
      for (int dt = 0; dt < NT; ++dt)
        dqT[dt] = mfma32(read_tr_swz<D>(Ks, 32 * kh + 16 * u, dt, l), sb, dqT[dt]);   // K_j^T dS^T
    }
  }
  __syncthreads();
  float* myx = xch + (size_t)qh * (NT * 16) * 64;
  if (kh == 1) {
#pragma unroll
    for (int dt = 0; dt < NT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) myx[(dt * 16 + r) * 64 + l] = dqT[dt][r];
  }
  __syncthreads();
  if (kh == 0 && qok) {
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
  constexpr int lds = PairLds<D>::BYTES;
  SLA_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_dkdv_mfma_kernel<D>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, lds));
  {
    KernelTimer kt("bwd_sparse_kv", st);
    bwd_dkdv_mfma_kernel<D><<<dim3(s.T * s.BH), 256, lds, st>>>(
        (const bf16*)a.Q, (const bf16*)a.K, (const bf16*)a.V, (const bf16*)a.dO, a.L, Ds, a.col_ptr,
        a.col_rows, a.col_order, dKlin, dVlin, s.N, s.T, s.n_h, s.scale, (bf16*)a.dK, (bf16*)a.dV);
  }
  SLA_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_dq_mfma_kernel<D>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, lds));
  {
    KernelTimer kt("bwd_sparse_q", st);
    bwd_dq_mfma_kernel<D><<<dim3(xcd_grid(s.T), s.BH), 256, lds, st>>>(
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
