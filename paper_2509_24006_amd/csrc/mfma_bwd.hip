// bf16 matrix-core backward kernels for the critical blocks (Algorithm 2, M_c = 1 branch;
// Eq. 7 with the 1/sqrt(d) factor on dQ and dK):
//   bwd_dkdv_mfma  one workgroup per key block j, walking the column table:
//                  dV_j += P^T dO_i, dK_j += dS^T Q_i / sqrt(d)
//   bwd_dq_mfma    one workgroup per query block i, walking the row table:
//                  dQ_i += dS K_j / sqrt(d)   (S, dP are recomputed; no atomics, one owner)
// P = exp(S - L) and dS = P (dP - D^s) are formed in float from MFMA accumulators.
//
// Streaming tiles are staged ROW-MAJOR in LDS once (double-buffered: the next step's tiles are
// in flight in registers during the arithmetic and written to the other buffer before the
// single barrier of a step).  Where a product needs the tile transposed (contraction over its
// rows) the operand is read with the transposing LDS read instead of keeping a second copy.
#include "mfma_common.h"

namespace sla {
namespace {

// Row stride (elements) of a row-major tile that is read both by rows (16-byte reads, one row
// per lane) and transposed: 304 bytes keeps both patterns off the worst bank conflicts.
constexpr int kRS(int D) { return D + 24; }

template <int D>
struct StreamLds {
  static constexpr int RS = kRS(D);
  static constexpr int TILE = kBlk * RS;          // elements of one row-major tile
  static constexpr int STEP = 4 * TILE;           // two pairs x two tensors
  static constexpr int STAT_BYTES = 2 * 2 * 2 * kBlk * 4;   // [buf][tile][L, D^s][64]
  static constexpr int BYTES = 2 * STEP * 2 + STAT_BYTES;
};

// Loads one 64 x D tile (rows beyond `valid_rows` read as zero) into registers / stores it.
template <int D>
__device__ __forceinline__ void load_tile_regs(const bf16* base, int valid_rows, u32x4 (&x)[D / 32]) {
  const __amdgpu_buffer_rsrc_t r = tile_rsrc(base, valid_rows * D * 2);
#pragma unroll
  for (int c = 0; c < D / 32; ++c) x[c] = __builtin_amdgcn_raw_buffer_load_b128(r, (threadIdx.x + 256 * c) * 16, 0, 0);
}

template <int D>
__device__ __forceinline__ void store_tile_regs(bf16* dst, const u32x4 (&x)[D / 32]) {
  constexpr int RS = kRS(D);
#pragma unroll
  for (int c = 0; c < D / 32; ++c) {
    const int ch = threadIdx.x + 256 * c;
    const int row = ch / (D / 8), c8 = ch - row * (D / 8);
    *reinterpret_cast<u32x4*>(dst + row * RS + 8 * c8) = x[c];
  }
}

// ------------------------------------------------------------------ dK, dV
// Wavefront (kh, par): kh = which 32 of the block's 64 keys, par = which of the two query
// tiles of a step.  S and dP are formed as [query][key] so that each lane owns one key; P
// and dS then feed the second products (contraction over queries) straight from registers.
template <int D>
__global__ __launch_bounds__(256) void bwd_dkdv_mfma_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ K, const bf16* __restrict__ V,
    const bf16* __restrict__ dO, const float* __restrict__ L, const float* __restrict__ Ds,
    const int32_t* __restrict__ col_ptr, const int32_t* __restrict__ col_rows,
    const int32_t* __restrict__ col_order, const float* __restrict__ dKlin,
    const float* __restrict__ dVlin, int N, int Tn, int n_h, float scale, bf16* __restrict__ dK,
    bf16* __restrict__ dV) {
  using Lds = StreamLds<D>;
  constexpr int RS = Lds::RS, NT = D / 32, KT = D / 16, CH = D / 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* tiles = reinterpret_cast<bf16*>(smem);
  float* stats = reinterpret_cast<float*>(smem + 2 * Lds::STEP * 2);
  float* xch = reinterpret_cast<float*>(smem);
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, g = l >> 5, ln = l & 31;
  const int kh = w & 1, par = w >> 1;
  // longest column lists first, across all heads: the r-th heaviest key block of every head
  // precedes the (r+1)-th of any head, so the tail of the launch is made of short lists
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
  const int steps = (cnt + 1) >> 1;
  u32x4 qreg[2][CH], greg[2][CH];
  float streg = 0.0f;
  auto load_step = [&](int s) {
    const bool two = 2 * s + 1 < cnt;
    const int i0 = list[beg + 2 * s];
    const int i1 = two ? list[beg + 2 * s + 1] : i0;
    const int r0 = min(kBlk, N - i0 * kBlk), r1 = two ? min(kBlk, N - i1 * kBlk) : 0;
    load_tile_regs<D>(Qb + (size_t)i0 * kBlk * D, r0, qreg[0]);
    load_tile_regs<D>(dOb + (size_t)i0 * kBlk * D, r0, greg[0]);
    load_tile_regs<D>(Qb + (size_t)i1 * kBlk * D, r1, qreg[1]);
    load_tile_regs<D>(dOb + (size_t)i1 * kBlk * D, r1, greg[1]);
    // thread t < 256: tile p = t / 128, kind = (t / 64) % 2 (L or D^s), query t % 64
    const int p = tid >> 7, kind = (tid >> 6) & 1, q = tid & 63;
    const int ii = p ? i1 : i0;
    const bool ok = q < (p ? r1 : r0);
    if (kind == 0) streg = ok ? Lb[ii * kBlk + q] * kLog2e : INFINITY;   // rows past the end give P = 0
    else streg = ok ? Dsb[ii * kBlk + q] : 0.0f;
  };
  auto store_step = [&](int buf) {
    bf16* base = tiles + buf * Lds::STEP;
    store_tile_regs<D>(base, qreg[0]);
    store_tile_regs<D>(base + Lds::TILE, greg[0]);
    store_tile_regs<D>(base + 2 * Lds::TILE, qreg[1]);
    store_tile_regs<D>(base + 3 * Lds::TILE, greg[1]);
    stats[buf * 4 * kBlk + tid] = streg;
  };
  if (steps > 0) {
    load_step(0);
    store_step(0);
  }
  __syncthreads();
  for (int s = 0; s < steps; ++s) {
    const int buf = s & 1;
    const bool two = 2 * s + 1 < cnt;
    if (s + 1 < steps) load_step(s + 1);
    if (par == 0 || two) {
      const bf16* Qs = tiles + buf * Lds::STEP + par * 2 * Lds::TILE;
      const bf16* Gs = Qs + Lds::TILE;
      const float* Ls = stats + buf * 4 * kBlk + par * 2 * kBlk;
      const float* Dq = Ls + kBlk;
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
            const float pv = kok ? fast_exp2(fmaf(sm[mt][4 * r4 + r], sl2, -lq[r])) : 0.0f;
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
          const bf16x8 ag = read_tr_operand(Gs, RS, 16 * u, 32 * et, l);   // dO_i^T
          dvT[et] = mfma32(ag, pb, dvT[et]);
          const bf16x8 aq = read_tr_operand(Qs, RS, 16 * u, 32 * et, l);   // Q_i^T
          dkT[et] = mfma32(aq, sb, dkT[et]);
        }
      }
    }
    if (s + 1 < steps) store_step(buf ^ 1);
    __syncthreads();
  }
  // ---- add the two query-tile streams, then the linear-branch parts, and store
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
__global__ __launch_bounds__(256) void bwd_dq_mfma_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ K, const bf16* __restrict__ V,
    const bf16* __restrict__ dO, const float* __restrict__ L, const float* __restrict__ Ds,
    const int32_t* __restrict__ row_idx, const float* __restrict__ dQlin, int N, int Tn, int n_h,
    float scale, bf16* __restrict__ dQ) {
  using Lds = StreamLds<D>;
  constexpr int RS = Lds::RS, NT = D / 32, KT = D / 16, CH = D / 32;
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
  u32x4 kreg[2][CH], vreg[2][CH];
  auto load_step = [&](int s) {
    const bool two = 2 * s + 1 < n_h;
    const int j0 = lut[2 * s];
    const int j1 = two ? lut[2 * s + 1] : j0;
    const int c0 = min(kBlk, N - j0 * kBlk), c1 = two ? min(kBlk, N - j1 * kBlk) : 0;
    load_tile_regs<D>(Kb + (size_t)j0 * kBlk * D, c0, kreg[0]);
    load_tile_regs<D>(Vb + (size_t)j0 * kBlk * D, c0, vreg[0]);
    load_tile_regs<D>(Kb + (size_t)j1 * kBlk * D, c1, kreg[1]);
    load_tile_regs<D>(Vb + (size_t)j1 * kBlk * D, c1, vreg[1]);
  };
  auto store_step = [&](int buf) {
    bf16* base = tiles + buf * Lds::STEP;
    store_tile_regs<D>(base, kreg[0]);
    store_tile_regs<D>(base + Lds::TILE, vreg[0]);
    store_tile_regs<D>(base + 2 * Lds::TILE, kreg[1]);
    store_tile_regs<D>(base + 3 * Lds::TILE, vreg[1]);
  };
  if (steps > 0) {
    load_step(0);
    store_step(0);
  }
  __syncthreads();
  for (int s = 0; s < steps; ++s) {
    const int buf = s & 1;
    const bool two = 2 * s + 1 < n_h;
    const int jmine = lut[par && two ? 2 * s + 1 : 2 * s];
    const int cols = min(kBlk, N - jmine * kBlk);
    if (s + 1 < steps) load_step(s + 1);
    if (par == 0 || two) {
      const bf16* Ks = tiles + buf * Lds::STEP + par * 2 * Lds::TILE;
      const bf16* Vs = Ks + Lds::TILE;
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
          float pv = fast_exp2(fmaf(sT[mt][r], sl2, -Lq));
          if (cols < kBlk && 32 * mt + c_row(r, g) >= cols) pv = 0.0f;
          dpT[mt][r] = pv * (dpT[mt][r] - Dq);
        }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const bf16x8 sb = c_to_operand(dpT[u >> 1], u & 1);
#pragma unroll
        for (int dt = 0; dt < NT; ++dt) {
          const bf16x8 ak = read_tr_operand(Ks, RS, 16 * u, 32 * dt, l);   // K_j^T
          dqT[dt] = mfma32(ak, sb, dqT[dt]);
        }
      }
    }
    if (s + 1 < steps) store_step(buf ^ 1);
    __syncthreads();
  }
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
  constexpr int lds = StreamLds<D>::BYTES;
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
    bwd_dq_mfma_kernel<D><<<grid, 256, lds, st>>>(
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
