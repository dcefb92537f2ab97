// bf16 matrix-core backward kernels of the linear branch and of Proj (Algorithm 2 first loop and
// last line, Eq. 8, plus the chain rule of Eq. 6 and through phi):
//   bwd_pre_mfma    per query block: dO^l = dO W^T, D^s, D^l, dH_i, dZ_i, dQ^phi_i -> dQ (linear part)
//   bwd_link_mfma   per key block:   dK^phi_j = V_j dH^T + 1 dZ^T -> dK (linear part), dV_j (linear part)
//   dw_mfma         dW = sum_n (O^l_n)^T dO_n, per-workgroup partial sums
// One lane owns one token (query or key) in every product whose result is per token, so the
// row-wise quantities (softmax statistics of phi, D^l, the normaliser phi(Q) Z) are per-lane scalars.
#include "mfma_common.h"

namespace sla {
namespace {

constexpr int kRSl(int D) { return D + 8; }

// Stages a d x d bf16 matrix stored [b][a] (b-major) into LDS transposed, [a][b] (stride RS).
template <int D>
__device__ __forceinline__ void stage_matrix_t(const bf16* __restrict__ src, bf16* dst, int RS) {
  for (int pidx = threadIdx.x; pidx < (D / 4) * (D / 4); pidx += 256) {
    const int a4 = pidx % (D / 4), b4 = pidx / (D / 4);
    u32x2 x[4];
#pragma unroll
    for (int bb = 0; bb < 4; ++bb)
      x[bb] = *reinterpret_cast<const u32x2*>(src + (size_t)(4 * b4 + bb) * D + 4 * a4);
    store_patch_t(dst, RS, 4 * a4, 4 * b4, x);
  }
}

// ------------------------------------------------------------------ query side
template <int D>
struct PreLds {
  static constexpr int RS = kRSl(D);
  static constexpr int G_ELEMS = kBlk * D;      // dO^l row-major [q][b], unpadded, 16-byte chunks swizzled
  static constexpr int GT_ELEMS = D * kVS;      // dO^l transposed [b][q]
  static constexpr int AT_ELEMS = D * kVS;      // (phi(Q)/den)^T [c][q]
  static constexpr int H_ELEMS = D * RS;        // H_i [a][b]; reuses the two transposed tiles
  static_assert(H_ELEMS <= GT_ELEMS + AT_ELEMS, "H_i must fit over the transposed tiles");
  static constexpr int F_OFF = (G_ELEMS + GT_ELEMS + AT_ELEMS) * 2;
  static constexpr int BYTES = F_OFF + 4 * kBlk * 4;   // Dl partial [par][q], dot partial [par][q]
};

// (three workgroups per CU: the kernel is a chain of short phases that wait on memory, and the
// LDS footprint is kept just under a third of a CU's for that)
template <int D>
__global__ __launch_bounds__(256, 3) void bwd_pre_mfma_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ dO, const bf16* __restrict__ W,
    const bf16* __restrict__ Os, const bf16* __restrict__ Ol, const bf16* __restrict__ H16,
    const float* __restrict__ Zs, int N,
    int Tn, int n_0, int phi, float* __restrict__ Ds, bf16* __restrict__ dHZ,
    float* __restrict__ dQlin) {
  using Lds = PreLds<D>;
  constexpr int RS = Lds::RS, NT = D / 32, KT = D / 16, HT = NT / 2;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* Gs = reinterpret_cast<bf16*>(smem);
  bf16* Gt = Gs + Lds::G_ELEMS;
  bf16* At = Gt + Lds::GT_ELEMS;
  bf16* Hs = Gt;   // staged once dH_i, dZ_i no longer need the transposed tiles
  float* dlp = reinterpret_cast<float*>(smem + Lds::F_OFF);   // [par][64]
  float* dotp = dlp + 2 * kBlk;                               // [par][64]
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, g = l >> 5, ln = l & 31;
  const int qh = w & 1, par = w >> 1;
  const int i = blockIdx.x, bh = blockIdx.y;
  const int q0 = i * kBlk, rows = min(kBlk, N - q0);
  const int qrow = qh * 32 + ln;
  const bool qok = qrow < rows;
  const size_t qoff = ((size_t)bh * N + q0 + qrow) * D;
  bf16x8 gf[KT];
#pragma unroll
  for (int t = 0; t < KT; ++t)
    gf[t] = qok ? *reinterpret_cast<const bf16x8*>(dO + qoff + 16 * t + 8 * g) : zero_bf16x8();
  // D^s = rowsum(dO * O^s)
  if (par == 0) {
    float ds = 0.0f;
    if (qok) {
#pragma unroll
      for (int t = 0; t < KT; ++t) {
        const bf16x8 o = *reinterpret_cast<const bf16x8*>(Os + qoff + 16 * t + 8 * g);
#pragma unroll
        for (int s = 0; s < 8; ++s) ds = fmaf((float)gf[t][s], (float)o[s], ds);
      }
    }
    ds = half_sum(ds);
    if (g == 0 && qok) Ds[(size_t)bh * N + q0 + qrow] = ds;
  }
  if (n_0 == 0) return;   // no linear branch: nothing else to do (uniform over the grid)
  const bf16* Hrow = H16 + ((size_t)bh * Tn + i) * (D * D);
  const float* Z = Zs + ((size_t)bh * Tn + i) * D;
  // dO^l^T[b][q] = sum_e W[b][e] dO[q][e]; this wave: b-tiles par*HT .. par*HT+HT-1
  f32x16 gl[HT];
  float dl = 0.0f;
#pragma unroll
  for (int h2 = 0; h2 < HT; ++h2) {
    const int bt = par * HT + h2;
    gl[h2] = zero_f32x16();
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(W + (size_t)(32 * bt + ln) * D + 16 * t + 8 * g);
      gl[h2] = mfma32(a, gf[t], gl[h2]);
    }
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      const int b0 = 32 * bt + 8 * r4 + 4 * g;
      bf16x4 ol4;
      if (qok) ol4 = *reinterpret_cast<const bf16x4*>(Ol + qoff + b0);
      bf16x4 pk;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float v = gl[h2][4 * r4 + r];
        pk[r] = (__bf16)v;
        if (qok) dl = fmaf(v, (float)ol4[r], dl);
        Gt[(b0 + r) * kVS + qrow] = __float2bfloat16(v);
      }
      *reinterpret_cast<bf16x4*>(Gs + qrow * D + (((b0 >> 3) ^ swz<D>(qrow)) << 3) + (b0 & 7)) = pk;
    }
  }
  dl = half_sum(dl);
  if (g == 0) dlp[par * kBlk + qrow] = dl;
  // phi(Q), its normaliser, and a = phi(Q) / den transposed into LDS (this wave: half of the features)
  bf16x8 qf[KT];
#pragma unroll
  for (int t = 0; t < KT; ++t)
    qf[t] = qok ? *reinterpret_cast<const bf16x8*>(Q + qoff + 16 * t + 8 * g) : zero_bf16x8();
  float qmx, qinv;
  phi_stats<KT>(qf, phi, qmx, qinv);
  float den = 0.0f;
  float yq[KT][8];
#pragma unroll
  for (int t = 0; t < KT; ++t) {
    const f32x4 z0 = *reinterpret_cast<const f32x4*>(Z + 16 * t + 8 * g);
    const f32x4 z1 = *reinterpret_cast<const f32x4*>(Z + 16 * t + 8 * g + 4);
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const float y = (float)(__bf16)phi_val((float)qf[t][s], phi, qmx, qinv);
      yq[t][s] = y;
      den = fmaf(y, s < 4 ? z0[s] : z1[s - 4], den);
    }
  }
  den = half_sum(den);
  const float dinv = qok ? 1.0f / den : 0.0f;
#pragma unroll
  for (int t = 0; t < KT; ++t) {
    if ((t >= KT / 2) != (par == 1)) continue;
#pragma unroll
    for (int s = 0; s < 8; ++s) At[(16 * t + 8 * g + s) * kVS + qrow] = __float2bfloat16(yq[t][s] * dinv);
  }
  __syncthreads();
  const float Dl = dlp[qrow] + dlp[kBlk + qrow];
  bf16* out = dHZ + ((size_t)bh * Tn + i) * (D * D + D);
  // dZ_i[c] = - sum_q a[q][c] D^l_q
  if (tid < D) {
    float z = 0.0f;
    for (int q = 0; q < kBlk; ++q)
      z = fmaf(__bfloat162float(At[tid * kVS + q]), dlp[q] + dlp[kBlk + q], z);
    out[(size_t)D * D + tid] = __float2bfloat16(-z);
  }
  // dH_i^T[b][c] = sum_q dO^l[q][b] a[q][c]; wave w owns b-tile w.  The product is formed with b
  // along the lanes (C tile rows = c), so that a lane holds consecutive c of one stored row.
  static_assert(NT <= 4, "one b-tile per wave");
  f32x16 acc[NT];
#pragma unroll
  for (int ct = 0; ct < NT; ++ct) acc[ct] = zero_f32x16();
  if (w < NT) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(Gt + (32 * w + ln) * kVS + 16 * u + 8 * g);
#pragma unroll
      for (int ct = 0; ct < NT; ++ct) {
        const bf16x8 b = *reinterpret_cast<const bf16x8*>(At + (32 * ct + ln) * kVS + 16 * u + 8 * g);
        acc[ct] = mfma32(b, a, acc[ct]);
      }
    }
  }
  __syncthreads();   // the transposed tiles are free: they stage the output rows, then H_i
  static_assert(4 * 32 * (64 * NT + 16) <= (Lds::GT_ELEMS + Lds::AT_ELEMS) * 2, "staging fits over the transposed tiles");
  if (w < NT)
    store_rows_bf16<NT>(reinterpret_cast<unsigned char*>(Gt) + w * (32 * (64 * NT + 16)), acc, out + (size_t)(32 * w) * D, D,
                        32, l);
  __syncthreads();
  stage_matrix_t<D>(Hrow, Hs, RS);
  __syncthreads();
  // dQ^phi^T[c][q] = (sum_b H[c][b] dO^l[q][b] - D^l_q Z[c]) / den_q; this wave: c-tiles of par
  f32x16 dq[HT];
  float dot = 0.0f;
  float yc[HT][16];
#pragma unroll
  for (int h2 = 0; h2 < HT; ++h2) {
    const int ct = par * HT + h2;
    dq[h2] = zero_f32x16();
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(Hs + (32 * ct + ln) * RS + 16 * t + 8 * g);
      const bf16x8 b = *reinterpret_cast<const bf16x8*>(Gs + qrow * D + (((2 * t + g) ^ swz<D>(qrow)) << 3));
      dq[h2] = mfma32(a, b, dq[h2]);
    }
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      const int c0 = 32 * ct + 8 * r4 + 4 * g;
      const f32x4 z4 = *reinterpret_cast<const f32x4*>(Z + c0);
      bf16x4 q4;
#pragma unroll
      for (int r = 0; r < 4; ++r) q4[r] = (__bf16)0.0f;
      if (qok) q4 = *reinterpret_cast<const bf16x4*>(Q + qoff + c0);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float v = (dq[h2][4 * r4 + r] - Dl * z4[r]) * dinv;
        const float x = (float)q4[r];
        const float y = phi == 0 ? phi_val(x, 0, qmx, qinv) : (x > 0.0f ? 1.0f : fast_exp2(x * kLog2e));
        dq[h2][4 * r4 + r] = v;
        yc[h2][4 * r4 + r] = y;
        dot = fmaf(v, y, dot);
      }
    }
  }
  dot = half_sum(dot);
  if (g == 0) dotp[par * kBlk + qrow] = dot;
  __syncthreads();
  const float dtot = phi == 0 ? dotp[qrow] + dotp[kBlk + qrow] : 0.0f;
  if (qok) {
#pragma unroll
    for (int h2 = 0; h2 < HT; ++h2) {
      const int ct = par * HT + h2;
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        f32x4 o4;
#pragma unroll
        for (int r = 0; r < 4; ++r) o4[r] = yc[h2][4 * r4 + r] * (dq[h2][4 * r4 + r] - dtot);
        *reinterpret_cast<f32x4*>(dQlin + qoff + 32 * ct + 8 * r4 + 4 * g) = o4;
      }
    }
  }
}

// ------------------------------------------------------------------ dW partial sums
// dW = sum over tokens of O^l^T dO (gradient of Proj, Eq. 6).  Workgroup g sums over token tiles
// g, g + G, ...; the two tiles of a step come in as LDS tiles, double-buffered, and both operands
// are contracted over tile rows (transposing reads).  Wave w owns rows c in [32 w, 32 w + 32) of dW.
template <int D>
__global__ __launch_bounds__(256, 2) void dw_mfma_kernel(const bf16* __restrict__ Ol,
                                                         const bf16* __restrict__ dO, int BH, int N,
                                                         int Tn, float* __restrict__ part) {
  using T = SwzTile<D>;
  constexpr int NT = D / 32;
  constexpr int BUF = 2 * T::BYTES;
  constexpr int RB = 16 * T::ROW_BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * BUF];
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, g = l >> 5, ln = l & 31;
  const int ldv = tile_lane_offset<D>(w, l);
  const unsigned lds0 = lds_base(smem) + wave_uniform(w) * 1024;
  f32x16 acc[NT];
#pragma unroll
  for (int et = 0; et < NT; ++et) acc[et] = zero_f32x16();
  const int total = BH * Tn;
  auto issue = [&](int t, int buf) {
    const int bh = t / Tn, i = t - bh * Tn;
    const int rows = min(kBlk, N - i * kBlk);
    const size_t base = ((size_t)bh * N + (size_t)i * kBlk) * D;
    issue_tile_load<D>(Ol + base, rows, lds0, buf * BUF, ldv);
    issue_tile_load<D>(dO + base, rows, lds0, buf * BUF + T::BYTES, ldv);
  };
  TileAddr<D> ad;
  ad.init(0, l);
  if ((int)blockIdx.x < total) issue(blockIdx.x, 0);
  int buf = 0;
  for (int t = blockIdx.x; t < total; t += gridDim.x) {
    wait_vm0();
    __syncthreads();   // this step's tiles have landed; the other buffer is fully consumed
    if (t + (int)gridDim.x < total) issue(t + gridDim.x, buf ^ 1);
    const int off = buf * BUF;
    buf ^= 1;
    if (w < NT) {
#pragma unroll
      for (int u = 0; u < kBlk / 16; ++u) {
        const bf16x8 a = lds_tr<D>(smem, ad.tr(0, w) + off + u * RB, ad.tr(1, w) + off + u * RB);   // O^l^T rows c
#pragma unroll
        for (int et = 0; et < NT; ++et) {
          const bf16x8 b = lds_tr<D>(smem, ad.tr(0, et) + off + T::BYTES + u * RB, ad.tr(1, et) + off + T::BYTES + u * RB);
          acc[et] = mfma32(a, b, acc[et]);
        }
      }
    }
  }
  if (w < NT) {
    float* out = part + (size_t)blockIdx.x * D * D;
#pragma unroll
    for (int et = 0; et < NT; ++et)
#pragma unroll
      for (int r = 0; r < 16; ++r) out[(size_t)(32 * w + c_row(r, g)) * D + 32 * et + ln] = acc[et][r];
  }
}

#define SLA_TRY(x)                   \
  do {                               \
    hipError_t e_ = (x);             \
    if (e_ != hipSuccess) return e_; \
  } while (0)

template <int D>
hipError_t pre_impl(const Shape& s, const BwdArgs& a, float* Ds, bf16* dHZ, float* dQlin,
                    float* dWpart, int nparts, hipStream_t st) {
  constexpr int lds = PreLds<D>::BYTES;
  SLA_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_pre_mfma_kernel<D>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, lds));
  {
    KernelTimer kt("bwd_pre", st);
    bwd_pre_mfma_kernel<D><<<dim3(s.T, s.BH), 256, lds, st>>>(
        (const bf16*)a.Q, (const bf16*)a.dO, (const bf16*)a.W, (const bf16*)a.Os, (const bf16*)a.Ol,
        (const bf16*)a.HZ, (const float*)((const char*)a.HZ + state_z_offset(s)), s.N, s.T, s.n_0, s.phi,
        Ds, dHZ, dQlin);
  }
  {
    KernelTimer kt("dw_partial", st);
    dw_mfma_kernel<D><<<nparts, 256, 0, st>>>((const bf16*)a.Ol, (const bf16*)a.dO, s.BH, s.N, s.T, dWpart);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t mfma_backward_pre(const Shape& s, const BwdArgs& a, float* Ds, void* dHZ16, float* dQlin,
                             float* dWpart, int nparts, hipStream_t st) {
  bf16* dHZ = reinterpret_cast<bf16*>(dHZ16);
  return s.d == 64 ? pre_impl<64>(s, a, Ds, dHZ, dQlin, dWpart, nparts, st)
                   : pre_impl<128>(s, a, Ds, dHZ, dQlin, dWpart, nparts, st);
}

}  // namespace sla
