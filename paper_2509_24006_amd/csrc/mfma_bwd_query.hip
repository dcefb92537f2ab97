// bf16 matrix-core backward kernels of the query side (Algorithm 2 first loop, Eq. 8 and the chain
// rule of Eq. 6 and through phi; Eq. 7's dQ) and of Proj:
//   pre_body        per query block: dO^l = dO W^T, D^s, D^l, dH_i, dZ_i, dQ^phi_i -> dQ (linear part)
//                   (the key-side counterpart is the prologue of the dK/dV kernel)
//   bwd_dq_mfma     one workgroup per query block i, walking the row table:
//                   dQ_i += dS K_j / sqrt(d)   (S, dP are recomputed; no atomics, one owner);
//                   with query blocks of one tile it runs pre_body first, in the same launch
//   dw_mfma         dW = sum_n (O^l_n)^T dO_n, per-workgroup partial sums
// One lane owns one token (query or key) in every product whose result is per token, so the
// row-wise quantities (softmax statistics of phi, D^l, the normaliser phi(Q) Z) are per-lane scalars.
#include "mfma_common.h"

namespace sla {
namespace {

// ------------------------------------------------------------------ query side
// Per query block i (Alg. 2, first loop; Eq. 8 and the chain rule of Eq. 6):
//   D^s = rowsum(dO * O^s);  dO^l = dO W^T;  D^l = rowsum(dO^l * O^l);  a = phi(Q) / (phi(Q) Z_i)
//   dH_i = a^T dO^l (stored transposed, [b][c]);  dZ_i = -a^T D^l
//   dQ^phi = (dO^l H_i^T - D^l Z_i^T) / (phi(Q) Z_i), then through the Jacobian of phi
// Every input tile (dO, O^s, O^l, Q, H_i) comes in as an LDS tile; dO^l and a are written back as
// row-major tiles so that products contracted over the queries read them with the transposing
// read; dH rows and the dQ part leave as whole rows.
template <int D>
struct PreLds {
  static constexpr int TILE = SwzTile<D>::BYTES;
  // slots: 0 dO, then dO^l | 1 O^s, then a, then rows 64.. of H_i | 2 O^l, then rows 0..63 of H_i | 3 Q
  // (a fifth slot for H_i would let all of it arrive early, but 5 tiles + 1 KB is just over half a CU's LDS)
  static constexpr int F_OFF = 4 * TILE;
  static constexpr int BYTES = F_OFF + 4 * kBlk * 4 + D * 4;   // D^l partial [par][q], dot partial [par][q], Z_i
  static constexpr int STG = 32 * (64 * (D / 32) + 16);   // staging of one wave, laid over slots 1..3
  static_assert(4 * STG <= 3 * TILE, "output staging fits over three slots");
};

// FUSED: the body runs as the prologue of the row-wise dQ kernel (below) for the same query block.
// It then leaves the block's Q and dO operand fragments (qf, gf), every lane's D^s (ds_lane) and the
// linear-branch part of dQ (lin: this wave's half of the features, in the register layout of the
// dQ^T accumulators) in registers instead of writing that part to memory.
template <int D, bool FUSED>
__device__ __forceinline__ void pre_body(
    unsigned char* smem, const int i, const int bh,
    const bf16* __restrict__ Q, const bf16* __restrict__ dO, const bf16* __restrict__ W,
    const bf16* __restrict__ Os, const bf16* __restrict__ Ol, const bf16* __restrict__ H16,
    const float* __restrict__ Zs, int N,
    int Tn, Lay lay, int n_0, int phi, float* __restrict__ Ds, bf16* __restrict__ dHZ,
    bf16* __restrict__ dQlin, bf16x8 (&qf)[D / 16], bf16x8 (&gf)[D / 16], float& ds_lane, f32x16 (&lin)[D / 64]) {
  using Lds = PreLds<D>;
  using T = SwzTile<D>;
  constexpr int NT = D / 32, KT = D / 16, HT = NT / 2;
  constexpr int RB = 16 * T::ROW_BYTES;
  constexpr int S0 = 0, S1 = Lds::TILE, S2 = 2 * Lds::TILE, S3 = 3 * Lds::TILE;
  float* dlp = reinterpret_cast<float*>(smem + Lds::F_OFF);   // [par][64]
  float* dotp = dlp + 2 * kBlk;                               // [par][64]
  float* zl = dotp + 2 * kBlk;                                // Z_i [D]
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, g = l >> 5, ln = l & 31;
  const int qh = w & 1, par = w >> 1;
  const int q0 = i * kBlk, rows = min(kBlk, N - q0);
  const int qrow = qh * 32 + ln;
  const bool qok = qrow < rows;
  const size_t base = ((size_t)bh * N + q0) * D;
  const int ldv = tile_lane_offset<D>(w, l);
  const int wu = wave_uniform(w);
  const unsigned lds0 = lds_base(smem) + wu * 1024;
  const bf16* Hrow = H16 + ((size_t)bh * Tn + i) * (D * D);   // stored [b][c] = H_i[c][b]
  TileLoader<D> tl;   // tiles of the caller's dO and Q (base: the library's own packed tensors)
  tl.init(lds_base(smem), w, l, 2 * lay.ts);
  tl.load(head_rsrc<D>(dO + lay.head(bh), N, 2 * lay.ts), i, S0);
  issue_tile_load<D>(Os + base, rows, lds0, S1, ldv);
  if (n_0 > 0) issue_tile_load<D>(Ol + base, rows, lds0, S2, ldv);
  if (n_0 > 0 || FUSED) tl.load(head_rsrc<D>(Q + lay.head(bh), N, 2 * lay.ts), i, S3);
  // rows of W for this wave's dO^l tiles, and Z_i, requested together with the tiles
  bf16x8 wfr[HT][KT];
  if (n_0 > 0) {
#pragma unroll
    for (int h2 = 0; h2 < HT; ++h2)
#pragma unroll
      for (int t = 0; t < KT; ++t)
        wfr[h2][t] = *reinterpret_cast<const bf16x8*>(W + (size_t)(32 * (par * HT + h2) + ln) * D + 16 * t + 8 * g);
    if (tid < D) zl[tid] = Zs[((size_t)bh * Tn + i) * D + tid];
  }
  wait_vm0_known();   // (known to the compiler: it then adds no waits of its own for the W rows, which
                      // would also wait for the D^s store below)
  __syncthreads();
  TileAddr<D> qa;   // rows 32 qh + ln of a tile
  qa.init(32 * qh, l);
#pragma unroll
  for (int t = 0; t < KT; ++t) gf[t] = lds_row(smem, qa.row(t) + S0);
  // D^s = rowsum(dO * O^s) (every wave needs it when the dQ loop follows; one of a query's two writes it)
  ds_lane = 0.0f;
  if (par == 0 || FUSED) {
    float ds = 0.0f;
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      const bf16x8 o = lds_row(smem, qa.row(t) + S1);
#pragma unroll
      for (int s = 0; s < 8; ++s) ds = fmaf((float)gf[t][s], (float)o[s], ds);
    }
    ds = half_sum(ds);
    if (par == 0 && g == 0 && qok) Ds[(size_t)bh * N + q0 + qrow] = ds;
    ds_lane = ds;
  }
  if (n_0 > 0 || FUSED) {
#pragma unroll
    for (int t = 0; t < KT; ++t) qf[t] = lds_row(smem, qa.row(t) + S3);
  }
  if (n_0 == 0) {   // no linear branch: nothing else to do (uniform over the grid)
#pragma unroll
    for (int h2 = 0; h2 < HT; ++h2) lin[h2] = zero_f32x16();
    return;
  }
  __syncthreads();   // dO and O^s are consumed: their slots take dO^l and a
  const int rowb = qrow * T::ROW_BYTES, rsw = swz<D>(qrow);
  // dO^l^T[b][q] = sum_e W[b][e] dO[q][e]; this wave: b-tiles par*HT .. par*HT+HT-1
  float dl = 0.0f;
#pragma unroll
  for (int h2 = 0; h2 < HT; ++h2) {
    const int bt = par * HT + h2;
    f32x16 gl = zero_f32x16();
#pragma unroll
    for (int t = 0; t < KT; ++t) gl = mfma32(wfr[h2][t], gf[t], gl);
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      const int b0 = 32 * bt + 8 * r4 + 4 * g;
      const int off = rowb + (((b0 >> 3) ^ rsw) << 4) + (b0 & 7) * 2;
      const bf16x4 ol4 = *reinterpret_cast<const bf16x4*>(smem + S2 + off);
      bf16x4 pk;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        // D^l from the same rounded dO^l that enters the products below: in
        // dO^l H_i^T - D^l Z_i^T the two terms nearly cancel, and a dO^l that differed between
        // them by its rounding would leave an error of the size of the terms, not of the result
        pk[r] = (__bf16)gl[4 * r4 + r];
        dl = fmaf((float)pk[r], (float)ol4[r], dl);
      }
      *reinterpret_cast<bf16x4*>(smem + S0 + off) = pk;
    }
  }
  dl = half_sum(dl);
  if (g == 0) dlp[par * kBlk + qrow] = dl;
  // phi(Q), its normaliser, and a = phi(Q) / den as a row-major tile (this wave: half of the features)
  float qmx = 0.0f, qinv = 1.0f;
  float den = 0.0f;
  float yq[KT][8];
  if (phi == 0) {   // softmax over the features: the exponentials are formed once
    qmx = -INFINITY;
#pragma unroll
    for (int t = 0; t < KT; ++t)
#pragma unroll
      for (int s = 0; s < 8; ++s) qmx = fmaxf(qmx, (float)qf[t][s]);
    qmx = half_max(qmx);
    float sum = 0.0f;
#pragma unroll
    for (int t = 0; t < KT; ++t)
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        yq[t][s] = fast_exp2(((float)qf[t][s] - qmx) * kLog2e);
        sum += yq[t][s];
      }
    sum = half_sum(sum);
    qinv = 1.0f / sum;
  }
#pragma unroll
  for (int t = 0; t < KT; ++t) {
    const f32x4 z0 = *reinterpret_cast<const f32x4*>(zl + 16 * t + 8 * g);
    const f32x4 z1 = *reinterpret_cast<const f32x4*>(zl + 16 * t + 8 * g + 4);
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const float x = (float)qf[t][s];
      const float y = (float)(__bf16)(phi == 0 ? yq[t][s] * qinv : (x > 0.0f ? x + 1.0f : fast_exp2(x * kLog2e)));
      yq[t][s] = y;
      den = fmaf(y, s < 4 ? z0[s] : z1[s - 4], den);
    }
  }
  den = half_sum(den);
  const float dinv = qok ? 1.0f / den : 0.0f;
#pragma unroll
  for (int t = 0; t < KT; ++t) {
    if ((t >= KT / 2) != (par == 1)) continue;
    bf16x8 av;
#pragma unroll
    for (int s = 0; s < 8; ++s) av[s] = (__bf16)(yq[t][s] * dinv);
    *reinterpret_cast<bf16x8*>(smem + S1 + rowb + (((2 * t + g) ^ rsw) << 4)) = av;
  }
  __syncthreads();   // dO^l and a are complete; O^l is consumed: its slot takes rows 0..63 of H_i
  issue_tile_load<D>(Hrow, min(kBlk, D), lds0, S2, ldv);
  const float Dl = dlp[qrow] + dlp[kBlk + qrow];
  bf16* out = dHZ + ((size_t)bh * Tn + i) * (D * D + D);
  // dH_i^T[b][c] = sum_q dO^l[q][b] a[q][c]: both operands contracted over tile rows; formed with b
  // along the lanes (C tile rows = c), so that a lane holds consecutive c of one stored row.
  // Wave w owns b-tile w.  dZ_i[c] = - sum_q a[q][c] D^l_q rides along as one more column: the wave
  // multiplies its own c-tile of a^T by D^l (in the k order of the transposing read).
  static_assert(NT <= 4, "one b-tile per wave");
  TileAddr<D> ad;
  ad.init(0, l);
  f32x16 acc[NT];
#pragma unroll
  for (int ct = 0; ct < NT; ++ct) acc[ct] = zero_f32x16();
  if (w < NT) {
    f32x16 zacc = zero_f32x16();
#pragma unroll
    for (int u = 0; u < kBlk / 16; ++u) {
      const bf16x8 bo = lds_tr<D>(smem, ad.tr(0, w) + S0 + u * RB, ad.tr(1, w) + S0 + u * RB);
      // slots 0..3: queries 16 u + 4 g .., slots 4..7: queries 16 u + 8 + 4 g ..; D^l as the sum of two
      // bf16 values (the terms of dZ cancel: one bf16 value per D^l would not do)
      bf16x8 dlb, dlc;
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const int qq = 16 * u + 4 * g + (s & 3) + 2 * (s & 4);
        const float v = dlp[qq] + dlp[kBlk + qq];
        dlb[s] = (__bf16)v;
        dlc[s] = (__bf16)(v - (float)dlb[s]);
      }
#pragma unroll
      for (int ct = 0; ct < NT; ++ct) {
        const bf16x8 ao = lds_tr<D>(smem, ad.tr(0, ct) + S1 + u * RB, ad.tr(1, ct) + S1 + u * RB);
        acc[ct] = mfma32(ao, bo, acc[ct]);
        if (ct == w) zacc = mfma32(ao, dlc, mfma32(ao, dlb, zacc));   // every column of this tile: sum_q a[q][c] D^l_q
      }
    }
    if (ln == 0) {
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        bf16x4 pk;
#pragma unroll
        for (int r = 0; r < 4; ++r) pk[r] = (__bf16)(-zacc[4 * r4 + r]);
        *reinterpret_cast<bf16x4*>(out + (size_t)D * D + 32 * w + 8 * r4 + 4 * g) = pk;
      }
    }
  }
  __syncthreads();   // a is consumed: its slot takes the other rows of H_i
  if (D > kBlk) issue_tile_load<D>(Hrow + (size_t)kBlk * D, D - kBlk, lds0, S1, ldv);
  wait_vm0();
  __syncthreads();
  // dQ^phi^T[c][q] = (sum_b H[c][b] dO^l[q][b] - D^l_q Z[c]) / den_q; this wave: c-tiles of par.  H^T is
  // read with the transposing read, whose k order is the one a C tile hands over, so dO^l is picked
  // up in that order too (two 8-byte pieces per k-step: features 16 t + 4 g .. and 16 t + 8 + 4 g ..)
  f32x16 dq[HT];
  float dot = 0.0f;
  float yc[HT][16];
#pragma unroll
  for (int h2 = 0; h2 < HT; ++h2) dq[h2] = zero_f32x16();
#pragma unroll
  for (int t = 0; t < KT; ++t) {
    const bf16x4 v0 = *reinterpret_cast<const bf16x4*>(smem + S0 + rowb + (((2 * t) ^ rsw) << 4) + 8 * g);
    const bf16x4 v1 = *reinterpret_cast<const bf16x4*>(smem + S0 + rowb + (((2 * t + 1) ^ rsw) << 4) + 8 * g);
    bf16x8 gb;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      gb[e] = v0[e];
      gb[4 + e] = v1[e];
    }
    const int mbase = (t / 4 ? S1 : S2) + (t % 4) * RB;   // rows b = 16 t .. of the stored matrix
#pragma unroll
    for (int h2 = 0; h2 < HT; ++h2) {
      const int ct = par * HT + h2;
      dq[h2] = mfma32(lds_tr<D>(smem, ad.tr(0, ct) + mbase, ad.tr(1, ct) + mbase), gb, dq[h2]);
    }
  }
#pragma unroll
  for (int h2 = 0; h2 < HT; ++h2) {
    const int ct = par * HT + h2;
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      const int c0 = 32 * ct + 8 * r4 + 4 * g;
      const f32x4 z4 = *reinterpret_cast<const f32x4*>(zl + c0);
      const bf16x4 q4 = *reinterpret_cast<const bf16x4*>(smem + S3 + rowb + (((c0 >> 3) ^ rsw) << 4) + (c0 & 7) * 2);
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
  __syncthreads();   // also: every wave is done with the tiles, slots 1..3 become the output staging
  const float dtot = phi == 0 ? dotp[qrow] + dotp[kBlk + qrow] : 0.0f;
  unsigned char* stage = smem + S1 + wu * Lds::STG;
  if (w < NT) store_rows_bf16<NT>(stage, acc, out + (size_t)(32 * w) * D, D, 32, l);
#pragma unroll
  for (int h2 = 0; h2 < HT; ++h2)
#pragma unroll
    for (int r = 0; r < 16; ++r) lin[h2][r] = yc[h2][r] * (dq[h2][r] - dtot);
  // (bf16: the row-wise kernel adds this part to its float sum and rounds once more; a float
  // round trip would move 2 x 4 bytes per element instead of 2 x 2)
  if (!FUSED) store_rows_bf16<HT>(stage, lin, dQlin + base + (size_t)(32 * qh) * D + par * (D / 2), D, rows - 32 * qh, l);
}

// The query side on its own (query blocks of several tiles, whose dQ kernel shares a workgroup
// between two tiles): one workgroup per 64-token tile.
template <int D>
__global__ __launch_bounds__(256, 2) void bwd_pre_mfma_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ dO, const bf16* __restrict__ W,
    const bf16* __restrict__ Os, const bf16* __restrict__ Ol, const bf16* __restrict__ H16,
    const float* __restrict__ Zs, int N,
    int Tn, Lay lay, int n_0, int phi, float* __restrict__ Ds, bf16* __restrict__ dHZ,
    bf16* __restrict__ dQlin) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16x8 qf[D / 16], gf[D / 16];
  f32x16 lin[D / 64];
  float ds;
  pre_body<D, false>(smem, blockIdx.x, blockIdx.y, Q, dO, W, Os, Ol, H16, Zs, N, Tn, lay, n_0, phi, Ds, dHZ, dQlin, qf,
                     gf, ds, lin);
}

// LDS of the row-wise dQ kernel: two pair buffers (K_j and V_j of the step in use and of the next
// one); Q_i and dO_i come in through the second buffer before the loop, the output staging is laid
// over the buffers after it.
template <int D>
struct PairLds {
  static constexpr int TILE = SwzTile<D>::BYTES;
  static constexpr int BUF = 2 * TILE;                   // the two tiles of a pair
  static constexpr int BYTES = 2 * BUF;
  static constexpr int SP = D + 4;                        // row pitch (floats) of the output staging
  static_assert(kBlk * SP * 4 <= BYTES, "the output staging of a tile fits over the pair buffers");
  // the second group of an eight-wave workgroup: its Q_i, dO_i tiles, later its output staging
  static constexpr int GROUP = (kBlk * SP * 4 > BUF ? kBlk * SP * 4 : BUF);
};

// ------------------------------------------------------------------ dQ
// Wave (qh, kh): S^T and dP^T are [key][query], one query per lane, so L and D^s are per-lane
// scalars and dS^T feeds dQ^T = K^T dS^T from registers.  The two kh waves hold partial sums
// over their keys and are added at the end.
// QT = 2 (query blocks of 128 or 256 tokens): two adjacent 64-query tiles, which walk the same
// list of key blocks, share a workgroup of eight waves and every K_j, V_j tile it fetches; each
// group of four waves has an LDS area of its own for its Q_i, dO_i tiles and its output staging
// (the second group's lies behind the pair buffers).
// FUSED (QT = 1): the workgroup first runs the query side of the linear branch for its query block
// (pre_body above: D^s, dH_i, dZ_i, the linear part of dQ) and then walks the row list.  The two
// parts want the same tiles (Q_i, dO_i), the linear part of dQ becomes the start value of the
// accumulators instead of a round trip through memory, and one launch less.
struct PreArgs {
  const bf16 *W, *Os, *Ol, *H16;
  const float* Zs;
  int n_0, phi;
  float* Ds_out;
  bf16* dHZ;
};
template <int D, int QT, bool FUSED>
__global__ __launch_bounds__(256 * QT, QT == 1 ? (D == 64 ? 3 : 2) : 1) void bwd_dq_mfma_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ K, const bf16* __restrict__ V,
    const bf16* __restrict__ dO, const float* __restrict__ L, const float* __restrict__ Ds,
    const int32_t* __restrict__ row_idx, const bf16* __restrict__ dQlin, int N, int Tn, Lay lay, int n_h,
    float scale, bf16* __restrict__ dQ, PreArgs pa) {
  static_assert(!FUSED || QT == 1, "the fused form has one query tile per workgroup");
  using Lds = PairLds<D>;
  using T = SwzTile<D>;
  constexpr int NT = D / 32, KT = D / 16;
  constexpr int RB = 16 * T::ROW_BYTES;
  constexpr int NW = 4 * QT;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int wall = threadIdx.x >> 6, l = threadIdx.x & 63, g = l >> 5, ln = l & 31;
  const int grp = QT == 1 ? 0 : wave_uniform(wall >> 2), w = wall & 3, tid = threadIdx.x & 255;
  const int qh = w & 1, kh = w >> 1;
  const int ib = xcd_local_block(blockIdx.x, (Tn + QT - 1) / QT), bh = blockIdx.y;
  if (ib < 0) return;
  // (a last block of a single tile: the second group runs along with no valid query and stores nothing)
  const int i = QT * ib + grp;
  // group 0 takes Q_i, dO_i in through the second pair buffer and stages its output over the pair
  // buffers; group 1 has DqLds<D>::GROUP bytes behind them for both
  unsigned char* gsm = smem + (grp ? Lds::BYTES - Lds::BUF : 0);
  const int q0 = i * kBlk, rows = max(0, min(kBlk, N - q0));
  const int qrow = qh * 32 + ln;
  const bool qok = qrow < rows;
  const int32_t* lut = row_idx + ((size_t)bh * Tn + QT * ib) * n_h;   // the same list for every tile of the block
  const float sl2 = scale * kLog2e;
  bf16x8 qf[KT], gf[KT];
  f32x16 lin[NT / 2];
  float ds_pre = 0.0f;
  if constexpr (FUSED) {
    // (the first part's own copies of the Q and dO fragments are not kept: holding them across it
    // costs more registers than the loop below leaves, and the tiles come back from the L2 together
    // with the first K, V pair)
    bf16x8 qf0[KT], gf0[KT];
    pre_body<D, true>(smem, i, bh, Q, dO, pa.W, pa.Os, pa.Ol, pa.H16, pa.Zs, N, Tn, lay, pa.n_0, pa.phi, pa.Ds_out,
                      pa.dHZ, nullptr, qf0, gf0, ds_pre, lin);
    __syncthreads();   // every wave is done with the first part's tiles and staging areas
  }
  TileLoader<D, NW> tl;   // K_j, V_j: all waves of the workgroup
  TileLoader<D> tq;       // Q_i, dO_i: the four waves of a group, into the group's area
  tl.init(lds_base(smem), wall, l, 2 * lay.ts);
  tq.init(lds_base(smem) + (grp ? Lds::BYTES - Lds::BUF : 0), w, l, 2 * lay.ts);
  const BufDesc descK = head_rsrc<D>(K + lay.head(bh), N, 2 * lay.ts);
  const BufDesc descV = head_rsrc<D>(V + lay.head(bh), N, 2 * lay.ts);
  // key block indices of steps s, s + 1, s + 2, fetched a step before the loads that need them
  int j0 = 0, j1 = 0, j2 = 0;
  auto issue = [&](int jj, const int bufi) __attribute__((always_inline)) {
    tl.load(descK, jj, bufi * Lds::BUF);
    tl.load(descV, jj, bufi * Lds::BUF + Lds::TILE);
  };
  // Q_i and dO_i come in as tiles through the second pair buffer (whole rows per load, zeros past
  // the end of the sequence) and are picked up from there in operand layout
  {
    const int it = min(i, Tn - 1);
    tq.load(head_rsrc<D>(Q + lay.head(bh), N, 2 * lay.ts), it, Lds::BUF);
    tq.load(head_rsrc<D>(dO + lay.head(bh), N, 2 * lay.ts), it, Lds::BUF + Lds::TILE);
  }
  if (n_h > 0) {
    j0 = lut[0];
    j1 = lut[min(1, n_h - 1)];
    j2 = lut[min(2, n_h - 1)];
    issue(j0, 0);
  }
  const float Lq = qok ? L[(size_t)bh * N + q0 + qrow] * kLog2e : INFINITY;
  float nDq;
  f32x16 dqT[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) dqT[t] = zero_f32x16();
  if constexpr (FUSED) {
    nDq = qok ? -ds_pre : 0.0f;
    // the linear part of dQ, this wave's half of the features, as the start value of those
    // accumulators (the sum is multiplied by 1/sqrt(d) at the end)
    const float rscale = 1.0f / scale;
#pragma unroll
    for (int dt = 0; dt < NT; ++dt) {
      const bool mine = dt / (NT / 2) == kh;   // (no run-time index into the accumulator array)
#pragma unroll
      for (int r = 0; r < 16; ++r) dqT[dt][r] = mine ? lin[dt % (NT / 2)][r] * rscale : 0.0f;
    }
  } else {
    nDq = qok ? -Ds[(size_t)bh * N + q0 + qrow] : 0.0f;
  }
  wait_vm0();
  __syncthreads();
  {
    TileAddr<D> qa;
    qa.init(32 * qh, l);
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      qf[t] = lds_row(gsm, qa.row(t) + Lds::BUF);
      gf[t] = lds_row(gsm, qa.row(t) + Lds::BUF + Lds::TILE);
    }
  }
#pragma unroll
  for (int t = 0; t < KT; ++t) {
    pin_loaded(qf[t]);
    pin_loaded(gf[t]);
  }
  // (the first step's barrier orders these reads before the loads that reuse the buffer)
  TileAddr<D> ad;   // this wave reads rows 32 kh .. of K_j and V_j
  ad.init(32 * kh, l);
  auto step = [&](int s, const int buf) __attribute__((always_inline)) {
    const int KO = buf * Lds::BUF, VO = KO + Lds::TILE;
    const int cols = min(kBlk, N - j0 * kBlk);
    const int j3 = lut[min(s + 3, n_h - 1)];
    ad.refresh();
    wait_vm0();
    __syncthreads();   // tiles of step s have landed for every wave; step s-1 is fully consumed
    if (s + 1 < n_h) issue(j1, buf ^ 1);
    // all LDS reads of the first two products up front, then the products
    bf16x8 ka[KT], va[KT], ta[2][NT];
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      ka[t] = lds_row(smem, ad.row(t) + KO);
      va[t] = lds_row(smem, ad.row(t) + VO);
    }
    sched_fence();
    // a lane's 16 entries of dP^T belong to its one query: the accumulator starts at -D^s of that
    // query instead of zero and comes out as dP - D^s
    f32x16 sT = zero_f32x16(), dpT;
#pragma unroll
    for (int r = 0; r < 16; ++r) dpT[r] = nDq;
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      sT = mfma32(ka[t], qf[t], sT);
      dpT = mfma32(va[t], gf[t], dpT);
    }
    // K_j^T for the third product arrives under the softmax arithmetic
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int dt = 0; dt < NT; ++dt)
        ta[u][dt] = lds_tr<D>(smem, ad.tr(0, dt) + KO + u * RB, ad.tr(1, dt) + KO + u * RB);
    sched_fence();
#pragma unroll
    for (int r = 0; r < 16; ++r) sT[r] = fast_exp2(fmaf(sT[r], sl2, -Lq));
    // keys past the end of the sequence (last key block only): P = 0.  A branch of the whole wave,
    // taken on one step per row at most; written into the exponential loop it costs three vector
    // instructions per score on every step.
    if (wave_uniform(cols) < kBlk) {
      int first_invalid = wave_uniform(cols - 32 * kh);   // (opaque to the compiler: the comparisons below stay inside the branch)
      asm volatile("" : "+s"(first_invalid));
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (c_row(r, g) >= first_invalid) sT[r] = 0.0f;
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) dpT[r] = sT[r] * dpT[r];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const bf16x8 sb = c_to_operand(dpT, u);
#pragma unroll
      for (int dt = 0; dt < NT; ++dt) dqT[dt] = mfma32(ta[u][dt], sb, dqT[dt]);   // K_j^T dS^T
    }
    j0 = j1;
    j1 = j2;
    j2 = j3;
  };
  for (int s = 0; s < n_h; s += 2) {
    step(s, 0);
    if (s + 1 < n_h) step(s + 1, 1);
  }
  // ---- add the two key halves in a row-major staging area, then every thread takes 16-byte
  // pieces of whole rows: adds the linear-branch part and stores (coalesced both ways).  The
  // linear-branch pieces are requested first, all at once, and arrive under the exchange.
  constexpr int C4 = D / 4;                  // 16-byte pieces per row
  constexpr int NIT = kBlk * C4 / 256;       // pieces per thread
  bf16x4 lq[NIT];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int idx = it * 256 + tid, row = idx / C4, c4 = idx % C4;
#pragma unroll
    for (int r = 0; r < 4; ++r) lq[it][r] = (__bf16)0.0f;
    if (dQlin && row < rows)   // (the library's own tensor: packed bf16 rows)
      lq[it] = *reinterpret_cast<const bf16x4*>(dQlin + ((size_t)bh * N + q0 + row) * D + 4 * c4);
  }
  __syncthreads();   // every wave is done with the tiles
  constexpr int SP = Lds::SP;
  float* stg = reinterpret_cast<float*>(grp ? gsm + Lds::BUF : smem);   // [64 queries][SP]
  const int srow = qrow * SP + 4 * g;
  if (kh == 1) {
#pragma unroll
    for (int dt = 0; dt < NT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4)
        *reinterpret_cast<f32x4*>(stg + srow + 32 * dt + 8 * r4) =
            f32x4{dqT[dt][4 * r4], dqT[dt][4 * r4 + 1], dqT[dt][4 * r4 + 2], dqT[dt][4 * r4 + 3]};
  }
  __syncthreads();
  if (kh == 0) {
#pragma unroll
    for (int dt = 0; dt < NT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        f32x4 a = *reinterpret_cast<const f32x4*>(stg + srow + 32 * dt + 8 * r4);
#pragma unroll
        for (int r = 0; r < 4; ++r) a[r] += dqT[dt][4 * r4 + r];
        *reinterpret_cast<f32x4*>(stg + srow + 32 * dt + 8 * r4) = a;
      }
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int idx = it * 256 + tid, row = idx / C4, c4 = idx % C4;
    if (row < rows) {
      const f32x4 sv = *reinterpret_cast<const f32x4*>(stg + row * SP + 4 * c4);
      bf16x4 pk;
#pragma unroll
      for (int r = 0; r < 4; ++r) pk[r] = (__bf16)(sv[r] * scale + (float)lq[it][r]);
      *reinterpret_cast<bf16x4*>(dQ + lay.head(bh) + (size_t)(q0 + row) * lay.ts + 4 * c4) = pk;
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
                                                         int Tn, Lay lay, float* __restrict__ part) {
  using T = SwzTile<D>;
  constexpr int NT = D / 32;
  constexpr int BUF = 2 * T::BYTES;
  constexpr int RB = 16 * T::ROW_BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * BUF];
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, g = l >> 5, ln = l & 31;
  const int ldv = tile_lane_offset<D>(w, l);
  const unsigned lds0 = lds_base(smem) + wave_uniform(w) * 1024;
  TileLoader<D> tl;   // tiles of the caller's dO
  tl.init(lds_base(smem), w, l, 2 * lay.ts);
  f32x16 acc[NT];
#pragma unroll
  for (int et = 0; et < NT; ++et) acc[et] = zero_f32x16();
  const int total = BH * Tn;
  auto issue = [&](int t, int buf) {
    const int bh = t / Tn, i = t - bh * Tn;
    const int rows = min(kBlk, N - i * kBlk);
    const size_t base = ((size_t)bh * N + (size_t)i * kBlk) * D;
    issue_tile_load<D>(Ol + base, rows, lds0, buf * BUF, ldv);
    tl.load(head_rsrc<D>(dO + lay.head(bh), N, 2 * lay.ts), i, buf * BUF + T::BYTES);
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

// dW partial sums of the whole call (launched between the query side and the column sums)
template <int D>
hipError_t dw_impl(const Shape& s, const BwdArgs& a, float* dWpart, int nparts, hipStream_t st) {
  KernelTimer kt("dw_partial", st);
  dw_mfma_kernel<D><<<nparts, 256, 0, st>>>((const bf16*)a.Ol, (const bf16*)a.dO, s.BH, s.N, s.T, s.lay(), dWpart);
  return hipGetLastError();
}

// Query side of the backward pass: the linear branch's first loop and the row-wise dQ kernel.  With
// query blocks of one tile (or an odd number of tiles) both run in one launch; with two tiles per
// workgroup in the dQ kernel the linear part runs as a kernel of its own and hands its part of dQ
// over in memory.
template <int D>
hipError_t query_impl(const Shape& s, const BwdArgs& a, float* Ds, bf16* dHZ, bf16* dQlin, hipStream_t st) {
  const float* Zs = (const float*)((const char*)a.HZ + state_z_offset(s));
  const PreArgs pa{(const bf16*)a.W, (const bf16*)a.Os, (const bf16*)a.Ol, (const bf16*)a.HZ, Zs, s.n_0, s.phi, Ds, dHZ};
  constexpr int lds_q = PairLds<D>::BYTES, lds_p = PreLds<D>::BYTES;
  if (s.rq % 2 == 0 && wide_query_tiles()) {
    SLA_TRY(ensure_dyn_lds(bwd_pre_mfma_kernel<D>, lds_p));
    {
      KernelTimer kt("bwd_pre", st);
      bwd_pre_mfma_kernel<D><<<dim3(s.T, s.BH), 256, lds_p, st>>>(
          (const bf16*)a.Q, (const bf16*)a.dO, pa.W, pa.Os, pa.Ol, pa.H16, Zs, s.N, s.T, s.lay(), s.n_0, s.phi, Ds, dHZ,
          dQlin);
    }
    const int bytes = lds_q + PairLds<D>::GROUP;
    SLA_TRY(ensure_dyn_lds(bwd_dq_mfma_kernel<D, 2, false>, bytes));
    KernelTimer kt("bwd_sparse_q", st);
    bwd_dq_mfma_kernel<D, 2, false><<<dim3(xcd_grid((s.T + 1) / 2), s.BH), 512, bytes, st>>>(
        (const bf16*)a.Q, (const bf16*)a.K, (const bf16*)a.V, (const bf16*)a.dO, a.L, Ds, a.row_idx,
        s.n_0 > 0 ? dQlin : nullptr, s.N, s.T, s.lay(), s.n_h, s.scale, (bf16*)a.dQ, pa);
  } else {
    constexpr int bytes = lds_q > lds_p ? lds_q : lds_p;
    SLA_TRY(ensure_dyn_lds(bwd_dq_mfma_kernel<D, 1, true>, bytes));
    KernelTimer kt("bwd_query", st);
    bwd_dq_mfma_kernel<D, 1, true><<<dim3(xcd_grid(s.T), s.BH), 256, bytes, st>>>(
        (const bf16*)a.Q, (const bf16*)a.K, (const bf16*)a.V, (const bf16*)a.dO, a.L, nullptr, a.row_idx, nullptr, s.N,
        s.T, s.lay(), s.n_h, s.scale, (bf16*)a.dQ, pa);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t mfma_backward_query(const Shape& s, const BwdArgs& a, float* Ds, void* dHZ16, float* dQlin,
                               hipStream_t st) {
  bf16* dHZ = reinterpret_cast<bf16*>(dHZ16);
  bf16* dQl = reinterpret_cast<bf16*>(dQlin);   // bf16 rows in the float-sized buffer
  return s.d == 64 ? query_impl<64>(s, a, Ds, dHZ, dQl, st) : query_impl<128>(s, a, Ds, dHZ, dQl, st);
}

hipError_t mfma_backward_dw(const Shape& s, const BwdArgs& a, float* dWpart, int nparts, hipStream_t st) {
  return s.d == 64 ? dw_impl<64>(s, a, dWpart, nparts, st) : dw_impl<128>(s, a, dWpart, nparts, st);
}

}  // namespace sla
