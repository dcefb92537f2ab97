// bf16 matrix-core backward kernel of the key side (Algorithm 2, M_c = 1 branch, and its last line;
// Eq. 7 with the 1/sqrt(d) factor on dK):
//   bwd_dkdv_mfma  one workgroup per key block j, walking the column table:
//                  dV_j += P^T dO_i, dK_j += dS^T Q_i / sqrt(d), started from the linear branch's
//                  dK_j, dV_j (the row-wise dQ kernel lives in mfma_bwd_query.hip)
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

// ------------------------------------------------------------------ dK, dV
// First products (S, dP): wave (kh, x) takes keys 32 kh .., queries 32 x .. of the pair; S and dP
// are [query][key], one key per lane.  Second products (dV^T = dO^T P, dK^T = Q^T dS): the same wave
// takes keys 32 kh .. and the feature half x, over all 64 queries.  P and dS therefore cross
// between the two waves of a key half, through LDS in operand layout (16 bytes per lane and
// k-step).  Each wave owns its quarter of dK_j, dV_j outright: 64 accumulator registers at d = 128
// instead of 128 for per-query-half partial sums, which is what leaves room to run the LDS reads
// several operands ahead of the products, and no summation at the end.
// L_q and D^s_q enter the first products as one more k-step: the A operand carries (L_q / scale)
// resp. D^s_q split into two bf16 terms, the B operand -1, so that the accumulators come out as
// S - L / scale and dP - D^s (error of the split: 2^-17 relative).  No per-step table in LDS, and
// P = exp2(c (S - L / scale)), dS = P (dP - D^s) cost one multiplication each.
template <int D>
struct KvLds {
  static constexpr int TILE = SwzTile<D>::BYTES;
  static constexpr int BUF = 2 * TILE;                   // Q_i and dO_i of a pair
  static constexpr int XOFF = 2 * BUF;                   // exchange: [kh][k-step 0..3][P | dS][lane] x 16 bytes
  static constexpr int XBYTES = 2 * 4 * 2 * 64 * 16;
  static constexpr int BYTES = XOFF + XBYTES;            // 80 KB at d = 128: half a CU
  static constexpr int STG = 32 * (64 * (D / 64) + 16);  // output staging of one wave, laid over the tiles
};

template <int D, int PHI>
__global__ __launch_bounds__(256, 2) void bwd_dkdv_mfma_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ K, const bf16* __restrict__ V,
    const bf16* __restrict__ dO, const float* __restrict__ L, const float* __restrict__ Ds,
    const int32_t* __restrict__ col_ptr, const int32_t* __restrict__ col_rows,
    const int32_t* __restrict__ col_order, const bf16* __restrict__ dHcol,
    const float* __restrict__ dZcol, int N, int Tn, Lay lay, int n_h, float scale,
    bf16* __restrict__ dK, bf16* __restrict__ dV) {
  using Lds = KvLds<D>;
  using T = SwzTile<D>;
  constexpr int NT = D / 32, KT = D / 16, HT = NT / 2;
  constexpr int RB = 16 * T::ROW_BYTES;
  constexpr int phi = PHI;   // feature map: 0 softmax over the features, 1 elu + 1
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, g = l >> 5, ln = l & 31;
  const int kh = w & 1, xh = w >> 1;
  // Longest column lists first, across all heads: the r-th heaviest key block of every head
  // precedes the (r+1)-th of any head.  The lists are very uneven (on video-like inputs the
  // heaviest key block of a head serves a third of all query blocks, the median one a dozen), and
  // the heaviest list alone lasts a good part of the launch, so every heavy list has to start at
  // once.  (Going head by head instead would let an XCD's workgroups share one head's Q and dO
  // tiles in its L2, but it starts the last head's heavy lists late: measured 1.5x slower.)
  // Within that order the heads are dealt to the XCDs (workgroups go to them round robin) in
  // halves -- the even or the odd ranks of a head -- so that an XCD's L2 serves the Q and dO tiles
  // of few heads at a time; most tile loads of this kernel miss the L2.
  const int BH = gridDim.x / Tn;
  int bh, rank;
  if (BH % 8 == 0 && BH >= 32 && Tn >= 128) {
    // Many long heads: every XCD takes its BH / 8 heads one after the other, each heaviest list first.
    // Its workgroups then share one head's Q and dO tiles and, being neighbours in rank, walk
    // their lists at about the same pace; a head is a small part of the launch, so the late start
    // of the last head's heavy lists costs little.
    const int hp = BH / 8;
    const int x = blockIdx.x & 7, m = blockIdx.x >> 3;
    bh = hp * x + m / Tn;
    rank = m % Tn;
  } else if ((2 * BH) % 8 == 0 && Tn % 2 == 0) {
    const int upx = 2 * BH / 8;   // half-heads per XCD
    const int x = blockIdx.x & 7, m = blockIdx.x >> 3;
    const int u = upx * x + m % upx;
    bh = u >> 1;
    rank = 2 * (m / upx) + (u & 1);
  } else {
    bh = blockIdx.x % BH;
    rank = blockIdx.x / BH;
  }
  const int j = col_order[(size_t)bh * Tn + rank];
  const int k0 = j * kBlk, cols = min(kBlk, N - k0);
  const int krow = kh * 32 + ln;
  const bool kok = krow < cols;
  bf16x8 kf[KT], vf[KT];
  f32x16 dvT[HT], dkT[HT];
#pragma unroll
  for (int t = 0; t < HT; ++t) {
    dvT[t] = zero_f32x16();
    dkT[t] = zero_f32x16();
  }
  const int32_t* ptr = col_ptr + (size_t)bh * (Tn + 1);
  const int32_t* list = col_rows + (size_t)bh * Tn * n_h;
  const int beg = ptr[j], cnt = ptr[j + 1] - beg;
  const float sl2 = scale * kLog2e, rscale = 1.0f / scale;
  TileLoader<D> tl;   // tiles of the caller's tensors (ldv, lds0 below: the library's packed ones)
  tl.init(lds_base(smem), w, l, 2 * lay.ts);
  const BufDesc descQ = head_rsrc<D>(Q + lay.head(bh), N, 2 * lay.ts);
  const BufDesc descG = head_rsrc<D>(dO + lay.head(bh), N, 2 * lay.ts);
  const float* Lb = L + (size_t)bh * N;
  const float* Dsb = Ds + (size_t)bh * N;
  const int ldv = tile_lane_offset<D>(w, l);
  const int wu = wave_uniform(w);
  const unsigned lds0 = lds_base(smem) + wu * 1024;
  // the row index of a step is fetched two steps ahead, so the tile loads never wait for it:
  // icur = query block of the pair that is in flight or in use, inext = the one after it
  int icur = cnt > 0 ? list[beg] : 0, inext = cnt > 1 ? list[beg + 1] : icur;
  auto issue = [&](int ii, const int bufi) __attribute__((always_inline)) {
    const int off = bufi * Lds::BUF;
    tl.load(descQ, ii, off);
    tl.load(descG, ii, off + Lds::TILE);
  };
  // K_j and V_j come in as tiles (whole rows per load, zeros past the end of the sequence) and are
  // picked up from LDS in operand layout.  With a linear branch, the aggregated dH^T of this key
  // block (d x d, stored [b][a]) comes in with them, through the second pair buffer (rows 0..63
  // in the Q slot, the rest in the dO slot), K_j and V_j through the first, which is handed to the
  // first pair's tiles as soon as the operands are in registers; dZ_j goes to registers directly.
  const int kvoff = dHcol ? 0 : Lds::BUF;
  tl.load(head_rsrc<D>(K + lay.head(bh), N, 2 * lay.ts), j, kvoff);
  tl.load(head_rsrc<D>(V + lay.head(bh), N, 2 * lay.ts), j, kvoff + Lds::TILE);
  f32x4 z4[HT][4];
  if (dHcol) {
    const bf16* M = dHcol + ((size_t)bh * Tn + j) * (D * D);
    issue_tile_load<D>(M, min(kBlk, D), lds0, Lds::BUF, ldv);
    if (D > kBlk) issue_tile_load<D>(M + (size_t)kBlk * D, D - kBlk, lds0, Lds::BUF + Lds::TILE, ldv);
    const float* dZ = dZcol + ((size_t)bh * Tn + j) * D;
#pragma unroll
    for (int dt = 0; dt < HT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) z4[dt][r4] = *reinterpret_cast<const f32x4*>(dZ + 32 * (xh * HT + dt) + 8 * r4 + 4 * g);
  } else if (cnt > 0) {
    issue(icur, 0);
  }
  wait_vm0_known();
  if (dHcol) {   // (tell the compiler too, or it waits for dZ later, with the first pair's loads in flight)
#pragma unroll
    for (int dt = 0; dt < HT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) pin_loaded(z4[dt][r4]);
  }
  __syncthreads();
  bf16x4 kc[HT][4];   // K_j at the positions of this wave's dK^T registers (linear branch only)
  {
    TileAddr<D> ka;
    ka.init(32 * kh, l);
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      kf[t] = lds_row(smem, ka.row(t) + kvoff);
      vf[t] = lds_row(smem, ka.row(t) + kvoff + Lds::TILE);
    }
    if (dHcol) {
      const int krw = krow * T::ROW_BYTES + 8 * g, ksw = swz<D>(krow);
#pragma unroll
      for (int dt = 0; dt < HT; ++dt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int a0 = 32 * (xh * HT + dt) + 8 * r4 + 4 * g;
          kc[dt][r4] = *reinterpret_cast<const bf16x4*>(smem + krw + (((a0 >> 3) ^ ksw) << 4));
        }
    }
  }
#pragma unroll
  for (int t = 0; t < KT; ++t) {
    pin_loaded(kf[t]);
    pin_loaded(vf[t]);
  }
  if (dHcol) {
    // ---- linear branch of Alg. 2 for key block j, as the start value of the accumulators:
    // dV += phi(K_j) dH_j and dK += d phi(K_j) / d K_j applied to (V_j dH_j^T + dZ_j), this wave's
    // feature half of each.
#pragma unroll
    for (int dt = 0; dt < HT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) pin_loaded(kc[dt][r4]);
    __syncthreads();   // K_j and V_j are in registers everywhere: their buffer takes the first pair
    if (cnt > 0) issue(icur, 0);
    float kmx, kinv;
    TileAddr<D> ma;
    ma.init(0, l);
    {
      // dV^T[b][n] = sum_a M[b][a] phi(K)[n][a]: rows b of M are the A operand
      bf16x8 kp[KT];
      phi_fragments<KT>(kf, phi, kp, kmx, kinv);
      if (!kok) {
#pragma unroll
        for (int t = 0; t < KT; ++t) kp[t] = zero_bf16x8();
      }
#pragma unroll
      for (int dt = 0; dt < HT; ++dt) {
        const int bt = xh * HT + dt;
#pragma unroll
        for (int t = 0; t < KT; ++t)
          dvT[dt] = mfma32(lds_row(smem, ma.row(t) + Lds::BUF + (bt / 2) * Lds::TILE + (bt % 2) * 2 * RB), kp[t], dvT[dt]);
      }
    }
    // d phi(K)^T[a][n] = sum_b M[b][a] V[n][b] + dZ[a]: M^T through the transposing read, whose
    // k order is the one a C tile hands over, so the V operand is brought into that order too
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      const bf16x8 vb = to_tr_order(vf[t]);
      const int mb = Lds::BUF + (t / 4) * Lds::TILE + (t % 4) * RB;   // rows b = 16 t .. of M
#pragma unroll
      for (int dt = 0; dt < HT; ++dt) {
        const int at = xh * HT + dt;
        dkT[dt] = mfma32(lds_tr<D>(smem, ma.tr(0, at) + mb, ma.tr(1, at) + mb), vb, dkT[dt]);
      }
    }
    // y = phi(K) (softmax map) or d phi / d K (the other one) at the positions of the dK^T
    // registers, formed once
    float yk[HT][16];
    float dot = 0.0f;
#pragma unroll
    for (int dt = 0; dt < HT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float x = (float)kc[dt][r4][r];
          const float y = phi == 0 ? phi_val(x, 0, kmx, kinv) : (x > 0.0f ? 1.0f : fast_exp2(x * kLog2e));
          const float v = dkT[dt][4 * r4 + r] + z4[dt][r4][r];
          dkT[dt][4 * r4 + r] = v;
          yk[dt][4 * r4 + r] = y;
          dot = fmaf(v, y, dot);
        }
    dot = half_sum(dot);
    float* dotx = reinterpret_cast<float*>(smem + Lds::XOFF);   // [x][64 keys]
    if (g == 0) dotx[xh * kBlk + krow] = dot;
    __syncthreads();   // (also: dH^T is consumed before the first step refills its buffer)
    const float dtot = phi == 0 ? dotx[krow] + dotx[kBlk + krow] : 0.0f;
#pragma unroll
    for (int dt = 0; dt < HT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        // the epilogue multiplies the whole dK sum by scale
        dkT[dt][r] = kok ? yk[dt][r] * (dkT[dt][r] - dtot) * rscale : 0.0f;
    __syncthreads();   // the sums above are read before the first step writes the exchange area
  }
  TileAddr<D> ad;   // first products: rows 32 x .. of Q_i, dO_i by rows
  ad.init(32 * xh, l);
  TileAddr<D> at;   // second products: transposing reads, feature tiles x HT ..
  at.init(0, l);
  // B operand of the extra k-step: -1 at k = 0, 1
  bf16x8 bneg;
#pragma unroll
  for (int e = 0; e < 8; ++e) bneg[e] = (__bf16)((g == 0 && e < 2) ? -1.0f : 0.0f);
  const int xw = Lds::XOFF + ((kh * 4 + 2 * xh) * 2 * 64 + l) * 16;   // this wave's exchange writes
  const int xr = Lds::XOFF + (kh * 4 * 2 * 64 + l) * 16;              // ... and reads
  const int xwave = Lds::XOFF + (kh * 4 + 2 * xh) * 2 * 64 * 16;      // start of this wave's part (uniform)
  const unsigned xstat = lds_base(smem) + wave_uniform(xwave);
  auto step = [&](int s, const int buf) __attribute__((always_inline)) {
    const int QO = buf * Lds::BUF, GO = QO + Lds::TILE;
    ad.refresh();
    at.refresh();
    wait_vm0_known();
    __syncthreads();   // tiles of step s have landed for every wave; step s-1 is fully consumed
    // L and D^s of this step's 64 queries are requested now, ahead of the next pair's tile loads in
    // the queue (loads return in order), and picked up after the first products.  They go global ->
    // LDS like the tiles (nothing the compiler could wait for, copy or spill), into the first 512
    // bytes of this wave's own part of the exchange area: the last reads of that part (the second
    // products of the previous step) are behind the barrier above, and the wave overwrites it with
    // P and dS only after it has read the statistics back.  Rows past the end read as 0; their Q
    // and dO rows are zero too, so the finite P they get adds nothing.
    {
      const int rows = min(kBlk, N - icur * kBlk), lo = lane_id() * 4;
      load_to_lds4(tile_rsrc(Lb + (size_t)icur * kBlk, rows * 4), lo, xstat);
      load_to_lds4(tile_rsrc(Dsb + (size_t)icur * kBlk, rows * 4), lo, xstat + 256);
    }
    // (the last step requests its own pair once more, into the other buffer, where nobody reads
    // it: every step then has the same number of loads in flight and one wait serves all)
    issue(s + 1 < cnt ? inext : icur, buf ^ 1);
    icur = inext;
    inext = list[beg + min(s + 2, cnt - 1)];
    // LDS reads run PF operand pairs ahead of the products that consume them (software pipeline
    // written out by hand: left alone, the compiler reads each operand right before its product
    // and every product then waits a full LDS latency).
    constexpr int PF = 4;
    bf16x8 qa[PF], ga[PF];
    auto read_s = [&](int t) __attribute__((always_inline)) {
      qa[t % PF] = lds_row(smem, ad.row(t) + QO);
      ga[t % PF] = lds_row(smem, ad.row(t) + GO);
    };
#pragma unroll
    for (int t = 0; t < PF; ++t) read_s(t);
    sched_fence();
    f32x16 sm = zero_f32x16(), dp = zero_f32x16();
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      sm = mfma32(qa[t % PF], kf[t], sm);
      dp = mfma32(ga[t % PF], vf[t], dp);
      if (t + PF < KT) read_s(t + PF);
      sched_fence();
    }
    // the extra k-step: A operands (hi, lo) at k = 0, 1 of the lanes with g = 0
    wait_vm<2 * T::IPW>();   // the statistics are there, the tile loads may still fly
    {
      const int qo = (32 * xh + (lane_id() & 31)) * 4;
      const float lcur = *reinterpret_cast<const float*>(smem + xwave + qo) * rscale;
      const float dcur = *reinterpret_cast<const float*>(smem + xwave + 256 + qo);
      bf16x8 aL = zero_bf16x8(), aD = zero_bf16x8();
      const __bf16 lh = (__bf16)lcur, dh = (__bf16)dcur;
      const __bf16 ll = (__bf16)(lcur - (float)lh), dl = (__bf16)(dcur - (float)dh);
      aL[0] = g == 0 ? lh : (__bf16)0.0f;
      aL[1] = g == 0 ? ll : (__bf16)0.0f;
      aD[0] = g == 0 ? dh : (__bf16)0.0f;
      aD[1] = g == 0 ? dl : (__bf16)0.0f;
      sm = mfma32(aL, bneg, sm);
      dp = mfma32(aD, bneg, dp);
    }
    // operand i of the second products: i = 2 HT ks + 2 dt + which; which 0: dO^T rows of feature
    // tile x HT + dt (for dV), which 1: Q^T (for dK); k = pair rows 16 ks ..
    constexpr int PT = 6, NOP = 8 * HT;
    bf16x8 ta[PT];
    auto read_t = [&](int i) __attribute__((always_inline)) {
      const int ks = i / (2 * HT), et = xh * HT + (i % (2 * HT)) / 2, base = (i % 2 ? QO : GO) + ks * RB;
      ta[i % PT] = lds_tr<D>(smem, at.tr(0, et) + base, at.tr(1, et) + base);
    };
    // the first transposed operands arrive under the softmax arithmetic
#pragma unroll
    for (int i = 0; i < PT; ++i) read_t(i);
    sched_fence();
    // P[q][key] = exp(S - L_q), dS = P (dP - D^s_q).  A lane past the end of the key block (its K
    // and V rows are zero) computes finite values that stay in its own columns of dK^T and dV^T,
    // which are never stored.
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float pv = fast_exp2(sm[r] * sl2);
      sm[r] = pv;
      dp[r] *= pv;
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      *reinterpret_cast<bf16x8*>(smem + xw + (2 * u) * 1024) = c_to_operand(sm, u);
      *reinterpret_cast<bf16x8*>(smem + xw + (2 * u + 1) * 1024) = c_to_operand(dp, u);
    }
    __syncthreads();   // P and dS of all 64 queries are there for both waves of the key half
    bf16x8 pb[4], sb[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      pb[ks] = lds_row(smem, xr + (2 * ks) * 1024);
      sb[ks] = lds_row(smem, xr + (2 * ks + 1) * 1024);
    }
    sched_fence();
#pragma unroll
    for (int i = 0; i < NOP; ++i) {
      const int ks = i / (2 * HT), dt = (i % (2 * HT)) / 2;
      if (i % 2 == 0) dvT[dt] = mfma32(ta[i % PT], pb[ks], dvT[dt]);   // dO_i^T P
      else dkT[dt] = mfma32(ta[i % PT], sb[ks], dkT[dt]);              // Q_i^T dS
      if (i + PT < NOP) read_t(i + PT);
      sched_fence();
    }
  };
  for (int s = 0; s < cnt; s += 2) {
    step(s, 0);
    if (s + 1 < cnt) step(s + 1, 1);
  }
  // ---- each wave owns keys 32 kh .., features (D / 2) x .. of dK_j and dV_j: whole-row stores
  // through its own staging area
  wait_vm0_known();        // the last step's surplus request has landed
  __syncthreads();   // every wave is done with the tiles
  unsigned char* stage = smem + wu * Lds::STG;
  const size_t o0 = lay.head(bh) + (size_t)(k0 + 32 * kh) * lay.ts + (D / 2) * xh;
  store_rows_bf16<HT>(stage, dvT, dV + o0, lay.ts, cols - 32 * kh, l);
#pragma unroll
  for (int dt = 0; dt < HT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) dkT[dt][r] *= scale;
  store_rows_bf16<HT>(stage, dkT, dK + o0, lay.ts, cols - 32 * kh, l);
}

#define SLA_TRY(x)                   \
  do {                               \
    hipError_t e_ = (x);             \
    if (e_ != hipSuccess) return e_; \
  } while (0)

template <int D>
hipError_t sparse_impl(const Shape& s, const BwdArgs& a, const float* Ds, const void* dHZcol, hipStream_t st) {
  const float* dZcol = dHZcol ? reinterpret_cast<const float*>((const char*)dHZcol + state_z_offset(s)) : nullptr;
  auto launch_kv = [&](auto kern) -> hipError_t {
    SLA_TRY(ensure_dyn_lds(kern, KvLds<D>::BYTES));
    KernelTimer kt("bwd_sparse_kv", st);
    kern<<<dim3(s.T * s.BH), 256, KvLds<D>::BYTES, st>>>(
        (const bf16*)a.Q, (const bf16*)a.K, (const bf16*)a.V, (const bf16*)a.dO, a.L, Ds, a.col_ptr, a.col_rows,
        a.col_order, (const bf16*)dHZcol, dZcol, s.N, s.T, s.lay(), s.n_h, s.scale, (bf16*)a.dK, (bf16*)a.dV);
    return hipSuccess;
  };
  SLA_TRY(s.phi == 0 ? launch_kv(bwd_dkdv_mfma_kernel<D, 0>) : launch_kv(bwd_dkdv_mfma_kernel<D, 1>));
  return hipGetLastError();
}

}  // namespace

hipError_t mfma_backward_sparse(const Shape& s, const BwdArgs& a, const float* Ds, const void* dHZcol, hipStream_t st) {
  return s.d == 64 ? sparse_impl<64>(s, a, Ds, dHZcol, st) : sparse_impl<128>(s, a, Ds, dHZcol, st);
}

}  // namespace sla
