// bf16 matrix-core forward path of SLA on gfx950 (Algorithm 1 and Eq. 6):
//   states_mfma     h_j = phi(K_j)^T V_j, z_j = rowsum(phi(K_j)^T)            (precompute line)
//   aggregate_mfma  H_i = sum_{j marginal} h_j as a dense GEMM with the 0/1 indicator of
//                   the marginal blocks (the accumulation line, batched over all rows)
//   fwd_mfma        online-softmax attention over the critical blocks of a query block,
//                   the closing line (O^s, L, O^l) and O = O^s + O^l W
// All contractions run on v_mfma_f32_32x32x16_bf16 with float accumulation.
#include <type_traits>
#include "mfma_common.h"

namespace sla {
namespace {

typedef __hip_bfloat16 bf16;

// ------------------------------------------------------------------ W^T, k-permuted
// WTp[e'][16 u + perm16(r)] = W[16 u + r][e']: the A operand of O^l W in the transposed
// product (O^T = W^T (O^l)^T), whose B operand comes straight out of C registers.
// (done by one extra workgroup of the state kernel's launch)
template <int D>
__device__ __forceinline__ void prep_w(const bf16* __restrict__ W, bf16* __restrict__ WTp, int tid) {
  for (int idx = tid; idx < D * D; idx += 256) {
    const int e = idx / D, ep = idx - e * D;
    WTp[ep * D + (e & ~15) + perm16(e & 15)] = W[idx];
  }
}

// ------------------------------------------------------------------ key-block states

// h_j^T[e][c] = sum_keys V[key][e] phi(K)[key][c], z_j[c] = sum_keys phi(K)[key][c] for one key
// block (Alg. 1, precompute line).  K_j and V_j come in as LDS tiles; phi is applied to the K tile
// in place; both operands of the product are contracted over tile rows, i.e. read with the
// transposing LDS read; the product is formed with e along the lanes so that the rows of h^T leave
// whole.  Wave w owns rows e in [32 w, 32 w + 32).
template <int D>
__global__ __launch_bounds__(256, 4) void states_mfma_kernel(const bf16* __restrict__ K,
                                                             const bf16* __restrict__ V, int N, int Tn, Lay lay,
                                                             int phi, bf16* __restrict__ hz,
                                                             const bf16* __restrict__ W, bf16* __restrict__ WTp) {
  using T = SwzTile<D>;
  constexpr int NT = D / 32;
  constexpr int STG = 32 * (64 * NT + 16);           // store_rows_bf16<NT> area of one wave
  constexpr int LDSB = 2 * T::BYTES > NT * STG ? 2 * T::BYTES : NT * STG;
  __shared__ __attribute__((aligned(16))) unsigned char smem[LDSB];
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, g = l >> 5;
  const int j = blockIdx.x, bh = blockIdx.y;
  if (j == Tn) {   // the extra column of the grid: head 0's workgroup prepares the projection matrix
    if (bh == 0) prep_w<D>(W, WTp, tid);
    return;
  }
  const int n0 = j * kBlk, cnt = min(kBlk, N - n0);
  const int wu = wave_uniform(w);
  {
    TileLoader<D> tl;
    tl.init(lds_base(smem), w, l, 2 * lay.ts);
    tl.load(head_rsrc<D>(K + lay.head(bh), N, 2 * lay.ts), j, 0);
    tl.load(head_rsrc<D>(V + lay.head(bh), N, 2 * lay.ts), j, T::BYTES);
  }
  wait_vm0();
  __syncthreads();
  // phi on the K tile in place: four threads per key row, a quarter of the features each
  {
    const int row = tid >> 2, part = tid & 3;
    constexpr int CPP = D / 32;   // 16-byte chunks per thread
    // (a thread visits its chunks in an order rotated by its row: the sixteen lanes that access LDS
    // together, four rows of four parts, then touch sixteen different chunk positions)
    const int rot = row & (CPP - 1);
    bf16x8 x[CPP];
#pragma unroll
    for (int c = 0; c < CPP; ++c)
      x[c] = *reinterpret_cast<const bf16x8*>(smem + swz_chunk_off<D>(row, part * CPP + ((c + rot) & (CPP - 1))));
    float mx = 0.0f, inv = 1.0f;
    if (phi == 0) {
      mx = -INFINITY;
#pragma unroll
      for (int c = 0; c < CPP; ++c)
#pragma unroll
        for (int e = 0; e < 8; ++e) mx = fmaxf(mx, (float)x[c][e]);
      mx = fmaxf(mx, __shfl_xor(mx, 1, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 2, 64));
      float sum = 0.0f;
#pragma unroll
      for (int c = 0; c < CPP; ++c)
#pragma unroll
        for (int e = 0; e < 8; ++e) sum += fast_exp2(((float)x[c][e] - mx) * kLog2e);
      sum += __shfl_xor(sum, 1, 64);
      sum += __shfl_xor(sum, 2, 64);
      inv = 1.0f / sum;
    }
    const bool ok = row < cnt;   // rows past the end of the sequence contribute nothing, also to z_j
#pragma unroll
    for (int c = 0; c < CPP; ++c) {
#pragma unroll
      for (int e = 0; e < 8; ++e) x[c][e] = (__bf16)(ok ? phi_val((float)x[c][e], phi, mx, inv) : 0.0f);
      *reinterpret_cast<bf16x8*>(smem + swz_chunk_off<D>(row, part * CPP + ((c + rot) & (CPP - 1)))) = x[c];
    }
  }
  __syncthreads();
  bf16* out = hz + ((size_t)bh * Tn + j) * (D * D + D);
  f32x16 acc[NT];
  if (w < NT) {
    TileAddr<D> ad;
    ad.init(0, l);
    constexpr int RB = 16 * T::ROW_BYTES;
    bf16x8 ones;
#pragma unroll
    for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;
    f32x16 zc = zero_f32x16();
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) acc[ct] = zero_f32x16();
#pragma unroll
    for (int t = 0; t < kBlk / 16; ++t) {
      const bf16x8 vb = lds_tr<D>(smem, ad.tr(0, w) + T::BYTES + t * RB, ad.tr(1, w) + T::BYTES + t * RB);   // V^T, rows e
#pragma unroll
      for (int ct = 0; ct < NT; ++ct) {
        const bf16x8 ka = lds_tr<D>(smem, ad.tr(0, ct) + t * RB, ad.tr(1, ct) + t * RB);   // phi(K)^T, rows c
        acc[ct] = mfma32(ka, vb, acc[ct]);   // C[c][e]: lane = e, registers = c
        if (ct == w) zc = mfma32(ka, ones, zc);   // every column of this C tile is z_j[32 w ..]
      }
    }
    if ((l & 31) == 0) {
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        bf16x4 pk;
#pragma unroll
        for (int r = 0; r < 4; ++r) pk[r] = (__bf16)zc[4 * r4 + r];
        *reinterpret_cast<bf16x4*>(out + (size_t)D * D + 32 * w + 8 * r4 + 4 * g) = pk;
      }
    }
  }
  __syncthreads();   // the tiles are free: each wave stages its rows over them
  if (w < NT) store_rows_bf16<NT>(smem + wu * STG, acc, out + (size_t)(32 * w) * D, D, 32, l);
}

// ------------------------------------------------------------------ forward main kernel
// One workgroup (4 wavefronts) per query block, one critical key block per step.  Wavefront
// (qh, par): qh = which 32 of the 64 query rows, par = which 32 of the step's 64 keys.
// Everything is held transposed (S^T = K Q^T, O^T = V^T P^T) so that each lane owns one query:
// softmax statistics are per-lane scalars and P goes from C registers straight into the B
// operand of the second product.  Each wave runs its own online softmax over its key halves;
// the two streams of a query half are merged at the end.  K_j and V_j go global -> LDS
// directly (swizzled, two barriers per step); V is read transposed.
// The scores of step s + 1 are formed under the exponentials of step s.
//
// The step loop is written for few instructions (a wave issues one every five to eight cycles
// whatever its kind, and a SIMD has two waves): tile slots fixed per step parity (two copies of
// the step, every LDS offset an immediate), per-lane LDS addresses held in registers, one M0 value
// per tile (RunLoader), the key block table read one entry per step through a running offset, the
// few conditions as branches of the whole wave.
template <int D>
struct FwdLds {
  // Slot 2p holds the K tile and slot 2p + 1 the V tile of the steps of parity p.  The scores S_s
  // are formed during step s - 1.  A wave copies its operands of step s (rows of K_{s+1}, V_s) to
  // registers at the top of the step; after a barrier of its own the two slots take K_{s+3} and
  // V_{s+2}: every tile is requested two steps before it is needed (an L2 miss costs more than
  // one step) although only two tiles of each kind have a slot.
  // After the loop the slots hold the exchange between the two key streams, H_i and the
  // projection matrix; the softmax statistics have a KB of their own behind the slots.
  static constexpr int TILE = SwzTile<D>::BYTES;
  static constexpr int XCH_HALF = (D / 2) * 64 * 4;       // C registers of one query half
  static_assert(XCH_HALF <= TILE, "exchange areas are laid over tile slots");
  static constexpr int STAT = 4 * TILE;                  // softmax statistics of the four waves (1 KB)
  static constexpr int ZOFF = STAT + 1024;               // Z_i (D floats)
  static constexpr int BYTES = ZOFF + D * 4;
};
// Query blocks of 128 (or 256) tokens: QT = 2 adjacent 64-query tiles, which have the same list of
// critical key blocks, share one workgroup of eight waves.  K_j and V_j are then fetched into LDS
// once for both tiles (half the L2 -> LDS traffic and half the load instructions per score); each
// group of four waves works on its tile exactly as a four-wave workgroup does, and has an LDS area
// of its own (the second group's lies behind the first's) for what follows the loop.

template <int D, int QT>
__global__ __launch_bounds__(256 * QT, QT == 1 ? 2 : 1) void fwd_mfma_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ K, const bf16* __restrict__ V,
    const bf16* __restrict__ WTp, const int32_t* __restrict__ row_idx, const bf16* __restrict__ H16,
    const float* __restrict__ Zs,
    int N, int Tn, Lay lay, int n_h, int n_0, int phi, float scale_log2e, bf16* __restrict__ O,
    bf16* __restrict__ Os, bf16* __restrict__ Ol, float* __restrict__ L) {
  using Lds = FwdLds<D>;
  constexpr int NT = D / 32, KT = D / 16;
  constexpr int NW = 4 * QT;   // waves that fill a K or V tile together
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, wall = tid >> 6, l = tid & 63, g = l >> 5, ln = l & 31;
  const int grp = QT == 1 ? 0 : wave_uniform(wall >> 2), w = wall & 3;   // tile of the workgroup, wave of the tile
  const int qh = w & 1, par = w >> 1;
  const int ib = xcd_local_block(blockIdx.x, (Tn + QT - 1) / QT), bh = blockIdx.y;
  if (ib < 0) return;
  // a last block of a single tile: the second group runs along (it shares the tile loads and the
  // barriers) on the last tile's tables with no valid query, and stores nothing
  const int i = QT * ib + grp, ic = min(i, Tn - 1);
  unsigned char* gsm = smem + grp * Lds::BYTES;   // this group's area for everything behind the loop
  const int q0 = i * kBlk, rows = max(0, min(kBlk, N - q0));
  const int qrow = qh * 32 + ln;                  // this lane's query inside the block
  const bool qok = qrow < rows;
  const size_t qoff = lay.head(bh) + (size_t)(q0 + qrow) * lay.ts;
  bf16x8 qf[KT];
#pragma unroll
  for (int t = 0; t < KT; ++t)
    qf[t] = qok ? *reinterpret_cast<const bf16x8*>(Q + qoff + 16 * t + 8 * g) : zero_bf16x8();
  f32x16 oT[NT];
#pragma unroll
  for (int et = 0; et < NT; ++et) oT[et] = zero_f32x16();
  float m = -INFINITY, lsum = 0.0f;
  const int32_t* lut = row_idx + ((size_t)bh * Tn + QT * ib) * n_h;   // the same list for every tile of the block
  const float c2 = scale_log2e;                    // exp(x / sqrt(d)) = exp2(x * c2)
  using T = SwzTile<D>;
  RunLoader<D, NW> tl;    // tiles of the caller's K and V: all waves of the workgroup, into the slots
  TileLoader<D> tm;       // packed d x d matrices: the four waves of a group, into the group's area
  tl.init(lds_base(smem), wall, l, 2 * lay.ts);
  tm.init(lds_base(smem) + grp * Lds::BYTES, w, l, 2 * D);
  constexpr int IPW = RunLoader<D, NW>::IPW;
  const BufDesc descK = head_rsrc<D>(K + lay.head(bh), N, 2 * lay.ts);
  const BufDesc descV = head_rsrc<D>(V + lay.head(bh), N, 2 * lay.ts);
  // a d x d bf16 matrix (aggregated state H_i, prepared projection matrix) goes global -> LDS like
  // the tiles: rows 0..63 into the slot at off0, the rest into the one at off1
  auto issue_matrix = [&](const bf16* M, int off0, int off1) {
    const BufDesc dm = tile_rsrc(M, D * D * 2);
    tm.load(dm, 0, off0);
    if (D > kBlk) tm.load(dm, 1, off1);
  };
  // H_i together with Z_i (one dword per lane of the first D / 64 waves, global -> LDS like the tiles:
  // a load the compiler sees would be waited for behind the projection matrix's loads, which
  // are requested before it is used)
  auto issue_state = [&](int off0, int off1) {
    issue_matrix(H16 + ((size_t)bh * Tn + ic) * (D * D), off0, off1);
    if (w < D / 64)
      load_to_lds4(tile_rsrc(Zs + ((size_t)bh * Tn + ic) * D, D * 4), (w * 64 + l) * 4,
                   lds_base(smem) + grp * Lds::BYTES + Lds::ZOFF + w * 256);
  };
  // Slots at the end of the loop, with p the parity of the last step: H_i goes to the slots of
  // K_{last+1} (never filled) and V_last, both free from the last step's second barrier on, the
  // exchange areas to the other two once the loop is over.
  const int pl = n_h > 0 ? (n_h - 1) & 1 : 0;
  const int h0 = (2 - 2 * pl) * Lds::TILE, h1 = (2 * pl + 1) * Lds::TILE;
  const int x0 = 2 * pl * Lds::TILE, x1 = (3 - 2 * pl) * Lds::TILE;
  float* ml = reinterpret_cast<float*>(gsm + Lds::STAT);   // [par][qh][32][2]
  // byte offsets (inside a head) of the key blocks of steps s .. s + 3; the table entry behind the
  // fourth is fetched a step before the load that needs it
  int kb0 = 0, kb1 = 0, kb2 = 0, kb3 = 0;
  if (n_h > 0) {
    kb0 = lut[0] * tl.tile_step;
    kb1 = lut[min(1, n_h - 1)] * tl.tile_step;
    kb2 = lut[min(2, n_h - 1)] * tl.tile_step;
    kb3 = lut[min(3, n_h - 1)] * tl.tile_step;
    tl.template load<0>(descK, kb0);
    tl.template load<Lds::TILE>(descV, kb0);
    if (n_h > 1) {
      tl.template load<2 * Lds::TILE>(descK, kb1);
      tl.template load<3 * Lds::TILE>(descV, kb1);
    }
  } else if (n_0 > 0) {
    issue_state(h0, h1);
  }
  unsigned lo = 16;                                  // byte offset of the next table entry to fetch
  const unsigned lomax = 4u * (unsigned)max(n_h - 1, 0);
  // a sequence whose last key block is partial: its offset and its number of keys
  const int off_tail = (N % kBlk) ? (Tn - 1) * tl.tile_step : -1;
  const int tail_cols = N - (N / kBlk) * kBlk;
#pragma unroll
  for (int t = 0; t < KT; ++t) pin_loaded(qf[t]);
  // per-lane LDS offsets of this wave's operand reads inside a tile (rows 32 par .. of both tiles)
  int kaddr[KT], vaddr[2][NT];
  {
    TileAddr<D> ad;
    ad.init(32 * par, l);
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      kaddr[t] = ad.row(t);
      asm volatile("" : "+v"(kaddr[t]));
    }
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int et = 0; et < NT; ++et) {
        vaddr[h][et] = ad.tr(h, et);
        asm volatile("" : "+v"(vaddr[h][et]));
      }
  }
  tl.pin();
  // The scores of a step are formed one step ahead, so that their matrix products (a chain on
  // one accumulator, during which the wave could issue nothing else) run under the exponentials
  // of the current step: S_0 here, S_{s+1} inside step s.
  f32x16 sT = zero_f32x16();
  if (n_h > 0) {
    if (n_h > 1) wait_vm<3 * IPW>();   // K_0 has landed; V_0, K_1 and V_1 may stay in flight
    else wait_vm<IPW>();
    __syncthreads();
    bf16x8 k0[KT];
#pragma unroll
    for (int t = 0; t < KT; ++t) k0[t] = lds_row(smem, kaddr[t]);
    __syncthreads();                   // every wave holds its rows of K_0: the slot takes K_2
    if (n_h > 2) tl.template load<0>(descK, kb2);
#pragma unroll
    for (int t = 0; t < KT; ++t) sT = mfma32(k0[t], qf[t], sT);
    if (n_h > 2) wait_vm<2 * IPW>();   // V_0 and K_1 have landed
    else wait_vm0();
    __syncthreads();
  }
  // One step; P = parity of s.  On entry K_{s+1} and V_s are in their slots for every wave, sT
  // holds S_s; sN receives S_{s+1}.  The wave copies its operands of the step to registers first;
  // a second barrier then frees both slots for K_{s+3} and V_{s+2}, two steps before they are
  // needed.  The few conditions are wave-uniform branches (two scalar instructions each).
  auto step = [&](auto Pc, int s, f32x16& sT, f32x16& sN) __attribute__((always_inline)) {
    constexpr int P = decltype(Pc)::value;
    constexpr int VS = (2 * P + 1) * Lds::TILE;    // V_s, then V_{s+2}
    constexpr int KN = 2 * (1 - P) * Lds::TILE;    // K_{s+1}, then K_{s+3}
    bf16x8 ka[KT], va[2][NT];
#pragma unroll
    for (int t = 0; t < KT; ++t) ka[t] = lds_row(smem, kaddr[t] + KN);
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int et = 0; et < NT; ++et)
        va[u][et] = lds_tr<D>(smem, vaddr[0][et] + VS + u * 16 * T::ROW_BYTES, vaddr[1][et] + VS + u * 16 * T::ROW_BYTES);
    // ---- online softmax on raw scores (the 1/sqrt(d) and log2 e factors ride on the exp2
    // argument); one query per lane
    if (kb0 == off_tail) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (32 * par + c_row(r, g) >= tail_cols) sT[r] = -INFINITY;
    }
    float mx = sT[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sT[r]);
    mx = half_max(mx);
    const float mnew = fmaxf(m, mx);
    // The reference point m of the exponentials follows the running maximum lazily: only when
    // some query's maximum has moved up by more than 2^kLazy (always at its first valid key), so
    // that the accumulators are rescaled on few steps.  P is then at most 2^kLazy instead of 1,
    // which neither float nor bf16 mind, and L = m + log(sum) comes out the same.
    constexpr float kLazy = 8.0f;
    if (__any((mnew - m) * c2 > kLazy)) {
      const float alpha = fast_exp2((m - mnew) * c2);
      lsum *= alpha;
#pragma unroll
      for (int et = 0; et < NT; ++et)
#pragma unroll
        for (int r = 0; r < 16; ++r) oT[et][r] *= alpha;
      m = mnew;
    }
    const float moff = m == -INFINITY ? 0.0f : -m * c2;   // a half with no valid key yet
    __syncthreads();   // every wave holds its operands of this step: both slots are refilled
    if (s + 3 < n_h) tl.template load<KN>(descK, kb3);
    if (s + 2 < n_h) tl.template load<VS>(descV, kb2);
    else if (s + 1 == n_h && n_0 > 0) issue_state(h0, h1);   // arrives under the last step
    const int jn = *reinterpret_cast<const int32_t*>(reinterpret_cast<const char*>(lut) + min(lo, lomax));
    lo += 4;
    sched_fence();
    static_assert(KT == 8 || KT == 4, "two or four exponentials per product of the next scores");
    sN = zero_f32x16();
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      sN = mfma32(ka[t], qf[t], sN);   // S_{s+1} (in the last step: of a slot that holds no tile, unused)
#pragma unroll
      for (int r = t * (16 / KT); r < (t + 1) * (16 / KT); ++r) sT[r] = fast_exp2(fmaf(sT[r], c2, moff));
    }
    // The row sum is taken over the float exponentials by plain additions (the packed dot
    // product that would add two bf16 values per instruction runs on the matrix pipe and holds
    // up the products).
    float psum = 0.0f;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const bf16x8 pf = c_to_operand(sT, u);
#pragma unroll
      for (int e = 0; e < 8; ++e) psum += sT[8 * u + e];
#pragma unroll
      for (int et = 0; et < NT; ++et) oT[et] = mfma32(va[u][et], pf, oT[et]);
    }
    lsum += psum;
    kb0 = kb1;
    kb1 = kb2;
    kb2 = kb3;
    kb3 = jn * tl.tile_step;
    sched_fence();     // (the matrix products above are issued before this wait)
    // K_{s+2} and V_{s+1}, requested a step ago, have landed; the two tiles requested in this
    // step may stay in flight (near the end fewer were requested: everything is waited for)
    if (s + 4 < n_h) wait_vm<2 * IPW>();
    else wait_vm0();
    __syncthreads();
  };
  {
    const std::integral_constant<int, 0> p0;
    const std::integral_constant<int, 1> p1;
    f32x16 sU = zero_f32x16();
    for (int s = 0; s < n_h; s += 2) {
      step(p0, s, sT, sU);
      if (s + 1 < n_h) step(p1, s + 1, sU, sT);
    }
  }
  // ---- merge the two key-tile streams (par 0 / par 1) of each query half
  lsum = half_sum(lsum);
  if (g == 0) {
    ml[((par * 2 + qh) * 32 + ln) * 2 + 0] = m;
    ml[((par * 2 + qh) * 32 + ln) * 2 + 1] = lsum;
  }
  wait_vm0();        // this wave's share of H_i has landed
  __syncthreads();   // also: all waves are done with the K / V tiles
  const float m_o = ml[(((par ^ 1) * 2 + qh) * 32 + ln) * 2 + 0];
  const float l_o = ml[(((par ^ 1) * 2 + qh) * 32 + ln) * 2 + 1];
  float cw = 0.0f, Lval = -INFINITY;
  if (n_h > 0) {
    const float mstar = fmaxf(m, m_o);   // raw-score units
    const float a_me = fast_exp2((m - mstar) * c2), a_ot = fast_exp2((m_o - mstar) * c2);
    const float ltot = lsum * a_me + l_o * a_ot;
    cw = a_me / ltot;
    Lval = mstar * c2 * kLn2 + logf(ltot);
  }
#pragma unroll
  for (int et = 0; et < NT; ++et)
#pragma unroll
    for (int r = 0; r < 16; ++r) oT[et][r] *= cw;
  float* myx = reinterpret_cast<float*>(gsm + (qh ? x1 : x0));   // exchange, then this query half's staging
  unsigned char* mystage = reinterpret_cast<unsigned char*>(myx);
  if (par == 1) {
#pragma unroll
    for (int et = 0; et < NT; ++et)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4)
        *reinterpret_cast<f32x4*>(myx + ((et * 4 + r4) * 64 + l) * 4) =
            f32x4{oT[et][4 * r4], oT[et][4 * r4 + 1], oT[et][4 * r4 + 2], oT[et][4 * r4 + 3]};
  }
  __syncthreads();
  const size_t orow0 = ((size_t)bh * N + q0 + 32 * qh) * D;   // first query of this wave
  const int wrows = rows - 32 * qh;                           // valid ones among its 32
  if (par == 0) {
#pragma unroll
    for (int et = 0; et < NT; ++et)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const f32x4 xv = *reinterpret_cast<const f32x4*>(myx + ((et * 4 + r4) * 64 + l) * 4);
#pragma unroll
        for (int r = 0; r < 4; ++r) oT[et][4 * r4 + r] += xv[r];
      }
    if (L && g == 0 && qok) L[(size_t)bh * N + q0 + qrow] = Lval;
    if (Os) store_rows_bf16<NT>(mystage, oT, Os + orow0, D, wrows, l);
  }
  // ---- linear branch: wave par computes O^l for features [par D/2, (par+1) D/2) of its queries
  // (both waves accumulate their share of O^l W into oT; par 1 starts again from zero)
  if (par == 1) {
#pragma unroll
    for (int et = 0; et < NT; ++et) oT[et] = zero_f32x16();
  }
  if (n_0 > 0) {
    __syncthreads();   // the exchange area is free: the projection matrix goes there
    issue_matrix(WTp, x0, x1);
    // phi(Q) of this lane's query: the lane holds features 16 t + 8 g + s, its partner the rest
    const float* Z = reinterpret_cast<const float*>(gsm + Lds::ZOFF);
    bf16x8 qp[KT];
    phi_fragments<KT>(qf, phi, qp);
    float den = 0.0f;
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      const f32x4 z0 = *reinterpret_cast<const f32x4*>(Z + 16 * t + 8 * g);
      const f32x4 z1 = *reinterpret_cast<const f32x4*>(Z + 16 * t + 8 * g + 4);
#pragma unroll
      for (int s2 = 0; s2 < 8; ++s2) den = fmaf((float)qp[t][s2], s2 < 4 ? z0[s2] : z1[s2 - 4], den);
    }
    den = half_sum(den);
    const float dinv = 1.0f / den;
    constexpr int HT = NT / 2;     // e-tiles per wave
    TileAddr<D> ma;                // rows 32 (et % 2) + ln of a 64-row tile: + 2 RB per odd tile
    ma.init(0, l);
    constexpr int RB = 16 * T::ROW_BYTES;
    f32x16 ol[HT];
#pragma unroll
    for (int h2 = 0; h2 < HT; ++h2) {
      const int et = par * HT + h2;
      ol[h2] = zero_f32x16();
#pragma unroll
      for (int t = 0; t < KT; ++t)
        ol[h2] = mfma32(lds_row(gsm, ma.row(t) + (et / 2 ? h1 : h0) + (et % 2) * 2 * RB), qp[t], ol[h2]);
#pragma unroll
      for (int r = 0; r < 16; ++r) ol[h2][r] *= dinv;
    }
    wait_vm0();
    __syncthreads();   // the projection matrix has landed; H_i is no longer needed
    // O^T[e'][q] += sum_{e in this wave's tiles} W[e][e'] O^l[q][e]
#pragma unroll
    for (int h2 = 0; h2 < HT; ++h2) {
      const int et = par * HT + h2;
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const bf16x8 b = c_to_operand(ol[h2], u);
#pragma unroll
        for (int ep = 0; ep < NT; ++ep)
          oT[ep] = mfma32(lds_row(gsm, ma.row(2 * et + u) + (ep / 2 ? x1 : x0) + (ep % 2) * 2 * RB), b, oT[ep]);
      }
    }
    if (Ol)
      store_rows_bf16<HT>(gsm + (w < 2 ? h0 : h1) + (w & 1) * (32 * (64 * HT + 16)), ol, Ol + orow0 + par * (D / 2), D,
                          wrows, l);
    __syncthreads();   // everyone is done with the projection matrix
    if (par == 1) {
#pragma unroll
      for (int et = 0; et < NT; ++et)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4)
          *reinterpret_cast<f32x4*>(myx + ((et * 4 + r4) * 64 + l) * 4) =
              f32x4{oT[et][4 * r4], oT[et][4 * r4 + 1], oT[et][4 * r4 + 2], oT[et][4 * r4 + 3]};
    }
    __syncthreads();
    if (par == 0) {
#pragma unroll
      for (int et = 0; et < NT; ++et)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const f32x4 xv = *reinterpret_cast<const f32x4*>(myx + ((et * 4 + r4) * 64 + l) * 4);
#pragma unroll
          for (int r = 0; r < 4; ++r) oT[et][4 * r4 + r] += xv[r];
        }
    }
  }
  if (par == 0) {
    store_rows_bf16<NT>(mystage, oT, O + lay.head(bh) + (size_t)(q0 + 32 * qh) * lay.ts, lay.ts, wrows, l);
    if (n_0 == 0 && Ol) {   // no marginal block: O^l is identically zero
#pragma unroll
      for (int et = 0; et < NT; ++et) oT[et] = zero_f32x16();
      store_rows_bf16<NT>(mystage, oT, Ol + orow0, D, wrows, l);
    }
  }
}

__global__ void fill_zero_f32_kernel(float* __restrict__ p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    p[i] = 0.0f;
}

#define SLA_TRY(x)                   \
  do {                               \
    hipError_t e_ = (x);             \
    if (e_ != hipSuccess) return e_; \
  } while (0)

template <int D>
hipError_t forward_impl(const Shape& s, const FwdArgs& a, bf16* hz16, bf16* WTp, hipStream_t st) {
  const int row_len = s.state_row();
  float* Zs = reinterpret_cast<float*>(reinterpret_cast<char*>(a.HZ) + state_z_offset(s));
  if (s.n_0 > 0) {
    {
      KernelTimer kt("states", st);
      states_mfma_kernel<D><<<dim3(s.T + 1, s.BH), 256, 0, st>>>((const bf16*)a.K, (const bf16*)a.V, s.N, s.T,
                                                               s.lay(), s.phi, hz16, (const bf16*)a.W, WTp);
    }
    SLA_TRY(mfma_aggregate(hz16, a.ind, s, a.HZ, Zs, st));
  } else if (a.Os) {   // saved states must read as zero
    KernelTimer kt("fill_zero", st);
    fill_zero_f32_kernel<<<1024, 256, 0, st>>>(a.HZ, (size_t)s.BH * s.T * row_len);
  }
  constexpr int lds = FwdLds<D>::BYTES;
  auto launch = [&](auto kern, int qt) -> hipError_t {
    SLA_TRY(ensure_dyn_lds(kern, qt * lds));
    KernelTimer kt("fwd_sparse", st);
    kern<<<dim3(xcd_grid((s.T + qt - 1) / qt), s.BH), 256 * qt, qt * lds, st>>>(
        (const bf16*)a.Q, (const bf16*)a.K, (const bf16*)a.V, WTp, a.row_idx, (const bf16*)a.HZ, Zs, s.N, s.T, s.lay(),
        s.n_h, s.n_0, s.phi, s.scale * kLog2e, (bf16*)a.O, (bf16*)a.Os, (bf16*)a.Ol, a.L);
    return hipSuccess;
  };
  // query blocks of an even number of tiles: tiles 2k and 2k + 1 have the same list and may share a
  // workgroup of eight waves (slower than two workgroups of four, hence on request only)
  if (s.rq % 2 == 0 && wide_query_tiles()) SLA_TRY(launch(fwd_mfma_kernel<D, 2>, 2));
  else SLA_TRY(launch(fwd_mfma_kernel<D, 1>, 1));
  return hipGetLastError();
}

}  // namespace

size_t mfma_forward_ws_bytes(const Shape& s) {
  return align_up((size_t)s.BH * s.T * s.state_row() * 2) + align_up((size_t)s.d * s.d * 2);
}

hipError_t mfma_forward(const Shape& s, const FwdArgs& a, char* ws, hipStream_t st) {
  bf16* hz16 = reinterpret_cast<bf16*>(ws);
  bf16* WTp = reinterpret_cast<bf16*>(ws + align_up((size_t)s.BH * s.T * s.state_row() * 2));
  return s.d == 64 ? forward_impl<64>(s, a, hz16, WTp, st) : forward_impl<128>(s, a, hz16, WTp, st);
}

}  // namespace sla
