// State aggregation of the linear branch as a dense matrix-core GEMM.
//
// Alg. 1 adds h_j, z_j into H_i, Z_i for every marginal block of row i, and Alg. 2 adds dH_i,
// dZ_i into the sums of key block j for every marginal block of column j.  Over all rows that is
//   out[i][:] = sum_k ind[i][k] in[k][:],   ind = 1 where the block is marginal, else 0,
// a T x T by T x (d*d + d) product per head.  The indicator is exact in bf16, the products are
// bf16 x bf16 with float accumulation.  Compared with adding the marginal blocks one by one
// (or subtracting the others from the total, App. A.3) the state rows are read once per 256
// output rows instead of once per row.
//
// The kernel is bound by HBM traffic (one read of the states, one write of the sums), so the
// design keeps everything else small: the indicator comes as bit masks, 8 bytes per row and
// k-step; the state tiles go global -> LDS directly (row-major, swizzled) through a ring of stages
// and are read with the transposing LDS read; the product is formed with the output rows along the
// lanes, so that the sums leave as whole 256-byte row pieces.  A workgroup of four waves owns 256
// output rows by 128 columns and two of them share a CU: while one fills its ring or stores its
// sums (a store drains the wave's whole memory queue: loads and stores complete in no fixed order
// relative to each other, so nothing can be waited for selectively behind it), the other computes.
// The workgroups that own the same columns run back to back on one XCD, so that the second read
// of the states comes from its L2.
#include "mfma_common.h"

namespace sla {
namespace {

constexpr int kStage = kBlk * 256;   // one k-step of states: 64 rows x 128 columns of bf16
constexpr int kStages = 4;           // ring of state tiles
constexpr int kOutStage = 32 * (64 * 4 + 16);   // store_rows_bf16<4> area of one wave
constexpr int kAggLds = kStages * kStage;       // the output staging is laid over the ring
constexpr int kAggRows = 256;        // output rows of one workgroup
static_assert(4 * kOutStage <= kAggLds, "staging of four waves fits in the ring");

// two adjacent indicator bits (bits s, s + 1 of x) -> a dword holding two bf16 (1.0 or 0.0)
__device__ __forceinline__ unsigned bits2bf(unsigned x, int s) {
  const unsigned y = (x >> s) & 3u;
  return (((y << 15) | y) & 0x00010001u) * 0x3f80u;
}

// Column tile ct < dd / 128: columns [128 ct, +128) of the matrix part, written in bf16; column
// tile dd / 128: the vector part (the last d entries of a state row), written in float.
// blockIdx.x = 8 (mtiles cg + mh) + x for column tile 8 cg + x and row tile mh: the round-robin
// deal puts the row tiles of one column tile on the same XCD, one after the other.
__global__ __launch_bounds__(256, 2) void aggregate_mfma_kernel(const bf16* __restrict__ in,
                                                                const unsigned long long* __restrict__ ind,
                                                                int T, int Tw, int row_len, int dd, int mtiles,
                                                                bf16* __restrict__ outH, float* __restrict__ outZ) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, g = l >> 5, ln = l & 31;
  const int rr = blockIdx.x >> 3;
  const int ct = (rr / mtiles) * 8 + (blockIdx.x & 7), mh = rr % mtiles, bh = blockIdx.y;
  if (ct > dd / 128) return;
  const bool zpart = ct == dd / 128;
  const int nbase = ct * 128, m0 = mh * kAggRows;
  const unsigned long long* ib = ind + (size_t)bh * T * Tw;
  const bf16* inb = in + (size_t)bh * T * row_len;
  const BufDesc rsrc = tile_rsrc(inb, T * row_len * 2);
  const int pitch = row_len * 2;
  const int wu = wave_uniform(w);
  const unsigned lds0 = lds_base(smem);
  f32x16 acc[2][4];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = zero_f32x16();
  const int ksteps = (T + kBlk - 1) / kBlk;
  // one wave-wide load deposits 4 rows x 256 bytes; wave w takes the 1 KB runs w, w + 4, w + 8 and
  // w + 12 of a stage; rows past T read as zeros (the vector part of a narrow head reads on into
  // the next row: those columns are not written)
  int vo[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int row = 4 * (4 * k + w) + (l >> 4), pc = l & 15;
    vo[k] = row * pitch + nbase * 2 + ((pc ^ swz<128>(row)) << 4);
  }
  int iks = 0, istage = 0;   // the next tile to request and its stage
  auto issue_next = [&]() {
    if (iks >= ksteps) return;
#pragma unroll
    for (int k = 0; k < 4; ++k)
      load_to_lds16(rsrc, vo[k], iks * kBlk * pitch, lds0 + istage * kStage + (4 * k + wu) * 1024);
    istage = istage == kStages - 1 ? 0 : istage + 1;
    ++iks;
  };
  // per-lane offsets of the transposing reads inside a stage: [8-row half][column tile]
  TileAddr<128> ad;
  ad.init(0, l);
  int tro[2][4];
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) tro[h][nt] = ad.tr(h, nt);
  constexpr int RB = 16 * SwzTile<128>::ROW_BYTES;
  const int row0 = m0 + 64 * w + ln;   // this lane's output rows: row0 and row0 + 32
#pragma unroll
  for (int k = 0; k < kStages - 1; ++k) issue_next();
  int stage = 0;
  for (int ks0 = 0; ks0 < ksteps; ks0 += 8) {
    // indicator words of the next eight k-steps for the lane's two rows
    unsigned long long wb[2][8];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int i = row0 + 32 * mt;
        wb[mt][q] = (i < T && ks0 + q < Tw) ? ib[(size_t)i * Tw + ks0 + q] : 0ull;
      }
    // (waited for here, once per eight k-steps, rather than at each first use below; the wait
    // also drains the tile loads in flight, which at the start are the ones needed first anyway)
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int q = 0; q < 8; ++q) pin_loaded(wb[mt][q]);
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int ks = ks0 + q;
      if (ks >= ksteps) break;
      // the lane's bits of this k-step, moved so that k = 16 u + 4 g sits at bit 16 u
      const unsigned long long x0 = wb[0][q] >> (4 * g), x1 = wb[1][q] >> (4 * g);
      // the tile has landed; the kStages - 2 tiles requested after it may still be in flight
      if (ks + kStages - 2 < ksteps) wait_vm<4 * (kStages - 2)>();
      else wait_vm0();
      __syncthreads();   // ... for every wave, and the stage of the previous tile is free
      issue_next();
      const int so = stage * kStage;
      stage = stage == kStages - 1 ? 0 : stage + 1;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        // slots 0..3 <- k = 16 u + 4 g .. + 3, slots 4..7 <- k = 16 u + 8 + 4 g .. + 3: the order
        // in which the transposing read hands over the state rows
        bf16x8 b[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
          const unsigned long long x = mt ? x1 : x0;
          const unsigned half = u < 2 ? (unsigned)x : (unsigned)(x >> 32);
          const int sh = 16 * (u & 1);
          u32x4 packed = {bits2bf(half, sh), bits2bf(half, sh + 2), bits2bf(half, sh + 8), bits2bf(half, sh + 10)};
          b[mt] = *reinterpret_cast<bf16x8*>(&packed);
        }
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
          const bf16x8 a = lds_tr<128>(smem, tro[0][nt] + so + u * RB, tro[1][nt] + so + u * RB);
#pragma unroll
          for (int mt = 0; mt < 2; ++mt) acc[mt][nt] = mfma32(a, b[mt], acc[mt][nt]);
        }
      }
    }
  }
  // C tiles: lane = output row, registers = columns 32 nt + c_row(r, g)
  if (zpart) {
    const int dz = row_len - dd;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      const int row = row0 + 32 * mt;
      if (row >= T) continue;
      float* o = outZ + ((size_t)bh * T + row) * dz;
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int c = 32 * nt + 8 * r4 + 4 * g;
          if (c < dz)
            *reinterpret_cast<f32x4*>(o + c) = f32x4{acc[mt][nt][4 * r4], acc[mt][nt][4 * r4 + 1],
                                                      acc[mt][nt][4 * r4 + 2], acc[mt][nt][4 * r4 + 3]};
        }
    }
  } else {
    __syncthreads();   // every wave has read the last tile: the ring becomes the staging areas
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      const int r0 = m0 + 64 * w + 32 * mt;
      if (r0 < T)
        store_rows_bf16<4>(smem + wu * kOutStage, acc[mt], outH + ((size_t)bh * T + r0) * dd + nbase, dd, T - r0, l);
    }
  }
}

// Short sequences (T <= 64: one k-step, one indicator word per row): a workgroup's four waves
// take four column tiles of the same 32 MT output rows, each wave with a stage of its own, so
// that no wave waits for another; the rows of the stage past T are fetched as zeros.
template <int MT>
__global__ __launch_bounds__(256, 2) void aggregate_short_kernel(const bf16* __restrict__ in,
                                                                 const unsigned long long* __restrict__ ind,
                                                                 int T, int row_len, int dd,
                                                                 bf16* __restrict__ outH, float* __restrict__ outZ) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, g = l >> 5, ln = l & 31;
  const int ct = blockIdx.x * 4 + w, bh = blockIdx.y;
  if (ct > dd / 128) return;   // (no barriers in this kernel)
  const bool zpart = ct == dd / 128;
  const int nbase = ct * 128;
  const unsigned long long* ib = ind + (size_t)bh * T;
  const bf16* inb = in + (size_t)bh * T * row_len;
  const BufDesc rsrc = tile_rsrc(inb, T * row_len * 2);
  const int pitch = row_len * 2;
  const int wu = wave_uniform(w);
  unsigned char* stage = smem + wu * kStage;
  const unsigned lds0 = lds_base(smem) + wu * kStage;
  const int nu = (T + 15) / 16;   // 16-row groups that hold valid rows
  for (int k = 0; k < 4 * nu; ++k) {
    const int row = 4 * k + (l >> 4), pc = l & 15;
    load_to_lds16(rsrc, row * pitch + nbase * 2 + ((pc ^ swz<128>(row)) << 4), 0, lds0 + k * 1024);
  }
  unsigned long long wb[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) wb[mt] = (ln + 32 * mt < T) ? ib[ln + 32 * mt] : 0ull;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) pin_loaded(wb[mt]);
  wait_vm0();
  TileAddr<128> ad;
  ad.init(0, l);
  constexpr int RB = 16 * SwzTile<128>::ROW_BYTES;
  f32x16 acc[MT][4];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = zero_f32x16();
  for (int u = 0; u < nu; ++u) {
    bf16x8 b[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const unsigned long long x = wb[mt] >> (4 * g);
      const unsigned half = (unsigned)(x >> (16 * u));   // u < 4: bits 16 u + 4 g ..
      u32x4 packed = {bits2bf(half, 0), bits2bf(half, 2), bits2bf(half, 8), bits2bf(half, 10)};
      b[mt] = *reinterpret_cast<bf16x8*>(&packed);
    }
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
      const bf16x8 a = lds_tr<128>(stage, ad.tr(0, nt) + u * RB, ad.tr(1, nt) + u * RB);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) acc[mt][nt] = mfma32(a, b[mt], acc[mt][nt]);
    }
  }
  if (zpart) {
    const int dz = row_len - dd;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int row = ln + 32 * mt;
      if (row >= T) continue;
      float* o = outZ + ((size_t)bh * T + row) * dz;
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int c = 32 * nt + 8 * r4 + 4 * g;
          if (c < dz)
            *reinterpret_cast<f32x4*>(o + c) = f32x4{acc[mt][nt][4 * r4], acc[mt][nt][4 * r4 + 1],
                                                      acc[mt][nt][4 * r4 + 2], acc[mt][nt][4 * r4 + 3]};
        }
    }
  } else {
    // the wave's own stage becomes its staging area (LDS serves a wave's accesses in order)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      if (32 * mt < T)
        store_rows_bf16<4>(stage, acc[mt], outH + ((size_t)bh * T + 32 * mt) * dd + nbase, dd, T - 32 * mt, l);
  }
}

}  // namespace

// out[i] = sum over k with bit k of ind[i] set of the bf16 state rows in[k] (d*d + d values each);
// ind is [BH][T][ceil(T/64)] 64-bit masks.  The d x d part goes to outH (bf16 [BH][T][d*d]), the d
// part to outZ (float).
hipError_t mfma_aggregate(const void* in, const unsigned long long* ind, const Shape& s, void* outH,
                          float* outZ, hipStream_t st) {
  const int row_len = s.state_row(), dd = s.d * s.d;
  const int Tw = (s.T + 63) / 64;
  if (dd % 128 != 0 || row_len - dd > 128) return hipErrorInvalidValue;
  hipError_t e = ensure_dyn_lds(aggregate_mfma_kernel, kAggLds);
  if (e != hipSuccess) return e;
  const int mtiles = (s.T + kAggRows - 1) / kAggRows;
  const int ntile = dd / 128 + 1;
  if (s.T <= 64) {
    auto kern = s.T <= 32 ? aggregate_short_kernel<1> : aggregate_short_kernel<2>;
    e = ensure_dyn_lds(kern, kAggLds);
    if (e != hipSuccess) return e;
    KernelTimer kt("aggregate", st);
    kern<<<dim3((ntile + 3) / 4, s.BH), 256, kAggLds, st>>>((const bf16*)in, ind, s.T, row_len, dd, (bf16*)outH, outZ);
    return hipGetLastError();
  }
  {
    KernelTimer kt("aggregate", st);
    aggregate_mfma_kernel<<<dim3(8 * ((ntile + 7) / 8) * mtiles, s.BH), 256, kAggLds, st>>>(
        (const bf16*)in, ind, s.T, Tw, row_len, dd, mtiles, (bf16*)outH, outZ);
  }
  return hipGetLastError();
}

}  // namespace sla
