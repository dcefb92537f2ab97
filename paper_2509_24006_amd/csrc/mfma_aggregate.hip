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
// Workgroup tile 256 (rows) x 128 (columns), k-step 64.  The state operand goes global -> LDS
// directly (row-major, swizzled, double-buffered) and is read with the transposing LDS read;
// the indicator operand is built in registers from 16-byte pieces of the padded int8 indicator.
#include "mfma_common.h"

namespace sla {
namespace {

constexpr int kTileB = kBlk * 256;   // 64 k-rows x 128 columns of bf16

// bytes (b0, b1, b2, b3) in {0,1} of `x` -> two dwords of bf16 pairs (1.0 or 0.0)
__device__ __forceinline__ void ind4(unsigned x, unsigned& lo, unsigned& hi) {
  lo = ((x & 0xffu) | ((x << 8) & 0xff0000u)) * 0x3f80u;
  hi = (((x >> 16) & 0xffu) | ((x >> 8) & 0xff0000u)) * 0x3f80u;
}

__global__ __launch_bounds__(256, 2) void aggregate_mfma_kernel(const bf16* __restrict__ in,
                                                                const int8_t* __restrict__ ind,
                                                                int T, int Tp, int row_len, int dd,
                                                                bf16* __restrict__ outH,
                                                                float* __restrict__ outZ) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, g = l >> 5, ln = l & 31;
  const int n0 = blockIdx.x * 128, m0 = blockIdx.y * 256, bh = blockIdx.z;
  const int8_t* ib = ind + (size_t)bh * T * Tp;
  const bf16* inb = in + (size_t)bh * T * row_len;
  const BufDesc rsrc = tile_rsrc(inb, T * row_len * 2);
  const int pitch = row_len * 2;
  const unsigned lds0 = lds_base(smem);
  f32x16 acc[2][4];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = zero_f32x16();
  const int ksteps = (T + kBlk - 1) / kBlk;
  // one wave-wide load deposits 4 rows x 256 bytes; wave w takes row groups w, w + 4, ...
  auto issue = [&](int ks) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int rg = 4 * k + w;
      const int row = 4 * rg + (l >> 4), pc = l & 15;
      const int voff = (ks * kBlk + row) * pitch + n0 * 2 + ((pc ^ swz<128>(row)) << 4);
      load_to_lds16(rsrc, voff, 0, lds0 + (ks & 1) * kTileB + rg * 1024);
    }
  };
  // indicator pieces of a k-step: rows m0 + 64 w + 32 mt + ln, 16 bytes per 16 k
  u32x4 ibn[2][4];
  auto load_ind = [&](int ks) {
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      const int i = m0 + 64 * w + 32 * mt + ln;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int k = ks * kBlk + 16 * u;
        ibn[mt][u] = (i < T && k < Tp) ? *reinterpret_cast<const u32x4*>(ib + (size_t)i * Tp + k)
                                       : u32x4{0u, 0u, 0u, 0u};
      }
    }
  };
  issue(0);
  load_ind(0);
  for (int ks = 0; ks < ksteps; ++ks) {
    wait_vm0();
    __syncthreads();
    u32x4 ib16[2][4];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int u = 0; u < 4; ++u) ib16[mt][u] = ibn[mt][u];
    if (ks + 1 < ksteps) {   // next step's tile and indicator pieces fly during this step's products
      issue(ks + 1);
      load_ind(ks + 1);
    }
    const unsigned char* Bs = smem + (ks & 1) * kTileB;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      // slots 0..3 <- k = 16u + 4g .. +3, slots 4..7 <- k = 16u + 8 + 4g .. +3
      bf16x8 a[2];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        const unsigned b0 = g ? ib16[mt][u].y : ib16[mt][u].x;
        const unsigned b1 = g ? ib16[mt][u].w : ib16[mt][u].z;
        unsigned p0, p1, p2, p3;
        ind4(b0, p0, p1);
        ind4(b1, p2, p3);
        u32x4 packed = {p0, p1, p2, p3};
        a[mt] = *reinterpret_cast<bf16x8*>(&packed);
      }
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) {
        const bf16x8 b = read_tr_swz<128>(Bs, 16 * u, nt, l);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) acc[mt][nt] = mfma32(a[mt], b, acc[mt][nt]);
      }
    }
  }
  // matrix part in bf16 (it is consumed as a bf16 MFMA operand), vector part in float
  bf16* oh = outH + (size_t)bh * T * dd;
  float* oz = outZ + (size_t)bh * T * (row_len - dd);
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
      const int col = n0 + 32 * nt + ln;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int row = m0 + 64 * w + 32 * mt + c_row(i, g);
        if (row < T && col < dd) oh[(size_t)row * dd + col] = __float2bfloat16(acc[mt][nt][i]);
        else if (row < T && col < row_len) oz[(size_t)row * (row_len - dd) + col - dd] = acc[mt][nt][i];
      }
    }
}

}  // namespace

// out[i] = sum over k with ind[i][k] = 1 of the bf16 state rows in[k] (d*d + d values each); ind is
// [BH][T][Tp] int8.  The d x d part goes to outH (bf16 [BH][T][d*d]), the d part to outZ (float).
hipError_t mfma_aggregate(const void* in, const int8_t* ind, const Shape& s, void* outH, float* outZ,
                          hipStream_t st) {
  const int row_len = s.state_row();
  const int Tp = (s.T + 15) / 16 * 16;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(aggregate_mfma_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, 2 * kTileB);
  if (e != hipSuccess) return e;
  KernelTimer kt("aggregate", st);
  aggregate_mfma_kernel<<<dim3((row_len + 127) / 128, (s.T + 255) / 256, s.BH), 256, 2 * kTileB, st>>>(
      (const bf16*)in, ind, s.T, Tp, row_len, s.d * s.d, (bf16*)outH, outZ);
  return hipGetLastError();
}

}  // namespace sla
