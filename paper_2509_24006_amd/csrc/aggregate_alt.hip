// The accumulation line of Alg. 1 (H_i = sum of h_j over the marginal blocks of row i) carried out
// the three ways the paper names, for comparison with the matrix-core product the library uses
// (mfma_aggregate.hip):
//   - one addition per marginal block (Alg. 1 as written),
//   - pre-aggregation (Appendix A.3): the sum over all key blocks, minus the other blocks,
//   - the Method of Four Russians (Appendix A.3): the sums of all 2^g subsets of every group of
//     g = 4 consecutive blocks are tabulated once, a row then adds one table entry per group.
// All three read bf16 state rows (d*d + d values: matrix, then vector), add in float, and write the
// matrix part in bf16 and the vector part in float, like the product.  A thread owns eight
// adjacent columns of the state row (16-byte loads; a wavefront reads 1 KB runs); the bits that
// steer a row are the same for the whole workgroup.
#include "sla_internal.h"

namespace sla {
namespace {

typedef __hip_bfloat16 bf16;
constexpr int kVec = 8;               // columns per thread: 16 bytes of a bf16 state row
constexpr int kCols = 256 * kVec;     // columns per workgroup
constexpr int kGroup = 4;             // g of the Four Russians tables

struct Acc {
  float v[kVec];
  __device__ __forceinline__ void zero() {
#pragma unroll
    for (int e = 0; e < kVec; ++e) v[e] = 0.0f;
  }
  __device__ __forceinline__ void add_row(const bf16* __restrict__ p) {   // 8 bf16 at p
    const uint4 raw = *reinterpret_cast<const uint4*>(p);
    const bf16* e8 = reinterpret_cast<const bf16*>(&raw);
#pragma unroll
    for (int e = 0; e < kVec; ++e) v[e] += __bfloat162float(e8[e]);
  }
  __device__ __forceinline__ void add_f32(const float* __restrict__ p) {   // 8 floats at p
    const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    v[0] += a.x; v[1] += a.y; v[2] += a.z; v[3] += a.w;
    v[4] += b.x; v[5] += b.y; v[6] += b.z; v[7] += b.w;
  }
  __device__ __forceinline__ void store_f32(float* __restrict__ p) const {
    *reinterpret_cast<float4*>(p) = float4{v[0], v[1], v[2], v[3]};
    *reinterpret_cast<float4*>(p + 4) = float4{v[4], v[5], v[6], v[7]};
  }
  // columns c .. c + 7 of output row `row`: the matrix part leaves in bf16, the vector part in float
  // (d*d is a multiple of 8, so the eight columns lie on one side)
  __device__ __forceinline__ void put(int c, int dd, size_t row, bf16* outH, float* outZ, int dz) const {
    if (c < dd) {
      bf16 o[kVec];
#pragma unroll
      for (int e = 0; e < kVec; ++e) o[e] = __float2bfloat16(v[e]);
      *reinterpret_cast<uint4*>(outH + row * dd + c) = *reinterpret_cast<const uint4*>(o);
    } else {
      store_f32(outZ + row * dz + (c - dd));
    }
  }
};

// bits of word q of a row that belong to existing key blocks
__device__ __forceinline__ unsigned long long valid_bits(int T, int q) {
  const int left = T - 64 * q;
  return left >= 64 ? ~0ull : ((1ull << left) - 1ull);
}

// adds in[64 q + b][c ..] for the set bits b of `w` (word q of a row's bit mask)
__device__ __forceinline__ void add_bits(Acc& a, const bf16* __restrict__ col, size_t row_len, unsigned long long w,
                                         int q) {
  while (w) {
    const int b = __ffsll((long long)w) - 1;
    w &= w - 1;
    a.add_row(col + (size_t)(64 * q + b) * row_len);
  }
}

// One addition per marginal block.  grid (ceil(row_len / 2048), T, BH)
__global__ __launch_bounds__(256) void agg_add_kernel(const bf16* __restrict__ in,
                                                      const unsigned long long* __restrict__ ind, int T, int Tw,
                                                      int row_len, int dd, bf16* __restrict__ outH,
                                                      float* __restrict__ outZ) {
  const int c = blockIdx.x * kCols + threadIdx.x * kVec, i = blockIdx.y, bh = blockIdx.z;
  if (c >= row_len) return;
  const bf16* col = in + (size_t)bh * T * row_len + c;
  const unsigned long long* w = ind + ((size_t)bh * T + i) * Tw;
  Acc a;
  a.zero();
  for (int q = 0; q < Tw; ++q) add_bits(a, col, row_len, w[q], q);
  a.put(c, dd, (size_t)bh * T + i, outH, outZ, row_len - dd);
}

// total[bh][c] = sum over all key blocks.  grid (ceil(row_len / 2048), BH)
__global__ __launch_bounds__(256) void agg_total_kernel(const bf16* __restrict__ in, int T, int row_len,
                                                        float* __restrict__ total) {
  const int c = blockIdx.x * kCols + threadIdx.x * kVec, bh = blockIdx.y;
  if (c >= row_len) return;
  const bf16* col = in + (size_t)bh * T * row_len + c;
  Acc a;
  a.zero();
  for (int k = 0; k < T; ++k) a.add_row(col + (size_t)k * row_len);
  a.store_f32(total + (size_t)bh * row_len + c);
}

// The total minus the blocks that are not marginal.  grid as agg_add_kernel
__global__ __launch_bounds__(256) void agg_preagg_kernel(const bf16* __restrict__ in,
                                                         const unsigned long long* __restrict__ ind,
                                                         const float* __restrict__ total, int T, int Tw,
                                                         int row_len, int dd, bf16* __restrict__ outH,
                                                         float* __restrict__ outZ) {
  const int c = blockIdx.x * kCols + threadIdx.x * kVec, i = blockIdx.y, bh = blockIdx.z;
  if (c >= row_len) return;
  const bf16* col = in + (size_t)bh * T * row_len + c;
  const unsigned long long* w = ind + ((size_t)bh * T + i) * Tw;
  Acc other, r;
  other.zero();
  for (int q = 0; q < Tw; ++q) add_bits(other, col, row_len, ~w[q] & valid_bits(T, q), q);
  r.zero();
  r.add_f32(total + (size_t)bh * row_len + c);
#pragma unroll
  for (int e = 0; e < kVec; ++e) r.v[e] -= other.v[e];
  r.put(c, dd, (size_t)bh * T + i, outH, outZ, row_len - dd);
}

// tab[bh][group][m][c] = sum of in[4 group + b][c] over the bits b of m, m = 0 .. 15 (float).
// grid (ceil(row_len / 2048), groups, BH)
__global__ __launch_bounds__(256) void fr_table_kernel(const bf16* __restrict__ in, int T, int groups, int row_len,
                                                       float* __restrict__ tab) {
  const int c = blockIdx.x * kCols + threadIdx.x * kVec, gr = blockIdx.y, bh = blockIdx.z;
  if (c >= row_len) return;
  Acc v[kGroup];
#pragma unroll
  for (int b = 0; b < kGroup; ++b) {
    const int k = kGroup * gr + b;
    v[b].zero();
    if (k < T) v[b].add_row(in + ((size_t)bh * T + k) * row_len + c);
  }
  float* t = tab + (((size_t)bh * groups + gr) << kGroup) * row_len + c;
#pragma unroll
  for (int m = 0; m < (1 << kGroup); ++m) {
    Acc s;
    s.zero();
#pragma unroll
    for (int b = 0; b < kGroup; ++b)
      if (m >> b & 1) {
#pragma unroll
        for (int e = 0; e < kVec; ++e) s.v[e] += v[b].v[e];
      }
    s.store_f32(t + (size_t)m * row_len);
  }
}

// One table entry per group of four blocks.  grid as agg_add_kernel
__global__ __launch_bounds__(256) void fr_lookup_kernel(const float* __restrict__ tab,
                                                        const unsigned long long* __restrict__ ind, int T, int Tw,
                                                        int groups, int row_len, int dd, bf16* __restrict__ outH,
                                                        float* __restrict__ outZ) {
  const int c = blockIdx.x * kCols + threadIdx.x * kVec, i = blockIdx.y, bh = blockIdx.z;
  if (c >= row_len) return;
  const unsigned long long* w = ind + ((size_t)bh * T + i) * Tw;
  const float* t = tab + (((size_t)bh * groups) << kGroup) * row_len + c;
  Acc a;
  a.zero();
  for (int gr = 0; gr < groups; ++gr) {
    const int m = (int)(w[gr >> 4] >> (kGroup * (gr & 15))) & 15;   // 16 groups per 64-bit word
    if (m) a.add_f32(t + (((size_t)gr << kGroup) + m) * row_len);
  }
  a.put(c, dd, (size_t)bh * T + i, outH, outZ, row_len - dd);
}

}  // namespace

size_t aggregate_alt_ws_bytes(const Shape& s, int method) {
  const size_t row_len = s.state_row();
  if (method == 2) return align_up((size_t)s.BH * row_len * 4);
  if (method == 3) return align_up(((size_t)s.BH * ((s.T + kGroup - 1) / kGroup) << kGroup) * row_len * 4);
  return 0;
}

// method 1: additions, 2: pre-aggregation, 3: Four Russians.  in: bf16 [BH][T][d*d + d]
hipError_t aggregate_alt(int method, const void* in, const unsigned long long* ind, const Shape& s, void* outH,
                         float* outZ, void* ws, hipStream_t st) {
  const int row_len = s.state_row(), dd = s.d * s.d, Tw = (s.T + 63) / 64;
  const int cb = (row_len + kCols - 1) / kCols;
  const bf16* h = (const bf16*)in;
  const dim3 rows(cb, s.T, s.BH);
  if (method == 1) {
    KernelTimer kt("agg_add", st);
    agg_add_kernel<<<rows, 256, 0, st>>>(h, ind, s.T, Tw, row_len, dd, (bf16*)outH, outZ);
  } else if (method == 2) {
    {
      KernelTimer kt("agg_total", st);
      agg_total_kernel<<<dim3(cb, s.BH), 256, 0, st>>>(h, s.T, row_len, (float*)ws);
    }
    KernelTimer kt("agg_preagg", st);
    agg_preagg_kernel<<<rows, 256, 0, st>>>(h, ind, (const float*)ws, s.T, Tw, row_len, dd, (bf16*)outH, outZ);
  } else if (method == 3) {
    const int groups = (s.T + kGroup - 1) / kGroup;
    {
      KernelTimer kt("agg_fr_table", st);
      fr_table_kernel<<<dim3(cb, groups, s.BH), 256, 0, st>>>(h, s.T, groups, row_len, (float*)ws);
    }
    KernelTimer kt("agg_fr_lookup", st);
    fr_lookup_kernel<<<rows, 256, 0, st>>>((const float*)ws, ind, s.T, Tw, groups, row_len, dd, (bf16*)outH, outZ);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace sla
