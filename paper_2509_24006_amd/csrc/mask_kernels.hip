// Mask step of SLA on gfx950: block mean-pooling, pooled scores, three-way classification
// (Eq. 2, Eq. 3, Alg. 1 mask line) and the row / column lookup tables of Appendix A.3.
//
// All arithmetic that decides the mask is float in one fixed order so that the integer
// result is reproducible: sequential add over a block's tokens, one IEEE division, a
// fused multiply-add chain over the features, one multiply by 1/sqrt(d).
#include "sla_internal.h"

namespace sla {
namespace {

// ---------------------------------------------------------------- pool
// A lane owns the 16 bytes of a token row that hold V adjacent features and walks the rows of
// its block in order (the sum over a block's tokens is sequential, see above); D / V lanes cover
// a block, so a wavefront pools 64 V / D blocks at once and each of its loads fetches whole
// rows.  blockIdx.y selects the tensor (Q with blocks of len0 tokens, Tn0 per head, or K with
// len1, Tn1).
template <typename T, int D>
__global__ __launch_bounds__(256) void pool_kernel(const T* __restrict__ X0, const T* __restrict__ X1, int BH, int N,
                                                   int Tn0, int len0, int Tn1, int len1, Lay lay,
                                                   float* __restrict__ out0, float* __restrict__ out1) {
  constexpr int V = 16 / sizeof(T), LPB = D / V, BPW = 64 / LPB;
  const T* X = blockIdx.y ? X1 : X0;
  float* out = blockIdx.y ? out1 : out0;
  const int Tn = blockIdx.y ? Tn1 : Tn0, len = blockIdx.y ? len1 : len0;
  const int lane = threadIdx.x & 63, sub = lane / LPB, fl = lane % LPB;
  const long blk = ((long)blockIdx.x * 4 + (threadIdx.x >> 6)) * BPW + sub;
  if (blk >= (long)BH * Tn) return;
  const int bh = (int)(blk / Tn), i = (int)(blk % Tn);
  const int cnt = min(len, N - i * len);
  const T* p = X + lay.head(bh) + (size_t)i * len * lay.ts + fl * V;
  float s[V];
#pragma unroll
  for (int v = 0; v < V; ++v) s[v] = 0.0f;
  // 16 rows are requested before the first is added (the sum itself stays in token order)
  int r = 0;
  for (; r + 16 <= cnt; r += 16) {
    uint4 raw[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) raw[k] = *reinterpret_cast<const uint4*>(p + (size_t)(r + k) * lay.ts);
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const T* e = reinterpret_cast<const T*>(&raw[k]);
#pragma unroll
      for (int v = 0; v < V; ++v) s[v] = s[v] + to_f32(e[v]);
    }
  }
  for (; r < cnt; ++r) {
    const uint4 raw = *reinterpret_cast<const uint4*>(p + (size_t)r * lay.ts);
    const T* e = reinterpret_cast<const T*>(&raw);
#pragma unroll
    for (int v = 0; v < V; ++v) s[v] = s[v] + to_f32(e[v]);
  }
  const float c = (float)cnt;
  float* o = out + (size_t)blk * D + fl * V;
#pragma unroll
  for (int v = 0; v < V; v += 4)
    *reinterpret_cast<float4*>(o + v) = float4{__fdiv_rn(s[v], c), __fdiv_rn(s[v + 1], c), __fdiv_rn(s[v + 2], c),
                                               __fdiv_rn(s[v + 3], c)};
}

// ---------------------------------------------------------------- scores
// 64x64 output tile per workgroup, 4x4 outputs per thread, features staged through LDS in
// chunks of 64 and read four at a time; each output keeps one fused multiply-add chain in
// ascending feature order.
// acc[a][b] = sum over features (ascending, one fused multiply-add chain) of
// qb[i0 + ty + 16 a][.] kb[j0 + tx + 16 b][.]; rows past Tq / T count as zeros.
__device__ __forceinline__ void score_tile(const float* __restrict__ qb, const float* __restrict__ kb, int Tq, int T,
                                           int d, int i0, int j0, float (*qs)[68], float (*ks)[68],
                                           float (&acc)[4][4]) {
  const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = 0.0f;
  for (int k0 = 0; k0 < d; k0 += 64) {
    // thread t brings 16 bytes: piece t % 16 of rows t / 16 + 16 q (d is a multiple of 64)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int r = (tid >> 4) + 16 * q, c = 4 * (tid & 15);
      const float4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
      *reinterpret_cast<float4*>(&qs[r][c]) =
          (i0 + r < Tq) ? *reinterpret_cast<const float4*>(qb + (size_t)(i0 + r) * d + k0 + c) : zero;
      *reinterpret_cast<float4*>(&ks[r][c]) =
          (j0 + r < T) ? *reinterpret_cast<const float4*>(kb + (size_t)(j0 + r) * d + k0 + c) : zero;
    }
    __syncthreads();
#pragma unroll 4
    for (int k = 0; k < 64; k += 4) {
      float4 av[4], bv[4];
#pragma unroll
      for (int a = 0; a < 4; ++a) av[a] = *reinterpret_cast<const float4*>(&qs[ty + 16 * a][k]);
#pragma unroll
      for (int b = 0; b < 4; ++b) bv[b] = *reinterpret_cast<const float4*>(&ks[tx + 16 * b][k]);
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          float x = acc[a][b];
          x = __fmaf_rn(av[a].x, bv[b].x, x);
          x = __fmaf_rn(av[a].y, bv[b].y, x);
          x = __fmaf_rn(av[a].z, bv[b].z, x);
          x = __fmaf_rn(av[a].w, bv[b].w, x);
          acc[a][b] = x;
        }
    }
    __syncthreads();
  }
}

__global__ __launch_bounds__(256) void score_kernel(const float* __restrict__ qbar,
                                                    const float* __restrict__ kbar, int Tq, int T, int d,
                                                    float scale, float* __restrict__ s) {
  __shared__ __attribute__((aligned(16))) float qs[64][68];
  __shared__ __attribute__((aligned(16))) float ks[64][68];
  const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
  const int bh = blockIdx.z, i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
  float acc[4][4];
  score_tile(qbar + (size_t)bh * Tq * d, kbar + (size_t)bh * T * d, Tq, T, d, i0, j0, qs, ks, acc);
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int i = i0 + ty + 16 * a;
    if (i >= Tq) continue;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const int j = j0 + tx + 16 * b;
      if (j < T) s[((size_t)bh * Tq + i) * T + j] = __fmul_rn(acc[a][b], scale);
    }
  }
}

// ---------------------------------------------------------------- classify
// Order-preserving map float -> uint32 (larger float <=> larger key); +0 and -0 coincide.
__device__ __forceinline__ uint32_t order_key(float f) {
  uint32_t b = __float_as_uint(f);
  if (b == 0x80000000u) b = 0u;
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// k-th largest key of a row held in LDS (k >= 1), found bit by bit: the result is the
// largest t with #{key >= t} >= k.  Entries whose key is 0 never count.
__device__ uint32_t kth_largest(const uint32_t* keys, int T, int k, int lane) {
  uint32_t prefix = 0;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cand = prefix | (1u << bit);
    int c = 0;
    for (int j = lane; j < T; j += 64) c += (keys[j] >= cand);
    if (wave_sum(c) >= k) prefix = cand;
  }
  return prefix;
}

// Marks with `label` the k entries that come first under (key descending, index
// ascending) among the entries with a non-zero key.
__device__ void mark_top(const uint32_t* keys, int8_t* lab, int T, int k, int8_t label, int lane) {
  if (k <= 0) return;
  const uint32_t thr = kth_largest(keys, T, k, lane);
  int c = 0;
  for (int j = lane; j < T; j += 64) c += (keys[j] > thr);
  int need = k - wave_sum(c);  // how many of the entries equal to thr are taken, lowest index first
  for (int j0 = 0; j0 < T; j0 += 64) {
    const int j = j0 + lane;
    const uint32_t key = (j < T) ? keys[j] : 0u;
    const bool eq = (j < T) && (key == thr);
    const unsigned long long m = __ballot(eq);
    const int before = __popcll(m & ((1ull << lane) - 1ull));
    if (j < T && (key > thr || (eq && before < need))) lab[j] = label;
    need -= __popcll(m);
  }
}

// The same with the row in registers (entry j = 64 i + lane in slot i, key 0 past the end): every
// count is a handful of wave votes tallied on the scalar side, no LDS and no cross-lane shuffles.
template <int KPL>
__device__ __forceinline__ void mark_top_reg(const uint32_t (&key)[KPL], int8_t (&lab)[KPL], int k, int8_t label,
                                             int lane) {
  if (k <= 0) return;
  uint32_t thr = 0;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cand = thr | (1u << bit);
    int c = 0;
#pragma unroll
    for (int i = 0; i < KPL; ++i) c += __popcll(__ballot(key[i] >= cand));
    if (c >= k) thr = cand;
  }
  int need = k;
#pragma unroll
  for (int i = 0; i < KPL; ++i) need -= __popcll(__ballot(key[i] > thr));
#pragma unroll
  for (int i = 0; i < KPL; ++i) {   // ascending index: slot by slot, lane by lane
    const bool eq = key[i] == thr;
    const unsigned long long m = __ballot(eq);
    const int before = __popcll(m & ((1ull << lane) - 1ull));
    if (key[i] > thr || (eq && before < need)) lab[i] = label;
    need -= __popcll(m);
  }
}

// One wavefront per row of the score matrix, rows of at most 64 KPL entries.
template <int KPL>
__global__ __launch_bounds__(256) void classify_reg_kernel(const float* __restrict__ s, int rows, int Tq, int rq,
                                                           int T, int n_h, int n_l, int8_t* __restrict__ Mc,
                                                           int32_t* __restrict__ row_idx,
                                                           int32_t* __restrict__ col_cnt) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * 4 + wave;
  if (row >= rows) return;   // (no barriers in this kernel)
  // the query tiles of this row of the mask: each gets a copy of the row's table entries
  const size_t t0 = (size_t)(row / Tq) * T + (size_t)(row % Tq) * rq;
  const int nrep = min(rq, T - (int)(row % Tq) * rq);
  if (lane < nrep) col_cnt[t0 + lane] = 0;   // one counter per (head, key block), cleared for the column count that follows
  const float* sr = s + (size_t)row * T;
  uint32_t key[KPL];
  int8_t lab[KPL];
#pragma unroll
  for (int i = 0; i < KPL; ++i) {
    const int j = 64 * i + lane;
    key[i] = j < T ? order_key(sr[j]) : 0u;
    lab[i] = 0;
  }
  mark_top_reg<KPL>(key, lab, n_h, (int8_t)1, lane);
  // negligible: lowest scores among the rest = largest inverted keys; critical entries and the
  // slots past the end get key 0 and drop out
#pragma unroll
  for (int i = 0; i < KPL; ++i) key[i] = (lab[i] == 1 || 64 * i + lane >= T) ? 0u : ~key[i];
  mark_top_reg<KPL>(key, lab, n_l, (int8_t)-1, lane);
  int base = 0;
#pragma unroll
  for (int i = 0; i < KPL; ++i) {
    const int j = 64 * i + lane;
    if (j < T) Mc[(size_t)row * T + j] = lab[i];
    const unsigned long long m = __ballot(lab[i] == 1);
    if (lab[i] == 1) {
      const int pos = base + __popcll(m & ((1ull << lane) - 1ull));
      for (int r = 0; r < nrep; ++r) row_idx[(t0 + r) * n_h + pos] = j;
    }
    base += __popcll(m);
  }
}

// One wavefront per row of the score matrix.
__global__ __launch_bounds__(256) void classify_kernel(const float* __restrict__ s, int rows, int Tq, int rq, int T,
                                                       int n_h, int n_l, int8_t* __restrict__ Mc,
                                                       int32_t* __restrict__ row_idx,
                                                       int32_t* __restrict__ col_cnt) {
  extern __shared__ unsigned char smem[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  uint32_t* keys = reinterpret_cast<uint32_t*>(smem) + (size_t)wave * T;
  int8_t* lab = reinterpret_cast<int8_t*>(smem + (size_t)4 * T * sizeof(uint32_t)) + (size_t)wave * T;
  const long row_raw = (long)blockIdx.x * 4 + wave;
  const bool live = row_raw < rows;  // surplus wavefronts redo the last row and store nothing
  const long row = live ? row_raw : rows - 1;
  const size_t t0 = (size_t)(row / Tq) * T + (size_t)(row % Tq) * rq;   // first query tile of this row of the mask
  const int nrep = min(rq, T - (int)(row % Tq) * rq);
  if (live && lane < nrep) col_cnt[t0 + lane] = 0;   // cleared for the column count that follows
  const float* sr = s + (size_t)row * T;
  for (int j = lane; j < T; j += 64) {
    keys[j] = order_key(sr[j]);
    lab[j] = 0;
  }
  __syncthreads();
  mark_top(keys, lab, T, n_h, (int8_t)1, lane);
  __syncthreads();
  // negligible: lowest scores among the rest = largest inverted keys; critical entries get
  // key 0 and drop out
  for (int j = lane; j < T; j += 64) keys[j] = (lab[j] == 1) ? 0u : ~keys[j];
  __syncthreads();
  mark_top(keys, lab, T, n_l, (int8_t)-1, lane);
  __syncthreads();
  int base = 0;
  for (int j0 = 0; j0 < T; j0 += 64) {
    const int j = j0 + lane;
    const int8_t v = (j < T) ? lab[j] : (int8_t)0;
    if (live && j < T) Mc[(size_t)row * T + j] = v;
    const unsigned long long m = __ballot(v == 1);
    if (live && v == 1) {
      const int pos = base + __popcll(m & ((1ull << lane) - 1ull));
      for (int r = 0; r < nrep; ++r) row_idx[(t0 + r) * n_h + pos] = j;
    }
    base += __popcll(m);
  }
}

// ---------------------------------------------------------------- column tables (CSC)

// tile[r][c] = label of query tile i0 + r and key block j0 + c (row (i0 + r) / rq of the head's
// M_c) for a 64 x 64 tile, 2 outside the matrix.  When rows are 16-byte aligned (T % 16 == 0)
// thread t brings piece t % 4 (16 bytes) of row t / 4 in one load.
__device__ __forceinline__ uint4 mask_piece(const int8_t* __restrict__ src, int T, int rq, int i0, int j0, int tid) {
  const int r = tid >> 2, p = tid & 3;
  const int i = i0 + r, j = j0 + 16 * p;
  uint4 v = {0x02020202u, 0x02020202u, 0x02020202u, 0x02020202u};
  if (i < T && j < T) v = *reinterpret_cast<const uint4*>(src + (size_t)(i / rq) * T + j);   // (j + 15 < T: T % 16 == 0)
  return v;
}
__device__ __forceinline__ void put_piece(int8_t (*tile)[68], uint4 v, int tid) {
  uint32_t* dst = reinterpret_cast<uint32_t*>(&tile[tid >> 2][16 * (tid & 3)]);
  dst[0] = v.x;
  dst[1] = v.y;
  dst[2] = v.z;
  dst[3] = v.w;
}
__device__ __forceinline__ void load_mask_tile_bytes(int8_t (*tile)[68], const int8_t* __restrict__ src, int T, int rq,
                                                     int i0, int j0, int l, int w) {
  for (int r = w; r < 64; r += 4) {
    const int i = i0 + r, j = j0 + l;
    tile[r][l] = (i < T && j < T) ? src[(size_t)(i / rq) * T + j] : (int8_t)2;
  }
}

// Marginal indicator as bit masks and the column counts, over query tiles i (of 64 tokens: label
// m(i, j) = Mc[i / rq][j]).  Bit b of ind[i][q] is set iff m(i, 64 q + b) == 0 (and the column
// exists), bit b of indT[j][q] iff m(64 q + b, j) == 0;
// cnt[j] (cleared by the classification kernel) receives the number of critical blocks of column
// j.  A workgroup takes a 64 x 64 tile of Mc through LDS; each wave votes 16 rows and 16 columns
// of it into 64-bit words.
__global__ __launch_bounds__(256) void indicator_kernel(const int8_t* __restrict__ Mc, int Tq, int rq, int T, int Tw,
                                                        unsigned long long* __restrict__ ind,
                                                        unsigned long long* __restrict__ indT,
                                                        int32_t* __restrict__ cnt) {
  __shared__ int8_t tile[64][68];
  const int bh = blockIdx.z, i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
  const int l = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int8_t* src = Mc + (size_t)bh * Tq * T;
  if (T % 16 == 0) put_piece(tile, mask_piece(src, T, rq, i0, j0, threadIdx.x), threadIdx.x);
  else load_mask_tile_bytes(tile, src, T, rq, i0, j0, l, w);
  __syncthreads();
  for (int r = w; r < 64; r += 4) {
    const unsigned long long rowbits = __ballot(tile[r][l] == 0);
    const int8_t cv = tile[l][r];
    const unsigned long long colbits = __ballot(cv == 0);
    const int ncrit = __popcll(__ballot(cv == 1));
    if (l == 0) {
      if (i0 + r < T) ind[((size_t)bh * T + i0 + r) * Tw + blockIdx.x] = rowbits;
      if (j0 + r < T) {
        indT[((size_t)bh * T + j0 + r) * Tw + blockIdx.y] = colbits;
        if (ncrit) atomicAdd(cnt + (size_t)bh * T + j0 + r, ncrit);
      }
    }
  }
}

// From the column counts of a head: col_ptr (exclusive prefix sums, T + 1 entries), col_order
// (col_order[rank] = j, rank = position of column j under count descending, index ascending: the
// column-wise backward kernel takes the longest lists first) and col_rows (the critical rows of
// every column, ascending).  A workgroup owns 64 columns of one head; every workgroup forms the
// prefix sum up to its columns from the head's counts by itself.
__global__ __launch_bounds__(256) void col_tables_kernel(const int8_t* __restrict__ Mc, int Tq, int rq, int T, int n_h,
                                                         const int32_t* __restrict__ cnt_g,
                                                         int32_t* __restrict__ ptr, int32_t* __restrict__ order,
                                                         int32_t* __restrict__ rows) {
  extern __shared__ int cnt[];          // T counts of the head
  __shared__ int part[4][64];
  __shared__ int wsum[4];
  __shared__ int cptr[64];
  __shared__ int8_t tile[64][68];
  const int bh = blockIdx.y, j0 = blockIdx.x * 64;
  const int tid = threadIdx.x, l = tid & 63, w = tid >> 6;
  const int32_t* cg = cnt_g + (size_t)bh * T;
  int before = 0;   // this thread's share of the counts of the columns before j0
  for (int j = tid; j < T; j += 256) {
    const int c = cg[j];
    cnt[j] = c;
    if (j < j0) before += c;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) before += __shfl_xor(before, o);
  if (l == 0) wsum[w] = before;
  __syncthreads();
  // pointers of this workgroup's columns: wave 0 scans its 64 counts
  if (w == 0) {
    const int j = j0 + l;
    const int c = j < T ? cnt[j] : 0;
    int incl = c;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int v = __shfl_up(incl, o);
      if (l >= o) incl += v;
    }
    const int p = wsum[0] + wsum[1] + wsum[2] + wsum[3] + incl - c;
    cptr[l] = p;
    if (j < T) ptr[(size_t)bh * (T + 1) + j] = p;
    if (j == T - 1) ptr[(size_t)bh * (T + 1) + T] = p + c;
  }
  // rank of this workgroup's columns; four threads share the comparisons of a column
  {
    const int j = j0 + l;
    int rank = 0;
    if (j < T) {
      const int c = cnt[j];
      const int chunk = (T + 3) / 4, lo = min(T, w * chunk), hi = min(T, lo + chunk);
      for (int k = lo; k < hi; ++k) rank += (cnt[k] > c) || (cnt[k] == c && k < j);
    }
    part[w][l] = rank;
  }
  __syncthreads();
  if (w == 0 && j0 + l < T) order[(size_t)bh * T + part[0][l] + part[1][l] + part[2][l] + part[3][l]] = j0 + l;
  if (n_h == 0) return;
  // rows of the critical blocks: tiles of 64 rows, wave w votes columns 16 w .. 16 w + 15
  const int8_t* src = Mc + (size_t)bh * Tq * T;
  int32_t* out = rows + (size_t)bh * T * n_h;
  int run[16];
#pragma unroll
  for (int c = 0; c < 16; ++c) run[c] = cptr[16 * w + c];
  auto vote = [&](int i0) {
#pragma unroll
    for (int c = 0; c < 16; ++c) {
      const bool crit = tile[l][16 * w + c] == 1;
      const unsigned long long m = __ballot(crit);
      if (crit) out[run[c] + __popcll(m & ((1ull << l) - 1ull))] = i0 + l;
      run[c] += __popcll(m);
    }
  };
  if (T % 16 == 0) {
    // eight tiles' loads in flight at a time
    for (int ib = 0; ib < T; ib += 512) {
      uint4 pre[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) pre[k] = mask_piece(src, T, rq, ib + 64 * k, j0, tid);
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        if (ib + 64 * k >= T) break;
        __syncthreads();   // the previous tile has been read
        put_piece(tile, pre[k], tid);
        __syncthreads();
        vote(ib + 64 * k);
      }
    }
  } else {
    for (int i0 = 0; i0 < T; i0 += 64) {
      __syncthreads();   // the previous tile has been read
      load_mask_tile_bytes(tile, src, T, rq, i0, j0, l, w);
      __syncthreads();
      vote(i0);
    }
  }
}


// ---------------------------------------------------------------- short sequences
// At most 64 key blocks: scores, classification and all tables of a head in one workgroup.  At
// that size each of the four kernels above is a few microseconds of work behind as many
// microseconds of launch.  Same arithmetic, same tables.  With `given` the scores are read
// instead of computed (classification of given scores).
__global__ __launch_bounds__(256) void mask_small_kernel(
    const float* __restrict__ qbar, const float* __restrict__ kbar, const float* __restrict__ given, int Tq, int rq,
    int T, int d, float scale, int n_h, int n_l, float* __restrict__ s_out, int8_t* __restrict__ Mc,
    int32_t* __restrict__ row_idx, unsigned long long* __restrict__ ind, unsigned long long* __restrict__ indT,
    int32_t* __restrict__ col_ptr, int32_t* __restrict__ col_order, int32_t* __restrict__ col_rows) {
  __shared__ __attribute__((aligned(16))) float qs[64][68];
  __shared__ __attribute__((aligned(16))) float ks[64][68];
  __shared__ float sc[64][65];
  __shared__ int8_t lab[64][68];   // labels of the rows of M_c; 2 past the end of a row
  __shared__ int cnt[64], cptr[64];
  const int bh = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const unsigned long long below = (1ull << lane) - 1ull;
  if (given) {
    const float* g = given + (size_t)bh * Tq * T;
    for (int e = tid; e < Tq * T; e += 256) sc[e / T][e % T] = g[e];
  } else {
    float acc[4][4];
    score_tile(qbar + (size_t)bh * Tq * d, kbar + (size_t)bh * T * d, Tq, T, d, 0, 0, qs, ks, acc);
    const int ty = tid >> 4, tx = tid & 15;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const int i = ty + 16 * a, j = tx + 16 * b;
        if (i < Tq && j < T) {
          const float v = __fmul_rn(acc[a][b], scale);
          sc[i][j] = v;
          s_out[((size_t)bh * Tq + i) * T + j] = v;
        }
      }
  }
  __syncthreads();
  // classification: a wave per row of M_c, the row in one register per lane
  for (int i = wave; i < Tq; i += 4) {
    uint32_t key[1];
    int8_t lb[1];
    key[0] = lane < T ? order_key(sc[i][lane]) : 0u;
    lb[0] = 0;
    mark_top_reg<1>(key, lb, n_h, (int8_t)1, lane);
    key[0] = (lb[0] == 1 || lane >= T) ? 0u : ~key[0];
    mark_top_reg<1>(key, lb, n_l, (int8_t)-1, lane);
    if (lane < T) Mc[((size_t)bh * Tq + i) * T + lane] = lb[0];
    lab[i][lane] = lane < T ? lb[0] : (int8_t)2;
    const unsigned long long m = __ballot(lb[0] == 1);
    if (lb[0] == 1) {
      const int pos = __popcll(m & below);
      const int nrep = min(rq, T - i * rq);   // the query tiles of this row
      for (int r = 0; r < nrep; ++r) row_idx[((size_t)bh * T + i * rq + r) * n_h + pos] = lane;
    }
  }
  __syncthreads();
  // bit masks and column counts over query tiles: tile r has the labels of row r / rq
  for (int r = wave; r < 64; r += 4) {
    const int8_t rv = (r < T) ? lab[r / rq][lane] : (int8_t)2;                 // row r, column = lane
    const int8_t cv = (r < T && lane < T) ? lab[lane / rq][r] : (int8_t)2;     // column r, query tile = lane
    const unsigned long long rowbits = __ballot(rv == 0), colbits = __ballot(cv == 0);
    const int ncrit = __popcll(__ballot(cv == 1));
    if (lane == 0) {
      cnt[r] = ncrit;
      if (r < T) {
        ind[(size_t)bh * T + r] = rowbits;
        indT[(size_t)bh * T + r] = colbits;
      }
    }
  }
  __syncthreads();
  if (wave == 0) {
    const int c = cnt[lane];
    int incl = c;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int v = __shfl_up(incl, o);
      if (lane >= o) incl += v;
    }
    cptr[lane] = incl - c;
    if (lane < T) {
      col_ptr[(size_t)bh * (T + 1) + lane] = incl - c;
      if (lane == T - 1) col_ptr[(size_t)bh * (T + 1) + T] = incl;
      int rank = 0;
      for (int k = 0; k < T; ++k) rank += (cnt[k] > c) || (cnt[k] == c && k < lane);
      col_order[(size_t)bh * T + rank] = lane;
    }
  }
  __syncthreads();
  if (n_h == 0) return;
  for (int j = wave; j < T; j += 4) {   // the critical query tiles of column j, ascending
    const bool crit = lane < T && lab[lane / rq][j] == 1;
    const unsigned long long m = __ballot(crit);
    if (crit) col_rows[(size_t)bh * T * n_h + cptr[j] + __popcll(m & below)] = lane;
  }
}

}  // namespace

// block means of Q (blocks of 64 rq tokens) and K (64) -> qbar (float [BH][Tq][d]), kbar (float [BH][T][d])
hipError_t launch_pool(const void* Q, const void* K, const Shape& s, float* qbar, float* kbar, hipStream_t st) {
  const int nblk = s.BH * s.T;
  const int bpw = s.dtype == 0 ? 256 / s.d : 512 / s.d;   // blocks per wavefront
  const dim3 grid((nblk + 4 * bpw - 1) / (4 * bpw), 2), block(256);
  const int lq = s.rq * kBlk;
  KernelTimer kt("pool", st);
  typedef __hip_bfloat16 bf;
  if (s.dtype == 0 && s.d == 64)
    pool_kernel<float, 64><<<grid, block, 0, st>>>((const float*)Q, (const float*)K, s.BH, s.N, s.Tq, lq, s.T, kBlk, s.lay(), qbar, kbar);
  else if (s.dtype == 0)
    pool_kernel<float, 128><<<grid, block, 0, st>>>((const float*)Q, (const float*)K, s.BH, s.N, s.Tq, lq, s.T, kBlk, s.lay(), qbar, kbar);
  else if (s.d == 64)
    pool_kernel<bf, 64><<<grid, block, 0, st>>>((const bf*)Q, (const bf*)K, s.BH, s.N, s.Tq, lq, s.T, kBlk, s.lay(), qbar, kbar);
  else
    pool_kernel<bf, 128><<<grid, block, 0, st>>>((const bf*)Q, (const bf*)K, s.BH, s.N, s.Tq, lq, s.T, kBlk, s.lay(), qbar, kbar);
  return hipGetLastError();
}

hipError_t launch_scores(const float* qbar, const float* kbar, const Shape& s, float* scores,
                         hipStream_t st) {
  const int nt = (s.T + 63) / 64;
  {
    KernelTimer kt("score", st);
    score_kernel<<<dim3(nt, (s.Tq + 63) / 64, s.BH), 256, 0, st>>>(qbar, kbar, s.Tq, s.T, s.d, s.scale, scores);
  }
  return hipGetLastError();
}

hipError_t launch_classify(const float* scores, const Shape& s, int8_t* Mc, int32_t* row_idx,
                           int32_t* col_cnt, hipStream_t st) {
  const int rows = s.BH * s.Tq;
  const size_t lds = (size_t)4 * s.T * (sizeof(uint32_t) + 1);
  {
    KernelTimer kt("classify", st);
    const dim3 grid((rows + 3) / 4);
    if (s.T <= 64) classify_reg_kernel<1><<<grid, 256, 0, st>>>(scores, rows, s.Tq, s.rq, s.T, s.n_h, s.n_l, Mc, row_idx, col_cnt);
    else if (s.T <= 128) classify_reg_kernel<2><<<grid, 256, 0, st>>>(scores, rows, s.Tq, s.rq, s.T, s.n_h, s.n_l, Mc, row_idx, col_cnt);
    else if (s.T <= 256) classify_reg_kernel<4><<<grid, 256, 0, st>>>(scores, rows, s.Tq, s.rq, s.T, s.n_h, s.n_l, Mc, row_idx, col_cnt);
    else if (s.T <= 512) classify_reg_kernel<8><<<grid, 256, 0, st>>>(scores, rows, s.Tq, s.rq, s.T, s.n_h, s.n_l, Mc, row_idx, col_cnt);
    else if (s.T <= 1024) classify_reg_kernel<16><<<grid, 256, 0, st>>>(scores, rows, s.Tq, s.rq, s.T, s.n_h, s.n_l, Mc, row_idx, col_cnt);
    else if (s.T <= 2048) classify_reg_kernel<32><<<grid, 256, 0, st>>>(scores, rows, s.Tq, s.rq, s.T, s.n_h, s.n_l, Mc, row_idx, col_cnt);
    else classify_kernel<<<grid, 256, lds, st>>>(scores, rows, s.Tq, s.rq, s.T, s.n_h, s.n_l, Mc, row_idx, col_cnt);
  }
  return hipGetLastError();
}

hipError_t launch_csc(const int8_t* Mc, const Shape& s, int32_t* col_cnt, int32_t* col_ptr, int32_t* col_rows,
                      unsigned long long* ind, unsigned long long* indT, int32_t* col_order, hipStream_t st) {
  const int Tw = (s.T + 63) / 64;
  {
    KernelTimer kt("indicator", st);
    indicator_kernel<<<dim3(Tw, Tw, s.BH), 256, 0, st>>>(Mc, s.Tq, s.rq, s.T, Tw, ind, indT, col_cnt);
  }
  {
    KernelTimer kt("col_tables", st);
    col_tables_kernel<<<dim3(Tw, s.BH), 256, s.T * sizeof(int), st>>>(Mc, s.Tq, s.rq, s.T, s.n_h, col_cnt, col_ptr, col_order,
                                                                      col_rows);
  }
  return hipGetLastError();
}

hipError_t launch_mask_small(const float* qbar, const float* kbar, const float* given, const Shape& s, float* scores,
                             int8_t* Mc, int32_t* row_idx, unsigned long long* ind, unsigned long long* indT,
                             int32_t* col_ptr, int32_t* col_order, int32_t* col_rows, hipStream_t st) {
  KernelTimer kt("mask_small", st);
  mask_small_kernel<<<s.BH, 256, 0, st>>>(qbar, kbar, given, s.Tq, s.rq, s.T, s.d, s.scale, s.n_h, s.n_l, scores, Mc,
                                          row_idx, ind, indT, col_ptr, col_order, col_rows);
  return hipGetLastError();
}

}  // namespace sla
