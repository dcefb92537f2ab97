// Device helpers for the bf16 matrix-core (MFMA) kernels on gfx950.
//
// One v_mfma_f32_32x32x16_bf16 multiplies A (32 x 16) by B (16 x 32) into C (32 x 32) per
// wavefront.  Register layout, lane l = 32 g + n (g = l / 32, n = l % 32):
//   A: lane holds row n,    eight k-values (slot s = 0..7) of k-group g
//   B: lane holds column n, eight k-values (slot s) of k-group g
//   C: lane holds column n, sixteen rows: register i -> row 8 (i / 4) + 4 g + (i % 4)
// The contraction runs over all 16 (g, s) pairs, so any assignment of k-indices to (g, s)
// gives the right product as long as A and B use the same one.  That freedom is what lets
// a C tile be fed back as a B operand without shuffling: registers 8 u .. 8 u + 7 of a C
// tile hold, for lane group g, the rows  16 u + {4g..4g+3} and 16 u + 8 + {4g..4g+3}.
// An A operand that has to match stores its k-index in the permuted order perm16() below.
#ifndef SLA_MFMA_COMMON_H_
#define SLA_MFMA_COMMON_H_

#include "sla_internal.h"

namespace sla {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// row of C register i for lane group g
__device__ __forceinline__ int c_row(int i, int g) { return ((i >> 2) << 3) + (g << 2) + (i & 3); }

// Position, inside a run of 16 consecutive k-indices, at which index kk is stored so that
// slots s = 0..7 of lane group g read positions 8 g + s and obtain the k-indices
// {4g..4g+3, 8+4g..8+4g+3}, the rows a C tile hands to lane group g.
__device__ __host__ __forceinline__ int perm16(int kk) {
  const int a = (kk >> 3) & 1, gg = (kk >> 2) & 1, r = kk & 3;
  return (gg << 3) + (a << 2) + r;
}

__device__ __forceinline__ bf16x8 zero_bf16x8() {
  bf16x8 z;
#pragma unroll
  for (int s = 0; s < 8; ++s) z[s] = (__bf16)0.0f;
  return z;
}

__device__ __forceinline__ f32x16 zero_f32x16() {
  f32x16 z;
#pragma unroll
  for (int s = 0; s < 16; ++s) z[s] = 0.0f;
  return z;
}

// eight consecutive floats -> bf16x8 (round to nearest even)
__device__ __forceinline__ bf16x8 cvt8(const float* p) {
  const f32x4 a = *reinterpret_cast<const f32x4*>(p);
  const f32x4 b = *reinterpret_cast<const f32x4*>(p + 4);
  bf16x8 r;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    r[s] = (__bf16)a[s];
    r[4 + s] = (__bf16)b[s];
  }
  return r;
}

// registers 8u..8u+7 of a C tile as a bf16 operand
__device__ __forceinline__ bf16x8 c_to_operand(const f32x16& c, int u) {
  bf16x8 r;
#pragma unroll
  for (int s = 0; s < 8; ++s) r[s] = (__bf16)c[8 * u + s];
  return r;
}

// 4 x 4 transpose of bf16 held as four 8-byte rows: out[i] = (in[0][i], in[1][i], in[2][i], in[3][i])
__device__ __forceinline__ void transpose4x4(const u32x2 (&in)[4], u32x2 (&out)[4]) {
  // in[k].x = (e0, e1), in[k].y = (e2, e3) of key k
  out[0].x = (in[0].x & 0xffffu) | (in[1].x << 16);
  out[0].y = (in[2].x & 0xffffu) | (in[3].x << 16);
  out[1].x = (in[0].x >> 16) | (in[1].x & 0xffff0000u);
  out[1].y = (in[2].x >> 16) | (in[3].x & 0xffff0000u);
  out[2].x = (in[0].y & 0xffffu) | (in[1].y << 16);
  out[2].y = (in[2].y & 0xffffu) | (in[3].y << 16);
  out[3].x = (in[0].y >> 16) | (in[1].y & 0xffff0000u);
  out[3].y = (in[2].y >> 16) | (in[3].y & 0xffff0000u);
}

typedef __hip_bfloat16 bf16;

// ---- transposing tile stage
// A 4-row x 4-feature patch (rows k4..k4+3, features f4..f4+3) of a row-major [rows][D]
// bf16 tile is loaded as four 8-byte pieces and stored transposed into an LDS tile laid out
// [feature][row position] (stride elements per feature) at row position `pos`.
__device__ __forceinline__ void load_patch(const bf16* __restrict__ src, int D, int k4, int f4,
                                           int rows_valid, u32x2 (&x)[4]) {
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    if (k4 + kk < rows_valid)
      x[kk] = *reinterpret_cast<const u32x2*>(src + (size_t)(k4 + kk) * D + f4);
    else
      x[kk] = u32x2{0u, 0u};
  }
}

__device__ __forceinline__ void store_patch_t(bf16* dst, int stride, int f4, int pos,
                                              const u32x2 (&x)[4]) {
  u32x2 y[4];
  transpose4x4(x, y);
#pragma unroll
  for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x2*>(dst + (f4 + i) * stride + pos) = y[i];
}

// position of row group kg (rows 4kg..4kg+3 of a 64-row tile) under perm16
__device__ __forceinline__ int pos_of_kg(int kg) { return ((kg >> 2) << 4) + perm16((kg & 3) << 2); }

constexpr int kVS = kBlk + 8;  // LDS stride (elements) of a transposed [feature][64 rows] tile

// One staging unit = rows 4rg..4rg+3, features 8fg..8fg+7 of a 64 x D row-major tile, loaded
// as four 16-byte pieces (zero beyond rows_valid).
__device__ __forceinline__ void load_unit(const bf16* __restrict__ src, int D, int rg, int fg,
                                          int rows_valid, u32x4 (&x)[4]) {
#pragma unroll
  for (int rr = 0; rr < 4; ++rr) {
    if (4 * rg + rr < rows_valid)
      x[rr] = *reinterpret_cast<const u32x4*>(src + (size_t)(4 * rg + rr) * D + 8 * fg);
    else
      x[rr] = u32x4{0u, 0u, 0u, 0u};
  }
}

// row-major copy: dst[row][feature], stride RS elements
__device__ __forceinline__ void store_unit_rows(bf16* dst, int RS, int rg, int fg, const u32x4 (&x)[4]) {
#pragma unroll
  for (int rr = 0; rr < 4; ++rr) *reinterpret_cast<u32x4*>(dst + (4 * rg + rr) * RS + 8 * fg) = x[rr];
}

// transposed copy: dst[feature][perm16 row position], stride kVS
__device__ __forceinline__ void store_unit_t(bf16* dst, int rg, int fg, const u32x4 (&x)[4]) {
  u32x2 lo[4], hi[4];
#pragma unroll
  for (int rr = 0; rr < 4; ++rr) {
    lo[rr] = u32x2{x[rr].x, x[rr].y};
    hi[rr] = u32x2{x[rr].z, x[rr].w};
  }
  store_patch_t(dst, kVS, 8 * fg, pos_of_kg(rg), lo);
  store_patch_t(dst, kVS, 8 * fg + 4, pos_of_kg(rg), hi);
}

// A operand (rows = 32 features f0.., k = 16 tile rows r0.. in the order a C tile hands them
// over, see perm16) read from a ROW-MAJOR LDS tile [row][feature] (stride elements) with the
// transposing LDS read: in each group of 16 lanes, lane 4e + a supplies the address of 4
// consecutive features of one row, and lane 4a + c receives feature c of the rows of lanes
// a, 4 + a, 8 + a, 12 + a.  Two reads give the eight k-values of a lane.
__device__ __forceinline__ bf16x8 read_tr_operand(const bf16* tile, int stride, int r0, int f0, int l) {
  typedef __attribute__((ext_vector_type(4))) short s16x4;
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  const int G = l >> 4, e = (l >> 2) & 3, a = l & 3;
  const bf16* p = tile + (r0 + 4 * (G >> 1) + e) * stride + f0 + 16 * (G & 1) + 4 * a;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 8 * stride));
  bf16x8 r;
  const bf16x4 lo4 = *reinterpret_cast<const bf16x4*>(&lo), hi4 = *reinterpret_cast<const bf16x4*>(&hi);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    r[i] = lo4[i];
    r[4 + i] = hi4[i];
  }
  return r;
}

// Raw buffer descriptor (base address, no stride, byte count, 32-bit raw format) over `bytes`
// bytes starting at p: loads through it return zero beyond the end.  p must be wave-uniform.
typedef u32x4 BufDesc;
__device__ __forceinline__ BufDesc tile_rsrc(const void* p, int bytes) {
  const unsigned long long a = reinterpret_cast<unsigned long long>(p);
  return BufDesc{(unsigned)a, (unsigned)(a >> 32) & 0xffffu, (unsigned)bytes, 0x00020000u};
}

typedef __attribute__((address_space(3))) void lds_void;

// One wave-wide 16-byte-per-lane load global -> LDS: lane L's 16 bytes at byte offset voff of the
// buffer plus the wave-uniform soff land at LDS byte address (lds_addr + 16 L), lds_addr uniform.
// Written as assembly on purpose: the compiler cannot tell which LDS bytes such a load writes,
// so for its own form of this load it waits for every outstanding one before the next LDS-writing
// load and before the next LDS read, which serialises the loads and exposes their whole latency.
// Here the ordering is the caller's job: wait_vm0() and a barrier before a tile is read, a
// barrier after its last read before it is overwritten.
__device__ __forceinline__ void load_to_lds16(BufDesc desc, int voff, int soff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :: "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(voff), "s"(desc), "s"(__builtin_amdgcn_readfirstlane(soff))
               : "memory");
}

// LDS byte address of the dynamic LDS array, as a wave-uniform integer
__device__ __forceinline__ unsigned lds_base(unsigned char* smem) {
  return __builtin_amdgcn_readfirstlane((unsigned)reinterpret_cast<size_t>((lds_void*)smem));
}

// p[idx] for 0 <= idx < count, else 0, without a branch (range-checked buffer load); p uniform
__device__ __forceinline__ float load_f32_or_zero(const float* p, int count, int idx) {
  const __amdgpu_buffer_rsrc_t r =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p), 0, count * 4, 0x00020000);
  return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, idx * 4, 0, 0));
}

// One wave-wide 4-byte-per-lane load global -> LDS: lane L's dword at byte offset voff of the buffer
// lands at LDS byte address lds_addr + 4 L (lds_addr wave-uniform); beyond the buffer's end it
// deposits zero.  Like load_to_lds16 it is invisible to the compiler's wait insertion; the data
// may be read from LDS after a wait_vm of the caller's that covers it.  Nothing lands in a
// register, so there is no register the compiler could copy or spill before the data has arrived.
__device__ __forceinline__ void load_to_lds4(BufDesc desc, int voff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
               :: "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(voff), "s"(desc)
               : "memory");
}

// lane index inside the wave, recomputed at every use (volatile: the compiler would otherwise
// hoist it out of a loop and may then spill it) instead of held in a register
__device__ __forceinline__ int lane_id() {
  int x;
  asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(x));
  return x;
}

// Nothing is scheduled across this point.  Used to keep the LDS reads of a step together and
// ahead of the matrix products that consume them, so that one LDS latency is exposed per group
// instead of one per product.
__device__ __forceinline__ void sched_fence() { __builtin_amdgcn_sched_barrier(0); }

// Reductions over the two halves of a wave: every lane gets op(x of lane l % 32, x of lane
// l % 32 + 32).  The swap of the upper half of one copy with the lower half of the other leaves
// the two values side by side in every lane: one VALU instruction instead of a trip through LDS.
__device__ __forceinline__ float half_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float half_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// A B-operand fragment in natural order (lane half g holds k = 8 g .. 8 g + 7) -> the order in
// which the transposing LDS read delivers the other operand (k = 4 g .. + 3 and 8 + 4 g .. + 3):
// the g = 0 lanes trade their upper four values for the lower four of the g = 1 lanes.
__device__ __forceinline__ bf16x8 to_tr_order(bf16x8 x) {
  u32x4 v = *reinterpret_cast<u32x4*>(&x);
  const auto r0 = __builtin_amdgcn_permlane32_swap(v.x, v.z, false, false);
  const auto r1 = __builtin_amdgcn_permlane32_swap(v.y, v.w, false, false);
  v.x = r0[0];
  v.z = r0[1];
  v.y = r1[0];
  v.w = r1[1];
  return *reinterpret_cast<bf16x8*>(&v);
}

// Makes the compiler finish the loads that produce x here.  Used on operand registers that are
// loaded before a pipelined loop: otherwise the wait for them lands at their first use inside the
// loop body, where it also waits -- on every trip -- for the tile loads just put in flight.
template <class T>
__device__ __forceinline__ void pin_loaded(T& x) {
  asm volatile("" : "+v"(x));
}

// ---- swizzled row-major tiles filled by direct global -> LDS loads
// A 64 x D bf16 tile lives in LDS unpadded (row = 2 D bytes); the 16-byte chunk c of row r sits
// at chunk position c ^ swz(r).  With swz(r) = 4 (r % 4) + (r / 4) % 4 both access patterns of
// the kernels are spread over the banks: one row per lane at a fixed chunk (16 consecutive rows
// hit 16 different chunk positions) and the transposing read (4 consecutive rows x 64 bytes).
// The tile is written by buffer loads that deposit 16 bytes per lane straight into LDS: lane L of
// a wave-wide load fills LDS chunk L of a 1 KB run, and fetches the global chunk that belongs
// there.  Loads beyond the tile's valid rows deposit zeros.
template <int D>
struct SwzTile {
  static constexpr int CPR = D / 8;             // chunks per row
  static constexpr int ROW_BYTES = 2 * D;
  static constexpr int BYTES = kBlk * ROW_BYTES;
  static constexpr int RPI = 1024 / ROW_BYTES;  // rows per wave-wide load
  static constexpr int IPW = kBlk / RPI / 4;    // loads per wave (4 waves share a tile)
};

template <int D>
__device__ __forceinline__ int swz(int row) {
  return (((row & 3) << 2) | ((row >> 2) & 3)) & (D / 8 - 1);
}


// byte offset (inside a tile) of the 16-byte chunk `c` of row `row`
template <int D>
__device__ __forceinline__ int swz_chunk_off(int row, int c) {
  return row * SwzTile<D>::ROW_BYTES + ((c ^ swz<D>(row)) << 4);
}

// All four waves of a workgroup enqueue the loads of one tile.  A wave-wide load deposits 1 KB;
// wave w takes the 1 KB runs w, w + 4, ... of the tile.  Load k of a lane fetches the chunk 4096 k
// bytes after that of load 0 (the swizzle has period 16 rows), so one per-lane offset serves all:
//   ldv  = tile_lane_offset<D>(w, l)                       per lane, fixed
//   lds0 = lds_base(smem) + 1024 * (wave index, uniform)   per wave, fixed
template <int D>
__device__ __forceinline__ int tile_lane_offset(int w, int l) {
  using T = SwzTile<D>;
  return swz_chunk_off<D>(T::RPI * w + l / T::CPR, l % T::CPR);
}
template <int D>
__device__ __forceinline__ void issue_tile_load(const bf16* gbase, int valid_rows, unsigned lds0, int lds_tile, int ldv) {
  using T = SwzTile<D>;
  const BufDesc rsrc = tile_rsrc(gbase, valid_rows * T::ROW_BYTES);
#pragma unroll
  for (int k = 0; k < T::IPW; ++k) load_to_lds16(rsrc, ldv, 4096 * k, lds0 + lds_tile + 4096 * k);
}

// The same for tiles whose rows lie tsB bytes apart in memory (a head of a [B,N,H,d] tensor; tsB =
// 2 D for packed rows) behind a descriptor that spans the whole head: the scalar offset selects
// the tile, and rows past the head's end read as zeros.
template <int D>
__device__ __forceinline__ BufDesc head_rsrc(const bf16* head_base, int N, int tsB) {
  return tile_rsrc(head_base, (N - 1) * tsB + 2 * D);
}
template <int D, int NW = 4>
struct TileLoader {
  using T = SwzTile<D>;
  static constexpr int IPW = kBlk / T::RPI / NW;   // loads per wave (NW waves share a tile)
  int ldv;        // this lane's byte offset inside a tile's memory image
  int kstep;      // bytes between the rows of two consecutive loads of a wave
  unsigned ldsw;  // LDS address of this wave's first KB of the tile at LDS offset 0
  int tile_step;  // bytes between consecutive 64-row tiles
  // w: this wave's index among the NW waves that fill a tile together
  __device__ __forceinline__ void init(unsigned lds_base_addr, int w, int l, int tsB) {
    const int row = T::RPI * w + l / T::CPR;
    ldv = row * tsB + (((l % T::CPR) ^ swz<D>(row)) << 4);
    kstep = NW * T::RPI * tsB;
    tile_step = kBlk * tsB;
    ldsw = lds_base_addr + __builtin_amdgcn_readfirstlane(w) * 1024;
  }
  // tile number `tile` of the head behind desc -> LDS offset lds_tile
  __device__ __forceinline__ void load(BufDesc desc, int tile, int lds_tile) const {
#pragma unroll
    for (int k = 0; k < IPW; ++k)
      load_to_lds16(desc, ldv, tile * tile_step + k * kstep, ldsw + lds_tile + 1024 * NW * k);
  }
};

// The loader of the step loops, built for few instructions per tile: a wave (one of NW that fill a
// tile together) fills a run of consecutive rows, IPW KB that are contiguous in LDS, so that one
// value of M0 serves all its loads of a tile and the instruction's immediate offset (which moves
// the LDS address and the memory address alike) steps through the run.  The swizzle of a row
// differs from load to load, hence one per-lane offset per load, each with the immediate taken
// out again (the rows of a load are at least 1 KB apart in memory, so none goes negative).
// Per tile: one scalar instruction for M0, the wait state it needs, IPW loads.
template <int D, int NW = 4>
struct RunLoader {
  using T = SwzTile<D>;
  static constexpr int IPW = kBlk / T::RPI / NW;
  static_assert(IPW == 1 || IPW == 2 || IPW == 4, "loads per wave and tile");
  int voff[IPW];
  unsigned ldsw;  // LDS address of this wave's run of the tile at LDS offset 0
  int tile_step;  // bytes between consecutive 64-row tiles in memory
  __device__ __forceinline__ void init(unsigned lds_base_addr, int w, int l, int tsB) {
#pragma unroll
    for (int k = 0; k < IPW; ++k) {
      const int row = T::RPI * (IPW * w + k) + l / T::CPR;
      voff[k] = row * tsB + (((l % T::CPR) ^ swz<D>(row)) << 4) - 1024 * k;
    }
    tile_step = __builtin_amdgcn_readfirstlane(kBlk * tsB);
    ldsw = lds_base_addr + __builtin_amdgcn_readfirstlane(w) * (1024 * IPW);
  }
  // keeps the per-lane offsets in their registers (the compiler would otherwise re-derive them
  // inside the loop, or spill them)
  __device__ __forceinline__ void pin() {
#pragma unroll
    for (int k = 0; k < IPW; ++k) asm volatile("" : "+v"(voff[k]));
  }
  // the tile at byte offset soff (wave-uniform) of the buffer -> the tile slot at LDS offset LDS_OFF
  template <int LDS_OFF>
  __device__ __forceinline__ void load(BufDesc desc, int soff_in) const {
    const int soff = __builtin_amdgcn_readfirstlane(soff_in);
    if constexpr (IPW == 4) {
      asm volatile(
          "s_add_u32 m0, %0, %1\n\ts_nop 0\n\t"
          "buffer_load_dwordx4 %2, %6, %7 offen lds\n\t"
          "buffer_load_dwordx4 %3, %6, %7 offen offset:1024 lds\n\t"
          "buffer_load_dwordx4 %4, %6, %7 offen offset:2048 lds\n\t"
          "buffer_load_dwordx4 %5, %6, %7 offen offset:3072 lds"
          ::"s"(ldsw), "n"(LDS_OFF), "v"(voff[0]), "v"(voff[1]), "v"(voff[2]), "v"(voff[3]), "s"(desc), "s"(soff)
          : "memory", "scc");
    } else if constexpr (IPW == 2) {
      asm volatile(
          "s_add_u32 m0, %0, %1\n\ts_nop 0\n\t"
          "buffer_load_dwordx4 %2, %4, %5 offen lds\n\t"
          "buffer_load_dwordx4 %3, %4, %5 offen offset:1024 lds"
          ::"s"(ldsw), "n"(LDS_OFF), "v"(voff[0]), "v"(voff[1]), "s"(desc), "s"(soff)
          : "memory", "scc");
    } else {
      asm volatile(
          "s_add_u32 m0, %0, %1\n\ts_nop 0\n\t"
          "buffer_load_dwordx4 %2, %3, %4 offen lds"
          ::"s"(ldsw), "n"(LDS_OFF), "v"(voff[0]), "s"(desc), "s"(soff)
          : "memory", "scc");
    }
  }
};

// A operand whose 32 rows are tile rows r0 + (l % 32) and whose k-values are features 16 t + 8 g ..
template <int D>
__device__ __forceinline__ bf16x8 read_row_swz(const unsigned char* tile, int r0, int t, int l) {
  return *reinterpret_cast<const bf16x8*>(tile + swz_chunk_off<D>(r0 + (l & 31), 2 * t + (l >> 5)));
}

// A operand with rows = features 32 et .. and k = tile rows r0 .. r0 + 15 (r0 a multiple of 16) in
// the order a C tile hands them over, via the transposing read (see read_tr_operand).
template <int D>
__device__ __forceinline__ bf16x8 read_tr_swz(const unsigned char* tile, int r0, int et, int l) {
  typedef __attribute__((ext_vector_type(4))) short s16x4;
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  const int G = l >> 4, e = (l >> 2) & 3, a = l & 3;
  const int chunk = 4 * et + 2 * (G & 1) + (a >> 1);
  const int row0 = r0 + 4 * (G >> 1) + e;
  const unsigned char* p0 = tile + swz_chunk_off<D>(row0, chunk) + 8 * (a & 1);
  const unsigned char* p1 = tile + swz_chunk_off<D>(row0 + 8, chunk) + 8 * (a & 1);
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p0));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p1));
  const bf16x4 lo4 = *reinterpret_cast<const bf16x4*>(&lo), hi4 = *reinterpret_cast<const bf16x4*>(&hi);
  bf16x8 r;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    r[i] = lo4[i];
    r[4 + i] = hi4[i];
  }
  return r;
}

// Per-lane byte offsets into a swizzled tile, kept as a handful of registers:
//   row(t)     16-byte chunk 2t + g of row r0 + (l % 32)                 (operand read by rows)
//   tr(h, et)  8 bytes of the transposing read h of feature tile et, tile rows r0 + 0..15; rows
//              r0 + 16u .. are a further 16u * ROW_BYTES away (the swizzle has period 16)
// Each offset is base + (constant ^ per-lane swizzle), one VALU operation at the point of use.
// Holding all of them in registers across the step loop costs more registers than the dK/dV
// kernel has, and what spills is reloaded from scratch with a wait that also drains the tile
// loads in flight.  refresh() at the top of a step keeps the compiler from hoisting them again.
template <int D>
struct TileAddr {
  int rb, sx;     // row reads: base, swizzle of the chunk-pair index
  int tb[2], fx;  // transposing reads: the two 8-row bases, swizzle of the feature tile index
  __device__ __forceinline__ void init(int r0, int l) {
    const int g = l >> 5, r = r0 + (l & 31);
    const int sw = swz<D>(r);
    rb = r * SwzTile<D>::ROW_BYTES + (((g ^ sw) & 1) << 4);
    sx = (sw & ~1) << 4;
    const int G = l >> 4, e = (l >> 2) & 3, a = l & 3;
    const int cl = 2 * (G & 1) + (a >> 1);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int rw = r0 + 8 * h + 4 * (G >> 1) + e;
      // chunk = 4 et + cl; its swizzled position is 4 (et ^ fe) + (cl ^ fb), fe and fb from the row
      const int f = swz<D>(rw);
      tb[h] = rw * SwzTile<D>::ROW_BYTES + (((cl ^ f) & 3) << 4) + 8 * (a & 1);
    }
    fx = (swz<D>(r0 + e) >> 2) << 6;
  }
  __device__ __forceinline__ void refresh() { asm volatile("" : "+v"(sx), "+v"(fx)); }
  __device__ __forceinline__ int row(int t) const { return rb + ((t << 5) ^ sx); }
  __device__ __forceinline__ int tr(int h, int et) const { return tb[h] + ((et << 6) ^ fx); }
  // the same with the per-lane base already moved to a tile slot: base = rb + slot (rows),
  // base = tb[h] + slot (transposing reads)
  __device__ __forceinline__ int row_at(int t, int base) const { return base + ((t << 5) ^ sx); }
  __device__ __forceinline__ int tr_at(int et, int base) const { return base + ((et << 6) ^ fx); }
};

typedef __attribute__((ext_vector_type(4))) short lds_s16x4_val;
typedef __attribute__((address_space(3))) lds_s16x4_val lds_s16x4_t;

// operand read by rows at a precomputed offset
__device__ __forceinline__ bf16x8 lds_row(const unsigned char* smem, int off) {
  return *reinterpret_cast<const bf16x8*>(smem + off);
}

// transposed operand from the two precomputed read offsets (off, off + 8 rows)
template <int D>
__device__ __forceinline__ bf16x8 lds_tr(const unsigned char* smem, int off0, int off1) {
  const lds_s16x4_val lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(smem + off0));
  const lds_s16x4_val hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(smem + off1));
  const bf16x4 lo4 = *reinterpret_cast<const bf16x4*>(&lo), hi4 = *reinterpret_cast<const bf16x4*>(&hi);
  bf16x8 r;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    r[i] = lo4[i];
    r[4 + i] = hi4[i];
  }
  return r;
}

__device__ __forceinline__ int wave_uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }

// Wave-local: NT C tiles of 32 rows (lane l % 32 = row, register r of tile t = column
// 32 t + c_row(r, l / 32)) go to LDS as bf16 rows and from there to global memory in 16-byte
// pieces of whole rows, instead of 8-byte pieces scattered over 32 rows.  `stage` is this wave's
// own LDS area of 32 * (64 NT + 16) bytes; dst points at row 0, column 0 of the tiles; rows at and
// beyond rows_valid are not written.
template <int NT>
__device__ __forceinline__ void store_rows_bf16(unsigned char* stage, const f32x16 (&c)[NT], bf16* dst,
                                                int row_stride, int rows_valid, int l) {
  constexpr int PB = 64 * NT + 16, PPR = 4 * NT;
  const int g = l >> 5, ln = l & 31;
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      bf16x4 pk;
#pragma unroll
      for (int r = 0; r < 4; ++r) pk[r] = (__bf16)c[t][4 * r4 + r];
      *reinterpret_cast<bf16x4*>(stage + ln * PB + (32 * t + 8 * r4 + 4 * g) * 2) = pk;
    }
#pragma unroll
  for (int it = 0; it < 32 * PPR / 64; ++it) {
    const int idx = it * 64 + l, row = idx / PPR, pc = idx % PPR;
    const u32x4 v = *reinterpret_cast<const u32x4*>(stage + row * PB + pc * 16);
    if (row < rows_valid) *reinterpret_cast<u32x4*>(dst + (size_t)row * row_stride + pc * 8) = v;
  }
}

// The float counterpart of store_rows_bf16: `stage` needs 32 * (128 NT + 16) bytes.
template <int NT>
__device__ __forceinline__ void store_rows_f32(unsigned char* stage, const f32x16 (&c)[NT], float* dst,
                                               int row_stride, int rows_valid, int l) {
  constexpr int PB = 128 * NT + 16, PPR = 8 * NT;
  const int g = l >> 5, ln = l & 31;
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4)
      *reinterpret_cast<f32x4*>(stage + ln * PB + (32 * t + 8 * r4 + 4 * g) * 4) =
          f32x4{c[t][4 * r4], c[t][4 * r4 + 1], c[t][4 * r4 + 2], c[t][4 * r4 + 3]};
#pragma unroll
  for (int it = 0; it < 32 * PPR / 64; ++it) {
    const int idx = it * 64 + l, row = idx / PPR, pc = idx % PPR;
    const u32x4 v = *reinterpret_cast<const u32x4*>(stage + row * PB + pc * 16);
    if (row < rows_valid) *reinterpret_cast<u32x4*>(dst + (size_t)row * row_stride + pc * 4) = v;
  }
}

// Workgroups are dealt to the 8 XCDs (each with its own L2) round-robin by linear index.  With a
// grid of 8 * ceil(T / 8) workgroups per head, XCD x gets the contiguous blocks
// [x ceil(T/8), (x+1) ceil(T/8)) in ascending order, so that neighbouring query blocks -- which
// share many of their critical key blocks -- run on the same L2 at about the same time.
// Returns the block index, or -1 for a padding workgroup.
__device__ __forceinline__ int xcd_local_block(int bx, int T) {
  const int C = (T + 7) >> 3;
  const int i = (bx & 7) * C + (bx >> 3);
  return i < T ? i : -1;
}
inline int xcd_grid(int T) { return 8 * ((T + 7) / 8); }

// all outstanding global loads of this wave (including those that write LDS) have completed
__device__ __forceinline__ void wait_vm0() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// The same as an instruction the compiler sees, not as text: its own wait insertion then knows
// that none of its loads is pending either.  For kernels that have compiler-visible loads before
// a loop of tile loads: otherwise the compiler may guard a register of such a load, long
// complete, with a wait inside the loop, which drains the tile loads in flight.
__device__ __forceinline__ void wait_vm0_known() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0); expcnt and lgkmcnt at their maximum = not waited for
  asm volatile("" ::: "memory");
}
// all but the N most recent ones have completed (loads complete in the order they were issued)
template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// phi statistics of a token whose features sit in B-operand fragments (lane holds features
// 16 t + 8 g + s, its partner lane l ^ 32 the others): softmax max and 1 / sum.
template <int KT>
__device__ __forceinline__ void phi_stats(const bf16x8 (&xf)[KT], int phi, float& mx, float& inv) {
  mx = 0.0f;
  inv = 1.0f;
  if (phi != 0) return;
  mx = -INFINITY;
#pragma unroll
  for (int t = 0; t < KT; ++t)
#pragma unroll
    for (int s = 0; s < 8; ++s) mx = fmaxf(mx, (float)xf[t][s]);
  mx = half_max(mx);
  float sum = 0.0f;
#pragma unroll
  for (int t = 0; t < KT; ++t)
#pragma unroll
    for (int s = 0; s < 8; ++s) sum += fast_exp2(((float)xf[t][s] - mx) * kLog2e);
  sum = half_sum(sum);
  inv = 1.0f / sum;
}

// phi of a token whose features sit in B-operand fragments, as bf16 operand fragments; for the
// softmax map every exponential is formed once (kept in registers between the sum and the values).
// mx, inv: the softmax statistics (0 and 1 for the other map), as phi_stats returns them.
template <int KT>
__device__ __forceinline__ void phi_fragments(const bf16x8 (&xf)[KT], int phi, bf16x8 (&out)[KT], float& mx, float& inv) {
  mx = 0.0f;
  inv = 1.0f;
  if (phi != 0) {
#pragma unroll
    for (int t = 0; t < KT; ++t)
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const float x = (float)xf[t][s];
        out[t][s] = (__bf16)(x > 0.0f ? x + 1.0f : fast_exp2(x * kLog2e));
      }
    return;
  }
  mx = -INFINITY;
#pragma unroll
  for (int t = 0; t < KT; ++t)
#pragma unroll
    for (int s = 0; s < 8; ++s) mx = fmaxf(mx, (float)xf[t][s]);
  mx = half_max(mx);
  float e[KT][8];
  float sum = 0.0f;
#pragma unroll
  for (int t = 0; t < KT; ++t)
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      e[t][s] = fast_exp2(((float)xf[t][s] - mx) * kLog2e);
      sum += e[t][s];
    }
  sum = half_sum(sum);
  inv = 1.0f / sum;
#pragma unroll
  for (int t = 0; t < KT; ++t)
#pragma unroll
    for (int s = 0; s < 8; ++s) out[t][s] = (__bf16)(e[t][s] * inv);
}
template <int KT>
__device__ __forceinline__ void phi_fragments(const bf16x8 (&xf)[KT], int phi, bf16x8 (&out)[KT]) {
  float mx, inv;
  phi_fragments<KT>(xf, phi, out, mx, inv);
}

__device__ __forceinline__ float phi_val(float x, int phi, float mx, float inv) {
  return phi == 0 ? fast_exp2((x - mx) * kLog2e) * inv : (x > 0.0f ? x + 1.0f : fast_exp2(x * kLog2e));
}

}  // namespace sla
#endif
