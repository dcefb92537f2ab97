// Internal declarations shared by the HIP translation units of the SLA library.
#ifndef SLA_INTERNAL_H_
#define SLA_INTERNAL_H_

#include <hip/hip_bf16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sla {

constexpr int kBlk = 64;  // tile of every kernel: b_kv, and b_q or the unit b_q is a multiple of (Section 6.1)

// Where the caller's Q, K, V, O, dO, dQ, dK, dV keep token n of head bh = b H + h: element
// offset head(bh) + n ts.  [B,H,N,d]: ts = d; [B,N,H,d]: ts = H d.  (Everything the library
// itself lays out -- saved tensors, workspaces -- is packed per head with rows d apart.)
struct Lay {
  long long bs, hs;   // elements between batches, between heads of a batch
  int ts, H;          // elements between tokens of a head; heads per batch
  __host__ __device__ size_t head(int bh) const { return (size_t)(bh / H) * bs + (size_t)(bh % H) * hs; }
};

// Shape of one call, derived on the host.
struct Shape {
  int BH, N, d, T, n_h, n_l, n_0;
  int Tq, rq;  // rows of M_c = query blocks of b_q = 64 rq tokens; row r of the 64-token grid has the labels of M_c row r / rq
  int phi;    // 0 softmax over features, 1 elu+1
  int dtype;  // 0 float, 1 bf16
  float scale;  // float 1/sqrt(d)
  Lay layv;     // where the caller's tensors keep their rows
  __host__ __device__ int state_row() const { return d * d + d; }
  Lay lay() const { return layv; }
};

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(__hip_bfloat16 x) { return __bfloat162float(x); }
__device__ __forceinline__ void from_f32(float& dst, float x) { dst = x; }
__device__ __forceinline__ void from_f32(__hip_bfloat16& dst, float x) { dst = __float2bfloat16(x); }

// ---- mask step (mask_kernels.hip)
hipError_t launch_pool(const void* Q, const void* K, const Shape& s, float* qbar, float* kbar, hipStream_t st);
hipError_t launch_scores(const float* qbar, const float* kbar, const Shape& s, float* scores,
                         hipStream_t st);
// col_cnt: [BH][T] ints of scratch: cleared by the classification, filled by the table build
hipError_t launch_classify(const float* scores, const Shape& s, int8_t* Mc, int32_t* row_idx,
                           int32_t* col_cnt, hipStream_t st);
hipError_t launch_csc(const int8_t* Mc, const Shape& s, int32_t* col_cnt, int32_t* col_ptr, int32_t* col_rows,
                      unsigned long long* ind, unsigned long long* indT, int32_t* col_order, hipStream_t st);

// T <= 64: scores (computed from qbar, kbar and written to `scores`, or read from `given`),
// classification and all tables in one launch
hipError_t launch_mask_small(const float* qbar, const float* kbar, const float* given, const Shape& s, float* scores,
                             int8_t* Mc, int32_t* row_idx, unsigned long long* ind, unsigned long long* indT,
                             int32_t* col_ptr, int32_t* col_order, int32_t* col_rows, hipStream_t st);

// ---- float-arithmetic path (simt_kernels.hip): every contraction in fp32 FMA
struct FwdArgs {
  const void *Q, *K, *V, *W;
  const int8_t* Mc;
  const unsigned long long* ind;   // marginal indicator bit masks
  const int32_t* row_idx;
  void* O;
  void *Os, *Ol;   // may be null (inference)
  float* L;        // may be null
  float* HZ;       // [BH,T] state rows (saved or workspace)
  float* hz;       // [BH,T] state rows of the key blocks (workspace)
};
hipError_t simt_forward(const Shape& s, const FwdArgs& a, hipStream_t st);

struct BwdArgs {
  const void *Q, *K, *V, *W, *dO;
  const int8_t* Mc;
  const unsigned long long* indT;  // marginal indicator bit masks, transposed
  const int32_t *row_idx, *col_ptr, *col_rows, *col_order;
  const void *Os, *Ol;
  const float *L, *HZ;
  void *dQ, *dK, *dV;
  float* dW;
  char* ws;  // workspace, ws_backward_bytes
};
size_t simt_backward_ws_bytes(const Shape& s);
// critical-block gradients on the matrix cores (mfma_bwd.hip).  dQlin: linear-branch part of dQ.
// dHZcol: dH and dZ summed over the marginal blocks of each key block (bf16 matrices, then float
// vectors at state_z_offset); the dK/dV kernel turns them into the linear-branch parts of dK and
// dV itself.  Both may be null (no marginal block).
hipError_t mfma_backward_sparse(const Shape& s, const BwdArgs& a, const float* Ds, const void* dHZcol, hipStream_t st);
hipError_t simt_backward(const Shape& s, const BwdArgs& a, hipStream_t st);

// ---- bf16 matrix-core path (mfma_fwd.hip)
size_t mfma_forward_ws_bytes(const Shape& s);
hipError_t mfma_forward(const Shape& s, const FwdArgs& a, char* ws, hipStream_t st);
// out[i] = sum over k with bit k of ind[i] set of the bf16 state rows in[k] (mfma_aggregate.hip)
hipError_t mfma_aggregate(const void* in, const unsigned long long* ind, const Shape& s, void* outH, float* outZ,
                          hipStream_t st);
// bf16 tensors keep the aggregated states as a bf16 block [BH][T][d*d] (matrices, transposed)
// followed by a float block [BH][T][d] (vectors); this is the byte offset of the second block.
inline size_t state_z_offset(const Shape& s) { return ((size_t)s.BH * s.T * s.d * s.d * 2 + 255) / 256 * 256; }

// the same sums by additions (method 1), pre-aggregation (2) or Four Russians tables (3), for
// comparison (aggregate_alt.hip)
size_t aggregate_alt_ws_bytes(const Shape& s, int method);
hipError_t aggregate_alt(int method, const void* in, const unsigned long long* ind, const Shape& s, void* outH,
                         float* outZ, void* ws, hipStream_t st);

// query side on the matrix cores (mfma_bwd_query.hip): D^s, dH_i / dZ_i rows (dHZ16), dQ.  dQlin:
// scratch for the linear part of dQ (only used with query blocks of two or four tiles).
hipError_t mfma_backward_query(const Shape& s, const BwdArgs& a, float* Ds, void* dHZ16, float* dQlin, hipStream_t st);
// partial sums of dW = sum O^l^T dO
hipError_t mfma_backward_dw(const Shape& s, const BwdArgs& a, float* dWpart, int nparts, hipStream_t st);

// Brackets one kernel launch with events when profiling is on (profile.hip).
class KernelTimer {
 public:
  KernelTimer(const char* name, hipStream_t st);
  ~KernelTimer();
 private:
  hipStream_t st_;
  long idx_;
};

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// Raises the dynamic-LDS limit of a kernel to `bytes`, once per kernel and device (profile.hip);
// every later call is a table lookup on the host.
hipError_t ensure_dyn_lds(const void* kernel, int bytes);
template <typename K>
hipError_t ensure_dyn_lds(K kernel, size_t bytes) {
  return ensure_dyn_lds(reinterpret_cast<const void*>(kernel), (int)bytes);
}

// Whether query blocks of an even number of tiles run the eight-wave kernels (sla_wide_query_tiles;
// profile.hip holds the flag).
bool wide_query_tiles();

}  // namespace sla
#endif
