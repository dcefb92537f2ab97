// C ABI of the SLA library (declared in include/sla.h): argument checks, buffer layout and
// kernel dispatch.  Host code only; every kernel lives in the other translation units.
#include <math.h>
#include <string.h>

#include <mutex>

#include "../../include/sla.h"
#include "sla_internal.h"

using namespace sla;

namespace {

constexpr int kMaxT = 3072;  // classify keeps 4 rows of keys and labels in 64 KB of LDS

int make_shape(const sla_params* p, Shape* s) {
  if (!p) return SLA_EINVAL;
  if (p->B <= 0 || p->H <= 0 || p->N <= 0 || p->d <= 0) return SLA_EINVAL;
  if (!(p->k_h >= 0.0 && p->k_h <= 1.0) || !(p->k_l >= 0.0 && p->k_l <= 1.0)) return SLA_EINVAL;
  if (p->bkv != kBlk || p->bq < kBlk || p->bq % kBlk || p->bq > 4 * kBlk) return SLA_EUNSUPPORTED;
  if (p->d != 64 && p->d != 128) return SLA_EUNSUPPORTED;
  if (p->phi != SLA_PHI_SOFTMAX && p->phi != SLA_PHI_ELU1) return SLA_EUNSUPPORTED;
  if (p->dtype != SLA_F32 && p->dtype != SLA_BF16) return SLA_EUNSUPPORTED;
  if (p->layout != SLA_BHND && p->layout != SLA_BNHD && p->layout != SLA_STRIDED) return SLA_EUNSUPPORTED;
  const long long T = ((long long)p->N + kBlk - 1) / kBlk;
  if (T > kMaxT) return SLA_EUNSUPPORTED;
  if ((long long)p->B * p->H > 65535) return SLA_EUNSUPPORTED;  // grid.y / grid.z limit
  s->BH = p->B * p->H;
  s->N = p->N;
  s->d = p->d;
  s->T = (int)T;
  s->rq = p->bq / kBlk;
  s->Tq = (int)(((long long)p->N + p->bq - 1) / p->bq);
  long long nh = (long long)floor(p->k_h * (double)T + 0.5);
  nh = nh < 0 ? 0 : (nh > T ? T : nh);
  long long nl = (long long)floor(p->k_l * (double)T + 0.5);
  nl = nl < 0 ? 0 : (nl > T - nh ? T - nh : nl);
  s->n_h = (int)nh;
  s->n_l = (int)nl;
  s->n_0 = (int)(T - nh - nl);
  s->phi = p->phi;
  s->dtype = p->dtype;
  {
    const long long N = p->N, H = p->H, d = p->d, esz = p->dtype == SLA_F32 ? 4 : 2;
    long long sb = H * N * d, sh = N * d, sn = d;
    if (p->layout == SLA_BNHD) {
      sb = N * H * d;
      sh = d;
      sn = H * d;
    } else if (p->layout == SLA_STRIDED) {
      sb = p->stride_b;
      sh = p->stride_h;
      sn = p->stride_n;
      const long long q = 16 / esz;   // elements per 16 bytes
      if (sb < 0 || sh < 0 || sn < d || sb % q || sh % q || sn % q) return SLA_EINVAL;
    }
    // tile offsets inside a head are 32-bit byte offsets
    if (N * sn * esz >= (1ll << 31)) return SLA_EUNSUPPORTED;
    s->layv = Lay{sb, sh, (int)sn, (int)H};
  }
  s->scale = 1.0f / sqrtf((float)p->d);
  return SLA_OK;
}

void fill_sizes(const Shape& s, sla_sizes_t* o) {
  memset(o, 0, sizeof(*o));
  const size_t BH = s.BH, T = s.T, Tq = s.Tq, N = s.N, d = s.d;
  const size_t esz = s.dtype == SLA_F32 ? 4 : 2;
  o->T = s.T;
  o->Tq = s.Tq;
  o->n_h = s.n_h;
  o->n_l = s.n_l;
  o->n_0 = s.n_0;
  o->mask_bytes = BH * Tq * T;
  size_t off = 0;
  o->lut_row_idx = off;
  off += align_up(BH * T * (size_t)s.n_h * 4 + 4);
  o->lut_col_ptr = off;
  off += align_up(BH * (T + 1) * 4);
  o->lut_col_rows = off;
  off += align_up(BH * T * (size_t)s.n_h * 4 + 4);
  const size_t Tw = (T + 63) / 64;
  o->lut_ind = off;
  off += align_up(BH * T * Tw * 8);
  o->lut_ind_t = off;
  off += align_up(BH * T * Tw * 8);
  o->lut_col_order = off;
  off += align_up(BH * T * 4);
  off += align_up(BH * T * 4);   // column counts: scratch of the table build, at the end of the buffer
  o->luts_bytes = off;
  off = 0;
  o->saved_Os = off;
  off += align_up(BH * N * d * esz);
  o->saved_Ol = off;
  off += align_up(BH * N * d * esz);
  o->saved_L = off;
  off += align_up(BH * N * 4);
  o->saved_HZ = off;
  o->saved_Z = s.dtype == SLA_BF16 ? off + state_z_offset(s) : off + d * d * 4;
  const size_t state = align_up(BH * T * (size_t)s.state_row() * 4);
  off += state;
  o->saved_bytes = off;
  off = 0;
  o->ws_mask_qbar = off;
  off += align_up(BH * Tq * d * 4);
  o->ws_mask_kbar = off;
  off += align_up(BH * T * d * 4);
  o->ws_mask_scores = off;
  off += align_up(BH * Tq * T * 4);
  o->ws_mask_bytes = off;
  // [0, state): H_i, Z_i when the caller passes no `saved`; then the key-block states
  const size_t hz_ws = s.dtype == SLA_BF16 ? mfma_forward_ws_bytes(s) : state;
  o->ws_forward_bytes = state + hz_ws;
  o->ws_backward_bytes = simt_backward_ws_bytes(s);
}

inline bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

// Workspace of sla_build_mask_static: pool(Q), pool(K) and the block scores of one call.  Every
// GPU the library runs on holds its own copy of the array, at its own address, until the process
// ends.  In host code the array's name is not a device address: the address is looked up once per
// device and only that pointer is handed to kernels.
static __device__ __align__(256) unsigned char scratch[SLA_STATIC_WS_BYTES];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

hipError_t scratch_of_current_device(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

int hip_status(hipError_t e) { return e == hipSuccess ? SLA_OK : SLA_EHIP; }

}  // namespace

extern "C" {

int sla_sizes(const sla_params* p, sla_sizes_t* out) {
  Shape s;
  if (!out) return SLA_EINVAL;
  const int rc = make_shape(p, &s);
  if (rc != SLA_OK) return rc;
  fill_sizes(s, out);
  return SLA_OK;
}

int sla_classify_scores(const sla_params* p, const float* scores, int8_t* Mc, void* luts,
                        void* stream) {
  Shape s;
  const int rc = make_shape(p, &s);
  if (rc != SLA_OK) return rc;
  if (!scores || !Mc || !luts || misaligned(scores) || misaligned(luts)) return SLA_EINVAL;
  sla_sizes_t z;
  fill_sizes(s, &z);
  hipStream_t st = (hipStream_t)stream;
  char* l = (char*)luts;
  if (s.T <= kBlk)
    return hip_status(launch_mask_small(nullptr, nullptr, scores, s, nullptr, Mc, (int32_t*)(l + z.lut_row_idx),
                                        (unsigned long long*)(l + z.lut_ind), (unsigned long long*)(l + z.lut_ind_t),
                                        (int32_t*)(l + z.lut_col_ptr), (int32_t*)(l + z.lut_col_order),
                                        (int32_t*)(l + z.lut_col_rows), st));
  int32_t* col_cnt = (int32_t*)(l + z.luts_bytes - align_up((size_t)s.BH * s.T * 4));
  hipError_t e = launch_classify(scores, s, Mc, (int32_t*)(l + z.lut_row_idx), col_cnt, st);
  if (e == hipSuccess)
    e = launch_csc(Mc, s, col_cnt, (int32_t*)(l + z.lut_col_ptr), (int32_t*)(l + z.lut_col_rows),
                   (unsigned long long*)(l + z.lut_ind), (unsigned long long*)(l + z.lut_ind_t),
                   (int32_t*)(l + z.lut_col_order), st);
  return hip_status(e);
}

int sla_build_mask(const sla_params* p, const void* Q, const void* K, int8_t* Mc, void* luts,
                   void* workspace, size_t workspace_bytes, void* stream) {
  Shape s;
  const int rc = make_shape(p, &s);
  if (rc != SLA_OK) return rc;
  if (!Q || !K || !Mc || !luts || !workspace) return SLA_EINVAL;
  if (misaligned(Q) || misaligned(K) || misaligned(luts) || misaligned(workspace)) return SLA_EINVAL;
  sla_sizes_t z;
  fill_sizes(s, &z);
  if (workspace_bytes < z.ws_mask_bytes) return SLA_ENOSPACE;
  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  float* qbar = (float*)(ws + z.ws_mask_qbar);
  float* kbar = (float*)(ws + z.ws_mask_kbar);
  float* sc = (float*)(ws + z.ws_mask_scores);
  hipError_t e = launch_pool(Q, K, s, qbar, kbar, st);
  if (e == hipSuccess && s.T <= kBlk) {
    char* l = (char*)luts;
    return hip_status(launch_mask_small(qbar, kbar, nullptr, s, sc, Mc, (int32_t*)(l + z.lut_row_idx),
                                        (unsigned long long*)(l + z.lut_ind), (unsigned long long*)(l + z.lut_ind_t),
                                        (int32_t*)(l + z.lut_col_ptr), (int32_t*)(l + z.lut_col_order),
                                        (int32_t*)(l + z.lut_col_rows), st));
  }
  if (e == hipSuccess) e = launch_scores(qbar, kbar, s, sc, st);
  if (e != hipSuccess) return SLA_EHIP;
  return sla_classify_scores(p, sc, Mc, luts, stream);
}

int sla_build_mask_static(const sla_params* p, const void* Q, const void* K, int8_t* Mc, void* luts,
                          void* stream) {
  Shape s;
  const int rc = make_shape(p, &s);
  if (rc != SLA_OK) return rc;
  sla_sizes_t z;
  fill_sizes(s, &z);
  if (z.ws_mask_bytes > (uint64_t)SLA_STATIC_WS_BYTES) return SLA_ENOSPACE;
  if (!Q || !K || !Mc || !luts) return SLA_EINVAL;
  void* ws = nullptr;
  if (scratch_of_current_device(&ws) != hipSuccess) return SLA_EHIP;
  // every byte of the workspace that the mask kernels read is written earlier in the same call,
  // so nothing has to be cleared between calls
  return sla_build_mask(p, Q, K, Mc, luts, ws, (size_t)SLA_STATIC_WS_BYTES, stream);
}

int sla_forward(const sla_params* p, const void* Q, const void* K, const void* V, const void* W,
                const int8_t* Mc, const void* luts, void* O, void* saved, void* workspace,
                size_t workspace_bytes, void* stream) {
  Shape s;
  const int rc = make_shape(p, &s);
  if (rc != SLA_OK) return rc;
  if (!Q || !K || !V || !W || !Mc || !luts || !O || !workspace) return SLA_EINVAL;
  if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(W) || misaligned(O) ||
      misaligned(luts) || misaligned(saved) || misaligned(workspace))
    return SLA_EINVAL;
  sla_sizes_t z;
  fill_sizes(s, &z);
  if (workspace_bytes < z.ws_forward_bytes) return SLA_ENOSPACE;
  char* ws = (char*)workspace;
  char* sv = (char*)saved;
  const char* l = (const char*)luts;
  FwdArgs a;
  a.Q = Q; a.K = K; a.V = V; a.W = W;
  a.Mc = Mc;
  a.row_idx = (const int32_t*)(l + z.lut_row_idx);
  a.ind = (const unsigned long long*)(l + z.lut_ind);
  a.O = O;
  a.Os = sv ? sv + z.saved_Os : nullptr;
  a.Ol = sv ? sv + z.saved_Ol : nullptr;
  a.L = sv ? (float*)(sv + z.saved_L) : nullptr;
  const size_t state = z.saved_bytes - z.saved_HZ;
  a.hz = (float*)(ws + state);
  a.HZ = sv ? (float*)(sv + z.saved_HZ) : (float*)ws;
  if (s.dtype == SLA_BF16) return hip_status(mfma_forward(s, a, ws + state, (hipStream_t)stream));
  return hip_status(simt_forward(s, a, (hipStream_t)stream));
}

int sla_backward(const sla_params* p, const void* Q, const void* K, const void* V, const void* W,
                 const int8_t* Mc, const void* luts, const void* saved, const void* dO, void* dQ,
                 void* dK, void* dV, float* dW, void* workspace, size_t workspace_bytes,
                 void* stream) {
  Shape s;
  const int rc = make_shape(p, &s);
  if (rc != SLA_OK) return rc;
  if (!Q || !K || !V || !W || !Mc || !luts || !saved || !dO || !dQ || !dK || !dV || !dW || !workspace)
    return SLA_EINVAL;
  if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(W) || misaligned(dO) ||
      misaligned(dQ) || misaligned(dK) || misaligned(dV) || misaligned(dW) || misaligned(luts) ||
      misaligned(saved) || misaligned(workspace))
    return SLA_EINVAL;
  sla_sizes_t z;
  fill_sizes(s, &z);
  if (workspace_bytes < z.ws_backward_bytes) return SLA_ENOSPACE;
  const char* sv = (const char*)saved;
  const char* l = (const char*)luts;
  BwdArgs a;
  a.Q = Q; a.K = K; a.V = V; a.W = W; a.dO = dO;
  a.Mc = Mc;
  a.row_idx = (const int32_t*)(l + z.lut_row_idx);
  a.col_ptr = (const int32_t*)(l + z.lut_col_ptr);
  a.col_rows = (const int32_t*)(l + z.lut_col_rows);
  a.indT = (const unsigned long long*)(l + z.lut_ind_t);
  a.col_order = (const int32_t*)(l + z.lut_col_order);
  a.Os = sv + z.saved_Os;
  a.Ol = sv + z.saved_Ol;
  a.L = (const float*)(sv + z.saved_L);
  a.HZ = (const float*)(sv + z.saved_HZ);
  a.dQ = dQ; a.dK = dK; a.dV = dV;
  a.dW = dW;
  a.ws = (char*)workspace;
  return hip_status(simt_backward(s, a, (hipStream_t)stream));
}

int sla_aggregate_ws_bytes(const sla_params* p, int method, uint64_t* bytes) {
  Shape s;
  if (!bytes) return SLA_EINVAL;
  const int rc = make_shape(p, &s);
  if (rc != SLA_OK) return rc;
  if (s.dtype != SLA_BF16 || method < SLA_AGG_GEMM || method > SLA_AGG_FOUR_RUSSIANS) return SLA_EUNSUPPORTED;
  *bytes = method == SLA_AGG_GEMM ? 0 : aggregate_alt_ws_bytes(s, method);
  return SLA_OK;
}

int sla_aggregate_states(const sla_params* p, int method, const void* luts, const void* h, void* outH,
                         float* outZ, void* workspace, size_t workspace_bytes, void* stream) {
  uint64_t need = 0;
  const int rc = sla_aggregate_ws_bytes(p, method, &need);
  if (rc != SLA_OK) return rc;
  if (!luts || !h || !outH || !outZ || (need && !workspace)) return SLA_EINVAL;
  if (misaligned(luts) || misaligned(h) || misaligned(outH) || misaligned(outZ) || misaligned(workspace))
    return SLA_EINVAL;
  if (workspace_bytes < need) return SLA_ENOSPACE;
  Shape s;
  make_shape(p, &s);
  sla_sizes_t z;
  fill_sizes(s, &z);
  const unsigned long long* ind = (const unsigned long long*)((const char*)luts + z.lut_ind);
  hipStream_t st = (hipStream_t)stream;
  if (method == SLA_AGG_GEMM) return hip_status(mfma_aggregate(h, ind, s, outH, outZ, st));
  return hip_status(aggregate_alt(method, h, ind, s, outH, outZ, workspace, st));
}

const char* sla_strerror(int code) {
  switch (code) {
    case SLA_OK: return "ok";
    case SLA_EINVAL: return "invalid argument (null or misaligned pointer, non-positive size, k outside [0,1])";
    case SLA_EUNSUPPORTED: return "unsupported configuration (block size, head dim, dtype, phi or sequence length)";
    case SLA_ENOSPACE: return "workspace too small (see sla_sizes)";
    case SLA_EHIP: return "a HIP call or kernel launch failed";
    default: return "unknown error code";
  }
}

}  // extern "C"
