// C ABI of the RSA library: argument validation and dispatch (declared in rsa.h).
#include <cmath>
#include <cstring>
#include <mutex>

#include "rsa_kernels.h"

namespace {

using rsa::Dims;

int validate(const rsa_desc *d, Dims *out) {
  if (!d) return RSA_ERR_NULL;
  if (d->B < 1 || d->Z < 1 || d->A < 1 || d->L < 1 || d->N < 1) return RSA_ERR_SHAPE;
  if (d->L % d->N != 0) return RSA_ERR_SHAPE;  // section 4.2: L divisible by the ring size
  if (d->rank_begin < 0 || d->rank_end > d->N || d->rank_begin >= d->rank_end) return RSA_ERR_SHAPE;
  if (d->A % 64 != 0 || d->A > 256) return RSA_ERR_UNSUPPORTED;
  if (d->dtype != RSA_F32 && d->dtype != RSA_BF16) return RSA_ERR_UNSUPPORTED;
  if (d->flags & ~(RSA_MODE_STAGED | RSA_OWN_ZIGZAG | RSA_DETERMINISTIC)) return RSA_ERR_UNSUPPORTED;
  const int mode = (int)(d->flags & RSA_MODE_STAGED);
  const int zigzag = (d->flags & RSA_OWN_ZIGZAG) ? 1 : 0;
  // the fused kernels are written for bf16 heads of 64 or 128 elements
  if (mode == RSA_MODE_FUSED && (d->dtype != RSA_BF16 || (d->A != 64 && d->A != 128))) return RSA_ERR_UNSUPPORTED;
  const int64_t c = d->L / d->N;
  if (c % 64 != 0) return RSA_ERR_UNSUPPORTED;
  if (zigzag && (mode == RSA_MODE_STAGED || c % 128 != 0)) return RSA_ERR_UNSUPPORTED;
  if (!(d->scale >= 0.0f) || !std::isfinite(d->scale)) return RSA_ERR_SHAPE;
  if ((int64_t)d->B * d->Z > 65535) return RSA_ERR_UNSUPPORTED;  // heads ride on gridDim.z
  out->B = d->B; out->Z = d->Z; out->A = d->A; out->N = d->N;
  out->rank_begin = d->rank_begin; out->rank_end = d->rank_end;
  out->causal = d->causal ? 1 : 0;
  out->mode = mode; out->zigzag = zigzag;
  out->L = d->L; out->c = c; out->Lq = (int64_t)(d->rank_end - d->rank_begin) * c;
  out->scale = d->scale > 0.0f ? d->scale : 1.0f / std::sqrt((float)d->A);
  out->deterministic = (d->flags & RSA_DETERMINISTIC) ? 1 : 0;
  // strides: all zero selects the dense layout; otherwise every stride must be positive, the
  // row stride a multiple of 16 bytes that holds a row, and only the fused kernels take them
  const int64_t *in[3] = {d->q_stride, d->kv_stride, d->o_stride};
  int64_t *st[3] = {out->qs, out->ks, out->os};
  const int64_t rows[3] = {out->Lq, out->L, out->Lq};
  out->strided = 0;
  for (int t = 0; t < 3; ++t) {
    const bool zero = in[t][0] == 0 && in[t][1] == 0 && in[t][2] == 0;
    const int64_t dense[3] = {(int64_t)d->Z * rows[t] * d->A, rows[t] * d->A, d->A};
    for (int k = 0; k < 3; ++k) st[t][k] = zero ? dense[k] : in[t][k];
    if (zero) continue;
    if (in[t][0] <= 0 || in[t][1] <= 0 || in[t][2] < d->A) return RSA_ERR_SHAPE;
    if (in[t][2] % 8 != 0 || in[t][2] > (1 << 24) || in[t][1] % 8 != 0 || in[t][0] % 8 != 0)
      return RSA_ERR_UNSUPPORTED;
    if (st[t][0] != dense[0] || st[t][1] != dense[1] || st[t][2] != dense[2]) out->strided = 1;
  }
  if (out->strided && mode == RSA_MODE_STAGED) return RSA_ERR_UNSUPPORTED;
  return RSA_OK;
}

inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Workspace layout of the staged mode (offsets in bytes, each block 256-aligned).
struct StagedWs {
  size_t strip32, strip32b, strip16, strip16b, acc_q, acc_k, acc_v, dvec, total;
};
StagedWs staged_layout(const Dims &d, int dtype, int pass) {
  const size_t heads = (size_t)d.B * d.Z;
  const size_t strip = heads * (size_t)d.c * (size_t)d.L;
  const size_t es = dtype == RSA_BF16 ? 2 : 4;
  StagedWs w{};
  size_t off = 0;
  w.strip32 = off; off += align256(strip * 4);                 // S (fp32)
  w.strip16 = off; off += align256(strip * es);                // P (dtype)
  w.acc_q = off; off += align256(heads * d.c * d.A * 4);       // Oacc or dQacc
  if (pass == 1) {
    w.strip32b = off; off += align256(strip * 4);              // dP (fp32)
    w.strip16b = off; off += align256(strip * es);             // dS (dtype)
    w.acc_k = off; off += align256(heads * d.L * d.A * 4);     // dKacc
    w.acc_v = off; off += align256(heads * d.L * d.A * 4);     // dVacc
    w.dvec = off; off += align256(heads * d.Lq * 4);           // D
  }
  w.total = off;
  return w;
}

// Fused backward: the row terms -D and -LSE / scale (fp32 per row)
size_t fused_bwd_base(const Dims &d) {
  const size_t rows = (size_t)d.B * d.Z * d.Lq;
  return 2 * align256(rows * 4);
}

// Fused backward with dQ from its own kernel: the row terms, then the partial dQ per split and
// row when the key walk is split.
size_t det_bwd_bytes(const Dims &d) {
  const size_t rows = (size_t)d.B * d.Z * d.Lq;
  const int ks = rsa::fused_key_splits(d);
  return fused_bwd_base(d) + (ks > 1 ? align256(ks * rows * d.A * 4) : 0);
}

// Fused path: the partial results of a split key walk (forward: unnormalised O and the pair
// (max, sum) per split and row; backward: partial dQ per split and row, after the base part).
size_t workspace_bytes(const Dims &d, int dtype, int pass) {
  if (d.mode == RSA_MODE_STAGED) return staged_layout(d, dtype, pass).total;
  const size_t rows = (size_t)d.B * d.Z * d.Lq;
  if (pass == 1) return det_bwd_bytes(d);
  bool big;
  int fs;
  rsa::fused_fwd_plan(d, &big, &fs);
  return fs > 1 ? align256(fs * rows * (d.A + 2) * 4) : 0;
}
// where the split walks' partial sums start in the backward workspace
inline float *fused_part(const Dims &d, void *ws) {
  return reinterpret_cast<float *>(static_cast<char *>(ws) + fused_bwd_base(d));
}

// Fused backward workspace: -D at the start, -LSE / scale next.
inline float *fused_nD(void *ws) { return static_cast<float *>(ws); }
inline float *fused_nL(const Dims &d, void *ws) {
  return reinterpret_cast<float *>(static_cast<char *>(ws) + align256((size_t)d.B * d.Z * d.Lq * 4));
}

inline int hip_status(hipError_t e) { return e == hipSuccess ? RSA_OK : RSA_ERR_HIP; }

#define RSA_TRY(expr)                             \
  do {                                            \
    hipError_t e_ = (expr);                       \
    if (e_ != hipSuccess) return RSA_ERR_HIP;     \
  } while (0)

int check_rank_chunk(const Dims &d, int n, int j) {
  if (n < d.rank_begin || n >= d.rank_end) return RSA_ERR_SHAPE;
  if (j < 0 || j >= d.N) return RSA_ERR_SHAPE;
  return RSA_OK;
}

// The paper's two-pass forward for the simulated ranks, one after the other.
int staged_forward(const Dims &d, int dtype, const void *Q, const void *K, const void *V, void *O,
                   float *LSE, char *ws, hipStream_t st) {
  const StagedWs w = staged_layout(d, dtype, 0);
  float *S = reinterpret_cast<float *>(ws + w.strip32);
  void *P = ws + w.strip16;
  float *Oacc = reinterpret_cast<float *>(ws + w.acc_q);
  const size_t es = dtype == RSA_BF16 ? 2 : 4;
  for (int n = d.rank_begin; n < d.rank_end; ++n) {
    for (int t = 0; t < d.N; ++t) {  // K ring pass, local chunk first
      const int j = (n - t + d.N) % d.N;
      RSA_TRY(rsa::staged_qk_step(d, dtype, n, j, Q, K, S, st));
    }
    RSA_TRY(rsa::staged_row_softmax(d, dtype, n, S, P, LSE, st));
    int first = 1;
    for (int t = 0; t < d.N; ++t) {  // V ring pass
      const int j = (n - t + d.N) % d.N;
      if (d.causal && j > n) continue;  // all-zero probabilities
      RSA_TRY(rsa::staged_av_step(d, dtype, n, j, P, V, Oacc, !first, st));
      first = 0;
    }
    char *On = static_cast<char *>(O) + (size_t)(n - d.rank_begin) * d.c * d.A * es;
    RSA_TRY(rsa::store_rows(dtype, Oacc, On, (int64_t)d.B * d.Z, d.c, d.A, d.c * d.A, d.Lq * d.A, st));
  }
  return RSA_OK;
}

int staged_backward(const Dims &d, int dtype, const void *dO, const void *Q, const void *K,
                    const void *V, const void *O, void *dQ, void *dK, void *dV, char *ws,
                    hipStream_t st) {
  const StagedWs w = staged_layout(d, dtype, 1);
  float *S = reinterpret_cast<float *>(ws + w.strip32);
  void *P = ws + w.strip16;
  float *dP = reinterpret_cast<float *>(ws + w.strip32b);
  void *dS = ws + w.strip16b;
  float *dQacc = reinterpret_cast<float *>(ws + w.acc_q);
  float *dKacc = reinterpret_cast<float *>(ws + w.acc_k);
  float *dVacc = reinterpret_cast<float *>(ws + w.acc_v);
  float *D = reinterpret_cast<float *>(ws + w.dvec);
  const size_t es = dtype == RSA_BF16 ? 2 : 4;
  const int64_t heads = (int64_t)d.B * d.Z;
  // chunks that no simulated rank looks at keep a zero gradient
  RSA_TRY(rsa::zero_f32(dKacc, heads * d.L * d.A, st));
  RSA_TRY(rsa::zero_f32(dVacc, heads * d.L * d.A, st));
  RSA_TRY(rsa::rowdot(d, dtype, 0, d.Lq, dO, O, D, st));
  // the softmax statistics are recomputed; the LSE written here is scratch
  float *lse_scratch = dQacc;  // (heads * c) floats fit in (heads * c * A)
  for (int n = d.rank_begin; n < d.rank_end; ++n) {
    Dims dn = d;  // a view in which rank n is the only rank, for the scratch LSE rows
    for (int t = 0; t < d.N; ++t) {
      const int j = (n - t + d.N) % d.N;
      RSA_TRY(rsa::staged_qk_step(d, dtype, n, j, Q, K, S, st));
    }
    dn.rank_begin = n; dn.rank_end = n + 1; dn.Lq = d.c;
    RSA_TRY(rsa::staged_row_softmax(dn, dtype, n, S, P, lse_scratch, st));
    for (int t = 0; t < d.N; ++t) {  // V ring pass of the backward: dP
      const int j = (n - t + d.N) % d.N;
      RSA_TRY(rsa::staged_dp_step(d, dtype, n, j, dO, V, dP, st));
    }
    RSA_TRY(rsa::staged_softmax_bwd(d, dtype, n, P, dP, D, dS, st));
    int first = 1;
    for (int t = 0; t < d.N; ++t) {  // K ring pass of the backward: dQ; partial dK, dV
      const int j = (n - t + d.N) % d.N;
      if (d.causal && j > n) continue;
      RSA_TRY(rsa::staged_dq_step(d, dtype, n, j, dS, K, dQacc, !first, st));
      RSA_TRY(rsa::staged_dk_step(d, dtype, n, j, dS, Q, dKacc, 1, st));
      RSA_TRY(rsa::staged_dv_step(d, dtype, n, j, P, dO, dVacc, 1, st));
      first = 0;
    }
    char *dQn = static_cast<char *>(dQ) + (size_t)(n - d.rank_begin) * d.c * d.A * es;
    RSA_TRY(rsa::store_rows(dtype, dQacc, dQn, heads, d.c, d.A, d.c * d.A, d.Lq * d.A, st));
  }
  RSA_TRY(rsa::store_rows(dtype, dKacc, dK, heads, d.L, d.A, d.L * d.A, d.L * d.A, st));
  RSA_TRY(rsa::store_rows(dtype, dVacc, dV, heads, d.L, d.A, d.L * d.A, d.L * d.A, st));
  return RSA_OK;
}

}  // namespace

extern "C" {

int rsa_version(void) { return 110; }

const char *rsa_strerror(int status) {
  switch (status) {
    case RSA_OK: return "ok";
    case RSA_ERR_NULL: return "a required pointer is NULL";
    case RSA_ERR_SHAPE: return "bad shape: sizes must be positive, L divisible by N, ranks within [0, N)";
    case RSA_ERR_UNSUPPORTED:
      return "unsupported: need a head size of 64 or 128 (staged mode: a multiple of 64 up to 256), L/N "
             "divisible by 64, 16-byte aligned pointers, bf16 for the fused mode";
    case RSA_ERR_WORKSPACE: return "workspace missing or too small";
    case RSA_ERR_HIP: return "a HIP call failed";
    default: return "unknown status";
  }
}

size_t rsa_workspace_bytes(const rsa_desc *d, int pass) {
  Dims dm;
  if (validate(d, &dm) != RSA_OK || (pass != 0 && pass != 1)) return 0;
  return workspace_bytes(dm, d->dtype, pass);
}

int rsa_forward(const rsa_desc *d, const void *Q, const void *K, const void *V, void *O, float *LSE,
                void *ws, size_t ws_bytes, void *stream) {
  Dims dm;
  int rc = validate(d, &dm);
  if (rc != RSA_OK) return rc;
  if (!Q || !K || !V || !O || !LSE) return RSA_ERR_NULL;
  if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || misaligned(LSE) || misaligned(ws))
    return RSA_ERR_UNSUPPORTED;
  const size_t need = workspace_bytes(dm, d->dtype, 0);
  if (need > 0 && (!ws || ws_bytes < need)) return RSA_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (dm.mode == RSA_MODE_STAGED)
    return staged_forward(dm, d->dtype, Q, K, V, O, LSE, static_cast<char *>(ws), st);
  return hip_status(rsa::fused_forward(dm, Q, K, V, O, LSE, st, static_cast<float *>(ws)));
}

int rsa_backward(const rsa_desc *d, const void *dO, const void *Q, const void *K, const void *V,
                 const void *O, const float *LSE, void *dQ, void *dK, void *dV, void *ws,
                 size_t ws_bytes, void *stream) {
  Dims dm;
  int rc = validate(d, &dm);
  if (rc != RSA_OK) return rc;
  if (!dO || !Q || !K || !V || !O || !LSE || !dQ || !dK || !dV) return RSA_ERR_NULL;
  if (misaligned(dO) || misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) ||
      misaligned(LSE) || misaligned(dQ) || misaligned(dK) || misaligned(dV) || misaligned(ws))
    return RSA_ERR_UNSUPPORTED;
  const size_t need = workspace_bytes(dm, d->dtype, 1);
  if (!ws || ws_bytes < need) return RSA_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (dm.mode == RSA_MODE_STAGED)
    return staged_backward(dm, d->dtype, dO, Q, K, V, O, dQ, dK, dV, static_cast<char *>(ws), st);
  return hip_status(rsa::fused_backward(dm, dO, Q, K, V, O, LSE, dQ, dK, dV, fused_nD(ws),
                                        fused_nL(dm, ws), st, fused_part(dm, ws), 1,
                                        rsa::fused_key_splits(dm)));
}

// The workspace of rsa_backward_static: one array per GPU, inside the library's code object.
// In host code the array's name is only a handle; its device address is looked up once per
// device (with that device current) and kept.
static __device__ __align__(256) unsigned char scratch[RSA_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void *scratch_addr[kMaxDevices] = {};

int scratch_of_current_device(void **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return RSA_ERR_HIP;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_addr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return RSA_ERR_HIP;
    scratch_addr[dev] = p;
  }
  *out = scratch_addr[dev];
  return RSA_OK;
}
}  // namespace

int rsa_backward_static(const rsa_desc *d, const void *dO, const void *Q, const void *K, const void *V,
                        const void *O, const float *LSE, void *dQ, void *dK, void *dV, void *stream) {
  Dims dm;
  int rc = validate(d, &dm);
  if (rc != RSA_OK) return rc;
  if (dm.mode != RSA_MODE_FUSED) return RSA_ERR_UNSUPPORTED;  // the staged strip is far larger
  if (workspace_bytes(dm, d->dtype, 1) > (size_t)RSA_STATIC_SCRATCH_BYTES) return RSA_ERR_WORKSPACE;
  void *ws = nullptr;
  if ((rc = scratch_of_current_device(&ws)) != RSA_OK) return rc;
  return rsa_backward(d, dO, Q, K, V, O, LSE, dQ, dK, dV, ws, RSA_STATIC_SCRATCH_BYTES, stream);
}

// ------------------------------------------------------------ step level ----
#define RSA_STEP_PROLOGUE(ptr_ok, ...)                            \
  Dims dm;                                                        \
  int rc = validate(d, &dm);                                      \
  if (rc != RSA_OK) return rc;                                    \
  if (!(ptr_ok)) return RSA_ERR_NULL;                             \
  { const void *ps_[] = {__VA_ARGS__};                            \
    for (const void *p_ : ps_) if (misaligned(p_)) return RSA_ERR_UNSUPPORTED; } \
  hipStream_t st = static_cast<hipStream_t>(stream)

int rsa_qk_step(const rsa_desc *d, int n, int j, const void *Q, const void *K, float *S, void *stream) {
  RSA_STEP_PROLOGUE(Q && K && S, Q, K, S);
  if (dm.strided) return RSA_ERR_UNSUPPORTED;  // the two-pass kernels take dense tensors only
  if ((rc = check_rank_chunk(dm, n, j)) != RSA_OK) return rc;
  return hip_status(rsa::staged_qk_step(dm, d->dtype, n, j, Q, K, S, st));
}

int rsa_row_softmax(const rsa_desc *d, int n, const float *S, void *P, float *LSE, void *stream) {
  RSA_STEP_PROLOGUE(S && P && LSE, S, P, LSE);
  if (dm.strided) return RSA_ERR_UNSUPPORTED;  // the two-pass kernels take dense tensors only
  if ((rc = check_rank_chunk(dm, n, 0)) != RSA_OK) return rc;
  return hip_status(rsa::staged_row_softmax(dm, d->dtype, n, S, P, LSE, st));
}

int rsa_av_step(const rsa_desc *d, int n, int j, const void *P, const void *V, float *Oacc,
                int accumulate, void *stream) {
  RSA_STEP_PROLOGUE(P && V && Oacc, P, V, Oacc);
  if (dm.strided) return RSA_ERR_UNSUPPORTED;  // the two-pass kernels take dense tensors only
  if ((rc = check_rank_chunk(dm, n, j)) != RSA_OK) return rc;
  return hip_status(rsa::staged_av_step(dm, d->dtype, n, j, P, V, Oacc, accumulate != 0, st));
}

int rsa_bwd_rowdot(const rsa_desc *d, int n, const void *dO, const void *O, float *D, void *stream) {
  RSA_STEP_PROLOGUE(dO && O && D, dO, O, D);
  if (dm.strided) return RSA_ERR_UNSUPPORTED;  // the two-pass kernels take dense tensors only
  if (n == -1) return hip_status(rsa::rowdot(dm, d->dtype, 0, dm.Lq, dO, O, D, st));
  if ((rc = check_rank_chunk(dm, n, 0)) != RSA_OK) return rc;
  return hip_status(rsa::rowdot(dm, d->dtype, (int64_t)(n - dm.rank_begin) * dm.c, dm.c, dO, O, D, st));
}

int rsa_dv_step(const rsa_desc *d, int n, int j, const void *P, const void *dO, float *dVacc,
                int accumulate, void *stream) {
  RSA_STEP_PROLOGUE(P && dO && dVacc, P, dO, dVacc);
  if (dm.strided) return RSA_ERR_UNSUPPORTED;  // the two-pass kernels take dense tensors only
  if ((rc = check_rank_chunk(dm, n, j)) != RSA_OK) return rc;
  return hip_status(rsa::staged_dv_step(dm, d->dtype, n, j, P, dO, dVacc, accumulate != 0, st));
}

int rsa_dp_step(const rsa_desc *d, int n, int j, const void *dO, const void *V, float *dP, void *stream) {
  RSA_STEP_PROLOGUE(dO && V && dP, dO, V, dP);
  if (dm.strided) return RSA_ERR_UNSUPPORTED;  // the two-pass kernels take dense tensors only
  if ((rc = check_rank_chunk(dm, n, j)) != RSA_OK) return rc;
  return hip_status(rsa::staged_dp_step(dm, d->dtype, n, j, dO, V, dP, st));
}

int rsa_softmax_bwd(const rsa_desc *d, int n, const void *P, const float *dP, const float *D,
                    void *dS, void *stream) {
  RSA_STEP_PROLOGUE(P && dP && D && dS, P, dP, D, dS);
  if (dm.strided) return RSA_ERR_UNSUPPORTED;  // the two-pass kernels take dense tensors only
  if ((rc = check_rank_chunk(dm, n, 0)) != RSA_OK) return rc;
  return hip_status(rsa::staged_softmax_bwd(dm, d->dtype, n, P, dP, D, dS, st));
}

int rsa_dq_step(const rsa_desc *d, int n, int j, const void *dS, const void *K, float *dQacc,
                int accumulate, void *stream) {
  RSA_STEP_PROLOGUE(dS && K && dQacc, dS, K, dQacc);
  if (dm.strided) return RSA_ERR_UNSUPPORTED;  // the two-pass kernels take dense tensors only
  if ((rc = check_rank_chunk(dm, n, j)) != RSA_OK) return rc;
  return hip_status(rsa::staged_dq_step(dm, d->dtype, n, j, dS, K, dQacc, accumulate != 0, st));
}

int rsa_dk_step(const rsa_desc *d, int n, int j, const void *dS, const void *Q, float *dKacc,
                int accumulate, void *stream) {
  RSA_STEP_PROLOGUE(dS && Q && dKacc, dS, Q, dKacc);
  if (dm.strided) return RSA_ERR_UNSUPPORTED;  // the two-pass kernels take dense tensors only
  if ((rc = check_rank_chunk(dm, n, j)) != RSA_OK) return rc;
  return hip_status(rsa::staged_dk_step(dm, d->dtype, n, j, dS, Q, dKacc, accumulate != 0, st));
}

int rsa_store(const rsa_desc *d, const float *src, void *dst, size_t count, void *stream) {
  RSA_STEP_PROLOGUE(src && dst, src, dst);
  if (count % 4 != 0) return RSA_ERR_SHAPE;
  return hip_status(rsa::store_rows(d->dtype, src, dst, 1, 1, (int64_t)count, 0, 0, st));
}

int rsa_bwd_preprocess(const rsa_desc *d, const void *dO, const void *O, const float *LSE,
                       void *ws, size_t ws_bytes, void *stream) {
  RSA_STEP_PROLOGUE(dO && O && LSE, dO, O, LSE, ws);
  if (d->dtype != RSA_BF16 || dm.mode != RSA_MODE_FUSED) return RSA_ERR_UNSUPPORTED;
  if (!ws || ws_bytes < det_bwd_bytes(dm)) return RSA_ERR_WORKSPACE;
  return hip_status(rsa::fused_bwd_preprocess(dm, dO, O, LSE, fused_nD(ws), fused_nL(dm, ws), st));
}

int rsa_bwd_dkdv(const rsa_desc *d, const void *dO, const void *Q, const void *K, const void *V,
                 const void *ws, size_t ws_bytes, void *dK, void *dV, void *stream) {
  RSA_STEP_PROLOGUE(dO && Q && K && V && dK && dV, dO, Q, K, V, ws, dK, dV);
  if (d->dtype != RSA_BF16 || dm.mode != RSA_MODE_FUSED) return RSA_ERR_UNSUPPORTED;
  if (!ws || ws_bytes < det_bwd_bytes(dm)) return RSA_ERR_WORKSPACE;
  void *w = const_cast<void *>(ws);
  return hip_status(rsa::fused_bwd_dkdv(dm, dO, Q, K, V, fused_nL(dm, w), fused_nD(w), dK, dV, st));
}

int rsa_bwd_dq(const rsa_desc *d, const void *dO, const void *Q, const void *K, const void *V,
               void *ws, size_t ws_bytes, void *dQ, void *stream) {
  RSA_STEP_PROLOGUE(dO && Q && K && V && dQ, dO, Q, K, V, ws, dQ);
  if (d->dtype != RSA_BF16 || dm.mode != RSA_MODE_FUSED) return RSA_ERR_UNSUPPORTED;
  if (!ws || ws_bytes < det_bwd_bytes(dm)) return RSA_ERR_WORKSPACE;
  return hip_status(rsa::fused_bwd_dq(dm, dO, Q, K, V, fused_nL(dm, ws), fused_nD(ws), dQ, st,
                                      fused_part(dm, ws), rsa::fused_key_splits(dm)));
}

// ----------------------------------------------- projections around RSA ----
namespace {
int proj_check(const rsa_desc *d, int32_t H, Dims *dm) {
  int rc = validate(d, dm);
  if (rc != RSA_OK) return rc;
  if (dm->mode != RSA_MODE_FUSED || d->dtype != RSA_BF16 || dm->strided) return RSA_ERR_UNSUPPORTED;
  if (H < 64) return RSA_ERR_SHAPE;
  if (H % 64 != 0) return RSA_ERR_UNSUPPORTED;
  // the GEMM kernel indexes rows and columns of its operands with 32 bits
  if ((int64_t)dm->B * dm->Lq >= (1LL << 31)) return RSA_ERR_UNSUPPORTED;
  return RSA_OK;
}
size_t proj_ws(const Dims &dm, int64_t H) {
  const int64_t M = (int64_t)dm.B * dm.Lq, ZA = (int64_t)dm.Z * dm.A;
  const int s1 = rsa::proj_wgrad_splits(ZA, H, M), s2 = rsa::proj_wgrad_splits(H, 3 * ZA, M);
  const size_t a = s1 > 1 ? (size_t)s1 * ZA * H * 4 : 0, b = s2 > 1 ? (size_t)s2 * H * 3 * ZA * 4 : 0;
  return align256(a > b ? a : b);
}
}  // namespace

size_t rsa_proj_workspace_bytes(const rsa_desc *d, int32_t H) {
  Dims dm;
  if (proj_check(d, H, &dm) != RSA_OK) return 0;
  return proj_ws(dm, H);
}

#define RSA_PROJ_PROLOGUE(ptr_ok, ...)                            \
  Dims dm;                                                        \
  int rc = proj_check(d, H, &dm);                                 \
  if (rc != RSA_OK) return rc;                                    \
  if (!(ptr_ok)) return RSA_ERR_NULL;                             \
  { const void *ps_[] = {__VA_ARGS__};                            \
    for (const void *p_ : ps_) if (misaligned(p_)) return RSA_ERR_UNSUPPORTED; } \
  hipStream_t st = static_cast<hipStream_t>(stream)

int rsa_qkv_proj(const rsa_desc *d, int32_t H, const void *X, const void *Wqkv, void *Q, void *K,
                 void *V, void *stream) {
  RSA_PROJ_PROLOGUE(X && Wqkv && Q && K && V, X, Wqkv, Q, K, V);
  return hip_status(rsa::proj_qkv(dm, H, X, Wqkv, Q, K, V, st));
}

int rsa_out_proj(const rsa_desc *d, int32_t H, const void *O, const void *Wo, void *Y, void *stream) {
  RSA_PROJ_PROLOGUE(O && Wo && Y, O, Wo, Y);
  return hip_status(rsa::proj_out(dm, H, O, Wo, Y, st));
}

int rsa_out_proj_bwd(const rsa_desc *d, int32_t H, const void *dY, const void *O, const void *Wo,
                     void *dO, float *dWo, void *ws, size_t ws_bytes, void *stream) {
  RSA_PROJ_PROLOGUE(dY && O && Wo && dO && dWo, dY, O, Wo, dO, dWo, ws);
  const size_t need = proj_ws(dm, H);
  if (need > 0 && (!ws || ws_bytes < need)) return RSA_ERR_WORKSPACE;
  return hip_status(rsa::proj_out_bwd(dm, H, dY, O, Wo, dO, dWo, static_cast<float *>(ws), st));
}

int rsa_qkv_proj_bwd(const rsa_desc *d, int32_t H, const void *dQ, const void *dK, const void *dV,
                     const void *X, const void *Wqkv, void *dX, float *dWqkv, void *ws,
                     size_t ws_bytes, void *stream) {
  RSA_PROJ_PROLOGUE(dQ && dK && dV && X && Wqkv && dX && dWqkv, dQ, dK, dV, X, Wqkv, dX, dWqkv, ws);
  const size_t need = proj_ws(dm, H);
  if (need > 0 && (!ws || ws_bytes < need)) return RSA_ERR_WORKSPACE;
  return hip_status(rsa::proj_qkv_bwd(dm, H, dQ, dK, dV, X, Wqkv, dX, dWqkv, static_cast<float *>(ws), st));
}

// ---------------------------------------------------------- Linformer ------
namespace {
// The attention of the ranks' rows to Kp projected keys: one chunk of Kp keys, no mask.
int linformer_dims(const rsa_desc *d, int32_t Kp, Dims *own, Dims *att) {
  int rc = validate(d, own);
  if (rc != RSA_OK) return rc;
  if (own->mode != RSA_MODE_FUSED || d->dtype != RSA_BF16 || own->zigzag || own->causal || own->strided)
    return RSA_ERR_UNSUPPORTED;
  if (Kp < 64) return RSA_ERR_SHAPE;
  if (Kp % 64 != 0) return RSA_ERR_UNSUPPORTED;
  // the GEMM kernel indexes rows and columns of its operands with 32 bits
  if (own->L >= (1LL << 31) || (int64_t)own->B * own->Z * own->A >= (1LL << 31)) return RSA_ERR_UNSUPPORTED;
  *att = *own;
  att->N = 1; att->rank_begin = 0; att->rank_end = 1;
  att->L = Kp; att->c = Kp;  // Lq stays: the ranks' rows
  att->ks[0] = (int64_t)own->Z * Kp * own->A; att->ks[1] = (int64_t)Kp * own->A; att->ks[2] = own->A;
  return RSA_OK;
}
size_t linformer_ws(const Dims &own, const Dims &att, int64_t Kp) {
  const int64_t Zt = (int64_t)own.B * own.Z;
  const size_t part = (size_t)rsa::linformer_splits(Kp, Zt, own.Lq, own.A) * Kp * Zt * own.A * 4;
  // backward: row terms, then the fp32 partial dV, dK of the split query walk
  const int qs = rsa::fused_bwd_dkdv_splits(att);
  size_t bwd = fused_bwd_base(att) + (qs > 1 ? (size_t)2 * qs * Zt * Kp * own.A * 4 : 0);
  if (rsa::shortkeys_supported(att)) bwd = rsa::shortkeys_bwd_ws_bytes(att);  // the one-kernel backward
  return align256(part > bwd ? part : bwd);
}
}  // namespace

size_t rsa_linformer_workspace_bytes(const rsa_desc *d, int32_t Kp) {
  Dims own, att;
  if (linformer_dims(d, Kp, &own, &att) != RSA_OK) return 0;
  return linformer_ws(own, att, Kp);
}

#define RSA_LINF_PROLOGUE(ptr_ok, ...)                            \
  Dims own, att;                                                  \
  int rc = linformer_dims(d, Kp, &own, &att);                     \
  if (rc != RSA_OK) return rc;                                    \
  if (!(ptr_ok)) return RSA_ERR_NULL;                             \
  { const void *ps_[] = {__VA_ARGS__};                            \
    for (const void *p_ : ps_) if (misaligned(p_)) return RSA_ERR_UNSUPPORTED; } \
  hipStream_t st = static_cast<hipStream_t>(stream);              \
  const int64_t row0 = (int64_t)own.rank_begin * own.c, Zt = (int64_t)own.B * own.Z; \
  (void)row0; (void)Zt

int rsa_linformer_project(const rsa_desc *d, int32_t Kp, const void *X, const void *E, void *Xp,
                          void *ws, size_t ws_bytes, void *stream) {
  RSA_LINF_PROLOGUE(X && E && Xp && ws, X, E, Xp, ws);
  if (ws_bytes < linformer_ws(own, att, Kp)) return RSA_ERR_WORKSPACE;
  const char *Xr = static_cast<const char *>(X) + row0 * own.A * 2;
  const char *Er = static_cast<const char *>(E) + row0 * Kp * 2;
  return hip_status(rsa::linformer_project(Zt, own.L, own.Lq, Kp, own.A, Xr, Er, Xp, static_cast<float *>(ws), st));
}

int rsa_linformer_forward(const rsa_desc *d, int32_t Kp, const void *Q, const void *Kp_, const void *Vp_,
                          void *O, float *LSE, void *stream) {
  RSA_LINF_PROLOGUE(Q && Kp_ && Vp_ && O && LSE, Q, Kp_, Vp_, O, LSE);
  if (rsa::shortkeys_supported(att)) return hip_status(rsa::shortkeys_forward(att, Q, Kp_, Vp_, O, LSE, st));
  return hip_status(rsa::fused_forward(att, Q, Kp_, Vp_, O, LSE, st, nullptr));
}

int rsa_linformer_backward(const rsa_desc *d, int32_t Kp, const void *dO, const void *Q, const void *Kp_,
                           const void *Vp_, const void *O, const float *LSE, void *dQ, void *dKp,
                           void *dVp, void *ws, size_t ws_bytes, void *stream) {
  RSA_LINF_PROLOGUE(dO && Q && Kp_ && Vp_ && O && LSE && dQ && dKp && dVp && ws, dO, Q, Kp_, Vp_, O, LSE,
                    dQ, dKp, dVp, ws);
  if (ws_bytes < linformer_ws(own, att, Kp)) return RSA_ERR_WORKSPACE;
  if (rsa::shortkeys_supported(att))
    return hip_status(rsa::shortkeys_backward(att, dO, Q, Kp_, Vp_, O, LSE, dQ, dKp, dVp,
                                              static_cast<float *>(ws), st));
  const int qs = rsa::fused_bwd_dkdv_splits(att);
  float *part = qs > 1 ? fused_part(att, ws) : nullptr;
  return hip_status(rsa::fused_backward(att, dO, Q, Kp_, Vp_, O, LSE, dQ, dKp, dVp, fused_nD(ws),
                                        fused_nL(att, ws), st, part, qs, 1));
}

int rsa_linformer_project_bwd(const rsa_desc *d, int32_t Kp, const void *dXp, const void *X, const void *E,
                              void *dX, float *dE, void *stream) {
  RSA_LINF_PROLOGUE(dXp && X && E && dX && dE, dXp, X, E, dX, dE);
  const char *Xr = static_cast<const char *>(X) + row0 * own.A * 2;
  const char *Er = static_cast<const char *>(E) + row0 * Kp * 2;
  char *dXr = static_cast<char *>(dX) + row0 * own.A * 2;
  float *dEr = dE + row0 * Kp;
  return hip_status(rsa::linformer_project_bwd(Zt, own.L, own.Lq, Kp, own.A, dXp, Xr, Er, dXr, dEr, st));
}

}  // extern "C"
