// Internal launch functions of the RSA library (host side).  Each returns the
// hipError_t of its launch.  Arguments are assumed validated by the C ABI layer.
#pragma once
#include "rsa_common.h"

namespace rsa {

// --- staged (two-pass) steps: section 3.1 stage 1, Eq. 1's softmax, Eq. 3 ---
hipError_t staged_qk_step(const Dims &d, int dtype, int n, int j, const void *Q, const void *K,
                          float *S, hipStream_t st);
hipError_t staged_row_softmax(const Dims &d, int dtype, int n, const float *S, void *P, float *LSE,
                              hipStream_t st);
hipError_t staged_av_step(const Dims &d, int dtype, int n, int j, const void *P, const void *V,
                          float *Oacc, int accumulate, hipStream_t st);
hipError_t staged_dv_step(const Dims &d, int dtype, int n, int j, const void *P, const void *dO,
                          float *dVacc, int accumulate, hipStream_t st);
hipError_t staged_dp_step(const Dims &d, int dtype, int n, int j, const void *dO, const void *V,
                          float *dP, hipStream_t st);
hipError_t staged_softmax_bwd(const Dims &d, int dtype, int n, const void *P, const float *dP,
                              const float *D, void *dS, hipStream_t st);
hipError_t staged_dq_step(const Dims &d, int dtype, int n, int j, const void *dS, const void *K,
                          float *dQacc, int accumulate, hipStream_t st);
hipError_t staged_dk_step(const Dims &d, int dtype, int n, int j, const void *dS, const void *Q,
                          float *dKacc, int accumulate, hipStream_t st);
// D rows [row_off, row_off + rows_per_head) of every head: D_i = sum_a dO_ia O_ia
hipError_t rowdot(const Dims &d, int dtype, int64_t row_off, int64_t rows_per_head, const void *dO,
                  const void *O, float *D, hipStream_t st);
// dst[b][r][:] (dtype) = src[b][r][:] (fp32); rows of `cols` elements, batch strides in elements
hipError_t store_rows(int dtype, const float *src, void *dst, int64_t batches,
                      int64_t rows_per_batch, int64_t cols, int64_t src_batch, int64_t dst_batch,
                      hipStream_t st);

// p[0..n) = 0 (n a multiple of 4), by a kernel
hipError_t zero_f32(float *p, int64_t n, hipStream_t st);

// --- fused (online-softmax) path, bf16, A = 64 or 128 ---
// Split of the walk over the keys (few query rows, many keys).  fused_fwd_plan: the forward's
// rows per work-group (big: 256, else 128) and its split count; part: its fp32 partial results,
// splits * B*Z*Lq * (A + 2) floats, or nullptr for no split.  fused_key_splits: the dQ kernel's count.
void fused_fwd_plan(const Dims &d, bool *big, int *splits);
int fused_key_splits(const Dims &d);
hipError_t fused_forward(const Dims &d, const void *Q, const void *K, const void *V, void *O,
                         float *LSE, hipStream_t st, float *part);
// nD = -rowsum(dO o O) and nL = -LSE / scale, (B,Z,Lq) fp32
hipError_t fused_bwd_preprocess(const Dims &d, const void *dO, const void *O, const float *LSE,
                                float *nD, float *nL, hipStream_t st);
// part / splits: optional split of the walk over the query rows (few keys, many rows): fp32
// partial dV and dK, 2 * splits * B*Z*L*A floats, added up in a fixed order; nullptr / 1: none
int fused_bwd_dkdv_splits(const Dims &d);
hipError_t fused_bwd_dkdv(const Dims &d, const void *dO, const void *Q, const void *K,
                          const void *V, const float *nL, const float *nD, void *dK, void *dV,
                          hipStream_t st, float *part = nullptr, int splits = 1);
// part / splits: the split key walk again, fp32 partial dQ, splits * B*Z*Lq * A floats
hipError_t fused_bwd_dq(const Dims &d, const void *dO, const void *Q, const void *K, const void *V,
                        const float *nL, const float *nD, void *dQ, hipStream_t st,
                        float *part = nullptr, int splits = 1);
hipError_t fused_backward(const Dims &d, const void *dO, const void *Q, const void *K,
                          const void *V, const void *O, const float *LSE, void *dQ, void *dK,
                          void *dV, float *nD, float *nL, hipStream_t st,
                          float *part = nullptr, int qsplits = 1, int ksplits = 1);

// out (bf16, layout lay) = the sum over `splits` fp32 partial results of n4 * 4 floats each, in a
// fixed order
hipError_t qsplit_reduce(const float *part, void *out, int64_t n4, int splits, int A, const OutLayout &lay,
                         hipStream_t st);

// --- attention to Kp = 128 or 256 keys that one work-group holds (Table 3's shape), bf16, A = 64 ---
// att: the dimensions with L = Kp keys, one chunk, Lq query rows.  The backward is one kernel (S, dP,
// dV, dK and dQ); part: fp32 partial dV, dK of the work-groups that share a head,
// shortkeys_bwd_ws_bytes(att) bytes (0: none needed).
bool shortkeys_supported(const Dims &att);
hipError_t shortkeys_forward(const Dims &att, const void *Q, const void *K, const void *V, void *O, float *LSE,
                             hipStream_t st);
size_t shortkeys_bwd_ws_bytes(const Dims &att);
hipError_t shortkeys_backward(const Dims &att, const void *dO, const void *Q, const void *K, const void *V,
                              const void *O, const float *LSE, void *dQ, void *dK, void *dV, float *part,
                              hipStream_t st);

// dX (Zt, L, A) rows [0, rows) from the pointer passed = E (rows, Kp) dXp (Zt, Kp, A), Kp <= 256
bool linformer_dx_supported(int64_t Kp, int A);
hipError_t linformer_dx(int64_t Zt, int64_t L, int64_t rows, int64_t Kp, int A, const void *dXp, const void *E,
                        void *dX, hipStream_t st);

// --- the linear maps around RSA (Table 2, rows Q/K/V and Linear), bf16, A = 64 or 128 ---
// X, dX, Y, dY: (B, Lq, H); W: (H, 3*Z*A), columns [Q | K | V] head-major; Wo: (Z*A, H);
// Q, K, V, O and their gradients: (B, Z, Lq, A); dW, dWo: fp32; part: k-split partial sums.
int proj_wgrad_splits(int64_t Mout, int64_t Nout, int64_t K);
hipError_t proj_qkv(const Dims &d, int64_t H, const void *X, const void *W, void *Q, void *K, void *V,
                    hipStream_t st);
hipError_t proj_out(const Dims &d, int64_t H, const void *O, const void *Wo, void *Y, hipStream_t st);
hipError_t proj_out_bwd(const Dims &d, int64_t H, const void *dY, const void *O, const void *Wo,
                        void *dO, float *dWo, float *part, hipStream_t st);
hipError_t proj_qkv_bwd(const Dims &d, int64_t H, const void *dQ, const void *dK, const void *dV,
                        const void *X, const void *W, void *dX, float *dW, float *part,
                        hipStream_t st);

// --- Linformer projections along the sequence (Table 3, row Projection), bf16, A = 64 or 128 ---
// Zt = B*Z heads; X, dX: (Zt, L, A), used from a first token on for `rows` tokens (the pointers
// passed are those of that first token); E: (rows, Kp); Xp, dXp: (Zt, Kp, A); dE fp32 (rows, Kp).
int linformer_splits(int64_t Kp, int64_t Zt, int64_t rows, int A);
hipError_t linformer_project(int64_t Zt, int64_t L, int64_t rows, int64_t Kp, int A, const void *X,
                             const void *E, void *Xp, float *part, hipStream_t st);
hipError_t linformer_project_bwd(int64_t Zt, int64_t L, int64_t rows, int64_t Kp, int A, const void *dXp,
                                 const void *X, const void *E, void *dX, float *dE, hipStream_t st);

}  // namespace rsa
