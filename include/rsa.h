/*
 * rsa.h -- C ABI of the Ring Self-Attention (RSA) library for AMD MI355X (gfx950).
 *
 * RSA (paper section 3.1) splits a sequence of L tokens into N chunks of
 * c = L/N rows; device ("rank") n holds Q^n, K^n, V^n and obtains
 * Attention^n(Q^n, K, V) = softmax(Q^n K^T / sqrt(d_k)) V (Eq. 1) by letting
 * the K chunks, then the V chunks, travel round the ring (Eq. 3).  This
 * library runs the ranks of the ring on ONE GPU: the chunks of K and V are
 * resident in device memory and "ring step t of rank n" is the visit of chunk
 * j = (n - t) mod N, local chunk first.  There is no inter-GPU traffic.
 *
 * Conventions for every entry point
 *  - All tensor pointers are DEVICE pointers, row-major with the last index
 *    contiguous, 16-byte aligned; dense unless the descriptor's stride fields
 *    say otherwise (fused mode).  The caller owns every buffer; the library
 *    never allocates, frees or keeps a pointer.
 *  - K, V, dK, dV are (B, Z, L, A).  Q, O, dO, dQ are (B, Z, Lq, A) with
 *    Lq = (rank_end - rank_begin) * c: the rows of ranks [rank_begin,
 *    rank_end) only.  LSE and D are (B, Z, Lq) fp32.
 *  - With a sub-range of ranks, dK and dV are that range's partial sums (what
 *    the ring's all-reduce of section 3.2.2 would add up).  dQ, dK, dV are
 *    overwritten, not accumulated into.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Work is enqueued asynchronously; no call synchronises, allocates or
 *    records a memset, so a sequence of calls can be captured in a HIP graph.
 *  - Every call returns an rsa_status.  Arguments are validated on the host
 *    before anything is launched; on error nothing has been enqueued.
 *  - dtype RSA_BF16: bf16 storage, fp32 accumulation and fp32 softmax, one
 *    round-to-nearest-even per stored element.  dtype RSA_F32: fp32
 *    throughout (staged mode only).
 *  - Supported: A = 64 or 128 in fused mode, any multiple of 64 up to 256 in
 *    staged mode; L divisible by N (section 4.2: the sequence length must be
 *    divisible by the sequence-parallel size); c divisible by 64.
 */
#ifndef RSA_H
#define RSA_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  RSA_OK = 0,
  RSA_ERR_NULL = -1,        /* a required pointer is NULL                    */
  RSA_ERR_SHAPE = -2,       /* non-positive size, L % N != 0, bad rank range */
  RSA_ERR_UNSUPPORTED = -3, /* A, dtype, chunk granularity, alignment, mode  */
  RSA_ERR_WORKSPACE = -4,   /* workspace NULL or smaller than required       */
  RSA_ERR_HIP = -5          /* a HIP launch reported an error                */
} rsa_status;

typedef enum { RSA_F32 = 0, RSA_BF16 = 1 } rsa_dtype;

/* flags: one mode, optionally or-ed with the bits below */
#define RSA_MODE_FUSED 0u  /* online-softmax kernels, no score strip in HBM   */
#define RSA_MODE_STAGED 1u /* the paper's two-pass layout: strip S^n in HBM   */
/* Zig-zag chunk ownership (fused mode only; an extension for the causal mask, which
 * the paper leaves open in section 3.1): the sequence is cut into 2N half-chunks of
 * h = c/2 rows and rank n owns half-chunks n and 2N-1-n, so that every rank sees the
 * same number of keys under the causal mask.  The c local rows of rank n in
 * Q, O, dO, dQ, LSE are then tokens [n h, (n+1) h) followed by tokens
 * [(2N-1-n) h, (2N-n) h); K, V, dK, dV stay in token order.  Ring step t of rank n
 * visits the two half-chunks of rank (n - t) mod N.  Needs h divisible by 64. */
#define RSA_OWN_ZIGZAG 2u
/* Request results that are bit-identical from run to run.  Every kernel of this library
 * already sums in a fixed order (the sums over ranks that the ring would all-reduce are
 * loops of one work-group; split walks are merged by a kernel in split order), so the
 * bit changes nothing today; it is accepted so that callers can state the requirement.
 * A backward that forms dQ inside the dK/dV sweep (S and dP computed once instead of
 * twice) would have to add every key block's share of dQ to an fp32 accumulator with
 * atomic adds; on this GPU those run at 0.34 T adds/s (1.4 TB/s), which for the
 * BERT-Large-shaped workload is 0.4 to 0.8 ms against the 0.2 ms of the dQ kernel it
 * would replace, so no such path is offered. */
#define RSA_DETERMINISTIC 4u

typedef struct {
  int32_t B, Z, A;   /* batch, heads, head size                              */
  int64_t L;         /* total sequence length                                */
  int32_t N;         /* ring size; c = L / N                                 */
  int32_t rank_begin, rank_end; /* simulated ranks [begin, end), 0-based     */
  int32_t causal;    /* 0: bidirectional (the paper); 1: key j visible to    */
                     /* query i iff j <= i in global token index (extension) */
  int32_t dtype;     /* rsa_dtype of Q, K, V, O, dO, dQ, dK, dV              */
  float scale;       /* 1/sqrt(d_k) of Eq. 1; 0 selects 1/sqrt(A)            */
  uint32_t flags;    /* RSA_MODE_* [| RSA_OWN_ZIGZAG] [| RSA_DETERMINISTIC]  */
  /* Strides in elements of the batch, head and row index (the last index is always
   * contiguous): q_stride for Q and dQ, kv_stride for K, V, dK, dV, o_stride for O
   * and dO.  All three zero = dense (B, Z, rows, A), i.e. {Z rows A, rows A, A}.
   * Non-dense layouts (e.g. heads interleaved as (B, rows, Z, A), or Q, K, V as
   * slices of one packed projection output) are taken by rsa_forward, rsa_backward
   * and the rsa_bwd_* calls in fused mode; row strides must be multiples of 8
   * elements (16 bytes) and at most 2^24.  LSE, D and the workspace are always dense. */
  int64_t q_stride[3], kv_stride[3], o_stride[3];
} rsa_desc;

int rsa_version(void);
const char *rsa_strerror(int status);

/* Bytes of device workspace rsa_forward (pass 0) or rsa_backward (pass 1)
 * needs for this descriptor; 0 if the descriptor is invalid. */
size_t rsa_workspace_bytes(const rsa_desc *d, int pass);

/*
 * RSA forward (section 3.1, Eq. 1 and Eq. 3): for every simulated rank n in
 * [rank_begin, rank_end) and ring step t, visit chunk j = (n - t) mod N:
 * scores of Q^n against K^j, full-row softmax over all L keys, O^n = sum_j
 * P^n_j V^j.  Writes O (dtype) and LSE_i = log sum_j exp(S_ij) (fp32).
 * ws: workspace of at least rsa_workspace_bytes(d, 0) bytes (may be NULL if
 * that is 0).  Staged mode keeps the score strip there; fused mode needs it
 * only when the descriptor has so few query rows for its keys (one rank's
 * share of a long sequence) that the pass over the keys is divided among
 * several work-groups per row tile, whose fp32 partial results it holds.
 */
int rsa_forward(const rsa_desc *d, const void *Q, const void *K, const void *V,
                void *O, float *LSE, void *ws, size_t ws_bytes, void *stream);

/*
 * RSA backward: the derivative of Eq. 1 with the ring structure of section
 * 3.2.2 (a V pass for dP, a K pass for dQ, sums over ranks for dK and dV):
 *   dV^j = sum_n (P^n_j)^T dO^n,  dP^n_j = dO^n (V^j)^T,
 *   D_i = sum_a dO_ia O_ia,       dS = P o (dP - D),
 *   dQ^n = s sum_j dS^n_j K^j,    dK^j = s sum_n (dS^n_j)^T Q^n.
 * O and LSE are the forward's outputs.
 */
int rsa_backward(const rsa_desc *d, const void *dO, const void *Q,
                 const void *K, const void *V, const void *O, const float *LSE,
                 void *dQ, void *dK, void *dV, void *ws, size_t ws_bytes,
                 void *stream);

/*
 * Step-level entry points: one ring step of one simulated rank, the paper's
 * two-pass layout (Table 2, rows Ring-QK^T and Ring-AV).  n is the rank (in
 * [rank_begin, rank_end)), j the chunk visited.  A "strip" is rank n's
 * (B, Z, c, L) matrix; column block j is columns [j*c, (j+1)*c).  Strips S and
 * dP are fp32; strips P and dS are in d->dtype.  Accumulators Oacc, dQacc
 * (B, Z, c, A) and dKacc, dVacc (B, Z, L, A) are fp32; `accumulate` = 0
 * overwrites the addressed block, 1 adds to it.
 */

/* Stage 1 (section 3.1): S^n_j = s Q^n (K^j)^T, masked entries -inf. */
int rsa_qk_step(const rsa_desc *d, int n, int j, const void *Q, const void *K,
                float *S, void *stream);
/* Eq. 1's softmax over the full row of L keys: P = softmax(S), LSE. */
int rsa_row_softmax(const rsa_desc *d, int n, const float *S, void *P,
                    float *LSE, void *stream);
/* Stage 2 (Eq. 3): Oacc (+)= P^n_j V^j. */
int rsa_av_step(const rsa_desc *d, int n, int j, const void *P, const void *V,
                float *Oacc, int accumulate, void *stream);
/* D_i = sum_a dO_ia O_ia for the rows of rank n; n = -1: every rank in
 * [rank_begin, rank_end). */
int rsa_bwd_rowdot(const rsa_desc *d, int n, const void *dO, const void *O,
                   float *D, void *stream);
/* dVacc^j (+)= (P^n_j)^T dO^n. */
int rsa_dv_step(const rsa_desc *d, int n, int j, const void *P, const void *dO,
                float *dVacc, int accumulate, void *stream);
/* dP^n_j = dO^n (V^j)^T. */
int rsa_dp_step(const rsa_desc *d, int n, int j, const void *dO, const void *V,
                float *dP, void *stream);
/* dS = P o (dP - D) over the whole strip of rank n. */
int rsa_softmax_bwd(const rsa_desc *d, int n, const void *P, const float *dP,
                    const float *D, void *dS, void *stream);
/* dQacc^n (+)= s dS^n_j K^j. */
int rsa_dq_step(const rsa_desc *d, int n, int j, const void *dS, const void *K,
                float *dQacc, int accumulate, void *stream);
/* dKacc^j (+)= s (dS^n_j)^T Q^n. */
int rsa_dk_step(const rsa_desc *d, int n, int j, const void *dS, const void *Q,
                float *dKacc, int accumulate, void *stream);
/* dst (d->dtype) = src (fp32), `count` elements: stores an accumulator. */
int rsa_store(const rsa_desc *d, const float *src, void *dst, size_t count,
              void *stream);

/*
 * The kernels of the deterministic fused backward on their own (bf16, fused mode),
 * for profiling and tests, on one workspace `ws` of at least
 * rsa_workspace_bytes(d, 1) bytes (checked on the host: RSA_ERR_WORKSPACE).  With
 * RSA_DETERMINISTIC rsa_backward runs the dQ kernel first, with the preprocess folded
 * into its prologue, then the dK/dV kernel; the three calls below in the order
 * given produce the same gradients up to the fp32 summation order of D.
 *  rsa_bwd_preprocess: fills ws with the row terms -D_i = -sum_a dO_ia O_ia and
 *    -LSE_i / s (fp32).  Both other kernels recompute
 *    P = exp2(s log2(e) (Q K^T - LSE / s)) tile by tile from the caller's Q and K
 *    (the factor is applied in fp32; no operand is rounded a second time) and
 *    read the row terms.
 *  rsa_bwd_dkdv: for every key chunk, the walk over the query rows of all
 *    simulated ranks -- dV = sum_n P^T dO, dK = s sum_n dS^T Q (the sums the
 *    ring all-reduces, section 3.2.2).  Also forms dP = dO V^T for its tiles.
 *  rsa_bwd_dq: for every rank, the K ring pass dQ^n = s sum_j dS^n_j K^j.  When the
 *    descriptor has few query rows and many keys (one rank's share of a long
 *    sequence) the pass over the keys is divided over several work-groups per
 *    row tile, as in rsa_forward and rsa_backward; their fp32 partial sums use
 *    the part of ws behind the row terms, which is why ws is writable.
 */
int rsa_bwd_preprocess(const rsa_desc *d, const void *dO, const void *O,
                       const float *LSE, void *ws, size_t ws_bytes,
                       void *stream);
int rsa_bwd_dkdv(const rsa_desc *d, const void *dO, const void *Q, const void *K,
                 const void *V, const void *ws, size_t ws_bytes, void *dK, void *dV,
                 void *stream);
int rsa_bwd_dq(const rsa_desc *d, const void *dO, const void *Q, const void *K,
               const void *V, void *ws, size_t ws_bytes, void *dQ, void *stream);

/*
 * rsa_backward for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels,
 * with the workspace in a static device array of RSA_STATIC_SCRATCH_BYTES inside the
 * library instead of a caller's buffer.  The call allocates and frees nothing.
 * Descriptors whose rsa_workspace_bytes(d, 1) exceeds that size are rejected with
 * RSA_ERR_WORKSPACE before anything is launched (RSA_DETERMINISTIC needs the least:
 * 8 bytes per query row unless the key walk is split).  Every call on a GPU uses
 * that GPU's one array: calls that overlap on one GPU (two streams, two threads) race,
 * and the array keeps the previous call's contents (the kernels clear what they
 * need cleared).  The first call on a device looks the array's address up
 * (hipGetSymbolAddress); make that call outside a stream capture.
 */
#define RSA_STATIC_SCRATCH_BYTES (32u << 20)
int rsa_backward_static(const rsa_desc *d, const void *dO, const void *Q, const void *K,
                        const void *V, const void *O, const float *LSE, void *dQ,
                        void *dK, void *dV, void *stream);

/*
 * The two linear maps around RSA on the simulated ranks' rows (Table 2, sequence
 * parallelism rows "Q/K/V" and "Linear"), bf16 with fp32 accumulation, fused mode
 * descriptors only.  H is the hidden size (a multiple of 64).  X, Y and their
 * gradients are (B, Lq, H); Q, K, V, O and their gradients are (B, Z, Lq, A), the
 * layout RSA reads and writes, so nothing is transposed in memory.  Wqkv is (H, 3 Z A)
 * row-major with columns [Q | K | V], each block head-major; Wo is (Z A, H).  The
 * paper prints no bias.  Weight gradients are fp32 and cover the rows of this call
 * (the sum over ranks is the all-reduce of the replicated weights); they are
 * overwritten.  ws: at least rsa_proj_workspace_bytes(d, H) bytes (partial sums of
 * the weight gradients over row blocks, added in a fixed order).
 */
size_t rsa_proj_workspace_bytes(const rsa_desc *d, int32_t H);
/* Q, K, V = heads of X Wqkv. */
int rsa_qkv_proj(const rsa_desc *d, int32_t H, const void *X, const void *Wqkv,
                 void *Q, void *K, void *V, void *stream);
/* Y = merge_heads(O) Wo. */
int rsa_out_proj(const rsa_desc *d, int32_t H, const void *O, const void *Wo,
                 void *Y, void *stream);
/* dO = heads of dY Wo^T; dWo = merge_heads(O)^T dY. */
int rsa_out_proj_bwd(const rsa_desc *d, int32_t H, const void *dY, const void *O,
                     const void *Wo, void *dO, float *dWo, void *ws,
                     size_t ws_bytes, void *stream);
/* dX = [dQ | dK | dV] Wqkv^T; dWqkv = X^T [dQ | dK | dV]. */
int rsa_qkv_proj_bwd(const rsa_desc *d, int32_t H, const void *dQ, const void *dK,
                     const void *dV, const void *X, const void *Wqkv, void *dX,
                     float *dWqkv, void *ws, size_t ws_bytes, void *stream);

/*
 * The Linformer variant of sequence-parallel attention (Table 3): keys and values are
 * projected along the sequence to Kp rows, every rank with its row block of the (L, Kp)
 * projection matrix, and the ranks' queries attend to the Kp projected rows (softmax of
 * Eq. 1 over them; no mask, so d->causal must be 0; fused mode, contiguous ownership).
 * Kp must be a multiple of 64.  bf16 with fp32 accumulation; dE is fp32.
 *  rsa_linformer_project: Xp (B, Z, Kp, A) = sum over the tokens l of ranks
 *    [rank_begin, rank_end) of E[l, :] X[b, z, l, :] -- the partial sum the ranks add up
 *    (all of it for the whole ring).  X is (B, Z, L, A), E is (L, Kp).  Called for K with E
 *    and for V with F.  ws: rsa_linformer_workspace_bytes(d, Kp) bytes.
 *  rsa_linformer_forward / _backward: Q, O, dO, dQ (B, Z, Lq, A); Kp_, Vp_, dKp, dVp
 *    (B, Z, Kp, A); dKp, dVp are the partial sums over the ranks' query rows.  The
 *    backward's ws is the same workspace.
 *  rsa_linformer_project_bwd: dX rows of the ranks' tokens = E dXp (other rows are left
 *    untouched), dE rows of the ranks' tokens = sum_{b,z} X dXp^T (other rows untouched).
 */
size_t rsa_linformer_workspace_bytes(const rsa_desc *d, int32_t Kp);
int rsa_linformer_project(const rsa_desc *d, int32_t Kp, const void *X, const void *E,
                          void *Xp, void *ws, size_t ws_bytes, void *stream);
int rsa_linformer_forward(const rsa_desc *d, int32_t Kp, const void *Q, const void *Kp_,
                          const void *Vp_, void *O, float *LSE, void *stream);
int rsa_linformer_backward(const rsa_desc *d, int32_t Kp, const void *dO, const void *Q,
                           const void *Kp_, const void *Vp_, const void *O,
                           const float *LSE, void *dQ, void *dKp, void *dVp, void *ws,
                           size_t ws_bytes, void *stream);
int rsa_linformer_project_bwd(const rsa_desc *d, int32_t Kp, const void *dXp, const void *X,
                              const void *E, void *dX, float *dE, void *stream);

#ifdef __cplusplus
}
#endif
#endif
