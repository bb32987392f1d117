// Staged (two-pass) Ring Self-Attention kernels: the paper's layout, in which
// rank n's score strip S^n (B, Z, c, L) lives in device memory between the
// K ring pass and the V ring pass (section 3.1; Table 2, rows Ring-QK^T and
// Ring-AV).  One ring step is one batched c x c x A (or c x A x c) GEMM per
// head; the softmax in between is a pure memory-bound row pass.
#include "rsa_kernels.h"

namespace rsa {

// ----------------------------------------------------------- GEMM step ------
// C[m][n] (+)= alpha * sum_k A(m,k) B(n,k), one 64 x 64 tile per work-group,
// one head per blockIdx.z.  An operand is "k-contiguous" when its k index is
// the fast one in memory (element (m,k) at base + m*ld + k) and
// "k-strided" otherwise (element (m,k) at base + k*ld + m); k-strided tiles
// are transposed on their way into LDS so that both tiles sit in LDS as
// [row][k] and every MFMA operand is one 16-byte LDS read.
constexpr int kTile = 64;

struct GemmArgs {
  const void *A, *B;
  float *C;
  int64_t a_batch, b_batch, c_batch;  // elements between heads
  int64_t lda, ldb, ldc;
  int K;                              // multiple of 64
  float alpha;
  int accumulate;
  int mask_mode;                      // 0 none, 1 causal per element, 2 whole block -inf
  int64_t mask_q0, mask_k0;           // global token index of C row 0 / column 0
};

template <bool KC>
__device__ __forceinline__ void load_tile_bf16(uint16_t *lds, const uint16_t *g, int64_t ld,
                                               int64_t r0, int64_t k0, int tid) {
  constexpr int P = 72;  // LDS row pitch in elements: 144 B keeps 16-byte row reads conflict-free
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int id = tid + it * 256;
    const int hi = id >> 3, lo = id & 7;
    if (KC) {
      const u32x4 v = *reinterpret_cast<const u32x4 *>(g + (r0 + hi) * ld + k0 + lo * 8);
      *reinterpret_cast<u32x4 *>(lds + hi * P + lo * 8) = v;
    } else {
      const u32x4 v = *reinterpret_cast<const u32x4 *>(g + (k0 + hi) * ld + r0 + lo * 8);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        lds[(lo * 8 + 2 * e) * P + hi] = (uint16_t)(v[e] & 0xffffu);
        lds[(lo * 8 + 2 * e + 1) * P + hi] = (uint16_t)(v[e] >> 16);
      }
    }
  }
}

__device__ __forceinline__ float masked(float x, int mode, int64_t q, int64_t k) {
  return (mode == 1 && k > q) ? -INFINITY : x;
}

template <bool A_KC, bool B_KC>
__global__ void __launch_bounds__(256) gemm_step_bf16(GemmArgs g) {
  constexpr int P = 72;
  __shared__ __attribute__((aligned(16))) uint16_t As[kTile * P];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[kTile * P];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t m0 = (int64_t)blockIdx.y * kTile, n0 = (int64_t)blockIdx.x * kTile;
  const int64_t head = blockIdx.z;
  float *C = g.C + head * g.c_batch;
  const int wm = (wave >> 1) * 32, wn = (wave & 1) * 32;
  const int col = lane & 31, half = lane >> 5;
  f32x16 acc = {0};
  if (g.mask_mode != 2) {
    const uint16_t *A = reinterpret_cast<const uint16_t *>(g.A) + head * g.a_batch;
    const uint16_t *B = reinterpret_cast<const uint16_t *>(g.B) + head * g.b_batch;
    for (int k0 = 0; k0 < g.K; k0 += kTile) {
      __syncthreads();
      load_tile_bf16<A_KC>(As, A, g.lda, m0, k0, tid);
      load_tile_bf16<B_KC>(Bs, B, g.ldb, n0, k0, tid);
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(As + (wm + col) * P + kk * 16 + half * 8);
        const bf16x8 b = *reinterpret_cast<const bf16x8 *>(Bs + (wn + col) * P + kk * 16 + half * 8);
        acc = mfma_32x32x16(a, b, acc);
      }
    }
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int64_t i = m0 + wm + (v >> 2) * 8 + half * 4 + (v & 3);
    const int64_t j = n0 + wn + col;
    float *p = C + i * g.ldc + j;
    float x = g.alpha * acc[v];
    if (g.mask_mode == 2) x = -INFINITY;
    x = masked(x, g.mask_mode, g.mask_q0 + i, g.mask_k0 + j);
    if (g.accumulate) x += *p;
    *p = x;
  }
}

// fp32 variant on the vector ALU: 4 x 4 outputs per thread, 32-deep k tiles.
template <bool KC>
__device__ __forceinline__ void load_tile_f32(float *lds, const float *g, int64_t ld, int64_t r0,
                                              int64_t k0, int tid) {
  constexpr int P = 33;
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int id = tid + it * 256;
    if (KC) {
      const int hi = id >> 3, lo = id & 7;  // row, 4-float chunk along k
      const f32x4 v = *reinterpret_cast<const f32x4 *>(g + (r0 + hi) * ld + k0 + lo * 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) lds[hi * P + lo * 4 + e] = v[e];
    } else {
      const int hi = id >> 4, lo = id & 15;  // k, 4-float chunk along rows
      const f32x4 v = *reinterpret_cast<const f32x4 *>(g + (k0 + hi) * ld + r0 + lo * 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) lds[(lo * 4 + e) * P + hi] = v[e];
    }
  }
}

template <bool A_KC, bool B_KC>
__global__ void __launch_bounds__(256) gemm_step_f32(GemmArgs g) {
  constexpr int P = 33, BK = 32;
  __shared__ float As[kTile * P];
  __shared__ float Bs[kTile * P];
  const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
  const int64_t m0 = (int64_t)blockIdx.y * kTile, n0 = (int64_t)blockIdx.x * kTile;
  const int64_t head = blockIdx.z;
  float *C = g.C + head * g.c_batch;
  float acc[4][4] = {};
  if (g.mask_mode != 2) {
    const float *A = reinterpret_cast<const float *>(g.A) + head * g.a_batch;
    const float *B = reinterpret_cast<const float *>(g.B) + head * g.b_batch;
    for (int k0 = 0; k0 < g.K; k0 += BK) {
      __syncthreads();
      load_tile_f32<A_KC>(As, A, g.lda, m0, k0, tid);
      load_tile_f32<B_KC>(Bs, B, g.ldb, n0, k0, tid);
      __syncthreads();
#pragma unroll 8
      for (int k = 0; k < BK; ++k) {
        float a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = As[(ty * 4 + i) * P + k];
#pragma unroll
        for (int j = 0; j < 4; ++j) b[j] = Bs[(tx * 4 + j) * P + k];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t r = m0 + ty * 4 + i;
    float *p = C + r * g.ldc + n0 + tx * 4;
    f32x4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float x = g.alpha * acc[i][j];
      if (g.mask_mode == 2) x = -INFINITY;
      x = masked(x, g.mask_mode, g.mask_q0 + r, g.mask_k0 + n0 + tx * 4 + j);
      o[j] = x;
    }
    if (g.accumulate) o += *reinterpret_cast<const f32x4 *>(p);
    *reinterpret_cast<f32x4 *>(p) = o;
  }
}

template <bool A_KC, bool B_KC>
static hipError_t launch_gemm(const GemmArgs &g, int M, int N, int heads, int dtype,
                              hipStream_t st) {
  dim3 grid(N / kTile, M / kTile, heads);
  if (dtype == RSA_BF16)
    hipLaunchKernelGGL((gemm_step_bf16<A_KC, B_KC>), grid, dim3(256), 0, st, g);
  else
    hipLaunchKernelGGL((gemm_step_f32<A_KC, B_KC>), grid, dim3(256), 0, st, g);
  return hipGetLastError();
}

static inline int64_t esz(int dtype) { return dtype == RSA_BF16 ? 2 : 4; }
static inline const void *offs(const void *p, int64_t elems, int dtype) {
  return static_cast<const char *>(p) + elems * esz(dtype);
}

hipError_t staged_qk_step(const Dims &d, int dtype, int n, int j, const void *Q, const void *K,
                          float *S, hipStream_t st) {
  GemmArgs g{};
  g.A = offs(Q, (int64_t)(n - d.rank_begin) * d.c * d.A, dtype);
  g.B = offs(K, (int64_t)j * d.c * d.A, dtype);
  g.C = S + (int64_t)j * d.c;
  g.a_batch = d.Lq * d.A; g.b_batch = d.L * d.A; g.c_batch = d.c * d.L;
  g.lda = d.A; g.ldb = d.A; g.ldc = d.L;
  g.K = d.A; g.alpha = d.scale; g.accumulate = 0;
  g.mask_mode = !d.causal ? 0 : (j > n ? 2 : (j == n ? 1 : 0));
  g.mask_q0 = (int64_t)n * d.c; g.mask_k0 = (int64_t)j * d.c;
  return launch_gemm<true, true>(g, (int)d.c, (int)d.c, d.B * d.Z, dtype, st);
}

hipError_t staged_av_step(const Dims &d, int dtype, int n, int j, const void *P, const void *V,
                          float *Oacc, int accumulate, hipStream_t st) {
  (void)n;
  GemmArgs g{};
  g.A = offs(P, (int64_t)j * d.c, dtype);
  g.B = offs(V, (int64_t)j * d.c * d.A, dtype);
  g.C = Oacc;
  g.a_batch = d.c * d.L; g.b_batch = d.L * d.A; g.c_batch = d.c * d.A;
  g.lda = d.L; g.ldb = d.A; g.ldc = d.A;
  g.K = (int)d.c; g.alpha = 1.0f; g.accumulate = accumulate;
  return launch_gemm<true, false>(g, (int)d.c, d.A, d.B * d.Z, dtype, st);
}

hipError_t staged_dv_step(const Dims &d, int dtype, int n, int j, const void *P, const void *dO,
                          float *dVacc, int accumulate, hipStream_t st) {
  GemmArgs g{};
  g.A = offs(P, (int64_t)j * d.c, dtype);  // A(m = key, k = query) = P[query][key]
  g.B = offs(dO, (int64_t)(n - d.rank_begin) * d.c * d.A, dtype);
  g.C = dVacc + (int64_t)j * d.c * d.A;
  g.a_batch = d.c * d.L; g.b_batch = d.Lq * d.A; g.c_batch = d.L * d.A;
  g.lda = d.L; g.ldb = d.A; g.ldc = d.A;
  g.K = (int)d.c; g.alpha = 1.0f; g.accumulate = accumulate;
  return launch_gemm<false, false>(g, (int)d.c, d.A, d.B * d.Z, dtype, st);
}

hipError_t staged_dp_step(const Dims &d, int dtype, int n, int j, const void *dO, const void *V,
                          float *dP, hipStream_t st) {
  GemmArgs g{};
  g.A = offs(dO, (int64_t)(n - d.rank_begin) * d.c * d.A, dtype);
  g.B = offs(V, (int64_t)j * d.c * d.A, dtype);
  g.C = dP + (int64_t)j * d.c;
  g.a_batch = d.Lq * d.A; g.b_batch = d.L * d.A; g.c_batch = d.c * d.L;
  g.lda = d.A; g.ldb = d.A; g.ldc = d.L;
  g.K = d.A; g.alpha = 1.0f; g.accumulate = 0;
  return launch_gemm<true, true>(g, (int)d.c, (int)d.c, d.B * d.Z, dtype, st);
}

hipError_t staged_dq_step(const Dims &d, int dtype, int n, int j, const void *dS, const void *K,
                          float *dQacc, int accumulate, hipStream_t st) {
  (void)n;
  GemmArgs g{};
  g.A = offs(dS, (int64_t)j * d.c, dtype);
  g.B = offs(K, (int64_t)j * d.c * d.A, dtype);
  g.C = dQacc;
  g.a_batch = d.c * d.L; g.b_batch = d.L * d.A; g.c_batch = d.c * d.A;
  g.lda = d.L; g.ldb = d.A; g.ldc = d.A;
  g.K = (int)d.c; g.alpha = d.scale; g.accumulate = accumulate;
  return launch_gemm<true, false>(g, (int)d.c, d.A, d.B * d.Z, dtype, st);
}

hipError_t staged_dk_step(const Dims &d, int dtype, int n, int j, const void *dS, const void *Q,
                          float *dKacc, int accumulate, hipStream_t st) {
  GemmArgs g{};
  g.A = offs(dS, (int64_t)j * d.c, dtype);
  g.B = offs(Q, (int64_t)(n - d.rank_begin) * d.c * d.A, dtype);
  g.C = dKacc + (int64_t)j * d.c * d.A;
  g.a_batch = d.c * d.L; g.b_batch = d.Lq * d.A; g.c_batch = d.L * d.A;
  g.lda = d.L; g.ldb = d.A; g.ldc = d.A;
  g.K = (int)d.c; g.alpha = d.scale; g.accumulate = accumulate;
  return launch_gemm<false, false>(g, (int)d.c, d.A, d.B * d.Z, dtype, st);
}

// --------------------------------------------------------- row softmax ------
// One wavefront per strip row of L fp32 scores: a first sweep keeps a running
// (max, sum) per lane, a wave reduction merges the 64 partial pairs, and a
// second sweep (the row is L2-resident by then) writes P.  Traffic per score:
// 4 B read from HBM, 2 B (bf16) or 4 B (fp32) written.
template <typename OutT>
__global__ void __launch_bounds__(256) row_softmax_kernel(const float *S, OutT *P, float *LSE,
                                                          int64_t rows, int64_t L, int64_t c,
                                                          int64_t Lq, int64_t row_off) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const float *s = S + row * L;
  float m = -INFINITY, l = 0.f;
  for (int64_t i = lane * 4; i < L; i += 256) {
    const f32x4 x = *reinterpret_cast<const f32x4 *>(s + i);
    const float mx = fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
    if (mx > m) {
      l *= exp2f((m - mx) * kLog2e);  // m = -inf gives 0
      m = mx;
    }
    if (m > -INFINITY)
      l += exp2f((x[0] - m) * kLog2e) + exp2f((x[1] - m) * kLog2e) +
           exp2f((x[2] - m) * kLog2e) + exp2f((x[3] - m) * kLog2e);
  }
  const float M = wave_max(m);
  l = (m > -INFINITY) ? l * exp2f((m - M) * kLog2e) : 0.f;
  const float lsum = wave_sum(l);
  const float inv = 1.0f / lsum;
  OutT *p = P + row * L;
  for (int64_t i = lane * 4; i < L; i += 256) {
    const f32x4 x = *reinterpret_cast<const f32x4 *>(s + i);
    float e[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) e[k] = exp2f((x[k] - M) * kLog2e) * inv;
    if constexpr (sizeof(OutT) == 2) {
      u32x2 o = {pack_bf16(e[0], e[1]), pack_bf16(e[2], e[3])};
      *reinterpret_cast<u32x2 *>(p + i) = o;
    } else {
      f32x4 o = {e[0], e[1], e[2], e[3]};
      *reinterpret_cast<f32x4 *>(p + i) = o;
    }
  }
  if (lane == 0) {
    const int64_t head = row / c, r = row % c;
    LSE[head * Lq + row_off + r] = M + logf(lsum);
  }
}

// The same for rows of L = 256 NV scores with NV <= 16: the row stays in the wave's registers
// (4 NV values per lane), so it is read from memory once, all its loads are in flight together,
// and the maximum is exact before the first exponential.
template <typename OutT, int NV>
__global__ void __launch_bounds__(256) row_softmax_reg_kernel(const float *S, OutT *P, float *LSE,
                                                              int64_t rows, int64_t c, int64_t Lq,
                                                              int64_t row_off) {
  constexpr int64_t L = 256 * NV;
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const float *s = S + row * L;
  f32x4 x[NV];
#pragma unroll
  for (int v = 0; v < NV; ++v) x[v] = *reinterpret_cast<const f32x4 *>(s + v * 256 + lane * 4);
  float m = -INFINITY;
#pragma unroll
  for (int v = 0; v < NV; ++v) m = fmaxf(m, fmaxf(fmaxf(x[v][0], x[v][1]), fmaxf(x[v][2], x[v][3])));
  const float M = wave_max(m);  // finite: every row has at least one unmasked score
  const float mc = M * kLog2e;
  float l = 0.f;
#pragma unroll
  for (int v = 0; v < NV; ++v)
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      x[v][k] = exp2f(fmaf(x[v][k], kLog2e, -mc));
      l += x[v][k];
    }
  const float lsum = wave_sum(l);
  const float inv = 1.0f / lsum;
  OutT *p = P + row * L;
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    if constexpr (sizeof(OutT) == 2) {
      u32x2 o = {pack_bf16(x[v][0] * inv, x[v][1] * inv), pack_bf16(x[v][2] * inv, x[v][3] * inv)};
      *reinterpret_cast<u32x2 *>(p + v * 256 + lane * 4) = o;
    } else {
      *reinterpret_cast<f32x4 *>(p + v * 256 + lane * 4) = x[v] * inv;
    }
  }
  if (lane == 0) {
    const int64_t head = row / c, r = row % c;
    LSE[head * Lq + row_off + r] = M + logf(lsum);
  }
}

// Longer rows, L = 1024 nv with nv <= 32: one work-group per row, 4 nv values per thread in
// registers, the maximum and the sum merged across the four waves through LDS.
template <typename OutT>
__global__ void __launch_bounds__(256) row_softmax_wg_kernel(const float *S, OutT *P, float *LSE, int nv,
                                                             int64_t c, int64_t Lq, int64_t row_off) {
  constexpr int NVMAX = 32;
  __shared__ float red[8];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t row = blockIdx.x, L = 1024 * (int64_t)nv;
  const float *s = S + row * L;
  f32x4 x[NVMAX];
  float m = -INFINITY;
#pragma unroll
  for (int v = 0; v < NVMAX; ++v)
    if (v < nv) {
      x[v] = *reinterpret_cast<const f32x4 *>(s + v * 1024 + tid * 4);
      m = fmaxf(m, fmaxf(fmaxf(x[v][0], x[v][1]), fmaxf(x[v][2], x[v][3])));
    }
  m = wave_max(m);
  if (lane == 0) red[wave] = m;
  __syncthreads();
  const float M = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));  // finite: some score is unmasked
  const float mc = M * kLog2e;
  float l = 0.f;
#pragma unroll
  for (int v = 0; v < NVMAX; ++v)
    if (v < nv) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        x[v][k] = exp2f(fmaf(x[v][k], kLog2e, -mc));
        l += x[v][k];
      }
    }
  l = wave_sum(l);
  if (lane == 0) red[4 + wave] = l;
  __syncthreads();
  const float lsum = (red[4] + red[5]) + (red[6] + red[7]);
  const float inv = 1.0f / lsum;
  OutT *p = P + row * L;
#pragma unroll
  for (int v = 0; v < NVMAX; ++v)
    if (v < nv) {
      if constexpr (sizeof(OutT) == 2) {
        u32x2 o = {pack_bf16(x[v][0] * inv, x[v][1] * inv), pack_bf16(x[v][2] * inv, x[v][3] * inv)};
        *reinterpret_cast<u32x2 *>(p + v * 1024 + tid * 4) = o;
      } else {
        *reinterpret_cast<f32x4 *>(p + v * 1024 + tid * 4) = x[v] * inv;
      }
    }
  if (tid == 0) {
    const int64_t head = row / c, r = row % c;
    LSE[head * Lq + row_off + r] = M + logf(lsum);
  }
}

template <typename OutT>
static bool launch_row_softmax_reg(const float *S, OutT *P, float *LSE, int64_t rows, int64_t L, int64_t c,
                                   int64_t Lq, int64_t row_off, hipStream_t st) {
  dim3 grid((unsigned)((rows + 3) / 4));
#define RSA_ROWSM(NV)                                                                              \
  if (L == 256 * NV) {                                                                             \
    hipLaunchKernelGGL((row_softmax_reg_kernel<OutT, NV>), grid, dim3(256), 0, st, S, P, LSE, rows, \
                       c, Lq, row_off);                                                            \
    return true;                                                                                   \
  }
  RSA_ROWSM(1) RSA_ROWSM(2) RSA_ROWSM(4) RSA_ROWSM(8) RSA_ROWSM(16)
#undef RSA_ROWSM
  if (L % 1024 == 0 && L <= 32768 && rows < (1LL << 31)) {
    hipLaunchKernelGGL((row_softmax_wg_kernel<OutT>), dim3((unsigned)rows), dim3(256), 0, st, S, P, LSE,
                       (int)(L / 1024), c, Lq, row_off);
    return true;
  }
  return false;
}

hipError_t staged_row_softmax(const Dims &d, int dtype, int n, const float *S, void *P, float *LSE,
                              hipStream_t st) {
  const int64_t rows = (int64_t)d.B * d.Z * d.c;
  const int64_t row_off = (int64_t)(n - d.rank_begin) * d.c;
  if (dtype == RSA_BF16 ? launch_row_softmax_reg(S, (uint16_t *)P, LSE, rows, d.L, d.c, d.Lq, row_off, st)
                        : launch_row_softmax_reg(S, (float *)P, LSE, rows, d.L, d.c, d.Lq, row_off, st))
    return hipGetLastError();
  dim3 grid((unsigned)((rows + 3) / 4));
  if (dtype == RSA_BF16)
    hipLaunchKernelGGL(row_softmax_kernel<uint16_t>, grid, dim3(256), 0, st, S, (uint16_t *)P, LSE,
                       rows, d.L, d.c, d.Lq, row_off);
  else
    hipLaunchKernelGGL(row_softmax_kernel<float>, grid, dim3(256), 0, st, S, (float *)P, LSE, rows,
                       d.L, d.c, d.Lq, row_off);
  return hipGetLastError();
}

// ------------------------------------------------------ softmax backward ----
// dS = P o (dP - D_row), one wavefront per strip row.
template <typename T>
__global__ void __launch_bounds__(256) softmax_bwd_kernel(const T *P, const float *dP,
                                                          const float *D, T *dS, int64_t rows,
                                                          int64_t L, int64_t c, int64_t Lq,
                                                          int64_t row_off) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const float Dr = D[(row / c) * Lq + row_off + row % c];
  const T *p = P + row * L;
  const float *g = dP + row * L;
  T *o = dS + row * L;
#pragma unroll 4
  for (int64_t i = lane * 4; i < L; i += 256) {
    const f32x4 gp = *reinterpret_cast<const f32x4 *>(g + i);
    float pv[4];
    if constexpr (sizeof(T) == 2) {
      const u32x2 u = *reinterpret_cast<const u32x2 *>(p + i);
      pv[0] = bf16_to_f32(u[0] & 0xffffu); pv[1] = bf16_to_f32(u[0] >> 16);
      pv[2] = bf16_to_f32(u[1] & 0xffffu); pv[3] = bf16_to_f32(u[1] >> 16);
      u32x2 r = {pack_bf16(pv[0] * (gp[0] - Dr), pv[1] * (gp[1] - Dr)),
                 pack_bf16(pv[2] * (gp[2] - Dr), pv[3] * (gp[3] - Dr))};
      *reinterpret_cast<u32x2 *>(o + i) = r;
    } else {
      const f32x4 u = *reinterpret_cast<const f32x4 *>(p + i);
      f32x4 r = {u[0] * (gp[0] - Dr), u[1] * (gp[1] - Dr), u[2] * (gp[2] - Dr),
                 u[3] * (gp[3] - Dr)};
      *reinterpret_cast<f32x4 *>(o + i) = r;
    }
  }
}

hipError_t staged_softmax_bwd(const Dims &d, int dtype, int n, const void *P, const float *dP,
                              const float *D, void *dS, hipStream_t st) {
  const int64_t rows = (int64_t)d.B * d.Z * d.c;
  const int64_t row_off = (int64_t)(n - d.rank_begin) * d.c;
  dim3 grid((unsigned)((rows + 3) / 4));
  if (dtype == RSA_BF16)
    hipLaunchKernelGGL(softmax_bwd_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t *)P,
                       dP, D, (uint16_t *)dS, rows, d.L, d.c, d.Lq, row_off);
  else
    hipLaunchKernelGGL(softmax_bwd_kernel<float>, grid, dim3(256), 0, st, (const float *)P, dP, D,
                       (float *)dS, rows, d.L, d.c, d.Lq, row_off);
  return hipGetLastError();
}

// --------------------------------------------------------------- row dot ----
// D_i = sum_a dO_ia O_ia over the A elements of a row (A a multiple of 64): 8 lanes per row,
// each taking 8 elements of every 64.
template <typename T>
__global__ void __launch_bounds__(256) rowdot_kernel(const T *dO, const T *O, float *D,
                                                     int64_t rows_per_head, int64_t Lq,
                                                     int64_t row_off, int64_t total_rows, int A) {
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t row = gid >> 3;
  const int sub = (int)(gid & 7);
  float acc = 0.f;
  int64_t idx = 0;
  if (row < total_rows) {
    const int64_t head = row / rows_per_head, r = row % rows_per_head;
    idx = head * Lq + row_off + r;
    for (int a0 = 0; a0 < A; a0 += 64) {
      const T *a = dO + idx * A + a0 + sub * 8;
      const T *b = O + idx * A + a0 + sub * 8;
      if constexpr (sizeof(T) == 2) {
        const u32x4 x = *reinterpret_cast<const u32x4 *>(a);
        const u32x4 y = *reinterpret_cast<const u32x4 *>(b);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          acc = fmaf(bf16_to_f32(x[e] & 0xffffu), bf16_to_f32(y[e] & 0xffffu), acc);
          acc = fmaf(bf16_to_f32(x[e] >> 16), bf16_to_f32(y[e] >> 16), acc);
        }
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) acc = fmaf(a[e], b[e], acc);
      }
    }
  }
  acc += __shfl_xor(acc, 1);
  acc += __shfl_xor(acc, 2);
  acc += __shfl_xor(acc, 4);
  if (row < total_rows && sub == 0) D[idx] = acc;
}

hipError_t rowdot(const Dims &d, int dtype, int64_t row_off, int64_t rows_per_head, const void *dO,
                  const void *O, float *D, hipStream_t st) {
  const int64_t total = (int64_t)d.B * d.Z * rows_per_head;
  dim3 grid((unsigned)((total * 8 + 255) / 256));
  if (dtype == RSA_BF16)
    hipLaunchKernelGGL(rowdot_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t *)dO,
                       (const uint16_t *)O, D, rows_per_head, d.Lq, row_off, total, d.A);
  else
    hipLaunchKernelGGL(rowdot_kernel<float>, grid, dim3(256), 0, st, (const float *)dO,
                       (const float *)O, D, rows_per_head, d.Lq, row_off, total, d.A);
  return hipGetLastError();
}

// ------------------------------------------------------------------ fill ----
// A kernel rather than a memset, so that a caller may capture the launch sequence in a graph.
__global__ void __launch_bounds__(256) zero_kernel(f32x4 *p, int64_t n4) {
  const f32x4 z = {0.f, 0.f, 0.f, 0.f};
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) p[i] = z;
}

hipError_t zero_f32(float *p, int64_t n, hipStream_t st) {  // n: a multiple of 4
  const int64_t n4 = n / 4;
  const int64_t blocks = (n4 + 255) / 256;
  hipLaunchKernelGGL(zero_kernel, dim3((unsigned)(blocks < 8192 ? blocks : 8192)), dim3(256), 0, st,
                     reinterpret_cast<f32x4 *>(p), n4);
  return hipGetLastError();
}

// ----------------------------------------------------------------- store ----
template <typename T>
__global__ void __launch_bounds__(256) store_kernel(const float *src, T *dst, int64_t rows,
                                                    int64_t cols, int64_t src_ld, int64_t dst_ld,
                                                    int64_t src_batch, int64_t dst_batch,
                                                    int64_t rows_per_batch) {
  // cols is a multiple of 4; one thread converts 4 consecutive elements
  const int64_t per_row = cols >> 2;
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (gid >= rows * per_row) return;
  const int64_t row = gid / per_row, q = gid % per_row;
  const int64_t b = row / rows_per_batch, r = row % rows_per_batch;
  const f32x4 x = *reinterpret_cast<const f32x4 *>(src + b * src_batch + r * src_ld + q * 4);
  T *o = dst + b * dst_batch + r * dst_ld + q * 4;
  if constexpr (sizeof(T) == 2) {
    u32x2 u = {pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3])};
    *reinterpret_cast<u32x2 *>(o) = u;
  } else {
    *reinterpret_cast<f32x4 *>(o) = x;
  }
}

hipError_t store_rows(int dtype, const float *src, void *dst, int64_t batches,
                      int64_t rows_per_batch, int64_t cols, int64_t src_batch, int64_t dst_batch,
                      hipStream_t st) {
  const int64_t rows = batches * rows_per_batch;
  const int64_t n = rows * (cols >> 2);
  if (n == 0) return hipSuccess;
  dim3 grid((unsigned)((n + 255) / 256));
  if (dtype == RSA_BF16)
    hipLaunchKernelGGL(store_kernel<uint16_t>, grid, dim3(256), 0, st, src, (uint16_t *)dst, rows,
                       cols, cols, cols, src_batch, dst_batch, rows_per_batch);
  else
    hipLaunchKernelGGL(store_kernel<float>, grid, dim3(256), 0, st, src, (float *)dst, rows, cols,
                       cols, cols, src_batch, dst_batch, rows_per_batch);
  return hipGetLastError();
}

}  // namespace rsa
