// The two linear maps around Ring Self-Attention on a rank's rows (paper Table 2, sequence
// parallelism rows "Q/K/V" and "Linear") and their derivatives, bf16 with fp32 accumulation:
//   Q/K/V:  (B, rows, H) x (H, AZ) -> (B, Z, rows, A), written head-split as RSA reads it
//   Linear: (B, Z, rows, A) x (AZ, H) -> (B, rows, H), read head-split as RSA writes it
// One MFMA GEMM kernel serves all six products.  An operand is a "view": a matrix cut into
// 64 x 64 tiles that are either blocks of a plain row-major matrix or the (64 rows, 64 elements of
// one head) blocks of up to three (B, Z, rows, A) tensors, A = 64 or 128, so no tensor is ever
// re-laid out in memory.
//
// Work-group: 256 x 256 outputs, 8 waves of 128 x 64 (4 x 2 MFMA blocks of 32 x 32), k in slabs
// of 64 through the swizzled LDS tiles of the attention kernels, double-buffered, one barrier
// per slab.  The product is formed transposed (accumulator rows = n, columns = m): a lane then
// owns one output row m and four consecutive n per register group; bf16 blocks leave through
// LDS as whole 128-byte row segments, fp32 blocks as 16-byte pieces.
#include "rsa_fused_tile.h"
#include "rsa_kernels.h"

namespace rsa {

// A bf16 matrix [R][C] served as 64 x 64 tiles.
struct MatView {
  const uint16_t *p[3];  // plain: p[0]; head-split: tensor cb / (Z * AH) holds column tile cb
  int64_t ld;            // row stride in elements (head-split: the head size A)
  int64_t rows;          // head-split: rows per (b, z) block (a multiple of 64)
  int Z;                 // head-split: heads per tensor
  int AH;                // head-split: column tiles per head (A / 64: 1 or 2), head-major order
  int split;             // 0: plain row-major; 1: (B, Z, rows, A) tensors, row index = b * rows + r
};

// A value that is the same in every lane, moved to scalar registers (integer division leaves
// its result in vector registers even when its operands are uniform).
__device__ __forceinline__ int64_t uniform64(int64_t x) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)x >> 32));
  return (int64_t)(((uint64_t)hi << 32) | lo);
}

// How the tiles of one operand move along k, slab by slab, with additions only (the divisions
// that place a head-split tile are done once, in TileCursor's constructor): `step` per slab, and
// after `period` steps an extra jump to the next batch element (mode 1) or to the next tensor of
// the view (mode 2: jump1 into tensor 1, jump2 into tensor 2).  With two column tiles per head
// (mode 3) a step is the 64 elements to the head's second half, every second step also jumps
// (jumpA) to the next head, and after Z heads comes the jump to the next tensor.
struct ViewWalk {
  int64_t ld, step, jump1, jump2, jumpA;
  int period, mode, Z;
  // krows: k runs over the row tiles of the view; else over its column tiles
  __device__ __forceinline__ ViewWalk(const MatView &v, bool krows) {
    jump1 = 0; jump2 = 0; jumpA = 0; period = 0x7fffffff; mode = 0; Z = v.Z;
    if (!v.split) {
      ld = v.ld;
      step = krows ? 64 * v.ld : 64;
    } else if (!krows) {  // k runs over heads, then over the tensors of the view
      ld = v.ld;
      const int64_t head = v.rows * v.ld;  // elements from one head to the next
      // after the last head of a tensor the pointer has moved Z heads; the next tensor starts over
      jump1 = (v.p[1] - v.p[0]) - (int64_t)v.Z * head;
      jump2 = (v.p[2] - v.p[1]) - (int64_t)v.Z * head;
      if (v.AH == 1) {
        step = head; period = v.Z; mode = 2;
      } else {
        step = 64; jumpA = head - 128; period = 2; mode = 3;
      }
    } else {  // k runs over the rows of a batch element, then over batch elements
      ld = v.ld;
      step = 64 * v.ld;
      jump1 = (int64_t)(v.Z - 1) * v.rows * v.ld;
      period = (int)(v.rows / 64); mode = 1;
    }
  }
};

struct TileCursor {
  const uint16_t *ptr;
  int cnt, which;  // which: tensor of the view; in mode 3 also the head inside it, times 4
  // krows: the tile index `fixed` selects columns and k (slab ks) selects rows; else the reverse
  __device__ __forceinline__ TileCursor(const MatView &v, bool krows, int64_t fixed, int64_t ks) {
    cnt = 0; which = 0;
    if (!v.split) {
      ptr = krows ? v.p[0] + ks * 64 * v.ld + fixed * 64 : v.p[0] + fixed * 64 * v.ld + ks * 64;
    } else {
      const uint32_t ct = (uint32_t)(krows ? fixed : ks), rt = (uint32_t)(krows ? ks : fixed);
      const uint32_t per_tensor = (uint32_t)(v.Z * v.AH);
      which = (int)(ct / per_tensor);
      const uint32_t rem = ct % per_tensor;
      const int64_t z = rem / (uint32_t)v.AH;
      const int ah = (int)(rem % (uint32_t)v.AH);
      const uint32_t m0 = rt * 64u, b = m0 / (uint32_t)v.rows, r0 = m0 % (uint32_t)v.rows;
      const uint16_t *t = which == 0 ? v.p[0] : (which == 1 ? v.p[1] : v.p[2]);
      ptr = t + (((int64_t)b * v.Z + z) * v.rows + r0) * v.ld + ah * 64;
      cnt = krows ? (int)(r0 / 64) : (v.AH == 1 ? (int)z : ah);
      if (!krows && v.AH == 2) which |= (int)z << 2;
    }
    ptr = reinterpret_cast<const uint16_t *>(uniform64(reinterpret_cast<int64_t>(ptr)));
    cnt = __builtin_amdgcn_readfirstlane(cnt);
    which = __builtin_amdgcn_readfirstlane(which);
  }
  template <bool WIDE>  // WIDE: some view of the product has two column tiles per head (mode 3)
  __device__ __forceinline__ void advance(const ViewWalk &w) {
    ptr += w.step;
    if (++cnt == w.period) {
      asm volatile("" ::: "memory");  // a real (rarely taken, uniform) branch instead of a chain of selects per slab
      cnt = 0;
      if (w.mode == 1) ptr += w.jump1;
      if (w.mode == 2) { ptr += which == 0 ? w.jump1 : w.jump2; ++which; }
      if (WIDE && w.mode == 3) {
        ptr += w.jumpA;
        which += 4;
        if ((which >> 2) == w.Z) { ptr += (which & 3) == 0 ? w.jump1 : w.jump2; which = (which & 3) + 1; }
      }
    }
  }
};

struct GemmArgs {
  MatView A, B;       // m-side and n-side operands
  int64_t M, N, K;    // multiples of 64
  int64_t kslabs;     // slabs of 64 k per split (split s takes slabs [s * kslabs, ...))
  void *out[3];       // plain: out[0] (+ split * M * out_ld elements for a k split); head-split: 3 tensors
  int64_t out_ld, out_rows;
  int out_Z, out_AH, out_split;  // head-split output: (B, out_Z, out_rows, 64 * out_AH) tensors
  int ntiles;         // 128-wide column tiles
};

// A_KROWS / B_KROWS: the operand's tiles hold k along their rows (the view is [K][M] or [K][N])
// instead of along their columns ([M][K], [N][K]).
// Work-group: 8 waves, 256 (m) x 256 (n) outputs; wave (wm, wn) of a 2 x 4 grid owns 128 x 64
// (4 x 2 MFMA blocks).  The tile is this large because a CU takes at most about 40 bytes per clock
// from global memory (measured, L2-resident data): a 128 x 128 tile needs 32 KiB per 512 matrix-pipe
// cycles and is bound by that at 30 % of the peak; this one needs 64 KiB per 2048.
// A slab of 64 k is 8 tiles = 64 KiB; the next slab is fetched into registers (8 x 16 bytes per
// lane) while the current one is used from LDS, then written to the other LDS buffer: one barrier
// per slab.  (Direct global->LDS loads would save the registers, but the compiler only lets LDS
// reads pass outstanding direct loads when the buffers are distinct objects, i.e. with two copies
// of the loop body, and two copies of a body with 128 accumulator registers do not agree on
// where the accumulators live.)
constexpr int kGemmBM = 256, kGemmBN = 256;
// WIDE: heads of 128 elements somewhere in the product (an operand view or the output).
template <bool A_KROWS, bool B_KROWS, bool OUT_F32, bool WIDE>
__global__ void __launch_bounds__(512, 1) proj_gemm_kernel(GemmArgs g) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[2][8][kTileBytes];  // [buffer][A0..A3, B0..B3]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;
  const int col = lane & 31, half = lane >> 5;
  const uint32_t wg = xcd_remap(blockIdx.x, gridDim.x);
  const int64_t m0 = (int64_t)(wg / g.ntiles) * kGemmBM, n0 = (int64_t)(wg % g.ntiles) * kGemmBN;
  const int64_t mt_last = g.M / 64 - 1, nt_last = g.N / 64 - 1;
  const int64_t ks_begin = (int64_t)blockIdx.y * g.kslabs;
  int64_t ks_end = ks_begin + g.kslabs;
  if (ks_end > g.K / 64) ks_end = g.K / 64;

  const TileLanes tl(lane);
  const ViewWalk wa(g.A, A_KROWS), wb(g.B, B_KROWS);
  // (a ragged edge refetches the last tile; its outputs are never stored)
  auto mt_of = [&](int t) { const int64_t mt = m0 / 64 + t; return mt > mt_last ? mt_last : mt; };
  auto nt_of = [&](int t) { const int64_t nt = n0 / 64 + t; return nt > nt_last ? nt_last : nt; };
  TileCursor ca[4] = {TileCursor(g.A, A_KROWS, mt_of(0), ks_begin), TileCursor(g.A, A_KROWS, mt_of(1), ks_begin),
                      TileCursor(g.A, A_KROWS, mt_of(2), ks_begin), TileCursor(g.A, A_KROWS, mt_of(3), ks_begin)};
  TileCursor cb[4] = {TileCursor(g.B, B_KROWS, nt_of(0), ks_begin), TileCursor(g.B, B_KROWS, nt_of(1), ks_begin),
                      TileCursor(g.B, B_KROWS, nt_of(2), ks_begin), TileCursor(g.B, B_KROWS, nt_of(3), ks_begin)};
  // this thread's 16-byte piece of every tile: row tid / 8, logical chunk tid % 8
  const int prow = tid >> 3, pcc = tid & 7;
  const int64_t ga_off = prow * wa.ld + pcc * 8, gb_off = prow * wb.ld + pcc * 8;
  const int l_off = tile_off(prow, pcc);
  u32x4 stg[8];
  // (loads through global-address-space pointers: a flat load would also count as an LDS
  // operation and every wait for an LDS read would then wait for the slab in flight)
  typedef __attribute__((address_space(1))) const u32x4 *gvec_t;
  auto fetch = [&]() __attribute__((always_inline)) {  // the slab the cursors point at, then move them on
#pragma unroll
    for (int t = 0; t < 4; ++t) stg[t] = *(gvec_t)(ca[t].ptr + ga_off);
#pragma unroll
    for (int t = 0; t < 4; ++t) stg[4 + t] = *(gvec_t)(cb[t].ptr + gb_off);
#pragma unroll
    for (int t = 0; t < 4; ++t) { ca[t].template advance<WIDE>(wa); cb[t].template advance<WIDE>(wb); }
  };
  auto put = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int t = 0; t < 8; ++t) *reinterpret_cast<u32x4 *>(lds[buf][t] + l_off) = stg[t];
  };

  f32x16 acc[2][4];  // [nb][mb]: rows n, columns m
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[nb][mb][v] = 0.f;

  int buf = 0;
  if (ks_begin < ks_end) {  // uniform over the work-group
    fetch();
    put(0);
  }
  __syncthreads();
  for (int64_t ks = ks_begin; ks < ks_end; ++ks) {
    const bool more = ks + 1 < ks_end;
    if (more) fetch();
    const unsigned char(*sc)[kTileBytes] = lds[buf];
    // the fragments of k-slice kk + 1 are read while the MFMAs of slice kk run
    bf16x8 af[2][4], bf[2][2];
    auto frags = [&](int kk, bf16x8(&a4)[4], bf16x8(&b2)[2]) __attribute__((always_inline)) {
#pragma unroll
      for (int mb = 0; mb < 4; ++mb) {
        const unsigned char *ta = sc[wm * 2 + (mb >> 1)];
        a4[mb] = A_KROWS ? tl.read_cols(ta, kk * 16, mb & 1)
                         : (B_KROWS ? tl.read_rows_perm(ta, (mb & 1) * 32, kk) : tl.read_rows(ta, (mb & 1) * 32, kk));
      }
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        const unsigned char *tb = sc[4 + wn];
        b2[nb] = B_KROWS ? tl.read_cols(tb, kk * 16, nb)
                         : (A_KROWS ? tl.read_rows_perm(tb, nb * 32, kk) : tl.read_rows(tb, nb * 32, kk));
      }
    };
    frags(0, af[0], bf[0]);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      if (kk < 3) frags(kk + 1, af[(kk + 1) & 1], bf[(kk + 1) & 1]);
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
          acc[nb][mb] = mfma_32x32x16(bf[kk & 1][nb], af[kk & 1][mb], acc[nb][mb]);
      __builtin_amdgcn_sched_barrier(0);  // keep the slices in this order
    }
    if (more) put(buf ^ 1);  // last read one slab ago, before the barrier that ended it
    __syncthreads();
    buf ^= 1;
  }

  // lane (col, half) holds, for output row m, the columns n = nb*32 + grp*8 + half*4 .. +4
  if (!OUT_F32) {
    // bf16: the wave's 128 x 64 block goes through two LDS tiles of its own (every wave is past
    // the loop's last barrier) and leaves as whole 128-byte row segments.
    unsigned char *t0 = lds[0][wave], *t1 = lds[1][wave];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) stage_block_T(mb < 2 ? t0 : t1, (mb & 1) * 32, acc[0][mb], acc[1][mb], 1.0f, lane);
    const int64_t nw = n0 + wn * 64;  // the block's 64 columns: (half of) one head of a head-split output
    if (nw < g.N) {
      int which = 0;
      int64_t zoff = 0, aoff = 0;
      const int out_AH = WIDE ? g.out_AH : 1;
      const int64_t out_A = 64 * out_AH;
      if (g.out_split) {
        const uint32_t hb = (uint32_t)(nw / 64), per_tensor = (uint32_t)(g.out_Z * out_AH);
        which = (int)(hb / per_tensor);
        const uint32_t rem = hb % per_tensor;
        zoff = rem / (uint32_t)out_AH;
        aoff = (rem % (uint32_t)out_AH) * 64;
      }
      uint16_t *base = static_cast<uint16_t *>(which == 0 ? g.out[0] : (which == 1 ? g.out[1] : g.out[2]));
#pragma unroll
      for (int it = 0; it < 16; ++it) {
        const int row = it * 8 + (lane >> 3), cc = lane & 7;  // row of the wave's 128
        const int64_t m = m0 + wm * 128 + row;
        if (m >= g.M) continue;
        const u32x4 w = *reinterpret_cast<const u32x4 *>((row < 64 ? t0 : t1) + tile_off(row & 63, cc));
        int64_t off;
        if (!g.out_split) {
          off = m * g.out_ld + nw + cc * 8;
        } else {
          const uint32_t b = (uint32_t)m / (uint32_t)g.out_rows, r = (uint32_t)m % (uint32_t)g.out_rows;
          off = (((int64_t)b * g.out_Z + zoff) * g.out_rows + r) * out_A + aoff + cc * 8;
        }
        *reinterpret_cast<u32x4 *>(base + off) = w;
      }
    }
    return;
  }
#pragma unroll
  for (int mb = 0; mb < 4; ++mb) {
    const int64_t m = m0 + wm * 128 + mb * 32 + col;
    if (m >= g.M) continue;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int grp = 0; grp < 4; ++grp) {
        const int64_t n = n0 + wn * 64 + nb * 32 + grp * 8 + half * 4;
        if (n >= g.N) continue;
        const int64_t off = ((int64_t)blockIdx.y * g.M + m) * g.out_ld + n;  // fp32 outputs are plain matrices
        const f32x16 &c = acc[nb][mb];
        const f32x4 w = {c[grp * 4 + 0], c[grp * 4 + 1], c[grp * 4 + 2], c[grp * 4 + 3]};
        *reinterpret_cast<f32x4 *>(static_cast<float *>(g.out[0]) + off) = w;
      }
  }
}

// out[i] = sum over s of part[s][i], s in fixed order: the deterministic end of a k split
__global__ void __launch_bounds__(256) ksplit_reduce_kernel(const float *part, float *out, int64_t n4,
                                                            int splits) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  f32x4 s = reinterpret_cast<const f32x4 *>(part)[i];
  for (int k = 1; k < splits; ++k) s += reinterpret_cast<const f32x4 *>(part)[(int64_t)k * n4 + i];
  reinterpret_cast<f32x4 *>(out)[i] = s;
}

static MatView plain(const void *p, int64_t ld) {
  MatView v{};
  v.p[0] = static_cast<const uint16_t *>(p); v.ld = ld; v.split = 0; v.rows = 64; v.Z = 1; v.AH = 1;
  return v;
}
static MatView heads(const void *p0, const void *p1, const void *p2, int64_t rows, int Z, int A = 64) {
  MatView v{};
  v.p[0] = static_cast<const uint16_t *>(p0); v.p[1] = static_cast<const uint16_t *>(p1);
  v.p[2] = static_cast<const uint16_t *>(p2); v.ld = A; v.rows = rows; v.Z = Z; v.AH = A / 64; v.split = 1;
  return v;
}

template <bool A_KROWS, bool B_KROWS, bool OUT_F32>
static hipError_t launch_gemm(GemmArgs &g, int splits, hipStream_t st) {
  g.ntiles = (int)((g.N + kGemmBN - 1) / kGemmBN);
  const int64_t mtiles = (g.M + kGemmBM - 1) / kGemmBM;
  g.kslabs = (g.K / 64 + splits - 1) / splits;
  dim3 grid((unsigned)(mtiles * g.ntiles), (unsigned)splits);
  const bool wide = (g.A.split && g.A.AH == 2) || (g.B.split && g.B.AH == 2) || (g.out_split && g.out_AH == 2);
  if (wide)
    hipLaunchKernelGGL((proj_gemm_kernel<A_KROWS, B_KROWS, OUT_F32, true>), grid, dim3(512), 0, st, g);
  else
    hipLaunchKernelGGL((proj_gemm_kernel<A_KROWS, B_KROWS, OUT_F32, false>), grid, dim3(512), 0, st, g);
  return hipGetLastError();
}

// k splits of a weight-gradient product: as many as still give every CU at most one work-group
// (the kernel runs one per CU; a second round costs more than the longer k walk of fewer splits,
// and every split writes and re-reads a full fp32 partial result)
int proj_wgrad_splits(int64_t Mout, int64_t Nout, int64_t K) {
  const int64_t tiles = ((Mout + kGemmBM - 1) / kGemmBM) * ((Nout + kGemmBN - 1) / kGemmBN);
  int64_t s = 256 / tiles;
  const int64_t slabs = K / 64;
  if (s > slabs / 4) s = slabs / 4;
  if (s < 1) s = 1;
  if (s > 64) s = 64;
  return (int)s;
}

hipError_t proj_qkv(const Dims &d, int64_t H, const void *X, const void *W, void *Q, void *K, void *V,
                    hipStream_t st) {
  GemmArgs g{};
  g.M = (int64_t)d.B * d.Lq; g.N = 3LL * d.Z * d.A; g.K = H;
  g.A = plain(X, H);          // [M][K]
  g.B = plain(W, g.N);        // [K][N]
  g.out[0] = Q; g.out[1] = K; g.out[2] = V;
  g.out_split = 1; g.out_rows = d.Lq; g.out_Z = d.Z; g.out_AH = d.A / 64;
  return launch_gemm<false, true, false>(g, 1, st);
}

hipError_t proj_out(const Dims &d, int64_t H, const void *O, const void *Wo, void *Y, hipStream_t st) {
  GemmArgs g{};
  g.M = (int64_t)d.B * d.Lq; g.N = H; g.K = (int64_t)d.Z * d.A;
  g.A = heads(O, nullptr, nullptr, d.Lq, d.Z, d.A);  // [M][K], column tile = (half of a) head
  g.B = plain(Wo, H);                           // [K][N]
  g.out[0] = Y; g.out_split = 0; g.out_ld = H;
  return launch_gemm<false, true, false>(g, 1, st);
}

hipError_t proj_out_bwd(const Dims &d, int64_t H, const void *dY, const void *O, const void *Wo,
                        void *dO, float *dWo, float *part, hipStream_t st) {
  const int64_t M = (int64_t)d.B * d.Lq, ZA = (int64_t)d.Z * d.A;
  {  // dO = dY Wo^T, head-split
    GemmArgs g{};
    g.M = M; g.N = ZA; g.K = H;
    g.A = plain(dY, H);   // [M][K]
    g.B = plain(Wo, H);   // [N][K]
    g.out[0] = dO; g.out_split = 1; g.out_rows = d.Lq; g.out_Z = d.Z; g.out_AH = d.A / 64;
    hipError_t e = launch_gemm<false, false, false>(g, 1, st);
    if (e != hipSuccess) return e;
  }
  // dWo = O^T dY: contraction over the rows
  GemmArgs g{};
  g.M = ZA; g.N = H; g.K = M;
  g.A = heads(O, nullptr, nullptr, d.Lq, d.Z, d.A);  // [K][M]
  g.B = plain(dY, H);                           // [K][N]
  const int splits = proj_wgrad_splits(ZA, H, M);
  g.out[0] = splits > 1 ? part : dWo; g.out_split = 0; g.out_ld = H;
  hipError_t e = launch_gemm<true, true, true>(g, splits, st);
  if (e != hipSuccess || splits == 1) return e;
  const int64_t n4 = ZA * H / 4;
  hipLaunchKernelGGL(ksplit_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st, part, dWo,
                     n4, splits);
  return hipGetLastError();
}

hipError_t proj_qkv_bwd(const Dims &d, int64_t H, const void *dQ, const void *dK, const void *dV,
                        const void *X, const void *W, void *dX, float *dW, float *part,
                        hipStream_t st) {
  const int64_t M = (int64_t)d.B * d.Lq, N3 = 3LL * d.Z * d.A;
  {  // dX = [dQ | dK | dV] W^T
    GemmArgs g{};
    g.M = M; g.N = H; g.K = N3;
    g.A = heads(dQ, dK, dV, d.Lq, d.Z, d.A);  // [M][K]
    g.B = plain(W, N3);                  // [N][K]
    g.out[0] = dX; g.out_split = 0; g.out_ld = H;
    hipError_t e = launch_gemm<false, false, false>(g, 1, st);
    if (e != hipSuccess) return e;
  }
  // dW = X^T [dQ | dK | dV]
  GemmArgs g{};
  g.M = H; g.N = N3; g.K = M;
  g.A = plain(X, H);                   // [K][M]
  g.B = heads(dQ, dK, dV, d.Lq, d.Z, d.A);  // [K][N]
  const int splits = proj_wgrad_splits(H, N3, M);
  g.out[0] = splits > 1 ? part : dW; g.out_split = 0; g.out_ld = N3;
  hipError_t e = launch_gemm<true, true, true>(g, splits, st);
  if (e != hipSuccess || splits == 1) return e;
  const int64_t n4 = H * N3 / 4;
  hipLaunchKernelGGL(ksplit_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st, part, dW,
                     n4, splits);
  return hipGetLastError();
}

// ---- Linformer projections along the sequence (Table 3, row Projection) ----
// out (Zt, Kp, A) bf16 = sum over the k splits of part[s][k][zt*A + a], in a fixed order
__global__ void __launch_bounds__(256) ksplit_reduce_heads_kernel(const float *part, uint16_t *out,
                                                                  int64_t Kp, int64_t Zt, int splits, int A) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;  // one group of 4 columns
  const int64_t n4 = Zt * (A / 4), total = Kp * n4;
  if (i >= total) return;
  const int64_t k = i / n4, c = (i % n4) * 4;
  f32x4 s = reinterpret_cast<const f32x4 *>(part)[i];
  for (int j = 1; j < splits; ++j) s += reinterpret_cast<const f32x4 *>(part)[(int64_t)j * total + i];
  const u32x2 w = {pack_bf16(s[0], s[1]), pack_bf16(s[2], s[3])};
  *reinterpret_cast<u32x2 *>(out + ((c / A) * Kp + k) * A + (c % A)) = w;
}

int linformer_splits(int64_t Kp, int64_t Zt, int64_t rows, int A) {
  return proj_wgrad_splits(Kp, Zt * A, rows);
}

// Xp (Zt, Kp, A) = E^T X over `rows` tokens: X (Zt, L, A) from token row0 on, E (rows, Kp) from row0 on
hipError_t linformer_project(int64_t Zt, int64_t L, int64_t rows, int64_t Kp, int A, const void *X,
                             const void *E, void *Xp, float *part, hipStream_t st) {
  GemmArgs g{};
  g.M = Kp; g.N = Zt * A; g.K = rows;
  g.A = plain(E, Kp);                               // [K = token][M = k]
  g.B = heads(X, nullptr, nullptr, L, (int)Zt, A);  // [K = token][N = (head, a)]; one "batch" of Zt heads
  const int splits = linformer_splits(Kp, Zt, rows, A);
  g.out[0] = part; g.out_split = 0; g.out_ld = g.N;
  hipError_t e = launch_gemm<true, true, true>(g, splits, st);
  if (e != hipSuccess) return e;
  const int64_t total = Kp * Zt * (A / 4);
  hipLaunchKernelGGL(ksplit_reduce_heads_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                     part, static_cast<uint16_t *>(Xp), Kp, Zt, splits, A);
  return hipGetLastError();
}

// dX rows (Zt, L, A) from row0 on = E dXp, and dE (rows, Kp) fp32 = sum over heads of X dXp^T
hipError_t linformer_project_bwd(int64_t Zt, int64_t L, int64_t rows, int64_t Kp, int A, const void *dXp,
                                 const void *X, const void *E, void *dX, float *dE, hipStream_t st) {
  if (linformer_dx_supported(Kp, A)) {
    hipError_t e = linformer_dx(Zt, L, rows, Kp, A, dXp, E, dX, st);
    if (e != hipSuccess) return e;
  } else {
    GemmArgs g{};
    g.M = rows; g.N = Zt * A; g.K = Kp;
    g.A = plain(E, Kp);                                  // [M = token][K = k]
    g.B = heads(dXp, nullptr, nullptr, Kp, (int)Zt, A);  // [K = k][N = (head, a)]
    g.out[0] = dX; g.out_split = 1; g.out_rows = L; g.out_Z = (int)Zt; g.out_AH = A / 64;
    hipError_t e = launch_gemm<false, true, false>(g, 1, st);
    if (e != hipSuccess) return e;
  }
  GemmArgs g{};
  g.M = rows; g.N = Kp; g.K = Zt * A;
  g.A = heads(X, nullptr, nullptr, L, (int)Zt, A);     // [M = token][K = (head, a)]
  g.B = heads(dXp, nullptr, nullptr, Kp, (int)Zt, A);  // [N = k][K = (head, a)]
  g.out[0] = dE; g.out_split = 0; g.out_ld = Kp;
  return launch_gemm<false, false, true>(g, 1, st);
}

}  // namespace rsa
