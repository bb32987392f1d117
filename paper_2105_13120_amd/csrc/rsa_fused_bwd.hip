// Fused Ring Self-Attention backward (bf16, A = 64): the derivative of Eq. 1
// with the ring structure of section 3.2.2, without the score strip in memory.
// P is recomputed from Q, K and the forward's LSE: P = exp(s QK^T - LSE).
//
//   preprocess: the row terms -D = -rowsum(dO o O) and -LSE / s; a kernel of its own for the
//     step-level entry point, the prologue of the dQ kernel in rsa_backward.
//   Both kernels recompute P = exp2(s log2e (Q K^T - LSE / s)): the matrix core forms the bracket
//   from the caller's bf16 Q and K as they are (its accumulator starts from -LSE / s) and the
//   factor s log2e is applied to the fp32 result, one multiply per score.  Folding that factor
//   into a bf16 operand instead would save the multiply and round the operand a second time:
//   an error of 2^-9 per element that is the same for every score of a key (or query), adds up
//   coherently in dK (or dQ) and more than doubles their largest error.
//   dkdv kernel: a work-group owns 4*32 keys and walks the query tiles of every
//     simulated rank, starting with the rank that holds those keys (ring
//     order); the sum over ranks that the ring would all-reduce is its loop.
//       S' = Q K^T - LSE / s, dP' = dO V^T - D      (A: Q / dO rows from LDS; B: K / V registers;
//                                                    the row terms are the accumulators' start)
//       P = exp2(s log2e S'), dS = P o dP'
//       dV^T += dO^T P, dK^T += Q^T dS   (A operand: LDS transpose reads; B: P / dS registers)
//   dq kernel: a work-group owns 4*R query rows and walks the K/V tiles in ring
//     order (the paper's second K ring pass):
//       S'^T = K Q^T - LSE / s, P^T = exp2(s log2e S'^T),
//       dP'^T = V dO^T - D, dS^T = P^T o dP'^T, dQ^T += K^T dS^T
#include "rsa_fused_tile.h"
#include "rsa_kernels.h"

namespace rsa {

struct BwdArgs {
  const uint16_t *Q, *K, *V, *dO;
  const float *nL, *nD;                 // -LSE / scale and -D per query row
  // dQ kernel with the preprocess folded in: it forms the row terms from O and LSE
  // itself and leaves them in nL_out, nD_out for the dK/dV kernel that follows
  const uint16_t *O;
  const float *LSE;
  float *nL_out, *nD_out;
  uint16_t *dQ, *dK, *dV;
  // fp32 partial sums per split: dV then dK of the dK/dV kernel with a split query walk,
  // dQ of the dQ kernel with a split key walk
  float *part;
  int64_t L, c, Lq;
  int64_t qs[3], ks[3], os[3];  // element strides (batch, head, row) of Q, dQ; K, V, dK, dV; O, dO
  RowMap map;  // local query row -> global token index
  int N, Z, tiles_per_head;
  float cl2, scale, inv_scale;  // scale log2(e), scale, 1 / scale
};

// ------------------------------------------------------------- preprocess ---
// nD_i = -sum_a dO_ia O_ia and nL_i = -LSE_i / scale: 8 lanes per row, 8 elements of every 64 each.
__global__ void __launch_bounds__(256) bwd_preprocess_kernel(const uint16_t *dO, const uint16_t *O,
                                                             const float *LSE, float *nD, float *nL,
                                                             int64_t rows, int A, float inv_scale,
                                                             OutLayout lay) {
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t row = gid >> 3;
  const int sub = (int)(gid & 7);
  float acc = 0.f;
  if (row < rows) {
    const int64_t base = lay.row_off(row);
    for (int a0 = 0; a0 < A; a0 += 64) {
      const int64_t off = base + a0 + sub * 8;
      const u32x4 x = *reinterpret_cast<const u32x4 *>(dO + off);
      const u32x4 y = *reinterpret_cast<const u32x4 *>(O + off);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc = fmaf(bf16_to_f32(x[e] & 0xffffu), bf16_to_f32(y[e] & 0xffffu), acc);
        acc = fmaf(bf16_to_f32(x[e] >> 16), bf16_to_f32(y[e] >> 16), acc);
      }
    }
  }
  acc += __shfl_xor(acc, 1);
  acc += __shfl_xor(acc, 2);
  acc += __shfl_xor(acc, 4);
  if (row < rows && sub == 0) {
    nD[row] = -acc;
    nL[row] = -LSE[row] * inv_scale;
  }
}

// ------------------------------------------------------------------ dK, dV ---
// Work-group: 4 waves x 32 keys.  K and V of a wave's keys stay in
// registers as B operands; the work-group walks the query rows in stages of NQ tiles of 64 rows
// of Q and dO, double-buffered in LDS and filled by direct global->LDS loads (no staging
// registers), one barrier per stage.
// The row terms of the softmax backward ride on the accumulator init of the MFMAs:
//   S'  = Q K^T - LSE / scale  (so P = exp2(scale log2e S') is one multiply and the exp2)
//   dP' = dO V^T - D           (so dS = P dP' is one multiply)
// and dK = scale * sum_i dS_ij Q_i.
// A head of 128 is two halves of 64 (AH = 2): two LDS tiles per 64 rows, S' and dP' contract over
// both, dV and dK have twice the accumulators, and the kernel runs one wave per SIMD.
template <int NQ, bool CAUSAL, int AH>
__global__ void __launch_bounds__(256, AH == 2 ? 1 : 2) fused_bwd_dkdv_kernel(BwdArgs a) {
  constexpr int KW = 32;      // keys per wave
  constexpr int BK = 4 * KW;  // keys per work-group
  constexpr int A = 64 * AH;
  // The two stage buffers are separate objects, each addressed by name, so that the
  // compiler knows a direct load into one cannot alias the LDS reads of the other.
  struct Stage {
    unsigned char Qt[NQ][AH][kTileBytes], dOs[NQ][AH][kTileBytes];
    float lse[NQ][64], d[NQ][64];
  };
  __shared__ __attribute__((aligned(16))) Stage stage0, stage1;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31, half = lane >> 5;
  const uint32_t wg = xcd_remap(blockIdx.x, gridDim.x);
  const int64_t head = wg / a.tiles_per_head;
  const int64_t key0 = (wg % a.tiles_per_head) * BK;  // first key of the work-group
  const int64_t wkey0 = key0 + wave * KW;             // first key of this wave

  const int64_t kv_off = head_offset(head, a.Z, a.ks);
  const uint16_t *Qh = a.Q + head_offset(head, a.Z, a.qs);
  const uint16_t *dOh = a.dO + head_offset(head, a.Z, a.os);
  const uint16_t *Kh = a.K + kv_off;
  const uint16_t *Vh = a.V + kv_off;
  const float *nLh = a.nL + head * a.Lq;
  const float *nDh = a.nD + head * a.Lq;
  const int64_t q_ld = a.qs[2], kv_ld = a.ks[2], o_ld = a.os[2];

  // K and V rows of this wave as B operands:
  // lane (col, half) holds row key = wkey0 + col, elements dk*16 + half*8 .. +8.
  bf16x8 kreg[4 * AH], vreg[4 * AH];
  {
    int64_t key = wkey0 + col;
    if (key >= a.L) key = a.L - 1;  // ragged tail: clamped here, not stored below
#pragma unroll
    for (int dk = 0; dk < 4 * AH; ++dk) {
      kreg[dk] = *reinterpret_cast<const bf16x8 *>(Kh + key * kv_ld + dk * 16 + half * 8);
      vreg[dk] = *reinterpret_cast<const bf16x8 *>(Vh + key * kv_ld + dk * 16 + half * 8);
    }
  }

  const TileLanes tl(lane);

  f32x16 dv[2 * AH], dk_[2 * AH];  // [db], transposed: rows = head dim, columns = keys
#pragma unroll
  for (int db = 0; db < 2 * AH; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) { dv[db][v] = 0.f; dk_[db][v] = 0.f; }

  // Stages of NQ query tiles in ring order: start at the rank that owns key0.
  const int nqt = (int)(a.Lq / 64);
  const int nst = (nqt + NQ - 1) / NQ;
  int start = 0;
  {
    const int64_t r = (int64_t)(a.map.owner(key0) - a.map.rb) * a.c;  // local row of that rank's first query
    if (r >= 0 && r < a.Lq) start = (int)(r / (64 * NQ));
  }
  auto st_of = [&](int i) { int q = start + i; return q >= nst ? q - nst : q; };
  // a stage matters if some row of it can see the first key of the work-group
  auto visible = [&](int i) {
    if (!CAUSAL) return true;
    const int qt = st_of(i) * NQ;
    bool v = false;
#pragma unroll
    for (int u = 0; u < NQ; ++u)
      v = v || (qt + u < nqt && a.map((int64_t)(qt + u) * 64) + 63 >= key0);
    return v;
  };
  // With few keys (Table 3's projected keys) the walk over the query stages is split over
  // gridDim.y work-groups, each writing fp32 partial sums that a second kernel adds up.
  const int per_split = (nst + (int)gridDim.y - 1) / (int)gridDim.y;
  const int i_begin = (int)blockIdx.y * per_split;
  const int i_end = i_begin + per_split < nst ? i_begin + per_split : nst;
  auto advance = [&](int i) { ++i; while (i < i_end && !visible(i)) ++i; return i; };

  const TileDMA dma_q(wave, lane, (int)q_ld), dma_o(wave, lane, (int)o_ld);
  auto load_stage = [&](int i, Stage &sn) __attribute__((always_inline)) {
    const int st = st_of(i);
#pragma unroll
    for (int u = 0; u < NQ; ++u) {
      int qt = st * NQ + u;
      if (qt >= nqt) qt = nqt - 1;  // past the last tile: refetch it (never used)
      const int64_t r0 = (int64_t)qt * 64;
#pragma unroll
      for (int ah = 0; ah < AH; ++ah) {
        dma_q.load(Qh + r0 * q_ld + ah * 64, sn.Qt[u][ah]);
        dma_o.load(dOh + r0 * o_ld + ah * 64, sn.dOs[u][ah]);
      }
      // the 64 row terms of the tile, one dword per lane: waves 0/1 fetch -LSE / scale, 2/3 fetch -D
      if ((wave & 1) == (u & 1)) {
        if (wave < 2) lds_dma4(nLh + r0 + lane, sn.lse[u]);
        else lds_dma4(nDh + r0 + lane, sn.d[u]);
      }
    }
  };

  int i = i_begin;
  if (i < i_end && !visible(i)) i = advance(i);
  if (i < i_end) load_stage(i, stage0);
  wait_vmem();
  __syncthreads();
  // one stage: start the loads of the next stage into sn, compute on sc
  auto stage = [&](Stage &sc, Stage &sn) __attribute__((always_inline)) {
    const int inext = advance(i);
    if (inext < i_end) load_stage(inext, sn);

    // The 32 MFMAs of a tile go in four groups of eight -- S', dP' of rows 0..31 (G0) and of
    // rows 32..63 (G1), then dV, dK over rows 0..31 (H0) and 32..63 (H1) -- and the vector work
    // of each half (V0, V1) sits beside the next group: G0 | G1 + V0 | H0 + V1 | H1.  MFMA and
    // vector instructions of one wave overlap only when they alternate in its instruction
    // stream, and an LDS read costs its full latency unless issued a phase early, so the
    // phases are fenced, every read after the tile's first is issued one phase before its
    // use, and the compiler interleaves inside a phase.
    bf16x8 qa[2][4 * AH], ga[2][4 * AH];
    f32x16 sacc[2], dpacc[2];
    const int qt0 = st_of(i) * NQ;
    auto active = [&](int u) {
      const int qt = qt0 + u;
      return qt < nqt && (!CAUSAL || a.map((int64_t)qt * 64) + 63 >= wkey0);
    };
    auto fetch = [&](int u, int qb) __attribute__((always_inline)) {
      // accumulators start from -LSE / scale and -D of their rows (same for all lanes of a half)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4 l4 = *reinterpret_cast<const f32x4 *>(&sc.lse[u][qb * 32 + g * 8 + half * 4]);
        const f32x4 d4 = *reinterpret_cast<const f32x4 *>(&sc.d[u][qb * 32 + g * 8 + half * 4]);
#pragma unroll
        for (int e = 0; e < 4; ++e) { sacc[qb][g * 4 + e] = l4[e]; dpacc[qb][g * 4 + e] = d4[e]; }
      }
#pragma unroll
      for (int dk = 0; dk < 4 * AH; ++dk) {
        qa[qb][dk] = tl.read_rows(sc.Qt[u][dk >> 2], qb * 32, dk & 3);
        ga[qb][dk] = tl.read_rows(sc.dOs[u][dk >> 2], qb * 32, dk & 3);
      }
    };
#pragma unroll
    for (int u = 0; u < NQ; ++u) {
      if (active(u)) {
        const int64_t qf = a.map((int64_t)(qt0 + u) * 64);  // token of the tile's first row
        const bool domask = CAUSAL && qf < wkey0 + KW - 1;
        bf16x8 pf[4], sf[4];  // [kk]: P and dS as B operands, k = query
        auto g12 = [&](int qb) __attribute__((always_inline)) {
#pragma unroll
          for (int dk = 0; dk < 4 * AH; ++dk) {
            sacc[qb] = mfma_32x32x16(qa[qb][dk], kreg[dk], sacc[qb]);
            dpacc[qb] = mfma_32x32x16(ga[qb][dk], vreg[dk], dpacc[qb]);
          }
        };
        auto softmax_bwd = [&](int qb) __attribute__((always_inline)) {
          f32x16 &sv = sacc[qb];
          const f32x16 &dp = dpacc[qb];
          if (domask) {
            // first visible row of the lane's key, relative to the block of 32 rows (32-bit compare)
            const int64_t d64 = wkey0 + col - qf - qb * 32 - half * 4;
            const int dfirst = d64 < -64 ? -64 : (int)d64;
#pragma unroll
            for (int v = 0; v < 16; ++v)
              if ((v >> 2) * 8 + (v & 3) < dfirst) sv[v] = -INFINITY;
          }
#pragma unroll
          for (int w2 = 0; w2 < 2; ++w2) {
            u32x4 w, x;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float p0 = __builtin_amdgcn_exp2f(sv[w2 * 8 + 2 * e] * a.cl2);
              const float p1 = __builtin_amdgcn_exp2f(sv[w2 * 8 + 2 * e + 1] * a.cl2);
              w[e] = pack_bf16(p0, p1);
              x[e] = pack_bf16(p0 * dp[w2 * 8 + 2 * e], p1 * dp[w2 * 8 + 2 * e + 1]);
            }
            pf[qb * 2 + w2] = __builtin_bit_cast(bf16x8, w);
            sf[qb * 2 + w2] = __builtin_bit_cast(bf16x8, x);
          }
        };
        bf16x8 gt[2][2][2 * AH], qt2[2][2][2 * AH];  // [qb][kk & 1][db]: dO^T and Q^T fragments
        auto fetch_t = [&](int qb) __attribute__((always_inline)) {
#pragma unroll
          for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
            for (int db = 0; db < 2 * AH; ++db) {
              gt[qb][k2][db] = tl.read_cols(sc.dOs[u][db >> 1], (qb * 2 + k2) * 16, db & 1);
              qt2[qb][k2][db] = tl.read_cols(sc.Qt[u][db >> 1], (qb * 2 + k2) * 16, db & 1);
            }
        };
        auto g34 = [&](int qb) __attribute__((always_inline)) {
#pragma unroll
          for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
            for (int db = 0; db < 2 * AH; ++db) {
              dv[db] = mfma_32x32x16(gt[qb][k2][db], pf[qb * 2 + k2], dv[db]);
              dk_[db] = mfma_32x32x16(qt2[qb][k2][db], sf[qb * 2 + k2], dk_[db]);
            }
        };
        // without a mask the tiles of a stage are all walked, and the first reads of every tile
        // after the stage's first were issued beside the previous tile's last MFMA group
        if (CAUSAL || u == 0) fetch(u, 0);
        __builtin_amdgcn_sched_barrier(0);
        fetch(u, 1);
        g12(0);
        __builtin_amdgcn_sched_barrier(0);
        fetch_t(0);
        g12(1);
        softmax_bwd(0);
        __builtin_amdgcn_sched_barrier(0);
        fetch_t(1);
        g34(0);
        softmax_bwd(1);
        __builtin_amdgcn_sched_barrier(0);
        // the first reads of the stage's next tile go beside this tile's last eight MFMAs
        // (their registers are free again), so that tile does not start by waiting for LDS
        // (past the end of the rows the tile is not walked and what was read is dropped)
        if (!CAUSAL && u + 1 < NQ) fetch(u + 1, 0);
        g34(1);
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    wait_vmem();
    __syncthreads();
    i = inext;
  };
  while (i < i_end) {
    stage(stage0, stage1);
    if (i >= i_end) break;
    stage(stage1, stage0);
  }

  if (gridDim.y > 1) {  // fp32 partial sums: [dV | dK][split][head][key][64]
    const int64_t heads = gridDim.x / a.tiles_per_head;
    const int64_t key = wkey0 + col;
    float *pv = a.part + (((int64_t)blockIdx.y * heads + head) * a.L + key) * A;
    float *pk = pv + (int64_t)gridDim.y * heads * a.L * A;
    if (key < a.L) {
#pragma unroll
      for (int db = 0; db < 2 * AH; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int off = db * 32 + g * 8 + half * 4;
          const f32x4 w = {dv[db][g * 4 + 0], dv[db][g * 4 + 1], dv[db][g * 4 + 2], dv[db][g * 4 + 3]};
          *reinterpret_cast<f32x4 *>(pv + off) = w;
          const f32x4 x = {dk_[db][g * 4 + 0] * a.scale, dk_[db][g * 4 + 1] * a.scale,
                           dk_[db][g * 4 + 2] * a.scale, dk_[db][g * 4 + 3] * a.scale};
          *reinterpret_cast<f32x4 *>(pk + off) = x;
        }
    }
    return;
  }

  // the wave's 32 x 64 blocks of dV and dK leave through its own LDS tile as whole 128-byte rows
  // (every wave is past the loop's last barrier and no load is in flight: the buffers are free)
  unsigned char *ot = wave < 2 ? stage0.Qt[wave][0] : stage0.dOs[wave - 2][0];
#pragma unroll
  for (int ah = 0; ah < AH; ++ah) {  // one half of the head at a time through the wave's tile
    stage_block_T(ot, 0, dv[2 * ah], dv[2 * ah + 1], 1.0f, lane);
    stage_block_T(ot, 32, dk_[2 * ah], dk_[2 * ah + 1], a.scale, lane);
    flush_rows<32>(ot, 0, a.dV + kv_off + wkey0 * kv_ld + ah * 64, a.L - wkey0, lane, (int)kv_ld);
    flush_rows<32>(ot, 32, a.dK + kv_off + wkey0 * kv_ld + ah * 64, a.L - wkey0, lane, (int)kv_ld);
  }
}

// ---------------------------------------------------------------------- dQ ---
template <int R, bool CAUSAL, bool PRE, int AH, int NK>  // NK: key tiles per stage (one barrier per stage)
__global__ void __launch_bounds__(256, R == 64 ? 1 : 2) fused_bwd_dq_kernel(BwdArgs a) {
  constexpr int QB = R / 32;
  constexpr int BM = 4 * R;
  constexpr int A = 64 * AH;  // a head of 128 is two halves of 64: two LDS tiles per 64 keys
  // two named stage buffers: see the dK/dV kernel
  __shared__ __attribute__((aligned(16))) unsigned char Ks0[NK][AH][kTileBytes], Ks1[NK][AH][kTileBytes];
  __shared__ __attribute__((aligned(16))) unsigned char Vs0[NK][AH][kTileBytes], Vs1[NK][AH][kTileBytes];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31, half = lane >> 5;
  const uint32_t wg = xcd_remap(blockIdx.x, gridDim.x, blockIdx.y);
  const int64_t head = wg / a.tiles_per_head;
  // under the causal mask later rows see more keys: the long work-groups of a head start first
  const int64_t row0 =
      (CAUSAL ? a.tiles_per_head - 1 - wg % a.tiles_per_head : wg % a.tiles_per_head) * BM;
  const int n = (a.map.rb + (int)(row0 / a.c)) % a.N;  // rank that owns the first row (see the forward)
  // last token any row of the work-group may look at (its 64-row tiles are runs of tokens)
  int64_t q_last = 0;
#pragma unroll
  for (int i = 0; i < BM / 64; ++i)
    if (row0 + i * 64 < a.Lq) {
      const int64_t e = a.map(row0 + i * 64) + 63;
      q_last = e > q_last ? e : q_last;
    }
  // tiles per run of consecutive tokens of a chunk: the chunk, or its half under zig-zag ownership
  const int tpc = (int)(a.c / kTileKeys);
  const int tpr = a.map.zigzag ? tpc / 2 : tpc;

  const int64_t kv_off = head_offset(head, a.Z, a.ks), q_off = head_offset(head, a.Z, a.qs);
  const int64_t o_off = head_offset(head, a.Z, a.os);
  const uint16_t *Qh = a.Q + q_off;
  const uint16_t *dOh = a.dO + o_off;
  const uint16_t *Kh = a.K + kv_off;
  const uint16_t *Vh = a.V + kv_off;
  const int64_t q_ld = a.qs[2], kv_ld = a.ks[2], o_ld = a.os[2];

  // Q and dO as B operands; -LSE / scale and -D of the lane's row, broadcast
  // over an accumulator, are what S'^T and dP'^T start from.
  bf16x8 qreg[QB][4 * AH], greg[QB][4 * AH];
  int64_t qrow[QB];
  int64_t qtok[QB];  // global token index of the lane's row
  f32x16 negl[QB], negd[QB];
  // first and last token of this wave's rows (R <= 64 rows inside one tile: a run of tokens)
  const int64_t wrow = row0 + wave * R < a.Lq ? row0 + wave * R : a.Lq - R;
  const int64_t wq_first = a.map(wrow);
  const int64_t wq_last = wq_first + R - 1;

  const TileLanes tl(lane);

  f32x16 dq[2 * AH][QB];
#pragma unroll
  for (int db = 0; db < 2 * AH; ++db)
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int v = 0; v < 16; ++v) dq[db][qb][v] = 0.f;

  // The ring walk: ring step t visits chunk (n - t) mod N.  Tiles are taken NK at a time;
  // a stage never straddles chunks when tiles-per-chunk is even, otherwise NK falls to 1.
  const int nk = (tpr % NK == 0) ? NK : 1;
  const int spc = tpc / nk;  // stages per chunk
  // the walk's stages, numbered t * spc + ks, divided over gridDim.y work-groups (see the forward)
  const int per_split = (a.N * spc + (int)gridDim.y - 1) / (int)gridDim.y;
  const int f_begin = (int)blockIdx.y * per_split;
  const int f_end = f_begin + per_split < a.N * spc ? f_begin + per_split : a.N * spc;
  auto k0_of = [&](int t, int ks) -> int64_t {
    int j = n - t;
    if (j < 0) j += a.N;
    return a.map.key_of(j, (int64_t)ks * nk * kTileKeys);
  };
  auto advance = [&](int &t, int &ks) -> bool {
    ++ks;
    for (;;) {
      if (ks >= spc) { ++t; ks = 0; }
      if (t * spc + ks >= f_end) return false;
      if (!CAUSAL || k0_of(t, ks) <= q_last) return true;
      ks = spc;
    }
  };
  const TileDMA dma(wave, lane, (int)kv_ld);
  auto load_stage = [&](int64_t k0, auto &Kn, auto &Vn) __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < NK; ++u) {
      if (u < nk) {
#pragma unroll
        for (int ah = 0; ah < AH; ++ah) {
          dma.load(Kh + (k0 + u * kTileKeys) * kv_ld + ah * 64, Kn[u][ah]);
          dma.load(Vh + (k0 + u * kTileKeys) * kv_ld + ah * 64, Vn[u][ah]);
        }
      }
    }
  };

  int t = f_begin / spc, kt = f_begin % spc;
  bool have = f_begin < f_end;
  if (CAUSAL && have && k0_of(t, kt) > q_last) have = advance(t, kt);
  if (have) load_stage(k0_of(t, kt), Ks0, Vs0);
  // The rows this wave keeps in registers are fetched after the first stage's tiles are on their
  // way, so that the two latencies overlap (short walks, e.g. a few hundred projected keys, are
  // mostly prologue).
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int64_t r = row0 + wave * R + qb * 32 + col;
    qrow[qb] = r < a.Lq ? r : a.Lq - 1;
    const int64_t blk = row0 + wave * R + qb * 32;  // the block of 32 rows is whole or absent
    qtok[qb] = a.map(blk < a.Lq ? blk : a.Lq - 32) + col;
#pragma unroll
    for (int dk = 0; dk < 4 * AH; ++dk) {
      qreg[qb][dk] = *reinterpret_cast<const bf16x8 *>(Qh + qrow[qb] * q_ld + dk * 16 + half * 8);
      greg[qb][dk] = *reinterpret_cast<const bf16x8 *>(dOh + qrow[qb] * o_ld + dk * 16 + half * 8);
    }
    float l2, dd;
    if (PRE) {
      // D = sum_a dO_a O_a: this lane holds half of the row's elements, the lane 32 away the rest
      float acc = 0.f;
#pragma unroll
      for (int dk = 0; dk < 4 * AH; ++dk) {
        const u32x4 x = __builtin_bit_cast(u32x4, greg[qb][dk]);
        const u32x4 y = *reinterpret_cast<const u32x4 *>(a.O + o_off + qrow[qb] * o_ld + dk * 16 + half * 8);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          acc = fmaf(bf16_to_f32(x[e] & 0xffffu), bf16_to_f32(y[e] & 0xffffu), acc);
          acc = fmaf(bf16_to_f32(x[e] >> 16), bf16_to_f32(y[e] >> 16), acc);
        }
      }
      dd = -xhalf_sum(acc);
      l2 = -a.LSE[head * a.Lq + qrow[qb]] * a.inv_scale;
      if (r < a.Lq && blockIdx.y == 0) {
        if (half == 0) {
          a.nD_out[head * a.Lq + r] = dd;
          a.nL_out[head * a.Lq + r] = l2;
        }
      }
    } else {
      l2 = a.nL[head * a.Lq + qrow[qb]];
      dd = a.nD[head * a.Lq + qrow[qb]];
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) { negl[qb][v] = l2; negd[qb][v] = dd; }
  }
  wait_vmem();
  __syncthreads();
  // one stage: start the loads of the next stage into (Kn, Vn), compute on (Kc, Vc)
  auto stage = [&](auto &Kc, auto &Vc, auto &Kn, auto &Vn) __attribute__((always_inline)) {
    const int64_t ks0 = k0_of(t, kt);
    int t2 = t, kt2 = kt;
    const bool have_next = advance(t2, kt2);
    if (have_next) load_stage(k0_of(t2, kt2), Kn, Vn);

#pragma unroll
    for (int u = 0; u < NK; ++u) {
    const int64_t k0 = ks0 + u * kTileKeys;
    if (u < nk && (!CAUSAL || k0 <= wq_last)) {
      const bool domask = CAUSAL && k0 + kTileKeys - 1 > wq_first;
      bf16x8 sf[QB][4];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        f32x16 s[QB], dp[QB];
#pragma unroll
        for (int dk = 0; dk < 4 * AH; ++dk) {
          const bf16x8 ka = tl.read_rows(Kc[u][dk >> 2], kb * 32, dk & 3);
          const bf16x8 va = tl.read_rows(Vc[u][dk >> 2], kb * 32, dk & 3);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) {
            s[qb] = mfma_32x32x16(ka, qreg[qb][dk], dk == 0 ? negl[qb] : s[qb]);
            dp[qb] = mfma_32x32x16(va, greg[qb][dk], dk == 0 ? negd[qb] : dp[qb]);
          }
        }
        if (domask) {  // uniform over the wave: only tiles on the diagonal pay for the mask
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) {
            // last visible key of the lane's row, relative to the block of 32 keys (32-bit compare)
            const int64_t d64 = qtok[qb] - k0 - kb * 32 - half * 4;
            const int dlast = d64 > 64 ? 64 : (int)d64;
#pragma unroll
            for (int v = 0; v < 16; ++v)
              if ((v >> 2) * 8 + (v & 3) > dlast) s[qb][v] = -INFINITY;
          }
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
          for (int v = 0; v < 16; ++v) dp[qb][v] *= __builtin_amdgcn_exp2f(s[qb][v] * a.cl2);
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            u32x4 w = {pack_bf16(dp[qb][u * 8 + 0], dp[qb][u * 8 + 1]), pack_bf16(dp[qb][u * 8 + 2], dp[qb][u * 8 + 3]),
                       pack_bf16(dp[qb][u * 8 + 4], dp[qb][u * 8 + 5]), pack_bf16(dp[qb][u * 8 + 6], dp[qb][u * 8 + 7])};
            sf[qb][kb * 2 + u] = __builtin_bit_cast(bf16x8, w);
          }
        }
      }
#pragma unroll
      for (int db = 0; db < 2 * AH; ++db)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          const bf16x8 ka = tl.read_cols(Kc[u][db >> 1], kk * 16, db & 1);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) dq[db][qb] = mfma_32x32x16(ka, sf[qb][kk], dq[db][qb]);
        }
    }

    }

    wait_vmem();
    __syncthreads();
    t = t2; kt = kt2; have = have_next;
  };
  while (have) {
    stage(Ks0, Vs0, Ks1, Vs1);
    if (!have) break;
    stage(Ks1, Vs1, Ks0, Vs0);
  }

  if (gridDim.y > 1) {  // fp32 partial sum of this split: [split][head][row][64]
    const int64_t heads = gridDim.x / a.tiles_per_head;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const int64_t r = row0 + wave * R + qb * 32 + col;
      if (r < a.Lq) {
        float *po = a.part + (((int64_t)blockIdx.y * heads + head) * a.Lq + r) * A + half * 4;
#pragma unroll
        for (int db = 0; db < 2 * AH; ++db)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const f32x4 w = {dq[db][qb][g * 4 + 0] * a.scale, dq[db][qb][g * 4 + 1] * a.scale,
                             dq[db][qb][g * 4 + 2] * a.scale, dq[db][qb][g * 4 + 3] * a.scale};
            *reinterpret_cast<f32x4 *>(po + db * 32 + g * 8) = w;
          }
      }
    }
    return;
  }

  // the wave's R x 64 block of dQ leaves through its own LDS tile as whole 128-byte rows
  unsigned char *ot = wave == 0 ? Ks0[0][0] : (wave == 1 ? Ks1[0][0] : (wave == 2 ? Vs0[0][0] : Vs1[0][0]));
  const int64_t wr0 = row0 + wave * R;
#pragma unroll
  for (int ah = 0; ah < AH; ++ah) {  // one half of the head at a time through the wave's tile
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) stage_block_T(ot, qb * 32, dq[2 * ah][qb], dq[2 * ah + 1][qb], a.scale, lane);
    flush_rows<R>(ot, 0, a.dQ + q_off + wr0 * q_ld + ah * 64, a.Lq - wr0, lane, (int)q_ld);
  }
}

// out (bf16) = sum over the splits of part[s][i], in a fixed order; n4 groups of four per split
// (the partial sums are dense (head, row, A); `lay` says where a row of the output tensor lives)
__global__ void __launch_bounds__(256) qsplit_reduce_kernel(const float *part, uint16_t *out, int64_t n4,
                                                            int splits, int A, OutLayout lay) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  f32x4 s = reinterpret_cast<const f32x4 *>(part)[i];
  for (int k = 1; k < splits; ++k) s += reinterpret_cast<const f32x4 *>(part)[(int64_t)k * n4 + i];
  const u32x2 w = {pack_bf16(s[0], s[1]), pack_bf16(s[2], s[3])};
  const int64_t e = i * 4;
  *reinterpret_cast<u32x2 *>(out + lay.row_off(e / A) + e % A) = w;
}

static BwdArgs make_bwd_args(const Dims &d, const void *dO, const void *Q, const void *K,
                             const void *V, const float *nL, const float *nD, void *dQ, void *dK,
                             void *dV) {
  BwdArgs a;
  a.Q = (const uint16_t *)Q;
  a.K = (const uint16_t *)K; a.V = (const uint16_t *)V;
  a.dO = (const uint16_t *)dO; a.nL = nL; a.nD = nD;
  a.dQ = (uint16_t *)dQ; a.dK = (uint16_t *)dK; a.dV = (uint16_t *)dV;
  a.part = nullptr;
  a.O = nullptr; a.LSE = nullptr; a.nL_out = nullptr; a.nD_out = nullptr;
  a.L = d.L; a.c = d.c; a.Lq = d.Lq; a.map = make_row_map(d);
  a.N = d.N; a.Z = d.Z; a.cl2 = d.scale * kLog2e; a.scale = d.scale; a.inv_scale = 1.0f / d.scale;
  for (int k = 0; k < 3; ++k) { a.qs[k] = d.qs[k]; a.ks[k] = d.ks[k]; a.os[k] = d.os[k]; }
  a.tiles_per_head = 0;
  return a;
}

hipError_t fused_bwd_preprocess(const Dims &d, const void *dO, const void *O, const float *LSE,
                                float *nD, float *nL, hipStream_t st) {
  const int64_t rows = (int64_t)d.B * d.Z * d.Lq;
  dim3 grid((unsigned)((rows * 8 + 255) / 256));
  hipLaunchKernelGGL(bwd_preprocess_kernel, grid, dim3(256), 0, st, (const uint16_t *)dO,
                     (const uint16_t *)O, LSE, nD, nL, rows, d.A, 1.0f / d.scale,
                     make_out_layout(d.os, d.Lq, d.Z));
  return hipGetLastError();
}

hipError_t qsplit_reduce(const float *part, void *out, int64_t n4, int splits, int A, const OutLayout &lay,
                         hipStream_t st) {
  hipLaunchKernelGGL(qsplit_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st, part,
                     (uint16_t *)out, n4, splits, A, lay);
  return hipGetLastError();
}

int fused_bwd_dkdv_splits(const Dims &d) {
  const int64_t wgs = (int64_t)d.B * d.Z * ((d.L + 127) / 128), stages = (d.Lq / 64 + 1) / 2;
  int64_t s = 1024 / wgs;  // aim at two work-groups per CU's worth of them
  if (s > stages / 8) s = stages / 8;
  if (s > 64) s = 64;
  return s < 2 ? 1 : (int)s;
}

hipError_t fused_bwd_dkdv(const Dims &d, const void *dO, const void *Q, const void *K,
                          const void *V, const float *nL, const float *nD, void *dK, void *dV,
                          hipStream_t st, float *part, int splits) {
  BwdArgs a = make_bwd_args(d, dO, Q, K, V, nL, nD, nullptr, dK, dV);
  a.tiles_per_head = (int)((d.L + 127) / 128);
  a.part = part;
  if (!part) splits = 1;
  dim3 grid((unsigned)((int64_t)d.B * d.Z * a.tiles_per_head), (unsigned)splits);
  if (d.A == 128) {
    if (d.causal)
      hipLaunchKernelGGL((fused_bwd_dkdv_kernel<2, true, 2>), grid, dim3(256), 0, st, a);
    else
      hipLaunchKernelGGL((fused_bwd_dkdv_kernel<2, false, 2>), grid, dim3(256), 0, st, a);
  } else if (d.causal) {
    hipLaunchKernelGGL((fused_bwd_dkdv_kernel<2, true, 1>), grid, dim3(256), 0, st, a);
  } else {
    hipLaunchKernelGGL((fused_bwd_dkdv_kernel<2, false, 1>), grid, dim3(256), 0, st, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || splits == 1) return e;
  const int64_t n4 = (int64_t)d.B * d.Z * d.L * (d.A / 4);
  const dim3 rg((unsigned)((n4 + 255) / 256));
  const OutLayout lay = make_out_layout(d.ks, d.L, d.Z);
  hipLaunchKernelGGL(qsplit_reduce_kernel, rg, dim3(256), 0, st, part, (uint16_t *)dV, n4, splits, d.A, lay);
  hipLaunchKernelGGL(qsplit_reduce_kernel, rg, dim3(256), 0, st, part + (int64_t)splits * n4 * 4,
                     (uint16_t *)dK, n4, splits, d.A, lay);
  return hipGetLastError();
}

template <bool PRE>
static void launch_dq(const Dims &d, const BwdArgs &a, dim3 grid, hipStream_t st) {
  if (d.A == 128) {  // one key tile (two LDS tiles) per stage
    if (d.causal)
      hipLaunchKernelGGL((fused_bwd_dq_kernel<32, true, PRE, 2, 1>), grid, dim3(256), 0, st, a);
    else
      hipLaunchKernelGGL((fused_bwd_dq_kernel<32, false, PRE, 2, 1>), grid, dim3(256), 0, st, a);
  } else if (d.causal) {
    hipLaunchKernelGGL((fused_bwd_dq_kernel<32, true, PRE, 1, 2>), grid, dim3(256), 0, st, a);
  } else {
    hipLaunchKernelGGL((fused_bwd_dq_kernel<32, false, PRE, 1, 2>), grid, dim3(256), 0, st, a);
  }
}

// dQ = sum of the split walks' partial sums
static hipError_t dq_reduce(const Dims &d, const float *part, void *dQ, int splits, hipStream_t st) {
  const int64_t n4 = (int64_t)d.B * d.Z * d.Lq * (d.A / 4);
  hipLaunchKernelGGL(qsplit_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st, part,
                     (uint16_t *)dQ, n4, splits, d.A, make_out_layout(d.qs, d.Lq, d.Z));
  return hipGetLastError();
}

hipError_t fused_bwd_dq(const Dims &d, const void *dO, const void *Q, const void *K, const void *V,
                        const float *nL, const float *nD, void *dQ, hipStream_t st, float *part,
                        int splits) {
  BwdArgs a = make_bwd_args(d, dO, Q, K, V, nL, nD, dQ, nullptr, nullptr);
  a.tiles_per_head = (int)((d.Lq + 127) / 128);
  a.part = part;
  if (!part) splits = 1;
  dim3 grid((unsigned)((int64_t)d.B * d.Z * a.tiles_per_head), (unsigned)splits);
  launch_dq<false>(d, a, grid, st);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || splits == 1) return e;
  return dq_reduce(d, part, dQ, splits, st);
}

// The dQ kernel with the preprocess in its prologue: also writes -D and -LSE / scale.
hipError_t fused_bwd_dq_pre(const Dims &d, const void *dO, const void *Q, const void *K, const void *V,
                            const void *O, const float *LSE, float *nL, float *nD, void *dQ,
                            hipStream_t st, float *part, int splits) {
  BwdArgs a = make_bwd_args(d, dO, Q, K, V, nullptr, nullptr, dQ, nullptr, nullptr);
  a.O = (const uint16_t *)O; a.LSE = LSE; a.nL_out = nL; a.nD_out = nD;
  a.tiles_per_head = (int)((d.Lq + 127) / 128);
  a.part = part;
  if (!part) splits = 1;
  dim3 grid((unsigned)((int64_t)d.B * d.Z * a.tiles_per_head), (unsigned)splits);
  launch_dq<true>(d, a, grid, st);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || splits == 1) return e;
  return dq_reduce(d, part, dQ, splits, st);
}

hipError_t fused_backward(const Dims &d, const void *dO, const void *Q, const void *K,
                          const void *V, const void *O, const float *LSE, void *dQ, void *dK,
                          void *dV, float *nD, float *nL, hipStream_t st, float *part,
                          int qsplits, int ksplits) {
  // the dQ kernel first: its prologue forms the row terms that the dK/dV kernel reads;
  // the two kernels' partial sums share `part`, one after the other.  (With heads of 128 the
  // prologue costs the dQ kernel more registers than it has: there the row terms come from
  // the preprocess kernel.)
  hipError_t e;
  if (d.A == 128) {
    e = fused_bwd_preprocess(d, dO, O, LSE, nD, nL, st);
    if (e != hipSuccess) return e;
    e = fused_bwd_dq(d, dO, Q, K, V, nL, nD, dQ, st, part, ksplits);
  } else {
    e = fused_bwd_dq_pre(d, dO, Q, K, V, O, LSE, nL, nD, dQ, st, part, ksplits);
  }
  if (e != hipSuccess) return e;
  return fused_bwd_dkdv(d, dO, Q, K, V, nL, nD, dK, dV, st, part, qsplits);
}

}  // namespace rsa
