// Fused Ring Self-Attention forward (bf16, A = 64 or 128).
//
// One work-group owns 4*R query rows of one head and walks the K/V chunks in
// ring order -- step t of rank n visits chunk j = (n - t) mod N, local chunk
// first (section 3.1) -- keeping a running row max and row sum, so the score
// strip S^n of Table 2 never reaches device memory.  The result is Eq. 1 /
// Eq. 3 exactly, up to summation order.
//
// K/V tiles reach LDS by direct global->LDS loads, two tiles per stage, double-buffered,
// one work-group barrier per stage.
//
// A head of 128 elements is handled as AH = 2 halves of 64: a 64-key tile is then two LDS tiles,
// the S^T contraction runs over both, and O^T has twice the accumulators.
//
// Data flow per 64-key tile and wave (R query rows):
//   S^T = K Q^T    A operand: K tile rows from LDS, B operand: Q^T in registers
//   softmax update on S^T: lane l owns query column l%32, so the row max and
//                  row sum are in-lane reductions plus one cross-half exchange
//   O^T += V^T P^T A operand: V^T through LDS transpose reads, B operand: P^T
//                  straight from the S^T accumulator registers (packed to bf16)
#include "rsa_fused_tile.h"
#include "rsa_kernels.h"

namespace rsa {

struct FwdArgs {
  const uint16_t *Q, *K, *V;
  uint16_t *O;
  float *LSE;
  int64_t L, c, Lq;
  int64_t qs[3], ks[3], os[3];  // element strides (batch, head, row) of Q; K and V; O
  RowMap map;            // local query row -> global token index
  int N, Z, tiles_per_head;
  float cl2;             // scale * log2(e)
  // split key walk (gridDim.y > 1): per split, head and row the unnormalised fp32 O and the pair
  // (stale max * cl2, row sum) it is relative to
  float *part_o, *part_ml;
};

template <int R, bool CAUSAL, int AH, int NK>  // NK: key tiles per stage (one barrier per stage)
__global__ void __launch_bounds__(256, (R == 32 && NK == 1 && AH == 1) ? 4 : 2) fused_fwd_kernel(FwdArgs a) {
  constexpr int QB = R / 32;
  constexpr int BM = 4 * R;
  constexpr int A = 64 * AH;
  // The two stage buffers are separate objects, each addressed by name: the compiler then
  // knows that a direct load into one buffer cannot alias the LDS reads of the other and
  // does not wait for the load before them.
  __shared__ __attribute__((aligned(16))) unsigned char Ks0[NK][AH][kTileBytes], Ks1[NK][AH][kTileBytes];
  __shared__ __attribute__((aligned(16))) unsigned char Vs0[NK][AH][kTileBytes], Vs1[NK][AH][kTileBytes];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31, half = lane >> 5;
  const uint32_t wg = xcd_remap(blockIdx.x, gridDim.x, blockIdx.y);
  const int64_t head = wg / a.tiles_per_head;
  // under the causal mask later rows see more keys: the long work-groups of a head start first
  const int64_t qt = CAUSAL ? a.tiles_per_head - 1 - wg % a.tiles_per_head : wg % a.tiles_per_head;
  const int64_t row0 = qt * BM;  // first local row of this work-group
  // rank that owns the first row (modulo N: with projected keys, Table 3, the rows are not
  // tokens of the key sequence and any chunk may come first)
  const int n = (a.map.rb + (int)(row0 / a.c)) % a.N;
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

  const int64_t kv_off = head_offset(head, a.Z, a.ks);
  const uint16_t *Qh = a.Q + head_offset(head, a.Z, a.qs);
  const uint16_t *Kh = a.K + kv_off;
  const uint16_t *Vh = a.V + kv_off;
  const int64_t q_ld = a.qs[2], kv_ld = a.ks[2], o_ld = a.os[2];

  // Q^T operand: lane (col, half) holds Q[row][dk*16 + half*8 .. +8]
  bf16x8 qreg[QB][4 * AH];
  int64_t qrow[QB];  // local row (clamped to the last row for a ragged tail)
  int64_t qtok[QB];  // its global token index
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    int64_t r = row0 + wave * R + qb * 32 + col;
    qrow[qb] = r < a.Lq ? r : a.Lq - 1;
    const int64_t blk = row0 + wave * R + qb * 32;  // the block of 32 rows is whole or absent
    qtok[qb] = a.map(blk < a.Lq ? blk : a.Lq - 32) + col;
#pragma unroll
    for (int dk = 0; dk < 4 * AH; ++dk)
      qreg[qb][dk] = *reinterpret_cast<const bf16x8 *>(Qh + qrow[qb] * q_ld + dk * 16 + half * 8);
  }
  // first and last token of this wave's rows (R <= 64 rows inside one tile: a run of tokens)
  const int64_t wrow = row0 + wave * R < a.Lq ? row0 + wave * R : a.Lq - R;
  const int64_t wq_first = a.map(wrow);
  const int64_t wq_last = wq_first + R - 1;

  const TileLanes tl(lane);

  f32x16 o[2 * AH][QB];
  float m[QB], mc[QB], l[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m[qb] = -INFINITY; mc[qb] = 0.f; l[qb] = 0.f;
#pragma unroll
    for (int db = 0; db < 2 * AH; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[db][qb][v] = 0.f;
  }

  // The ring walk: ring step t visits chunk (n - t) mod N.  Tiles are taken NK at a time;
  // a stage never straddles chunks when tiles-per-chunk is even, otherwise NK falls to 1.
  const int nk = (tpr % NK == 0) ? NK : 1;
  const int spc = tpc / nk;  // stages per chunk
  // With few work-groups the walk's stages, numbered t * spc + ks, are divided over gridDim.y
  // work-groups, each leaving an unnormalised partial result that a second kernel merges.
  const int per_split = (a.N * spc + (int)gridDim.y - 1) / (int)gridDim.y;
  const int f_begin = (int)blockIdx.y * per_split;
  const int f_end = f_begin + per_split < a.N * spc ? f_begin + per_split : a.N * spc;
  auto k0_of = [&](int t, int ks) -> int64_t {
    int j = n - t;
    if (j < 0) j += a.N;
    return a.map.key_of(j, (int64_t)ks * nk * kTileKeys);
  };
  // next stage of the ring walk that holds a visible key for some row of this work-group
  auto advance = [&](int &t, int &ks) -> bool {
    ++ks;
    for (;;) {
      if (ks >= spc) { ++t; ks = 0; }
      if (t * spc + ks >= f_end) return false;
      if (!CAUSAL || k0_of(t, ks) <= q_last) return true;
      ks = spc;  // later stages of this chunk start even further right
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
      // ---- S^T = K Q^T
      f32x16 s[2][QB];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        bf16x8 ka[4 * AH];
#pragma unroll
        for (int dk = 0; dk < 4 * AH; ++dk) ka[dk] = tl.read_rows(Kc[u][dk >> 2], kb * 32, dk & 3);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
          for (int v = 0; v < 16; ++v) s[kb][qb][v] = 0.f;
#pragma unroll
          for (int dk = 0; dk < 4 * AH; ++dk) s[kb][qb] = mfma_32x32x16(ka[dk], qreg[qb][dk], s[kb][qb]);
        }
      }
      if (CAUSAL && k0 + kTileKeys - 1 > wq_first) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          // last visible key of the lane's row, relative to the tile (clamped: 32-bit compare)
          const int64_t d64 = qtok[qb] - k0 - half * 4;
          const int dlast = d64 > 64 ? 64 : (int)d64;
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v)
              if (kb * 32 + (v >> 2) * 8 + (v & 3) > dlast) s[kb][qb][v] = -INFINITY;
        }
      }
      // ---- running max; the accumulators are rescaled only when some row's max
      // grew by more than 2^8 in the exp2 domain (exact: l and O share the stale max)
      float tm[QB];
      bool need = false;
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        float x = s[0][qb][0];
#pragma unroll
        for (int v = 1; v < 16; ++v) x = fmaxf(x, s[0][qb][v]);
#pragma unroll
        for (int v = 0; v < 16; ++v) x = fmaxf(x, s[1][qb][v]);
        tm[qb] = xhalf_max(x);
        need |= (tm[qb] - m[qb]) * a.cl2 > 8.0f;
      }
      if (__builtin_amdgcn_ballot_w64(need) != 0) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          // a row that has seen no key yet (a split walk can start right of it) keeps mc = 0
          const float mn = fmaxf(m[qb], tm[qb]);
          const bool seen = mn > -INFINITY;
          const float alpha = seen ? __builtin_amdgcn_exp2f((m[qb] - mn) * a.cl2) : 1.0f;
          m[qb] = mn;
          mc[qb] = seen ? mn * a.cl2 : 0.f;
          l[qb] *= alpha;
#pragma unroll
          for (int db = 0; db < 2 * AH; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[db][qb][v] *= alpha;
        }
      }
      // ---- P^T = exp2(S^T cl2 - m cl2), packed to bf16 as the B operand
      bf16x8 pf[QB][4];
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        float ls = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          float p[16];
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            p[v] = __builtin_amdgcn_exp2f(fmaf(s[kb][qb][v], a.cl2, -mc[qb]));
            ls += p[v];
          }
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            u32x4 w = {pack_bf16(p[u * 8 + 0], p[u * 8 + 1]), pack_bf16(p[u * 8 + 2], p[u * 8 + 3]),
                       pack_bf16(p[u * 8 + 4], p[u * 8 + 5]), pack_bf16(p[u * 8 + 6], p[u * 8 + 7])};
            pf[qb][kb * 2 + u] = __builtin_bit_cast(bf16x8, w);
          }
        }
        l[qb] += ls;
      }
      // ---- O^T += V^T P^T
#pragma unroll
      for (int db = 0; db < 2 * AH; ++db)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          const bf16x8 va = tl.read_cols(Vc[u][db >> 1], kk * 16, db & 1);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) o[db][qb] = mfma_32x32x16(va, pf[qb][kk], o[db][qb]);
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

  if (gridDim.y > 1) {  // partial result of this split
    const int64_t heads = gridDim.x / a.tiles_per_head;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const float lt = xhalf_sum(l[qb]);
      const int64_t r = row0 + wave * R + qb * 32 + col;
      if (r < a.Lq) {
        const int64_t pr = ((int64_t)blockIdx.y * heads + head) * a.Lq + r;
        float *po = a.part_o + pr * A + half * 4;
#pragma unroll
        for (int db = 0; db < 2 * AH; ++db)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const f32x4 w = {o[db][qb][g * 4 + 0], o[db][qb][g * 4 + 1], o[db][qb][g * 4 + 2], o[db][qb][g * 4 + 3]};
            *reinterpret_cast<f32x4 *>(po + db * 32 + g * 8) = w;
          }
        if (half == 0) {
          a.part_ml[pr * 2] = lt > 0.f ? mc[qb] : -INFINITY;
          a.part_ml[pr * 2 + 1] = lt;
        }
      }
    }
    return;
  }

  // ---- epilogue: O = O^T / l, LSE = s m + ln l.  The wave's R x 64 block of O goes through its
  // own LDS tile (every wave is past the loop's last barrier and no load is in flight, so the
  // stage buffers are free) and leaves as whole 128-byte rows.
  unsigned char *ot = wave == 0 ? Ks0[0][0] : (wave == 1 ? Ks1[0][0] : (wave == 2 ? Vs0[0][0] : Vs1[0][0]));
  float inv[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float lt = xhalf_sum(l[qb]);
    inv[qb] = 1.0f / lt;
    const int64_t r = row0 + wave * R + qb * 32 + col;
    if (r < a.Lq && half == 0) a.LSE[head * a.Lq + r] = (mc[qb] + __builtin_amdgcn_logf(lt)) * kLn2;
  }
  const int64_t wr0 = row0 + wave * R;
#pragma unroll
  for (int ah = 0; ah < AH; ++ah) {  // one half of the head at a time through the wave's tile
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) stage_block_T(ot, qb * 32, o[2 * ah][qb], o[2 * ah + 1][qb], inv[qb], lane);
    flush_rows<R>(ot, 0, a.O + head_offset(head, a.Z, a.os) + wr0 * o_ld + ah * 64, a.Lq - wr0, lane, (int)o_ld);
  }
}

// Merge of the split walks' partial results: with M the largest stale max of a row,
// O = sum_s 2^(mc_s - M) o_s / sum_s 2^(mc_s - M) l_s and LSE = (M + log2 of that denominator) ln 2.
// A split that saw no key of the row has mc = -inf and is left out.  A/4 lanes x 4 columns per row.
__global__ void __launch_bounds__(256) fwd_combine_kernel(const float *part_o, const float *part_ml,
                                                          uint16_t *O, float *LSE, int64_t rows, int splits,
                                                          int A, OutLayout lay) {
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int lanes = A >> 2;
  const int64_t row = gid / lanes;
  const int sub = (int)(gid % lanes);
  if (row >= rows) return;
  float M = -INFINITY;
  for (int s = 0; s < splits; ++s) M = fmaxf(M, part_ml[((int64_t)s * rows + row) * 2]);
  float lsum = 0.f;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < splits; ++s) {
    const int64_t pr = (int64_t)s * rows + row;
    const float mc = part_ml[pr * 2];
    if (mc > -INFINITY) {
      const float w = __builtin_amdgcn_exp2f(mc - M);
      lsum = fmaf(w, part_ml[pr * 2 + 1], lsum);
      acc += *reinterpret_cast<const f32x4 *>(part_o + pr * A + sub * 4) * w;
    }
  }
  const float inv = 1.0f / lsum;
  const u32x2 w = {pack_bf16(acc[0] * inv, acc[1] * inv), pack_bf16(acc[2] * inv, acc[3] * inv)};
  *reinterpret_cast<u32x2 *>(O + lay.row_off(row) + sub * 4) = w;
  if (sub == 0) LSE[row] = (M + __builtin_amdgcn_logf(lsum)) * kLn2;
}

template <int R, int AH, int NK>
static hipError_t launch_fwd(const Dims &d, const FwdArgs &a, int64_t heads, int splits, hipStream_t st) {
  dim3 grid((unsigned)(heads * a.tiles_per_head), (unsigned)splits);
  if (d.causal)
    hipLaunchKernelGGL((fused_fwd_kernel<R, true, AH, NK>), grid, dim3(256), 0, st, a);
  else
    hipLaunchKernelGGL((fused_fwd_kernel<R, false, AH, NK>), grid, dim3(256), 0, st, a);
  return hipGetLastError();
}

// Splits of the key walk for a kernel whose work-groups own `rows_per_wg` query rows (two
// work-groups per CU make 512 slots): 1 when the rows alone fill the chip.  Otherwise the smallest count whose work-groups fill whole rounds of the 512 slots
// to 95 % -- a round that is half empty costs as much as a full one -- with at least 16 stages
// of 128 keys left per split (shorter walks lose more to their prologue and to the merge than
// the better fill gains).  Under the causal mask walks differ in length, so at least three
// rounds are wanted; under zig-zag ownership half of the row tiles see almost no keys and do
// not count.  When no count qualifies, the largest one allowed.
static int key_splits_for(const Dims &d, int rows_per_wg) {
  int64_t wgs = (int64_t)d.B * d.Z * ((d.Lq + rows_per_wg - 1) / rows_per_wg);
  if (wgs >= 1024) return 1;
  int64_t stages = d.L / 128;  // the longest walk of a row tile
  if (d.causal && !d.zigzag && (int64_t)d.rank_end * d.c / 128 < stages) stages = (int64_t)d.rank_end * d.c / 128;
  const int64_t smax = stages / 16 < 32 ? stages / 16 : 32;
  if (smax < 2) return 1;
  if (d.causal && d.zigzag) wgs = (wgs + 1) / 2;
  const int64_t min_rounds = d.causal ? 3 : 1;
  for (int64_t s = 1; s <= smax; ++s) {
    const int64_t n = s * wgs, rounds = (n + 511) / 512;
    if (rounds >= min_rounds && n * 20 >= rounds * 512 * 19) return (int)s;
  }
  return (int)smax;
}

// the dQ kernel: 128 rows per work-group
int fused_key_splits(const Dims &d) { return key_splits_for(d, 128); }

// The forward: 64 rows per wave (256 per work-group) halve the LDS traffic per flop and are
// taken when their work-groups, times their splits, fill the 512 slots at least once; else 32
// rows per wave, which give twice the work-groups.  (A head of 128 elements takes 32 rows per
// wave and one key tile per stage: registers and LDS.)
void fused_fwd_plan(const Dims &d, bool *big, int *splits) {
  if (d.A == 64 && d.Lq % 256 == 0) {
    const int s = key_splits_for(d, 256);
    if ((int64_t)d.B * d.Z * (d.Lq / 256) * s >= 512) {
      *big = true; *splits = s;
      return;
    }
  }
  *big = false; *splits = key_splits_for(d, 128);
}

hipError_t fused_forward(const Dims &d, const void *Q, const void *K, const void *V, void *O,
                         float *LSE, hipStream_t st, float *part) {
  FwdArgs a;
  a.Q = (const uint16_t *)Q; a.K = (const uint16_t *)K; a.V = (const uint16_t *)V;
  a.O = (uint16_t *)O; a.LSE = LSE;
  a.L = d.L; a.c = d.c; a.Lq = d.Lq; a.map = make_row_map(d);
  a.N = d.N; a.Z = d.Z;
  for (int k = 0; k < 3; ++k) { a.qs[k] = d.qs[k]; a.ks[k] = d.ks[k]; a.os[k] = d.os[k]; }
  a.cl2 = d.scale * kLog2e;
  const int64_t heads = (int64_t)d.B * d.Z;
  bool big;
  int splits;
  fused_fwd_plan(d, &big, &splits);
  if (!part) splits = 1;
  const int64_t rows = heads * d.Lq;
  a.part_o = part;
  a.part_ml = part ? part + (int64_t)splits * rows * d.A : nullptr;
  a.tiles_per_head = big ? (int)(d.Lq / 256) : (int)((d.Lq + 127) / 128);
  hipError_t e = d.A == 128 ? launch_fwd<32, 2, 1>(d, a, heads, splits, st)
                 : big      ? launch_fwd<64, 1, 2>(d, a, heads, splits, st)
                            : launch_fwd<32, 1, 1>(d, a, heads, splits, st);
  if (e != hipSuccess || splits == 1) return e;
  const OutLayout lay = make_out_layout(d.os, d.Lq, d.Z);
  hipLaunchKernelGGL(fwd_combine_kernel, dim3((unsigned)((rows * (d.A / 4) + 255) / 256)), dim3(256), 0, st,
                     a.part_o, a.part_ml, (uint16_t *)O, LSE, rows, splits, d.A, lay);
  return hipGetLastError();
}

}  // namespace rsa
