// Attention to a short, fixed set of keys (bf16, A = 64): the Linformer variant of Table 3, where
// every query row of the ranks attends to the same Kp = 128 or 256 projected keys of its head.
// With all keys of a head inside one work-group the ring walk of the general kernels degenerates
// (two stages), and the backward no longer needs two kernels: a work-group that owns all keys sees,
// for a tile of query rows, the complete dS row, so dQ needs neither a second sweep with S and dP
// recomputed nor atomics.  One kernel forms S, dP, dV, dK and dQ: five GEMM units executed for the
// five of the derivative of Eq. 1, where the two-kernel backward executes seven.
//
//   backward, per work-group (NW waves, wave w owns keys 32 w .. 32 w + 31; K, V of those keys in
//   registers) and per tile t of 64 query rows of its share of the head's rows:
//       S'  = Q K^T - LSE / s, dP' = dO V^T - D         (the row terms are the accumulators' start)
//       P   = exp2(s log2e S'), dS = P o dP'
//       dV^T += dO^T P, dK^T += Q^T dS                  (as in the dK/dV kernel of the general path)
//       dS^T -> LDS (bf16, [key][query row])
//     and, one tile later (the barrier at the top of a tile publishes the previous tile's dS^T),
//       dQ^T = s K^T dS^T                               (16x16x32 MFMAs; a wave owns 16 rows x 128 / NW
//                                                        dims over all keys; K as [key][dim] tiles in LDS)
//   The tiles of Q and dO arrive by direct global->LDS loads two tiles ahead (a ring of three
//   buffers), so that D = rowsum(dO o O) of tile t + 1 can be formed during tile t from the dO tile
//   already in LDS and O rows fetched into registers: the preprocess costs no pass of its own.
//   dV, dK of the work-groups that share a head (its rows are split over them) leave as fp32 partial
//   sums, added in a fixed order by qsplit_reduce_kernel.
#include "rsa_fused_tile.h"
#include "rsa_kernels.h"

namespace rsa {

struct SkArgs {
  const uint16_t *Q, *K, *V, *dO, *O;
  const float *LSE;
  uint16_t *dQ, *dK, *dV;
  float *part;            // fp32 partial sums [dV | dK][split][head][key][64], or nullptr (splits == 1)
  int64_t Lq;             // query rows per head (a multiple of 64)
  int64_t qs[3], ks[3], os[3];
  int Z, splits, tiles_per_split;
  float cl2, scale, inv_scale;
};

// D = A(16x32) * B(32x16) + C.  Lane l supplies A[l%16][k(l/16, 0..7)] and B[k(l/16, 0..7)][l%16]
// (any assignment k(group, e) of the 32 k indices to the four lane groups, the same for both) and
// receives C[(l/16)*4 + v][l%16] in element v.
__device__ __forceinline__ f32x4 mfma_16x16x32(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// Operand of a 16x16x32 MFMA whose m (or n) index runs over 16 columns of a tile and whose k index
// runs over 32 tile rows: lane (j = l%16, g = l/16) gets, for e = 0..7,
//   tile[k0 + (e>>2)*16 + (g&1)*8 + (g>>1)*4 + (e&3)][cb*16 + j].
// The order of the rows over the lane groups is chosen so that the 32 lanes of a phase of the
// transpose read (groups 0, 1: rows 0..3 and 8..11; groups 2, 3: rows 4..7 and 12..15) touch all 64
// banks once under the tile's chunk swizzle.  k0: multiple of 32.
struct TileLanes16 {
  int off0;  // column block 0; block cb is off0 ^ (cb << 5): cb only moves the 16-byte chunk by 2 cb
  __device__ __forceinline__ explicit TileLanes16(int lane) {
    const int j = lane & 15, g = lane >> 4;
    const int row = (g & 1) * 8 + (g >> 1) * 4 + (j >> 2);
    off0 = tile_off(row, (j >> 1) & 1) + (j & 1) * 8;
  }
  __device__ __forceinline__ bf16x8 read(const unsigned char *tile, int k0, int cb) const {
    const int off = off0 ^ (cb << 5);
    const u32x2 lo = lds_read_tr16(tile + k0 * 128 + off);
    const u32x2 hi = lds_read_tr16(tile + (k0 + 16) * 128 + off);
    const u32x4 w = {lo[0], lo[1], hi[0], hi[1]};
    return __builtin_bit_cast(bf16x8, w);
  }
};

// An 8-byte LDS store that the compiler does not see as a memory access.  For this kernel's dS^T stores it
// cannot tell that they miss the ring buffers, and it would wait for every direct load in flight before the
// first of them: the tile requested at the top of a step would be waited for in the middle of that step.
// The stores are ordered by hand instead: a wave's LDS operations complete in order, and the wait at the top of
// every step names lgkmcnt(0) before the barrier that publishes them.
__device__ __forceinline__ void lds_store_b64_unseen(unsigned char *lds_ptr, u32x2 v) {
  typedef __attribute__((address_space(3))) unsigned char *lptr_t;
  const uint32_t addr = (uint32_t)(uintptr_t)(lptr_t)lds_ptr;
  asm volatile("ds_write_b64 %0, %1" : : "v"(addr), "v"(v) : "memory");
}
// vmcnt(0) and lgkmcnt(0): before a barrier behind which other waves read what this wave stored that way
__device__ __forceinline__ void wait_vmem_lds() { __builtin_amdgcn_s_waitcnt(0x0070); }

template <int NW>
__global__ void __launch_bounds__(64 * NW, 1) shortkeys_bwd_kernel(SkArgs a) {
  constexpr int KT = NW / 2;        // 64-key tiles
  constexpr int WPR = NW / 4;       // waves that share 16 rows of dQ
  constexpr int DB = 4 / WPR;       // 16-dim blocks of dQ per wave
  constexpr int RPL = 8 / NW;       // rows per lane in the D computation
  constexpr int OST = 32 * DB + 16; // bytes between rows of a wave's dQ staging block (padded)
  struct Ring { unsigned char Qt[kTileBytes], dOs[kTileBytes]; };
  // separate objects addressed by name: the compiler then knows that a direct load into one of
  // them cannot alias the LDS reads of the others
  __shared__ __attribute__((aligned(16))) Ring ring0, ring1, ring2;
  __shared__ __attribute__((aligned(16))) unsigned char dST[2][KT][kTileBytes];  // [tile parity]
  __shared__ __attribute__((aligned(16))) unsigned char Kt[KT][kTileBytes];
  __shared__ __attribute__((aligned(16))) unsigned char qst[NW][16 * OST];
  __shared__ __attribute__((aligned(16))) float nl[3][64], nd[3][64];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31, half = lane >> 5;
  const int64_t head = blockIdx.x / a.splits;
  const int split = blockIdx.x % a.splits;
  const int nqt = (int)(a.Lq / 64);
  const int t_begin = split * a.tiles_per_split;
  const int T = min(a.tiles_per_split, nqt - t_begin);  // tiles of this work-group
  if (T <= 0) return;  // (the host's split leaves none empty)

  const int64_t kv_off = head_offset(head, a.Z, a.ks);
  const int64_t q_ld = a.qs[2], kv_ld = a.ks[2], o_ld = a.os[2];
  const uint16_t *Qh = a.Q + head_offset(head, a.Z, a.qs) + (int64_t)t_begin * 64 * q_ld;
  const uint16_t *dOh = a.dO + head_offset(head, a.Z, a.os) + (int64_t)t_begin * 64 * o_ld;
  const uint16_t *Oh = a.O + head_offset(head, a.Z, a.os) + (int64_t)t_begin * 64 * o_ld;
  uint16_t *dQh = a.dQ + head_offset(head, a.Z, a.qs) + (int64_t)t_begin * 64 * q_ld;
  const float *LSEh = a.LSE + head * a.Lq + (int64_t)t_begin * 64;
  const uint16_t *Kh = a.K + kv_off;
  const uint16_t *Vh = a.V + kv_off;

  // K, V of the wave's 32 keys as B operands: lane (col, half) holds row col, elements dk*16 + half*8 ..
  bf16x8 kreg[4], vreg[4];
  {
    const int64_t key = wave * 32 + col;
#pragma unroll
    for (int dk = 0; dk < 4; ++dk) {
      kreg[dk] = *reinterpret_cast<const bf16x8 *>(Kh + key * kv_ld + dk * 16 + half * 8);
      vreg[dk] = *reinterpret_cast<const bf16x8 *>(Vh + key * kv_ld + dk * 16 + half * 8);
    }
  }
  const TileLanes tl(lane);
  const TileLanes16 tl16(lane);
  const TileDMAT<NW> dma_q(wave, lane, (int)q_ld), dma_o(wave, lane, (int)o_ld), dma_k(wave, lane, (int)kv_ld);

  f32x16 dv[2], dk_[2];  // transposed: rows = head dim (block db), columns = the wave's keys
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) { dv[db][v] = 0.f; dk_[db][v] = 0.f; }

  // rows of the D computation: lane handles 8 elements (chunk `sub`) of rows drow0 + rr * 8 NW
  // (lane-dependent parts of global addresses are kept as 32-bit offsets from uniform bases)
  const int drow0 = tid >> 3, sub = tid & 7;
  const int o_lane = drow0 * (int)o_ld + sub * 8;
  u32x4 oreg[RPL];
  float lreg[RPL];
  auto load_o = [&](int t) __attribute__((always_inline)) {
    const uint16_t *ot = Oh + (int64_t)t * 64 * o_ld;
    const float *lt = LSEh + (int64_t)t * 64;
#pragma unroll
    for (int rr = 0; rr < RPL; ++rr) {
      oreg[rr] = *reinterpret_cast<const u32x4 *>(ot + (o_lane + rr * 8 * NW * (int)o_ld));
      lreg[rr] = lt[drow0 + rr * 8 * NW];
    }
  };
  // row terms of tile t (its dO tile is in rg, its O rows in oreg) -> nl, nd [slot]
  auto row_terms = [&](const Ring &rg, int slot) __attribute__((always_inline)) {
#pragma unroll
    for (int rr = 0; rr < RPL; ++rr) {
      const int row = rr * 8 * NW + drow0;
      const u32x4 x = *reinterpret_cast<const u32x4 *>(rg.dOs + tile_off(row, sub));
      const u32x4 y = oreg[rr];
      float acc = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc = fmaf(bf16_to_f32(x[e] & 0xffffu), bf16_to_f32(y[e] & 0xffffu), acc);
        acc = fmaf(bf16_to_f32(x[e] >> 16), bf16_to_f32(y[e] >> 16), acc);
      }
      acc += __shfl_xor(acc, 1);
      acc += __shfl_xor(acc, 2);
      acc += __shfl_xor(acc, 4);
      if (sub == 0) {
        nd[slot][row] = -acc;
        nl[slot][row] = -lreg[rr] * a.inv_scale;
      }
    }
  };
  auto load_tile = [&](int t, Ring &rg) __attribute__((always_inline)) {
    dma_q.load(Qh + (int64_t)t * 64 * q_ld, rg.Qt);
    dma_o.load(dOh + (int64_t)t * 64 * o_ld, rg.dOs);
  };

  // where the wave's dS^T goes: rows (wave & 1) * 32 + col of key tile wave >> 1, 8 bytes (4 query
  // rows) at chunk qb * 4 + g, half `half`
  const int ds_row = (wave & 1) * 32 + col;
  const int ds_base = (wave >> 1) * kTileBytes + ds_row * 128 + half * 8;
  const int ds_rot = swz_rot(ds_row) << 4;

  // dQ of the previous tile from its dS^T
  const int dq_rows = (wave / WPR) * 16;          // the wave's 16 query rows
  const int dq_dim0 = (wave % WPR) * (16 * DB);   // its first dim
  // in two parts (k slices of 32 keys: [0, KT) and [KT, 2 KT)) that ride in the last phase of the next
  // tile's main sweep, whose eight MFMAs fill the gaps of this chain of LDS reads and small MFMAs
  f32x4 dq[DB];
  auto dq_part = [&](const unsigned char(*ds)[kTileBytes], int part) __attribute__((always_inline)) {
    if (part == 0) {
#pragma unroll
      for (int b = 0; b < DB; ++b) dq[b] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int ks = part * KT; ks < (part + 1) * KT; ++ks) {
      const bf16x8 bfrag = tl16.read(ds[ks >> 1], (ks & 1) * 32, dq_rows >> 4);
#pragma unroll
      for (int b = 0; b < DB; ++b)
        dq[b] = mfma_16x16x32(tl16.read(Kt[ks >> 1], (ks & 1) * 32, (dq_dim0 >> 4) + b), bfrag, dq[b]);
    }
  };
  // the wave's dQ block goes to its LDS staging block as bf16 (dq_stage) and leaves from there as
  // 16-byte pieces (dq_flush: a step later, behind the step's barrier, so that the wait for the
  // step's tile loads never waits for stores just issued)
  auto dq_stage = [&]() __attribute__((always_inline)) {
    // lane (n = l%16, mg = l/16) holds dims dq_dim0 + b*16 + mg*4 .. +3 of query row dq_rows + n
    const int n = lane & 15, mg = lane >> 4;
    const int st_off = wave * (16 * OST) + n * OST + mg * 8;
#pragma unroll
    for (int b = 0; b < DB; ++b) {
      const u32x2 w = {pack_bf16(dq[b][0] * a.scale, dq[b][1] * a.scale),
                       pack_bf16(dq[b][2] * a.scale, dq[b][3] * a.scale)};
      *reinterpret_cast<u32x2 *>(&qst[0][st_off + b * 32]) = w;
    }
  };
  auto dq_flush = [&](int t) __attribute__((always_inline)) {
    // 16 rows of 32 DB bytes (same wave: LDS operations complete in order)
    const unsigned char *st = qst[wave];
    constexpr int PPR = 2 * DB;  // pieces per row
    uint16_t *dq_t = dQh + ((int64_t)t * 64 + dq_rows) * q_ld + dq_dim0;
#pragma unroll
    for (int it = 0; it < (16 * PPR + 63) / 64; ++it) {
      const int p = it * 64 + lane, row = p / PPR, pc = p % PPR;
      if (row < 16)
        *reinterpret_cast<u32x4 *>(dq_t + (row * (int)q_ld + pc * 8)) =
            *reinterpret_cast<const u32x4 *>(st + row * OST + pc * 16);
    }
  };

  // S', dP', P, dS, dV, dK of one tile of 64 rows (in rg, row terms in slot) against the wave's keys,
  // one block of 32 rows after the other with one set of registers (the two waves of a SIMD overlap
  // each other's matrix and vector phases); every LDS read is issued a phase before its use.
  auto main_tile = [&](const Ring &rg, int slot, int par, const unsigned char(*ds_prev)[kTileBytes])
      __attribute__((always_inline)) {
    const int ds_off = par * (KT * kTileBytes) + ds_base;
    bf16x8 qa[4], ga[4];
    f32x16 sacc, dpacc;
    bf16x8 pf[2], sf[2];
    bf16x8 gt[2][2], qt2[2][2];
    auto rows = [&](int qb) __attribute__((always_inline)) {
#pragma unroll
      for (int dk = 0; dk < 4; ++dk) {
        qa[dk] = tl.read_rows(rg.Qt, qb * 32, dk);
        ga[dk] = tl.read_rows(rg.dOs, qb * 32, dk);
      }
    };
    auto init = [&](int qb) __attribute__((always_inline)) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4 l4 = *reinterpret_cast<const f32x4 *>(&nl[slot][qb * 32 + g * 8 + half * 4]);
        const f32x4 d4 = *reinterpret_cast<const f32x4 *>(&nd[slot][qb * 32 + g * 8 + half * 4]);
#pragma unroll
        for (int e = 0; e < 4; ++e) { sacc[g * 4 + e] = l4[e]; dpacc[g * 4 + e] = d4[e]; }
      }
    };
    auto g12 = [&]() __attribute__((always_inline)) {
#pragma unroll
      for (int dk = 0; dk < 4; ++dk) {
        sacc = mfma_32x32x16(qa[dk], kreg[dk], sacc);
        dpacc = mfma_32x32x16(ga[dk], vreg[dk], dpacc);
      }
    };
    auto softmax_bwd = [&](int qb) __attribute__((always_inline)) {
#pragma unroll
      for (int w2 = 0; w2 < 2; ++w2) {
        u32x4 w, x;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float p0 = __builtin_amdgcn_exp2f(sacc[w2 * 8 + 2 * e] * a.cl2);
          const float p1 = __builtin_amdgcn_exp2f(sacc[w2 * 8 + 2 * e + 1] * a.cl2);
          w[e] = pack_bf16(p0, p1);
          x[e] = pack_bf16(p0 * dpacc[w2 * 8 + 2 * e], p1 * dpacc[w2 * 8 + 2 * e + 1]);
        }
        pf[w2] = __builtin_bit_cast(bf16x8, w);
        sf[w2] = __builtin_bit_cast(bf16x8, x);
        // the lane's 2 x 4 query rows of this slice: rows qb*32 + g*8 + half*4 .. +3, g = 2 w2, 2 w2 + 1
#pragma unroll
        for (int gg = 0; gg < 2; ++gg) {
          const int cc = qb * 4 + w2 * 2 + gg;
          const u32x2 piece = {x[2 * gg], x[2 * gg + 1]};
          lds_store_b64_unseen(&dST[0][0][ds_off + ((cc << 4) ^ ds_rot)], piece);
        }
      }
    };
    auto cols = [&](int qb) __attribute__((always_inline)) {
#pragma unroll
      for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
        for (int db = 0; db < 2; ++db) {
          gt[k2][db] = tl.read_cols(rg.dOs, (qb * 2 + k2) * 16, db);
          qt2[k2][db] = tl.read_cols(rg.Qt, (qb * 2 + k2) * 16, db);
        }
    };
    auto g34 = [&]() __attribute__((always_inline)) {
#pragma unroll
      for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
        for (int db = 0; db < 2; ++db) {
          dv[db] = mfma_32x32x16(gt[k2][db], pf[k2], dv[db]);
          dk_[db] = mfma_32x32x16(qt2[k2][db], sf[k2], dk_[db]);
        }
    };
    rows(0);
    init(0);
    __builtin_amdgcn_sched_barrier(0);
    cols(0);
    g12();
    __builtin_amdgcn_sched_barrier(0);
    softmax_bwd(0);
    __builtin_amdgcn_sched_barrier(0);
    rows(1);
    g34();
    init(1);
    __builtin_amdgcn_sched_barrier(0);
    cols(1);
    g12();
    __builtin_amdgcn_sched_barrier(0);
    softmax_bwd(1);
    __builtin_amdgcn_sched_barrier(0);
    g34();
    dq_part(ds_prev, 0);
    dq_part(ds_prev, 1);
    __builtin_amdgcn_sched_barrier(0);
  };

  // prologue: K as [key][dim] tiles, tile 0 and its O rows; then the row terms of tile 0, and tile 1
#pragma unroll
  for (int kt = 0; kt < KT; ++kt) dma_k.load(Kh + (int64_t)kt * 64 * kv_ld, Kt[kt]);
  load_tile(0, ring0);
  load_o(0);
  wait_vmem();
  __syncthreads();
  row_terms(ring0, 0);
  if (T > 1) { load_tile(1, ring1); load_o(1); }

  // tile t: cur holds it, nxt holds tile t + 1 (arrived by the barrier), nn takes tile t + 2
  int t = 0;
  auto step = [&](Ring &cur, Ring &nxt, Ring &nn, int slot) __attribute__((always_inline)) {
    wait_vmem_lds();
    __syncthreads();
    if (t + 2 < T) load_tile(t + 2, nn);
    if (t + 1 < T) row_terms(nxt, slot == 2 ? 0 : slot + 1);
    if (t + 2 < T) load_o(t + 2);
    if (t > 1) dq_flush(t - 2);  // staged at the end of the previous step
    __builtin_amdgcn_sched_barrier(0);
    // (the first tile has no predecessor: its dQ parts run on whatever the buffer holds and are dropped)
    main_tile(cur, slot, t & 1, dST[(t - 1) & 1]);
    if (t > 0) dq_stage();  // dQ of tile t - 1
    ++t;
  };
  while (t < T) {
    step(ring0, ring1, ring2, 0);
    if (t >= T) break;
    step(ring1, ring2, ring0, 1);
    if (t >= T) break;
    step(ring2, ring0, ring1, 2);
  }
  wait_vmem_lds();
  __syncthreads();
  if (T > 1) dq_flush(T - 2);
  dq_part(dST[(T - 1) & 1], 0);
  dq_part(dST[(T - 1) & 1], 1);
  dq_stage();
  dq_flush(T - 1);

  // dV, dK of the wave's 32 keys
  const int64_t key0 = wave * 32;
  if (a.part) {  // fp32 partial sums: [dV | dK][split][head][key][64]
    const int64_t heads = gridDim.x / a.splits;
    const int64_t keys = 32 * NW;
    float *pv = a.part + (((int64_t)split * heads + head) * keys + key0 + col) * 64;
    float *pk = pv + (int64_t)a.splits * heads * keys * 64;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int off = db * 32 + g * 8 + half * 4;
        const f32x4 w = {dv[db][g * 4 + 0], dv[db][g * 4 + 1], dv[db][g * 4 + 2], dv[db][g * 4 + 3]};
        *reinterpret_cast<f32x4 *>(pv + off) = w;
        const f32x4 x = {dk_[db][g * 4 + 0] * a.scale, dk_[db][g * 4 + 1] * a.scale,
                         dk_[db][g * 4 + 2] * a.scale, dk_[db][g * 4 + 3] * a.scale};
        *reinterpret_cast<f32x4 *>(pk + off) = x;
      }
  } else {
    // through an LDS tile of the wave's own (the dS^T buffers hold one per wave) as whole rows
    __syncthreads();  // every wave's last dQ has read them
    unsigned char *ot = &dST[0][0][0] + wave * kTileBytes;
    stage_block_T(ot, 0, dv[0], dv[1], 1.0f, lane);
    stage_block_T(ot, 32, dk_[0], dk_[1], a.scale, lane);
    flush_rows<32>(ot, 0, a.dV + kv_off + key0 * kv_ld, 32, lane, (int)kv_ld);
    flush_rows<32>(ot, 32, a.dK + kv_off + key0 * kv_ld, 32, lane, (int)kv_ld);
  }
}

// ------------------------------------------------------------------ forward ---
// Eq. 1 for query rows that all attend to the same Kp <= 256 keys of their head: the keys' K and V
// tiles are loaded into LDS once per work-group, which then walks blocks of 256 query rows of the head
// (wave w: rows 64 w .. 64 w + 63 of the block) with no barrier and no load but the rows' own Q:
//   S^T = K Q^T (A: K tile rows from LDS, B: Q^T in registers), running max and sum per row
//   (lane = query column), O^T += V^T P^T (A: LDS transpose reads, B: P^T from the accumulator).
// The waves of a work-group drift apart, so one wave's row loads and stores run beside the others'
// matrix work.
struct SkFwdArgs {
  const uint16_t *Q, *K, *V;
  uint16_t *O;
  float *LSE;
  int64_t Lq;
  int64_t qs[3], ks[3], os[3];
  int Z, splits, blocks_per_split;
  float cl2;
};

template <int KT>
__global__ void __launch_bounds__(256, 2) shortkeys_fwd_kernel(SkFwdArgs a) {
  __shared__ __attribute__((aligned(16))) unsigned char Kt[KT][kTileBytes], Vt[KT][kTileBytes];
  __shared__ __attribute__((aligned(16))) unsigned char stg[4][32 * 128];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31, half = lane >> 5;
  const int64_t head = blockIdx.x / a.splits;
  const int split = blockIdx.x % a.splits;
  const int nblk = (int)((a.Lq + 255) / 256);
  const int b_begin = split * a.blocks_per_split;
  const int b_end = min(b_begin + a.blocks_per_split, nblk);
  if (b_begin >= b_end) return;

  const int64_t kv_off = head_offset(head, a.Z, a.ks);
  const int64_t q_ld = a.qs[2], kv_ld = a.ks[2], o_ld = a.os[2];
  const uint16_t *Qh = a.Q + head_offset(head, a.Z, a.qs);
  uint16_t *Oh = a.O + head_offset(head, a.Z, a.os);
  float *LSEh = a.LSE + head * a.Lq;
  {
    const TileDMA dma(wave, lane, (int)kv_ld);
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      dma.load(a.K + kv_off + (int64_t)kt * 64 * kv_ld, Kt[kt]);
      dma.load(a.V + kv_off + (int64_t)kt * 64 * kv_ld, Vt[kt]);
    }
  }
  const TileLanes tl(lane);
  unsigned char *ot = stg[wave];
  const int q_lane = col * (int)q_ld + half * 8;  // lane part of a Q row address (32-bit)
  wait_vmem();
  __syncthreads();

  // Q^T operand: lane (col, half) holds Q[row][dk*16 + half*8 .. +8]; the rows of the next block are
  // fetched as soon as the last S^T of the current one has been issued
  bf16x8 qreg[2][4];
  auto load_q = [&](int64_t r0) __attribute__((always_inline)) {
    if (r0 >= a.Lq) r0 = a.Lq - 64;  // past the end: any valid rows (not used)
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const uint16_t *qp = Qh + (r0 + qb * 32) * q_ld;
#pragma unroll
      for (int dk = 0; dk < 4; ++dk) qreg[qb][dk] = *reinterpret_cast<const bf16x8 *>(qp + (q_lane + dk * 16));
    }
  };
  load_q((int64_t)b_begin * 256 + wave * 64);
  for (int b = b_begin; b < b_end; ++b) {
    const int64_t wr0 = (int64_t)b * 256 + wave * 64;  // the wave's first row
    if (wr0 >= a.Lq) break;                             // (rows come in multiples of 64)
    f32x16 o[2][2];
    float m[2], mc[2], l[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      m[qb] = -INFINITY; mc[qb] = 0.f; l[qb] = 0.f;
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][qb][v] = 0.f;
    }
#pragma unroll
    for (int u = 0; u < KT; ++u) {
      f32x16 sc[2][2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        bf16x8 ka[4];
#pragma unroll
        for (int dk = 0; dk < 4; ++dk) ka[dk] = tl.read_rows(Kt[u], kb * 32, dk);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
          for (int v = 0; v < 16; ++v) sc[kb][qb][v] = 0.f;
#pragma unroll
          for (int dk = 0; dk < 4; ++dk) sc[kb][qb] = mfma_32x32x16(ka[dk], qreg[qb][dk], sc[kb][qb]);
        }
      }
      if (u == KT - 1) {
        __builtin_amdgcn_sched_barrier(0);
        load_q(wr0 + 256);
        __builtin_amdgcn_sched_barrier(0);
      }
      // running max; the accumulators are rescaled only when some row's max grew by more than
      // 2^8 in the exp2 domain (exact: l and O share the stale max)
      float tm[2];
      bool need = false;
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        float x = sc[0][qb][0];
#pragma unroll
        for (int v = 1; v < 16; ++v) x = fmaxf(x, sc[0][qb][v]);
#pragma unroll
        for (int v = 0; v < 16; ++v) x = fmaxf(x, sc[1][qb][v]);
        tm[qb] = xhalf_max(x);
        need |= (tm[qb] - m[qb]) * a.cl2 > 8.0f;
      }
      if (__builtin_amdgcn_ballot_w64(need) != 0) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
          const float mn = fmaxf(m[qb], tm[qb]);
          const float alpha = __builtin_amdgcn_exp2f((m[qb] - mn) * a.cl2);  // first tile: exp2(-inf) = 0
          m[qb] = mn;
          mc[qb] = mn * a.cl2;
          l[qb] *= alpha;
#pragma unroll
          for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[db][qb][v] *= alpha;
        }
      }
      bf16x8 pf[2][4];
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        float ls = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          float p[16];
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            p[v] = __builtin_amdgcn_exp2f(fmaf(sc[kb][qb][v], a.cl2, -mc[qb]));
            ls += p[v];
          }
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            u32x4 w = {pack_bf16(p[h * 8 + 0], p[h * 8 + 1]), pack_bf16(p[h * 8 + 2], p[h * 8 + 3]),
                       pack_bf16(p[h * 8 + 4], p[h * 8 + 5]), pack_bf16(p[h * 8 + 6], p[h * 8 + 7])};
            pf[qb][kb * 2 + h] = __builtin_bit_cast(bf16x8, w);
          }
        }
        l[qb] += ls;
      }
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          const bf16x8 va = tl.read_cols(Vt[u], kk * 16, db);
#pragma unroll
          for (int qb = 0; qb < 2; ++qb) o[db][qb] = mfma_32x32x16(va, pf[qb][kk], o[db][qb]);
        }
    }
    // O = O^T / l, LSE = (m cl2 + log2 l) ln 2; 32 rows at a time through the wave's LDS tile
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const float lt = xhalf_sum(l[qb]);
      const float inv = 1.0f / lt;
      if (half == 0) LSEh[wr0 + qb * 32 + col] = (mc[qb] + __builtin_amdgcn_logf(lt)) * kLn2;
      stage_block_T(ot, 0, o[0][qb], o[1][qb], inv, lane);
      flush_rows<32>(ot, 0, Oh + (wr0 + qb * 32) * o_ld, 32, lane, (int)o_ld);
    }
  }
}

int shortkeys_fwd_splits(const Dims &att) {
  const int64_t heads = (int64_t)att.B * att.Z, blocks = (att.Lq + 255) / 256;
  int best = 1;
  double best_cost = 1e30;
  for (int s = 1; s <= 128 && s <= blocks; ++s) {
    const int64_t per = (blocks + s - 1) / s;
    if (per * (s - 1) >= blocks) continue;
    const double cost = (double)((heads * s + 511) / 512) * (per + 1);  // + 1: the K/V load, in blocks
    if (cost < best_cost) { best_cost = cost; best = s; }
  }
  return best;
}

hipError_t shortkeys_forward(const Dims &att, const void *Q, const void *K, const void *V, void *O, float *LSE,
                             hipStream_t st) {
  SkFwdArgs a;
  a.Q = (const uint16_t *)Q; a.K = (const uint16_t *)K; a.V = (const uint16_t *)V;
  a.O = (uint16_t *)O; a.LSE = LSE; a.Lq = att.Lq; a.Z = att.Z;
  for (int k = 0; k < 3; ++k) { a.qs[k] = att.qs[k]; a.ks[k] = att.ks[k]; a.os[k] = att.os[k]; }
  a.splits = shortkeys_fwd_splits(att);
  a.blocks_per_split = (int)(((att.Lq + 255) / 256 + a.splits - 1) / a.splits);
  a.cl2 = att.scale * kLog2e;
  const dim3 grid((unsigned)((int64_t)att.B * att.Z * a.splits));
  if (att.L == 256)
    hipLaunchKernelGGL(shortkeys_fwd_kernel<4>, grid, dim3(256), 0, st, a);
  else
    hipLaunchKernelGGL(shortkeys_fwd_kernel<2>, grid, dim3(256), 0, st, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------- dX = E dXp ---
// The input gradient of the Linformer projection (Table 3, row Projection): for every head,
// dX (rows, A) = E (rows, Kp) dXp (Kp, A) with Kp <= 256.  As a GEMM its contraction is only Kp long, so a
// tiled kernel spends its time filling and draining its pipeline; here a work-group keeps its 128
// rows of E in registers (as B operands: wave w owns rows 32 w .. 32 w + 31) and streams the heads'
// dXp tiles through LDS, double-buffered, one barrier per 64 output columns:
//     dX^T (64 dims x 32 rows) += dXp^T (dims x 16 k) E^T (16 k x rows)     (A: LDS transpose reads)
// and the block leaves through the wave's LDS tile as whole 128-byte rows.
struct DxArgs {
  const uint16_t *E, *dXp;
  uint16_t *dX;
  int64_t rows, L, Kp;
  int A, AH, ntiles, tiles_per_group, groups;  // ntiles = heads * AH column tiles of 64
};

template <int KT>
__global__ void __launch_bounds__(256, 2) linformer_dx_kernel(DxArgs g) {
  struct Buf { unsigned char t[KT][kTileBytes]; };
  __shared__ __attribute__((aligned(16))) Buf buf0, buf1;
  __shared__ __attribute__((aligned(16))) unsigned char stg[4][32 * 128];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t blk = blockIdx.x / g.groups;
  const int grp = blockIdx.x % g.groups;
  const int64_t row0 = blk * 128;
  const int ct_begin = grp * g.tiles_per_group;
  const int nct = min(g.tiles_per_group, g.ntiles - ct_begin);
  if (nct <= 0) return;
  const TileLanes tl(lane);
  const TileDMAT<4> dma_e(wave, lane, (int)g.Kp), dma_b(wave, lane, g.A);

  // E rows of the block -> LDS (its 2 x KT tiles fill the two buffers) -> registers
  const int64_t last_rt = g.rows / 64 - 1;
#pragma unroll
  for (int kt = 0; kt < KT; ++kt) {
    const int64_t rt0 = min(row0 / 64, last_rt), rt1 = min(row0 / 64 + 1, last_rt);  // past the end: refetch
    dma_e.load(g.E + rt0 * 64 * g.Kp + kt * 64, buf0.t[kt]);
    dma_e.load(g.E + rt1 * 64 * g.Kp + kt * 64, buf1.t[kt]);
  }
  wait_vmem();
  __syncthreads();
  bf16x8 efrag[KT * 4];
#pragma unroll
  for (int ks = 0; ks < KT * 4; ++ks) {
    const unsigned char *te = (wave >> 1) ? buf1.t[ks >> 2] : buf0.t[ks >> 2];
    efrag[ks] = tl.read_rows_perm(te, (wave & 1) * 32, ks & 3);
  }
  __syncthreads();  // the buffers are free again

  auto load_b = [&](int ct, Buf &b) __attribute__((always_inline)) {
    const int head = ct / g.AH, ah = ct % g.AH;
    const uint16_t *src = g.dXp + (int64_t)head * g.Kp * g.A + ah * 64;
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) dma_b.load(src + (int64_t)kt * 64 * g.A, b.t[kt]);
  };
  unsigned char *ot = stg[wave];
  const int64_t wrow0 = row0 + wave * 32;
  auto tile = [&](int ct, const Buf &b) __attribute__((always_inline)) {
    f32x16 acc[2];
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;
    // a k slice is only two MFMAs, far less than the latency of an LDS read: the fragments are read
    // DEPTH slices ahead
    constexpr int DEPTH = 6, NS = KT * 4;
    bf16x8 af[NS][2];
    auto frags = [&](int ks) __attribute__((always_inline)) {
#pragma unroll
      for (int db = 0; db < 2; ++db) af[ks][db] = tl.read_cols(b.t[ks >> 2], (ks & 3) * 16, db);
    };
#pragma unroll
    for (int ks = 0; ks < DEPTH && ks < NS; ++ks) frags(ks);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < NS; ++ks) {
      if (ks + DEPTH < NS) frags(ks + DEPTH);
#pragma unroll
      for (int db = 0; db < 2; ++db) acc[db] = mfma_32x32x16(af[ks][db], efrag[ks], acc[db]);
      __builtin_amdgcn_sched_barrier(0);
    }
    stage_block_T(ot, 0, acc[0], acc[1], 1.0f, lane);
  };
  // the staged block leaves a step later, behind the step's barrier and beside the next tile's MFMAs
  auto flush = [&](int ct) __attribute__((always_inline)) {
    const int head = ct / g.AH, ah = ct % g.AH;
    flush_rows<32>(ot, 0, g.dX + ((int64_t)head * g.L + wrow0) * g.A + ah * 64, g.rows - wrow0, lane, g.A);
  };

  load_b(ct_begin, buf0);
  int i = 0;
  auto step = [&](Buf &cur, Buf &nxt) __attribute__((always_inline)) {
    wait_vmem();
    __syncthreads();
    if (i + 1 < nct) load_b(ct_begin + i + 1, nxt);
    if (i > 0) flush(ct_begin + i - 1);
    tile(ct_begin + i, cur);
    ++i;
  };
  while (i < nct) {
    step(buf0, buf1);
    if (i >= nct) break;
    step(buf1, buf0);
  }
  flush(ct_begin + nct - 1);
}

bool linformer_dx_supported(int64_t Kp, int A) { return Kp % 64 == 0 && Kp <= 256 && (A == 64 || A == 128); }

hipError_t linformer_dx(int64_t Zt, int64_t L, int64_t rows, int64_t Kp, int A, const void *dXp, const void *E,
                        void *dX, hipStream_t st) {
  DxArgs g;
  g.E = (const uint16_t *)E; g.dXp = (const uint16_t *)dXp; g.dX = (uint16_t *)dX;
  g.rows = rows; g.L = L; g.Kp = Kp; g.A = A; g.AH = A / 64; g.ntiles = (int)(Zt * g.AH);
  const int64_t blocks = (rows + 127) / 128;
  // groups of column tiles per row block: few, even rounds of the 512 work-groups the chip holds
  int best = 1;
  double best_cost = 1e30;
  for (int gr = 1; gr <= 16 && gr <= g.ntiles; ++gr) {
    const int per = (g.ntiles + gr - 1) / gr;
    if ((int64_t)per * (gr - 1) >= g.ntiles) continue;
    const double cost = (double)((blocks * gr + 511) / 512) * (per + 2);
    if (cost < best_cost) { best_cost = cost; best = gr; }
  }
  g.groups = best;
  g.tiles_per_group = (g.ntiles + best - 1) / best;
  const dim3 grid((unsigned)(blocks * best));
  switch (Kp / 64) {
    case 1: hipLaunchKernelGGL(linformer_dx_kernel<1>, grid, dim3(256), 0, st, g); break;
    case 2: hipLaunchKernelGGL(linformer_dx_kernel<2>, grid, dim3(256), 0, st, g); break;
    case 3: hipLaunchKernelGGL(linformer_dx_kernel<3>, grid, dim3(256), 0, st, g); break;
    default: hipLaunchKernelGGL(linformer_dx_kernel<4>, grid, dim3(256), 0, st, g); break;
  }
  return hipGetLastError();
}

bool shortkeys_supported(const Dims &att) {
  return att.A == 64 && (att.L == 128 || att.L == 256) && !att.causal && !att.strided && att.N == 1 &&
         att.Lq >= 64;
}

// Work-groups per head: the rows of a head are split so that the grid covers the 256 compute units
// (one work-group each) in as few, as even rounds as possible.
int shortkeys_splits(const Dims &att) {
  const int64_t heads = (int64_t)att.B * att.Z, tiles = att.Lq / 64;
  int best = 1;
  double best_cost = 1e30;
  for (int s = 1; s <= 64 && s <= tiles; ++s) {
    const int64_t per = (tiles + s - 1) / s;
    if ((per * (s - 1)) >= tiles) continue;  // the last split would be empty
    const int64_t rounds = (heads * s + 255) / 256;
    const double cost = (double)rounds * (per + 3);  // + 3: a work-group's prologue and epilogue, in tiles
    if (cost < best_cost) { best_cost = cost; best = s; }
  }
  return best;
}

size_t shortkeys_bwd_ws_bytes(const Dims &att) {
  const int s = shortkeys_splits(att);
  return s > 1 ? (size_t)2 * s * att.B * att.Z * att.L * 64 * 4 : 0;
}

hipError_t shortkeys_backward(const Dims &att, const void *dO, const void *Q, const void *K, const void *V,
                              const void *O, const float *LSE, void *dQ, void *dK, void *dV, float *part,
                              hipStream_t st) {
  SkArgs a;
  a.Q = (const uint16_t *)Q; a.K = (const uint16_t *)K; a.V = (const uint16_t *)V;
  a.dO = (const uint16_t *)dO; a.O = (const uint16_t *)O; a.LSE = LSE;
  a.dQ = (uint16_t *)dQ; a.dK = (uint16_t *)dK; a.dV = (uint16_t *)dV;
  a.Lq = att.Lq; a.Z = att.Z;
  for (int k = 0; k < 3; ++k) { a.qs[k] = att.qs[k]; a.ks[k] = att.ks[k]; a.os[k] = att.os[k]; }
  a.splits = shortkeys_splits(att);
  a.tiles_per_split = (int)((att.Lq / 64 + a.splits - 1) / a.splits);
  a.part = a.splits > 1 ? part : nullptr;
  if (a.splits > 1 && !part) return hipErrorInvalidValue;
  a.cl2 = att.scale * kLog2e; a.scale = att.scale; a.inv_scale = 1.0f / att.scale;
  const dim3 grid((unsigned)((int64_t)att.B * att.Z * a.splits));
  if (att.L == 256)
    hipLaunchKernelGGL(shortkeys_bwd_kernel<8>, grid, dim3(512), 0, st, a);
  else
    hipLaunchKernelGGL(shortkeys_bwd_kernel<4>, grid, dim3(256), 0, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || a.splits == 1) return e;
  const int64_t n4 = (int64_t)att.B * att.Z * att.L * (64 / 4);
  const OutLayout lay = make_out_layout(att.ks, att.L, att.Z);
  e = qsplit_reduce(part, dV, n4, a.splits, 64, lay, st);
  if (e != hipSuccess) return e;
  return qsplit_reduce(part + (int64_t)a.splits * n4 * 4, dK, n4, a.splits, 64, lay, st);
}

}  // namespace rsa
