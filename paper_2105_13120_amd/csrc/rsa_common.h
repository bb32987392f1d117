// Shared device helpers for the RSA kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rsa.h"

namespace rsa {

typedef __bf16 bf16_t;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// D = A(32x16) * B(16x32) + C on the matrix core.  Lane l supplies
// A[l%32][(l/32)*8 .. +8] and B[(l/32)*8 .. +8][l%32]; it receives
// C[(v/4)*8 + (l/32)*4 + v%4][l%32] in element v of the accumulator.
__device__ __forceinline__ f32x16 mfma_32x32x16(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Two fp32 -> packed bf16 (round to nearest even), low half = x.
__device__ __forceinline__ uint32_t pack_bf16(float x, float y) {
  f32x2 v = {x, y};
  bf16x2 r = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __builtin_bit_cast(float, (uint32_t)b << 16);
}

// LDS transpose read (ds_read_b64_tr_b16).  Within each group of 16 lanes,
// lane j passes the address of 4 consecutive 16-bit elements ("row j/4,
// columns (j%4)*4 .. +4" of a 4 x 16 block); lane i receives column i of that
// block: element k of the result is element i%4 of the row passed by lane
// 4*k + i/4.
__device__ __forceinline__ u32x2 lds_read_tr16(const void *lds_ptr) {
  typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
  typedef __attribute__((address_space(3))) s16x4 *lds_s16x4_ptr;
  s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds_ptr));
  return __builtin_bit_cast(u32x2, r);
}

// Direct 16-byte global->LDS load (global_load_lds_dwordx4): lane l of the wave fetches
// 16 bytes from its own global address and the hardware writes them to LDS at
// lds_base + 16 l; lds_base must be the same for the whole wave.  Completion is tracked
// by vmcnt: wait_vmem() before the barrier that publishes the data.
__device__ __forceinline__ void lds_dma16(const void *gsrc, void *lds_base) {
  typedef __attribute__((address_space(1))) const void *gptr_t;
  typedef __attribute__((address_space(3))) void *lptr_t;
  __builtin_amdgcn_global_load_lds((gptr_t)gsrc, (lptr_t)lds_base, 16, 0, 0);
}
// Same, 4 bytes per lane: lane l's dword lands at lds_base + 4 l.
__device__ __forceinline__ void lds_dma4(const void *gsrc, void *lds_base) {
  typedef __attribute__((address_space(1))) const void *gptr_t;
  typedef __attribute__((address_space(3))) void *lptr_t;
  __builtin_amdgcn_global_load_lds((gptr_t)gsrc, (lptr_t)lds_base, 4, 0, 0);
}
__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }  // vmcnt(0)

// Exchange between the two lanes l and l^32 (the two halves of a 32x32
// accumulator column).  v_permlane32_swap a, b swaps a[32..63] with b[0..31];
// with a = b = x on entry, lanes 0-31 end with (a, b) = (x[l], x[l+32]) and
// lanes 32-63 with (x[l-32], x[l]).  Written as inline asm because the
// compiler's builtin for this instruction folds its two results into one when
// both operands carry the same value.  The s_nop covers the wait states the
// instruction needs after a VALU write of its operands.
__device__ __forceinline__ void xhalf_pair(float x, float &lo, float &hi) {
  uint32_t a = __builtin_bit_cast(uint32_t, x), b = a;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
  lo = __builtin_bit_cast(float, a);
  hi = __builtin_bit_cast(float, b);
}
// v_permlane32_swap a, b in general: lanes 32..63 of a change places with lanes 0..31 of b.
__device__ __forceinline__ void permlane32_swap(uint32_t &a, uint32_t &b) {
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ float xhalf_max(float x) {
  float lo, hi;
  xhalf_pair(x, lo, hi);
  return fmaxf(lo, hi);
}
__device__ __forceinline__ float xhalf_sum(float x) {
  float lo, hi;
  xhalf_pair(x, lo, hi);
  return lo + hi;
}

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

// Work-group id remap for the 8 XCDs: hardware hands consecutive work-group
// ids to XCDs round-robin, so id i runs on XCD i % 8.  Returns a logical id
// such that each XCD gets one contiguous range of logical ids (work-groups
// that share K/V then share that XCD's L2).  `n` must be the grid size.
// `rot` turns the assignment of ranges to XCDs: with a second grid dimension that
// repeats the ids (splits of a walk), rot = blockIdx.y lets every XCD take every
// range in turn, so ranges of unequal work (causal mask) do not load the XCDs unequally.
__device__ __forceinline__ uint32_t xcd_remap(uint32_t id, uint32_t n, uint32_t rot = 0) {
  const uint32_t per = n >> 3;
  if (per == 0 || id >= per * 8) return id;  // tail keeps its id
  return ((id + rot) & 7) * per + (id >> 3);
}

// Derived sizes of a validated descriptor, shared by host code and kernels.
struct Dims {
  int B, Z, A, N, rank_begin, rank_end, causal;
  int mode;    // RSA_MODE_FUSED or RSA_MODE_STAGED
  int zigzag;  // 1: rank n owns half-chunks n and 2N-1-n (RSA_OWN_ZIGZAG)
  int64_t L, c, Lq;
  float scale;
  int deterministic;  // RSA_DETERMINISTIC was asked for (every path is deterministic already)
  // element strides of (batch, head, row) for Q/dQ, K/V/dK/dV and O/dO; strided = any not dense
  int64_t qs[3], ks[3], os[3];
  int strided;
};

// Element offset of row 0 of flat head index head = b * Z + z in a tensor whose batch, head and
// row strides are st[0], st[1], st[2].
__host__ __device__ inline int64_t head_offset(int64_t head, int Z, const int64_t *st) {
  return (head / Z) * st[0] + (head % Z) * st[1];
}

// Where a row of a strided output tensor lives, for kernels that walk (head, row) pairs flat:
// flat_row = head * rows_per_head + row.
struct OutLayout {
  int64_t st[3], rows_per_head;
  int Z;
  __host__ __device__ int64_t row_off(int64_t flat_row) const {
    return head_offset(flat_row / rows_per_head, Z, st) + (flat_row % rows_per_head) * st[2];
  }
};
inline OutLayout make_out_layout(const int64_t *st, int64_t rows_per_head, int Z) {
  OutLayout l;
  for (int k = 0; k < 3; ++k) l.st[k] = st[k];
  l.rows_per_head = rows_per_head; l.Z = Z;
  return l;
}

// Which global token a local query row is.  Contiguous ownership (the paper, section 3.1):
// rank n owns rows [n c, (n+1) c).  Zig-zag ownership: the sequence is cut into 2N
// half-chunks of h = c/2 rows and rank n owns half-chunks n and 2N-1-n, stored in that
// order, so that under the causal mask every rank sees the same number of keys.
// h is a multiple of 64: the 64 rows of a tile are consecutive tokens in both layouts.
struct RowMap {
  int64_t q0, c, h;
  int rb, last_half;  // first simulated rank; 2N - 1
  int zigzag;
  __host__ __device__ int64_t operator()(int64_t r) const {
    if (!zigzag) return q0 + r;
    const int64_t rho = rb + r / c, w = r % c;
    return w < h ? rho * h + w : (last_half - rho) * h + (w - h);
  }
  // first key of the rows [w, ...) of the chunk (pair of half-chunks) that rank j owns
  __host__ __device__ int64_t key_of(int j, int64_t w) const {
    if (!zigzag) return (int64_t)j * c + w;
    return w < h ? (int64_t)j * h + w : (int64_t)(last_half - j) * h + (w - h);
  }
  // rank that owns global token g
  __host__ __device__ int owner(int64_t g) const {
    if (!zigzag) return (int)(g / c);
    const int hc = (int)(g / h);
    return hc <= last_half / 2 ? hc : last_half - hc;
  }
};
inline RowMap make_row_map(const Dims &d) {
  RowMap m;
  m.q0 = (int64_t)d.rank_begin * d.c; m.c = d.c; m.h = d.c / 2;
  m.rb = d.rank_begin; m.last_half = 2 * d.N - 1; m.zigzag = d.zigzag;
  return m;
}

}  // namespace rsa
