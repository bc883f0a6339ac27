// Device-side building blocks shared by the MFMA kernels (gfx950): operand tiles in LDS, their swizzles, the
// global -> register -> LDS mover and the MFMA fragment reads.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace hydra {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;


__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
__device__ __forceinline__ bf16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);                                          // round to nearest even
  return (bf16_t)(u >> 16);
}


constexpr int BK = 64;
constexpr int CPR = BK / 8;  // 16-byte chunks per row of a contraction-contiguous tile
// swizzle of a contraction-contiguous tile: 16 neighbouring rows must land in 16 distinct 16-byte bank groups
__device__ __forceinline__ int kc_swz(int row) { return BK == 64 ? ((row >> 1) & 7) : ((row >> 2) & 3); }
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

// operands live in global memory: say so, or the loads become flat loads that also count as LDS traffic
typedef const __attribute__((address_space(1))) u32x4_t *gvec_ptr;

template <int R> __device__ __forceinline__ int rc_swz(int k) {
  return (R / 8 >= 16) ? ((k & 3) << 2) : (((k >> 1) & 1) << 2);
}

// Global -> register -> LDS mover of one operand.  All per-thread addressing is
// computed once: a slice load is base (uniform) + 32-bit per-thread offset.
//   RCL = 0: memory is [rows][K] (contraction contiguous): LDS [row][BK], chunk kc of row r at slot r*CPR + (kc ^ kc_swz(r))
//   RCL = 1: memory is [K][rows] (rows contiguous):        LDS [k][R],    chunk c of slice row k at slot k*(R/8) + (c ^ swz(k))
// Rows beyond the matrix are redirected to a valid row: they only feed rows /
// columns of C that are never stored.  The contraction tail is zero-filled.
template <int R, int RCL>
struct Mover {
  static constexpr int N = R * CPR / 256;  // 16-byte chunks per thread and slice
  static constexpr int CPK = R / 8;
  const bf16_t *base;   // uniform: element (row0, kbeg) of the operand
  int64_t kstep;        // uniform: elements per slice
  uint32_t off[N];      // per-thread element offset inside a slice
  int kloc[N];          // first contraction index of the chunk inside a slice
  int slot[N];          // LDS element offset
  __device__ __forceinline__ void init(const bf16_t *mat, int64_t ld, int row0, int rows, int kbeg, int tid) {
    if (!RCL) {
      base = mat + (int64_t)row0 * ld + kbeg;
      kstep = BK;
    } else {
      base = mat + (int64_t)kbeg * ld + row0;
      kstep = (int64_t)BK * ld;
    }
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int id = tid + i * 256;
      if (!RCL) {
        int row = id / CPR;
        const int kc = id % CPR;
        slot[i] = (row * CPR + (kc ^ kc_swz(row))) * 8;
        if (row0 + row >= rows) row = 0;
        off[i] = (uint32_t)(row * ld + kc * 8);
        kloc[i] = kc * 8;
      } else {
        const int k = id / CPK;
        int c = id % CPK;
        slot[i] = (k * CPK + (c ^ rc_swz<R>(k))) * 8;
        if (row0 + c * 8 >= rows) c = 0;
        off[i] = (uint32_t)(k * ld + c * 8);
        kloc[i] = k;
      }
    }
  }
  // slice t (0-based from kbeg), known to lie entirely inside the contraction range
  __device__ __forceinline__ void load_full(u32x4_t (&r)[N], int t) const {
    const bf16_t *b = base + t * kstep;
#pragma unroll
    for (int i = 0; i < N; ++i) r[i] = *(gvec_ptr)(b + off[i]);
  }
  // any slice; krem = contraction steps left at the start of the slice
  __device__ __forceinline__ void load_tail(u32x4_t (&r)[N], int t, int krem) const {
    const bf16_t *b = base + t * kstep;
#pragma unroll
    for (int i = 0; i < N; ++i) {
      u32x4_t v = {0u, 0u, 0u, 0u};
      if (kloc[i] < krem) v = *(gvec_ptr)(b + off[i]);
      r[i] = v;
    }
  }
  __device__ __forceinline__ void store(const u32x4_t (&r)[N], bf16_t *lds) const {
#pragma unroll
    for (int i = 0; i < N; ++i) *(u32x4_t *)(lds + slot[i]) = r[i];
  }
};

// LDS element offsets of the MFMA operand for 32 rows starting at rb and the 16 contraction steps
// kk16*16..+15 of a slice: lane L holds row rb + L%32, steps (L/32)*8 .. +7
template <int R, int RCL>
__device__ __forceinline__ void fragment_offsets(int rb, int kk16, int lane, int &o0, int &o1) {
  if (!RCL) {
    const int row = rb + (lane & 31), kc = kk16 * 2 + (lane >> 5);
    o0 = (row * CPR + (kc ^ kc_swz(row))) * 8;
    o1 = 0;
  } else {
    // transposing read: within each group of 16 lanes, lane i receives element i%4 of the 8 bytes
    // addressed by lanes i/4, i/4+4, i/4+8, i/4+12 of the group
    constexpr int CPK = R / 8;
    const int G = lane >> 4, sl = lane & 15;
    const int k = kk16 * 16 + (G >> 1) * 8 + (sl >> 2);
    const int m = rb + 16 * (G & 1) + 4 * (sl & 3);
    const int c = m >> 3, half = (m >> 2) & 1;
    o0 = (k * CPK + (c ^ rc_swz<R>(k))) * 8 + half * 4;
    o1 = ((k + 4) * CPK + (c ^ rc_swz<R>(k + 4))) * 8 + half * 4;
  }
}

template <int RCL>
__device__ __forceinline__ bf16x8_t fragment(const bf16_t *lds, int o0, int o1) {
  if (!RCL) {
    return *(const bf16x8_t *)(lds + o0);
  } else {
    const s16x4_t v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t *)(lds + o0));
    const s16x4_t v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t *)(lds + o1));
    union { s16x4_t h[2]; bf16x8_t f; } u;
    u.h[0] = v0;
    u.h[1] = v1;
    return u.f;
  }
}

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
// two fp32 -> packed bf16, round to nearest even (one instruction on gfx950)
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  const f32x2_t v = {a, b};
  union { bf16x2_t h; uint32_t u; } x;
  x.h = __builtin_convertvector(v, bf16x2_t);
  return x.u;
}
}  // namespace hydra
