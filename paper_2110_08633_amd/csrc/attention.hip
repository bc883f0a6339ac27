// Fused causal self-attention for the bf16 path (gfx950): scores, mask,
// softmax and the product with V in one kernel, and the matching backward
// kernels, so that no T x T matrix ever reaches HBM.  Only what lies on or
// below the diagonal is computed.
//
// The attention of one (sample, head): s[i,j] = q_i . k_j / sqrt(dh) for
// j <= i, p = softmax_j(s), o_i = sum_j p[i,j] v_j.  The forward kernel keeps,
// per row, only the log-sum-exp L_i = log sum_j exp(s[i,j]); the backward
// kernels rebuild p[i,j] = exp(s[i,j] - L_i) from q and k.
//
// Operand conventions are those of the GEMM kernels: v_mfma_f32_32x32x16_bf16
// with the column operand first, so a lane holds row L%32 of a 32x32 result and
// columns (r/4)*8 + (L/32)*4 + r%4 for r = 0..15.  K and V tiles of 64 keys
// are staged in LDS with the GEMM movers (K contraction-contiguous, V read with
// the transposing LDS read); probabilities go through a per-wavefront LDS patch
// to become the row operand of the second product.
#include "kernels.h"
#include "tile_ops.h"

namespace hydra {

namespace {

constexpr int AQ = 128;      // query rows per block, 32 per wavefront
constexpr int AK = 64;       // keys per tile (= BK)
constexpr int PP = AK + 8;   // pitch of the probability patch (bf16 elements): 144 bytes, conflict-free 16-byte reads
constexpr float LOG2E = 1.4426950408889634f, LN2 = 0.6931471805599453f;

__device__ __forceinline__ float xor32(float x) { return __shfl_xor(x, 32, 64); }

// column (within a 32-wide tile) of accumulator register r of this lane
__device__ __forceinline__ int acc_col(int r, int lane) { return (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3); }

__device__ __forceinline__ bf16x8_t load_frag_global(const bf16_t *p) {
  union { u32x4_t u; bf16x8_t f; } x;
  x.u = *(gvec_ptr)p;
  return x.f;
}

// A [64 rows][DH] bf16 tile of a row-major matrix, fetched once from global memory (16 bytes per lane, rows past
// the end of the sequence read as zero) and written to LDS in one or both of the operand layouts of tile_ops.h:
//   layout 0: DH/64 slices [row][64], contraction (head dimension) contiguous - operand of products over dh
//   layout 1: [row][DH] as a slice of 64 contraction steps (= rows)       - operand of products over the rows
template <int DH, int SETS = 2>
struct RowTile {
  static constexpr int CPT = DH / 8;            // 16-byte chunks per row
  static constexpr int N = 64 * CPT / 256;      // chunks per thread
  uint32_t off[N];
  int row[N], slot0[N], slot1[N];
  u32x4_t r[SETS][N];  // up to two tiles in flight: tile t travels in set t & 1 (always indexed by compile-time constants)
  __device__ __forceinline__ void init(int64_t ld, int tid) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int id = tid + i * 256;
      const int rw = id / CPT, c = id % CPT;
      row[i] = rw;
      off[i] = (uint32_t)(rw * ld + c * 8);
      slot0[i] = (c / 8) * AK * BK + (rw * CPR + ((c % 8) ^ kc_swz(rw))) * 8;
      slot1[i] = (rw * CPT + (c ^ rc_swz<DH>(rw))) * 8;
    }
  }
  // base: element (first row of the tile, first column of the head); rows_valid: rows of the tile inside the sequence
  template <int S>
  __device__ __forceinline__ void load(const bf16_t *base, int rows_valid) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      u32x4_t v = {0u, 0u, 0u, 0u};
      if (row[i] < rows_valid) v = *(gvec_ptr)(base + off[i]);
      r[S][i] = v;
    }
  }
  template <int S>
  __device__ __forceinline__ void store0(bf16_t *lds) const {
#pragma unroll
    for (int i = 0; i < N; ++i) *(u32x4_t *)(lds + slot0[i]) = r[S][i];
  }
  template <int S>
  __device__ __forceinline__ void store1(bf16_t *lds) const {
#pragma unroll
    for (int i = 0; i < N; ++i) *(u32x4_t *)(lds + slot1[i]) = r[S][i];
  }
};

template <int V> struct IntC { static constexpr int value = V; };

// four consecutive results of a lane's row -> bf16 -> the wavefront's patch [32][PP]
__device__ __forceinline__ void patch_put(bf16_t *patch, int lane, int nt, int q, const float (&w)[4]) {
  u32x2_t v;
  v.x = pack_bf16(w[0], w[1]);
  v.y = pack_bf16(w[2], w[3]);
  *(u32x2_t *)(patch + (lane & 31) * PP + nt * 32 + q * 8 + (lane >> 5) * 4) = v;
}
__device__ __forceinline__ bf16x8_t patch_get(const bf16_t *patch, int lane, int kk) {
  return *(const bf16x8_t *)(patch + (lane & 31) * PP + kk * 16 + (lane >> 5) * 8);
}
__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): this wavefront's LDS traffic has completed
  __builtin_amdgcn_wave_barrier();
}
// a lane's 32x32 result tile (row L%32) -> bf16 row segment at dst (already offset to the row and the tile)
__device__ __forceinline__ void store_tile_row(bf16_t *dst, int lane, const f32x16_t &a) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    u32x2_t w;
    w.x = pack_bf16(a[q * 4 + 0], a[q * 4 + 1]);
    w.y = pack_bf16(a[q * 4 + 2], a[q * 4 + 3]);
    *(u32x2_t *)(dst + q * 8 + (lane >> 5) * 4) = w;
  }
}

// ---------------------------------------------------------------------------
// forward: one block = 128 query rows of one (sample, head); wavefront w owns
// rows r0 = q0 + 32 w .. + 31 and keeps its Q fragments in registers.  One
// sweep over the key tiles up to the diagonal with a running row maximum and
// sum (the output is rescaled when the maximum grows and divided by the sum at
// the end).  K and V tiles are requested from global memory two tiles ahead
// (one tile's arithmetic is shorter than a trip to memory), rest in registers,
// and move into one of two LDS buffers one tile ahead; one barrier per tile.
// ---------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256) void attn_fwd_kernel(const bf16_t *__restrict__ qkv, bf16_t *__restrict__ o,
                                                       float *__restrict__ lse, int T, int H, int d,
                                                       float scale_log2e) {
  constexpr int NS = DH / 64;  // 64-wide slices of the head dimension
  constexpr int ND = DH / 32;  // 32-wide column tiles of the output
  constexpr int TILE = AK * DH;
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  bf16_t *const Ks = smem;              // [2][TILE] layout 0
  bf16_t *const Vs = Ks + 2 * TILE;     // [2][TILE] layout 1
  bf16_t *const Ps = Vs + 2 * TILE;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int qb = gridDim.x - 1 - blockIdx.x;  // blocks with the most keys first
  const int z = blockIdx.y, b = z / H, h = z % H;
  const int q0 = qb * AQ, r0 = q0 + wave * 32;
  const int64_t ld = 3 * (int64_t)d;
  const bf16_t *qp = qkv + (int64_t)b * T * ld + h * DH, *kp = qp + d, *vp = qp + 2 * d;
  const int myrow = r0 + (lane & 31);
  const int ldrow = min(myrow, T - 1);  // rows past the sequence compute on a valid row and store nothing

  bf16x8_t qf[DH / 16];
#pragma unroll
  for (int kk = 0; kk < DH / 16; ++kk) qf[kk] = load_frag_global(qp + ldrow * ld + kk * 16 + (lane >> 5) * 8);

  int ko[2][4], vo[ND][4][2];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    int unused;
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) fragment_offsets<AK, 0>(nt * 32, kk, lane, ko[nt][kk], unused);
#pragma unroll
    for (int nd = 0; nd < ND; ++nd) fragment_offsets<DH, 1>(nd * 32, kk, lane, vo[nd][kk][0], vo[nd][kk][1]);
  }
  bf16_t *const patch = Ps + wave * 32 * PP;
  const int kend = min(T, q0 + AQ);  // keys any row of the block can see
  const int ntile = (kend + AK - 1) / AK;
  const int my_last = r0 + 31;       // tiles starting beyond it hold nothing for this wavefront

  RowTile<DH> tk, tv;
  tk.init(ld, tid);
  tv.init(ld, tid);
  tk.template load<0>(kp, T);
  tv.template load<0>(vp, T);
  if (ntile > 1) {
    tk.template load<1>(kp + (int64_t)AK * ld, T - AK);
    tv.template load<1>(vp + (int64_t)AK * ld, T - AK);
  }
  tk.template store0<0>(Ks);
  tv.template store1<0>(Vs);
  __syncthreads();

  float m = -INFINITY, l = 0.f;
  f32x16_t acc[ND];
#pragma unroll
  for (int nd = 0; nd < ND; ++nd)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[nd][r] = 0.f;

  // one key tile; SET = jt & 1 is the register set tile jt travelled in (free again: tile jt is in LDS)
  auto tile_step = [&](int jt, auto setc) {
    constexpr int SET = decltype(setc)::value;
    const int j0 = jt * AK;
    const bf16_t *ks = Ks + SET * TILE, *vs = Vs + SET * TILE;
    if (jt + 2 < ntile) {  // tile jt + 2: global -> registers, in flight during this tile's and the next one's products
      tk.template load<SET>(kp + (int64_t)(j0 + 2 * AK) * ld, T - j0 - 2 * AK);
      tv.template load<SET>(vp + (int64_t)(j0 + 2 * AK) * ld, T - j0 - 2 * AK);
    }
    if (j0 <= my_last) {
      f32x16_t s[2];
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[nt][r] = 0.f;
#pragma unroll
        for (int sl = 0; sl < NS; ++sl)
#pragma unroll
          for (int kk = 0; kk < 4; ++kk)
            s[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fragment<0>(ks + sl * AK * BK, ko[nt][kk], 0),
                                                            qf[sl * 4 + kk], s[nt], 0, 0, 0);
      }
      // Vector-ALU work per score is what bounds this kernel (a wavefront instruction takes four clocks), so it is
      // kept to a maximum, a fused multiply-add, an exponential, an add and half a conversion: the scores stay
      // unscaled (the scale is positive, so it commutes with the maximum and is folded into the exponent's
      // multiply-add), and the causal mask is applied only in tiles that reach above the wavefront's first row.
      if (j0 + AK - 1 > r0) {
        const int over = j0 + (lane >> 5) * 4 - myrow;  // key - row of this lane's first column
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (over + nt * 32 + (r >> 2) * 8 + (r & 3) > 0) s[nt][r] = -INFINITY;
      }
      float tmax = s[0][0];
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) tmax = __builtin_fmaxf(tmax, s[nt][r]);
      tmax = __builtin_fmaxf(tmax, xor32(tmax));
      // The reference maximum m of a row (log2 domain) only has to keep the exponentials in range, so it is moved -
      // and the sum and the output rescaled - only when some row's maximum has outgrown it by more than 2^8; the
      // result does not depend on which reference is used.  Finite from the first tile on: key 0 is visible to
      // every row.
      const float tm = tmax * scale_log2e;
      if (__builtin_amdgcn_ballot_w64(tm > m + 8.f)) {
        const float mn = __builtin_fmaxf(m, tm);
        const float alpha = __builtin_amdgcn_exp2f(m - mn);
        m = mn;
        l *= alpha;
#pragma unroll
        for (int nd = 0; nd < ND; ++nd)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[nd][r] *= alpha;
      }
      float sum = 0.f;
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float p[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[nt][q * 4 + e], scale_log2e, -m));
            sum += p[e];
          }
          patch_put(patch, lane, nt, q, p);
        }
      l += sum;
      wave_lds_fence();
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const bf16x8_t pf = patch_get(patch, lane, kk);
#pragma unroll
        for (int nd = 0; nd < ND; ++nd)
          acc[nd] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fragment<1>(vs, vo[nd][kk][0], vo[nd][kk][1]), pf, acc[nd], 0,
                                                            0, 0);
      }
      wave_lds_fence();  // the patch has been read before the next tile overwrites it
    }
    if (jt + 1 < ntile) {
      tk.template store0<SET ^ 1>(Ks + (SET ^ 1) * TILE);
      tv.template store1<SET ^ 1>(Vs + (SET ^ 1) * TILE);
    }
    __syncthreads();
  };
  for (int jt = 0; jt < ntile; jt += 2) {
    tile_step(jt, IntC<0>());
    if (jt + 1 < ntile) tile_step(jt + 1, IntC<1>());
  }
  l += xor32(l);
  const float inv_l = 1.f / l;
  if (myrow < T) {
    if (lane < 32) lse[(int64_t)z * T + myrow] = (m + log2f(l)) * LN2;
    bf16_t *op = o + ((int64_t)b * T + myrow) * d + h * DH;
#pragma unroll
    for (int nd = 0; nd < ND; ++nd) {
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[nd][r] *= inv_l;
      store_tile_row(op + nd * 32, lane, acc[nd]);
    }
  }
}

// ---------------------------------------------------------------------------
// backward, part 1: dQ.  Same decomposition as the forward kernel (128 query
// rows per block, 32 per wavefront, key tiles up to the diagonal).  Per tile:
// p = exp(s - L), dP = dO V^T, dS = p (dP - D) / sqrt(dh) with
// D_i = sum_c dO[i,c] O[i,c] (written out for part 2), dQ += dS K.
// ---------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256) void attn_bwd_dq_kernel(const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ o,
                                                          const bf16_t *__restrict__ d_o, const float *__restrict__ lse,
                                                          float *__restrict__ dsum, bf16_t *__restrict__ dqkv, int T,
                                                          int H, int d, float scale) {
  constexpr int NS = DH / 64, ND = DH / 32;
  constexpr int TILE = AK * DH;
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  bf16_t *const Ks0 = smem;              // [2][TILE] K, layout 0 (scores)
  bf16_t *const Ks1 = Ks0 + 2 * TILE;    // [2][TILE] K, layout 1 (dQ += dS K contracts over keys)
  bf16_t *const Vs0 = Ks1 + 2 * TILE;    // [2][TILE] V, layout 0 (dP = dO V^T)
  bf16_t *const Ps = Vs0 + 2 * TILE;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int qb = gridDim.x - 1 - blockIdx.x;
  const int z = blockIdx.y, b = z / H, h = z % H;
  const int q0 = qb * AQ, r0 = q0 + wave * 32;
  const int64_t ld = 3 * (int64_t)d;
  const bf16_t *qp = qkv + (int64_t)b * T * ld + h * DH, *kp = qp + d, *vp = qp + 2 * d;
  const int myrow = r0 + (lane & 31);
  const int ldrow = min(myrow, T - 1);

  bf16x8_t qf[DH / 16], dof[DH / 16];
  float dsum_part = 0.f;
  {
    const bf16_t *dop = d_o + ((int64_t)b * T + ldrow) * d + h * DH, *op = o + ((int64_t)b * T + ldrow) * d + h * DH;
#pragma unroll
    for (int kk = 0; kk < DH / 16; ++kk) {
      const int c = kk * 16 + (lane >> 5) * 8;
      qf[kk] = load_frag_global(qp + ldrow * ld + c);
      dof[kk] = load_frag_global(dop + c);
      const bf16x8_t of = load_frag_global(op + c);
#pragma unroll
      for (int e = 0; e < 8; ++e) dsum_part += (float)dof[kk][e] * (float)of[e];
    }
  }
  const float Di = dsum_part + xor32(dsum_part);
  const float L2 = lse[(int64_t)z * T + ldrow] * LOG2E;
  if (lane < 32 && myrow < T) dsum[(int64_t)z * T + myrow] = Di;

  int ko[2][4], vo[ND][4][2];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    int unused;
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) fragment_offsets<AK, 0>(nt * 32, kk, lane, ko[nt][kk], unused);
#pragma unroll
    for (int nd = 0; nd < ND; ++nd) fragment_offsets<DH, 1>(nd * 32, kk, lane, vo[nd][kk][0], vo[nd][kk][1]);
  }
  bf16_t *const patch = Ps + wave * 32 * PP;
  const int kend = min(T, q0 + AQ);
  const int ntile = (kend + AK - 1) / AK;
  const int my_last = r0 + 31;
  const float scale_log2e = scale * LOG2E;
  const float nL2 = -L2, nDs = -Di * scale;

  RowTile<DH> tk, tv;
  tk.init(ld, tid);
  tv.init(ld, tid);
  tk.template load<0>(kp, T);
  tv.template load<0>(vp, T);
  if (ntile > 1) {
    tk.template load<1>(kp + (int64_t)AK * ld, T - AK);
    tv.template load<1>(vp + (int64_t)AK * ld, T - AK);
  }
  tk.template store0<0>(Ks0);
  tk.template store1<0>(Ks1);
  tv.template store0<0>(Vs0);
  __syncthreads();

  f32x16_t acc[ND];
#pragma unroll
  for (int nd = 0; nd < ND; ++nd)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[nd][r] = 0.f;

  // staging as in the forward kernel: tiles requested two ahead, SET = jt & 1
  auto tile_step = [&](int jt, auto setc) {
    constexpr int SET = decltype(setc)::value;
    const int j0 = jt * AK, cur = SET * TILE, nxt = (SET ^ 1) * TILE;
    if (jt + 2 < ntile) {
      tk.template load<SET>(kp + (int64_t)(j0 + 2 * AK) * ld, T - j0 - 2 * AK);
      tv.template load<SET>(vp + (int64_t)(j0 + 2 * AK) * ld, T - j0 - 2 * AK);
    }
    if (j0 <= my_last) {
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
        f32x16_t s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = dp[r] = 0.f;
#pragma unroll
        for (int sl = 0; sl < NS; ++sl)
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) {
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fragment<0>(Ks0 + cur + sl * AK * BK, ko[nt][kk], 0),
                                                        qf[sl * 4 + kk], s, 0, 0, 0);
            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fragment<0>(Vs0 + cur + sl * AK * BK, ko[nt][kk], 0),
                                                         dof[sl * 4 + kk], dp, 0, 0, 0);
          }
        // as in the forward kernel the vector-ALU work per score is kept minimal: the mask only where the tile
        // reaches above the wavefront's first row (a masked score of -inf gives p = 0 exactly), the scale folded
        // into two fused multiply-adds
        if (j0 + nt * 32 + 31 > r0) {
          const int over = j0 + nt * 32 + (lane >> 5) * 4 - myrow;
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (over + (r >> 2) * 8 + (r & 3) > 0) s[r] = -INFINITY;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float ds[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[q * 4 + e], scale_log2e, nL2));
            ds[e] = p * __builtin_fmaf(dp[q * 4 + e], scale, nDs);
          }
          patch_put(patch, lane, nt, q, ds);
        }
      }
      wave_lds_fence();
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const bf16x8_t df = patch_get(patch, lane, kk);
#pragma unroll
        for (int nd = 0; nd < ND; ++nd)
          acc[nd] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fragment<1>(Ks1 + cur, vo[nd][kk][0], vo[nd][kk][1]), df,
                                                            acc[nd], 0, 0, 0);
      }
      wave_lds_fence();
    }
    if (jt + 1 < ntile) {
      tk.template store0<SET ^ 1>(Ks0 + nxt);
      tk.template store1<SET ^ 1>(Ks1 + nxt);
      tv.template store0<SET ^ 1>(Vs0 + nxt);
    }
    __syncthreads();
  };
  for (int jt = 0; jt < ntile; jt += 2) {
    tile_step(jt, IntC<0>());
    if (jt + 1 < ntile) tile_step(jt + 1, IntC<1>());
  }
  if (myrow < T) {
    bf16_t *dq = dqkv + ((int64_t)b * T + myrow) * ld + h * DH;
#pragma unroll
    for (int nd = 0; nd < ND; ++nd) store_tile_row(dq + nd * 32, lane, acc[nd]);
  }
}

// ---------------------------------------------------------------------------
// backward, part 2: dK and dV.  One block = 128 keys of one (sample, head),
// wavefront w owns keys kr0 = k0 + 32 w .. + 31 and keeps their K and V
// fragments in registers.  It walks the query tiles (64 rows) from the diagonal
// to the end of the sequence, computing the transposed quantities directly:
// s^T = K Q^T, p^T = exp(s^T - L), dP^T = V dO^T, dS^T = p^T (dP^T - D)/sqrt(dh),
// dV += p^T dO, dK += dS^T Q.  No atomics: every key row has one owner.
// ---------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256) void attn_bwd_dkv_kernel(const bf16_t *__restrict__ qkv,
                                                           const bf16_t *__restrict__ d_o,
                                                           const float *__restrict__ lse,
                                                           const float *__restrict__ dsum, bf16_t *__restrict__ dqkv,
                                                           int T, int H, int d, float scale) {
  constexpr int NS = DH / 64, ND = DH / 32;
  constexpr int TILE = AK * DH;
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  bf16_t *const Qs0 = smem;              // [2][TILE] Q, layout 0 (s^T)
  bf16_t *const Qs1 = Qs0 + 2 * TILE;    // [2][TILE] Q, layout 1 (dK += dS^T Q contracts over queries)
  bf16_t *const Os0 = Qs1 + 2 * TILE;    // [2][TILE] dO, layout 0 (dP^T)
  bf16_t *const Os1 = Os0 + 2 * TILE;    // [2][TILE] dO, layout 1 (dV += p^T dO)
  bf16_t *const Ps = Os1 + 2 * TILE;
  float *const Ls = (float *)(Ps + 4 * 32 * PP);  // [2][128]: -log-sum-exp (log2 domain) and -D / sqrt(dh) of the tile's 64 queries
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kb = blockIdx.x;
  const int z = blockIdx.y, b = z / H, h = z % H;
  const int k0 = kb * AQ, kr0 = k0 + wave * 32;
  const int64_t ld = 3 * (int64_t)d;
  const bf16_t *qp = qkv + (int64_t)b * T * ld + h * DH, *kp = qp + d, *vp = qp + 2 * d;
  const bf16_t *dop = d_o + (int64_t)b * T * d + h * DH;
  const int mykey = kr0 + (lane & 31);
  const int ldkey = min(mykey, T - 1);

  bf16x8_t kf[DH / 16], vf[DH / 16];
#pragma unroll
  for (int kk = 0; kk < DH / 16; ++kk) {
    const int c = kk * 16 + (lane >> 5) * 8;
    kf[kk] = load_frag_global(kp + ldkey * ld + c);
    vf[kk] = load_frag_global(vp + ldkey * ld + c);
  }
  int ko[2][4], vo[ND][4][2];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    int unused;
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) fragment_offsets<AK, 0>(nt * 32, kk, lane, ko[nt][kk], unused);
#pragma unroll
    for (int nd = 0; nd < ND; ++nd) fragment_offsets<DH, 1>(nd * 32, kk, lane, vo[nd][kk][0], vo[nd][kk][1]);
  }
  bf16_t *const patch = Ps + wave * 32 * PP;
  const float scale_log2e = scale * LOG2E;

  f32x16_t dk[ND], dv[ND];
#pragma unroll
  for (int nd = 0; nd < ND; ++nd)
#pragma unroll
    for (int r = 0; r < 16; ++r) dk[nd][r] = dv[nd][r] = 0.f;

  // head width 128 has no registers left for a second tile in flight (it would spill): one tile ahead there
  constexpr bool FAR = DH <= 64;
  RowTile<DH, FAR ? 2 : 1> tq, to;
  tq.init(ld, tid);
  to.init(d, tid);
  const int ibeg = (k0 / AK) * AK;
  float stat0 = 0.f, stat1 = 0.f;  // this thread's entry of the statistics of the two tiles in flight
  auto load_stat = [&](int i0) -> float {
    float st = 0.f;
    if (tid < 128) {
      const int qi = i0 + (tid & 63);
      if (qi < T) st = tid < 64 ? -lse[(int64_t)z * T + qi] * LOG2E : -dsum[(int64_t)z * T + qi] * scale;
    }
    return st;
  };
  tq.template load<0>(qp + (int64_t)ibeg * ld, T - ibeg);
  to.template load<0>(dop + (int64_t)ibeg * d, T - ibeg);
  stat0 = load_stat(ibeg);
  if (FAR && ibeg + AK < T) {
    tq.template load<FAR ? 1 : 0>(qp + (int64_t)(ibeg + AK) * ld, T - ibeg - AK);
    to.template load<FAR ? 1 : 0>(dop + (int64_t)(ibeg + AK) * d, T - ibeg - AK);
    stat1 = load_stat(ibeg + AK);
  }
  tq.template store0<0>(Qs0);
  tq.template store1<0>(Qs1);
  to.template store0<0>(Os0);
  to.template store1<0>(Os1);
  if (tid < 128) Ls[tid] = stat0;
  __syncthreads();

  // one query tile; SET = it & 1.  Tiles are requested from global memory two ahead, as in the other two kernels.
  // (par = parity of the tile's index = its LDS buffer; with FAR it equals SET, otherwise only set 0 is used)
  auto tile_step = [&](int i0, int par, auto setc) {
    constexpr int SET = decltype(setc)::value;
    const int cur = par * TILE, nxt = (par ^ 1) * TILE;
    const float *ls = Ls + par * 128;
    const bool more = i0 + AK < T;
    if (FAR && i0 + 2 * AK < T) {
      tq.template load<FAR ? SET : 0>(qp + (int64_t)(i0 + 2 * AK) * ld, T - i0 - 2 * AK);
      to.template load<FAR ? SET : 0>(dop + (int64_t)(i0 + 2 * AK) * d, T - i0 - 2 * AK);
      (SET ? stat1 : stat0) = load_stat(i0 + 2 * AK);
    }
    if (!FAR && more) {
      tq.template load<0>(qp + (int64_t)(i0 + AK) * ld, T - i0 - AK);
      to.template load<0>(dop + (int64_t)(i0 + AK) * d, T - i0 - AK);
      stat0 = load_stat(i0 + AK);
    }
    if (i0 + AK - 1 >= kr0) {  // else every query of the tile precedes every key of this wavefront
      f32x16_t s[2], dp[2];
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[nt][r] = dp[nt][r] = 0.f;
#pragma unroll
        for (int sl = 0; sl < NS; ++sl)
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) {
            s[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fragment<0>(Qs0 + cur + sl * AK * BK, ko[nt][kk], 0),
                                                            kf[sl * 4 + kk], s[nt], 0, 0, 0);
            dp[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fragment<0>(Os0 + cur + sl * AK * BK, ko[nt][kk], 0),
                                                             vf[sl * 4 + kk], dp[nt], 0, 0, 0);
          }
        // p^T into the patch; dS^T replaces s in registers for the second round.  The mask is needed only where
        // the tile holds queries that precede keys of this wavefront; queries past the end of the sequence need
        // none (their Q and dO rows are zero-filled and their statistics zero, so they contribute exact zeros).
        // ls holds -L (log2 domain) and -D / sqrt(dh) of the tile's queries.
        if (i0 + nt * 32 < kr0 + 31) {
          const int under = mykey - (i0 + nt * 32 + (lane >> 5) * 4);  // key - query of this lane's first column
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (under - ((r >> 2) * 8 + (r & 3)) > 0) s[nt][r] = -INFINITY;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int qc = nt * 32 + q * 8 + (lane >> 5) * 4;  // first of this lane's four queries within the tile
          const f32x4_t nl = *(const f32x4_t *)(ls + qc), nd4 = *(const f32x4_t *)(ls + 64 + qc);
          float p4[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[nt][q * 4 + e], scale_log2e, nl[e]));
            p4[e] = p;
            s[nt][q * 4 + e] = p * __builtin_fmaf(dp[nt][q * 4 + e], scale, nd4[e]);
          }
          patch_put(patch, lane, nt, q, p4);
        }
      }
      wave_lds_fence();
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const bf16x8_t pf = patch_get(patch, lane, kk);
#pragma unroll
        for (int nd = 0; nd < ND; ++nd)
          dv[nd] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fragment<1>(Os1 + cur, vo[nd][kk][0], vo[nd][kk][1]), pf,
                                                           dv[nd], 0, 0, 0);
      }
      wave_lds_fence();
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float w4[4] = {s[nt][q * 4 + 0], s[nt][q * 4 + 1], s[nt][q * 4 + 2], s[nt][q * 4 + 3]};
          patch_put(patch, lane, nt, q, w4);
        }
      wave_lds_fence();
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const bf16x8_t pf = patch_get(patch, lane, kk);
#pragma unroll
        for (int nd = 0; nd < ND; ++nd)
          dk[nd] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fragment<1>(Qs1 + cur, vo[nd][kk][0], vo[nd][kk][1]), pf,
                                                           dk[nd], 0, 0, 0);
      }
      wave_lds_fence();
    }
    if (more) {
      constexpr int NS_ = FAR ? (SET ^ 1) : 0;  // register set the next tile travelled in
      tq.template store0<NS_>(Qs0 + nxt);
      tq.template store1<NS_>(Qs1 + nxt);
      to.template store0<NS_>(Os0 + nxt);
      to.template store1<NS_>(Os1 + nxt);
      if (tid < 128) Ls[(par ^ 1) * 128 + tid] = NS_ ? stat1 : stat0;
    }
    __syncthreads();
  };
  if (FAR) {
    for (int i0 = ibeg; i0 < T; i0 += 2 * AK) {
      tile_step(i0, 0, IntC<0>());
      if (i0 + AK < T) tile_step(i0 + AK, 1, IntC<1>());
    }
  } else {
    int it = 0;
    for (int i0 = ibeg; i0 < T; i0 += AK, ++it) tile_step(i0, it & 1, IntC<0>());
  }
  if (mykey < T) {
    bf16_t *dkp = dqkv + ((int64_t)b * T + mykey) * ld + d + h * DH, *dvp = dkp + d;
#pragma unroll
    for (int nd = 0; nd < ND; ++nd) {
      store_tile_row(dkp + nd * 32, lane, dk[nd]);
      store_tile_row(dvp + nd * 32, lane, dv[nd]);
    }
  }
}

}  // namespace

bool attention_fused_supported(int dtype, int dh) { return dtype == DT_BF16 && (dh == 64 || dh == 128); }

template <typename K>
static hipError_t set_lds(K kern, size_t bytes) {
  return hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

hipError_t launch_attention_fwd(const void *qkv, void *o, float *lse, int B, int H, int T, int dh, hipStream_t s) {
  const int d = H * dh;
  const float scale_log2e = LOG2E / sqrtf((float)dh);
  dim3 grid((T + AQ - 1) / AQ, B * H);
  const size_t lds = (size_t)(4 * AK * dh + 4 * 32 * PP) * 2;
  // causal half of both products
  ProfScope ps("attention_fwd", s, 2.0 * B * H * dh * ((double)T * (T + 1.0)), 0);
#define HYDRA_ATTN_FWD(DH_)                                                                                     \
  do {                                                                                                           \
    static hipError_t a1 = set_lds(attn_fwd_kernel<DH_>, lds);                                                   \
    if (a1 != hipSuccess) return a1;                                                                             \
    hipLaunchKernelGGL(attn_fwd_kernel<DH_>, grid, dim3(256), lds, s, (const bf16_t *)qkv, (bf16_t *)o, lse, T, H, \
                       d, scale_log2e);                                                                          \
  } while (0)
  if (dh == 64) HYDRA_ATTN_FWD(64);
  else if (dh == 128) HYDRA_ATTN_FWD(128);
  else return hipErrorInvalidValue;
#undef HYDRA_ATTN_FWD
  return hipGetLastError();
}

hipError_t launch_attention_bwd(const void *qkv, const void *o, const void *d_o, const float *lse, float *dsum,
                                void *dqkv, int B, int H, int T, int dh, hipStream_t s) {
  const int d = H * dh;
  const float scale = 1.0f / sqrtf((float)dh);
  dim3 grid((T + AQ - 1) / AQ, B * H);
  const size_t lds_dq = (size_t)(6 * AK * dh + 4 * 32 * PP) * 2;
  const size_t lds_dkv = (size_t)(8 * AK * dh + 4 * 32 * PP) * 2 + 256 * 4;
  // five causal products of T x T x dh each (s and dP in both kernels count once: the recomputation is overhead)
  ProfScope ps("attention_bwd", s, 5.0 * B * H * dh * ((double)T * (T + 1.0)), 0);
#define HYDRA_ATTN_BWD(DH_)                                                                                        \
  do {                                                                                                              \
    static hipError_t a1 = set_lds(attn_bwd_dq_kernel<DH_>, lds_dq), a2 = set_lds(attn_bwd_dkv_kernel<DH_>, lds_dkv); \
    if (a1 != hipSuccess) return a1;                                                                                \
    if (a2 != hipSuccess) return a2;                                                                                \
    hipLaunchKernelGGL(attn_bwd_dq_kernel<DH_>, grid, dim3(256), lds_dq, s, (const bf16_t *)qkv, (const bf16_t *)o, \
                       (const bf16_t *)d_o, lse, dsum, (bf16_t *)dqkv, T, H, d, scale);                             \
    hipLaunchKernelGGL(attn_bwd_dkv_kernel<DH_>, grid, dim3(256), lds_dkv, s, (const bf16_t *)qkv,                  \
                       (const bf16_t *)d_o, lse, dsum, (bf16_t *)dqkv, T, H, d, scale);                             \
  } while (0)
  if (dh == 64) HYDRA_ATTN_BWD(64);
  else if (dh == 128) HYDRA_ATTN_BWD(128);
  else return hipErrorInvalidValue;
#undef HYDRA_ATTN_BWD
  return hipGetLastError();
}

}  // namespace hydra
