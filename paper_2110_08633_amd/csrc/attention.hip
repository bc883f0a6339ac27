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
template <int DH>
struct RowTile {
  static constexpr int CPT = DH / 8;            // 16-byte chunks per row
  static constexpr int N = 64 * CPT / 256;      // chunks per thread
  uint32_t off[N];
  int row[N], slot0[N], slot1[N];
  u32x4_t r[N];
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
  __device__ __forceinline__ void load(const bf16_t *base, int rows_valid) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      u32x4_t v = {0u, 0u, 0u, 0u};
      if (row[i] < rows_valid) v = *(gvec_ptr)(base + off[i]);
      r[i] = v;
    }
  }
  __device__ __forceinline__ void store0(bf16_t *lds) const {
#pragma unroll
    for (int i = 0; i < N; ++i) *(u32x4_t *)(lds + slot0[i]) = r[i];
  }
  __device__ __forceinline__ void store1(bf16_t *lds) const {
#pragma unroll
    for (int i = 0; i < N; ++i) *(u32x4_t *)(lds + slot1[i]) = r[i];
  }
};

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
// the end).  The next tile's K and V are in flight from global memory while the
// current one is multiplied; two LDS buffers, one barrier per tile.
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
  tk.load(kp, T);
  tv.load(vp, T);
  tk.store0(Ks);
  tv.store1(Vs);
  __syncthreads();

  float m = -INFINITY, l = 0.f;
  f32x16_t acc[ND];
#pragma unroll
  for (int nd = 0; nd < ND; ++nd)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[nd][r] = 0.f;

  for (int jt = 0; jt < ntile; ++jt) {
    const int j0 = jt * AK;
    const bf16_t *ks = Ks + (jt & 1) * TILE, *vs = Vs + (jt & 1) * TILE;
    if (jt + 1 < ntile) {  // next tile: global -> registers, in flight during the products below
      tk.load(kp + (int64_t)(j0 + AK) * ld, T - j0 - AK);
      tv.load(vp + (int64_t)(j0 + AK) * ld, T - j0 - AK);
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
      float tmax = -INFINITY;
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = j0 + nt * 32 + acc_col(r, lane);
          const float v = (key <= myrow && key < T) ? s[nt][r] * scale_log2e : -INFINITY;
          s[nt][r] = v;
          tmax = fmaxf(tmax, v);
        }
      tmax = fmaxf(tmax, xor32(tmax));
      const float mn = fmaxf(m, tmax);  // finite from the first tile on: key 0 is visible to every row
      const float alpha = exp2f(m - mn);
      m = mn;
      float sum = 0.f;
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float p[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            p[e] = exp2f(s[nt][q * 4 + e] - mn);
            sum += p[e];
          }
          patch_put(patch, lane, nt, q, p);
        }
      l = l * alpha + sum;
#pragma unroll
      for (int nd = 0; nd < ND; ++nd)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[nd][r] *= alpha;
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
      tk.store0(Ks + ((jt + 1) & 1) * TILE);
      tv.store1(Vs + ((jt + 1) & 1) * TILE);
    }
    __syncthreads();
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

  RowTile<DH> tk, tv;
  tk.init(ld, tid);
  tv.init(ld, tid);
  tk.load(kp, T);
  tv.load(vp, T);
  tk.store0(Ks0);
  tk.store1(Ks1);
  tv.store0(Vs0);
  __syncthreads();

  f32x16_t acc[ND];
#pragma unroll
  for (int nd = 0; nd < ND; ++nd)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[nd][r] = 0.f;

  for (int jt = 0; jt < ntile; ++jt) {
    const int j0 = jt * AK, cur = (jt & 1) * TILE, nxt = ((jt + 1) & 1) * TILE;
    if (jt + 1 < ntile) {
      tk.load(kp + (int64_t)(j0 + AK) * ld, T - j0 - AK);
      tv.load(vp + (int64_t)(j0 + AK) * ld, T - j0 - AK);
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
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float ds[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int key = j0 + nt * 32 + q * 8 + (lane >> 5) * 4 + e;
            const float p = (key <= myrow && key < T) ? exp2f(s[q * 4 + e] * scale_log2e - L2) : 0.f;
            ds[e] = p * (dp[q * 4 + e] - Di) * scale;
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
      tk.store0(Ks0 + nxt);
      tk.store1(Ks1 + nxt);
      tv.store0(Vs0 + nxt);
    }
    __syncthreads();
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
  float *const Ls = (float *)(Ps + 4 * 32 * PP);  // [2][128]: log-sum-exp (log2 domain) and D of the tile's 64 queries
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

  RowTile<DH> tq, to;
  tq.init(ld, tid);
  to.init(d, tid);
  const int ibeg = (k0 / AK) * AK;
  float stat = 0.f;  // this thread's entry of the next tile's statistics
  auto load_stat = [&](int i0) {
    stat = 0.f;
    if (tid < 128) {
      const int qi = i0 + (tid & 63);
      if (qi < T) stat = tid < 64 ? lse[(int64_t)z * T + qi] * LOG2E : dsum[(int64_t)z * T + qi];
    }
  };
  tq.load(qp + (int64_t)ibeg * ld, T - ibeg);
  to.load(dop + (int64_t)ibeg * d, T - ibeg);
  load_stat(ibeg);
  tq.store0(Qs0);
  tq.store1(Qs1);
  to.store0(Os0);
  to.store1(Os1);
  if (tid < 128) Ls[tid] = stat;
  __syncthreads();

  int it = 0;
  for (int i0 = ibeg; i0 < T; i0 += AK, ++it) {
    const int cur = (it & 1) * TILE, nxt = ((it + 1) & 1) * TILE;
    const float *ls = Ls + (it & 1) * 128;
    const bool more = i0 + AK < T;
    if (more) {
      tq.load(qp + (int64_t)(i0 + AK) * ld, T - i0 - AK);
      to.load(dop + (int64_t)(i0 + AK) * d, T - i0 - AK);
      load_stat(i0 + AK);
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
        // p^T into the patch; dS^T replaces s in registers for the second round
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float p4[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int qc = nt * 32 + q * 8 + (lane >> 5) * 4 + e;  // query within the tile
            const int qi = i0 + qc;
            const float p = (qi >= mykey && qi < T) ? exp2f(s[nt][q * 4 + e] * scale_log2e - ls[qc]) : 0.f;
            p4[e] = p;
            s[nt][q * 4 + e] = p * (dp[nt][q * 4 + e] - ls[64 + qc]) * scale;
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
      tq.store0(Qs0 + nxt);
      tq.store1(Qs1 + nxt);
      to.store0(Os0 + nxt);
      to.store1(Os1 + nxt);
      if (tid < 128) Ls[((it + 1) & 1) * 128 + tid] = stat;
    }
    __syncthreads();
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
