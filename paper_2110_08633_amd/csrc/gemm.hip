// GEMM kernels for gfx950: bf16 MFMA (LDS-tiled, fp32 accumulate) and a plain
// fp32 kernel, both with the same fused epilogues (bias, residual, GELU,
// GELU', scale) and the same causal short-cuts for attention operands.
//
// The linear layers of a block (y = x*W + b), their input gradients
// (dx = dy*W^T) and weight gradients (dW = x^T*dy) and the batched attention
// products are all instances of C = alpha * op(A) * op(B) with a row-major C.
#include "kernels.h"

namespace hydra {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

struct GemmArgs {
  const void *A, *B;
  int M, N, K;
  int64_t lda, ldb, ldc;
  int nb2;
  int64_t sA1, sA2, sB1, sB2, sC1, sC2;
  float alpha;
  const float *bias, *resid;
  float *out_f32;
  void *out_act, *out_act2;
  const void *aux;
  int epi, causal;
  int tiles_m, tiles_n;
};

__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
__device__ __forceinline__ bf16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);                                          // round to nearest even
  return (bf16_t)(u >> 16);
}

template <typename T> __device__ __forceinline__ float ld_act(const void *p, int64_t i);
template <> __device__ __forceinline__ float ld_act<float>(const void *p, int64_t i) { return ((const float *)p)[i]; }
template <> __device__ __forceinline__ float ld_act<bf16_t>(const void *p, int64_t i) { return bf2f(((const bf16_t *)p)[i]); }
template <typename T> __device__ __forceinline__ void st_act(void *p, int64_t i, float v);
template <> __device__ __forceinline__ void st_act<float>(void *p, int64_t i, float v) { ((float *)p)[i] = v; }
template <> __device__ __forceinline__ void st_act<bf16_t>(void *p, int64_t i, float v) { ((bf16_t *)p)[i] = f2bf(v); }

// tanh-form GELU and its derivative (fp32)
__device__ __forceinline__ float gelu_f(float u) {
  const float c = 0.7978845608028654f;
  float t = tanhf(c * (u + 0.044715f * u * u * u));
  return 0.5f * u * (1.f + t);
}
__device__ __forceinline__ float dgelu_f(float u) {
  const float c = 0.7978845608028654f;
  float t = tanhf(c * (u + 0.044715f * u * u * u));
  float dt = (1.f - t * t) * c * (1.f + 3.f * 0.044715f * u * u);
  return 0.5f * (1.f + t) + 0.5f * u * dt;
}

template <typename ActT>
__device__ __forceinline__ void epilogue_store(const GemmArgs &g, int64_t coff, int row, int col, float acc) {
  float v = acc * g.alpha;
  if (g.bias) v += g.bias[col];
  const int64_t idx = coff + (int64_t)row * g.ldc + col;
  if (g.epi == EPI_GELU) {
    st_act<ActT>(g.out_act, idx, v);
    st_act<ActT>(g.out_act2, idx, gelu_f(v));
    return;
  }
  if (g.epi == EPI_DGELU) v *= dgelu_f(ld_act<ActT>(g.aux, idx));
  if (g.resid) v += g.resid[idx];
  if (g.out_f32) g.out_f32[idx] = v;
  if (g.out_act) st_act<ActT>(g.out_act, idx, v);
}

// ---------------------------------------------------------------------------
// bf16 MFMA kernel.  256 threads = 4 wavefronts arranged WM x WN over a
// BM x BN tile; K is consumed in slices of BK = 64 staged through LDS in
// K-contiguous form [row][BK + 8] (the 16-byte pad makes the 128-bit operand
// reads conflict-free).  Operands that are stored with the contraction index
// strided (ta / tb) are transposed in registers on their way into LDS.
// ---------------------------------------------------------------------------
constexpr int BK = 64;
constexpr int LDSP = BK + 8;  // row pitch in elements

// K-contiguous source: rows x BK tile, 16-byte chunks
template <int ROWS>
struct TileKC {
  static constexpr int NCH = ROWS * (BK / 8) / 256;  // chunks per thread
  u32x4_t r[NCH];
  __device__ __forceinline__ void load(const bf16_t *__restrict__ base, int64_t ld, int row0, int rows, int k0, int kend,
                                       int tid) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int id = tid + i * 256;
      const int row = id >> 3, kc = (id & 7) * 8;
      u32x4_t v = {0u, 0u, 0u, 0u};
      if (row0 + row < rows && k0 + kc < kend) v = *(const u32x4_t *)(base + (int64_t)(row0 + row) * ld + k0 + kc);
      r[i] = v;
    }
  }
  __device__ __forceinline__ void store(bf16_t *lds, int tid) const {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int id = tid + i * 256;
      const int row = id >> 3, kc = (id & 7) * 8;
      *(u32x4_t *)(lds + row * LDSP + kc) = r[i];
    }
  }
};

// row-contiguous source (stored [K][rows]): BK x ROWS tile read as 4(k) x 8(row)
// blocks, transposed in registers, written as 8-byte pieces [row][4 k]
template <int ROWS>
struct TileRC {
  static constexpr int TOTAL = (BK / 4) * (ROWS / 8);
  static constexpr int NBLK = (TOTAL + 255) / 256;
  static constexpr int RB = ROWS / 8;  // blocks along the row dimension
  u32x4_t r[NBLK][4];
  __device__ __forceinline__ void load(const bf16_t *__restrict__ base, int64_t ld, int row0, int rows, int k0, int kend,
                                       int tid) {
#pragma unroll
    for (int i = 0; i < NBLK; ++i) {
      const int id = tid + i * 256;
      const int rb = id % RB, kb = id / RB;
      const bool rok = (TOTAL % 256 == 0 || id < TOTAL) && row0 + rb * 8 < rows;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int k = k0 + kb * 4 + q;
        u32x4_t v = {0u, 0u, 0u, 0u};
        if (rok && k < kend) v = *(const u32x4_t *)(base + (int64_t)k * ld + row0 + rb * 8);
        r[i][q] = v;
      }
    }
  }
  __device__ __forceinline__ void store(bf16_t *lds, int tid) const {
#pragma unroll
    for (int i = 0; i < NBLK; ++i) {
      const int id = tid + i * 256;
      if (TOTAL % 256 != 0 && id >= TOTAL) continue;
      const int rb = id % RB, kb = id / RB;
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        // dword a of each source row holds rows (2a, 2a+1) of the block for one k
        u32x2_t lo, hi;
        lo.x = __builtin_amdgcn_perm(r[i][1][a], r[i][0][a], 0x05040100u);
        lo.y = __builtin_amdgcn_perm(r[i][3][a], r[i][2][a], 0x05040100u);
        hi.x = __builtin_amdgcn_perm(r[i][1][a], r[i][0][a], 0x07060302u);
        hi.y = __builtin_amdgcn_perm(r[i][3][a], r[i][2][a], 0x07060302u);
        *(u32x2_t *)(lds + (rb * 8 + 2 * a) * LDSP + kb * 4) = lo;
        *(u32x2_t *)(lds + (rb * 8 + 2 * a + 1) * LDSP + kb * 4) = hi;
      }
    }
  }
};

template <int ROWS, int T> struct TileSel { typedef TileKC<ROWS> type; };
template <int ROWS> struct TileSel<ROWS, 1> { typedef TileRC<ROWS> type; };

template <int BM, int BN, int WM, int WN, int TA, int TB>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const GemmArgs g) {
  constexpr int MI = BM / WM / 32, NJ = BN / WN / 32;
  __shared__ __attribute__((aligned(16))) bf16_t As[2][BM * LDSP];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[2][BN * LDSP];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int tile = blockIdx.x;
  const int tm = tile / g.tiles_n, tn = tile % g.tiles_n;
  const int m0 = tm * BM, n0 = tn * BN;
  if (g.causal == CAUSAL_SKIP_UPPER && n0 > m0 + BM - 1) return;
  const int z = blockIdx.y, z1 = z / g.nb2, z2 = z % g.nb2;
  const bf16_t *A = (const bf16_t *)g.A + z1 * g.sA1 + z2 * g.sA2;
  const bf16_t *B = (const bf16_t *)g.B + z1 * g.sB1 + z2 * g.sB2;
  const int64_t coff = z1 * g.sC1 + z2 * g.sC2;

  int kbeg = 0, kend = g.K;
  if (g.causal == CAUSAL_K_END) kend = min(g.K, m0 + BM);
  if (g.causal == CAUSAL_K_BEGIN) kbeg = (m0 / BK) * BK;

  typename TileSel<BM, TA>::type ta;
  typename TileSel<BN, TB>::type tb;

  f32x16_t acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = (kend - kbeg + BK - 1) / BK;
  if (nk > 0) {
    ta.load(A, g.lda, m0, g.M, kbeg, kend, tid);
    tb.load(B, g.ldb, n0, g.N, kbeg, kend, tid);
    ta.store(As[0], tid);
    tb.store(Bs[0], tid);
  }
  __syncthreads();
  const int arow = (wm * (BM / WM) + (lane & 31)) * LDSP + (lane >> 5) * 8;
  const int brow = (wn * (BN / WN) + (lane & 31)) * LDSP + (lane >> 5) * 8;
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) {
      ta.load(A, g.lda, m0, g.M, kbeg + (kt + 1) * BK, kend, tid);
      tb.load(B, g.ldb, n0, g.N, kbeg + (kt + 1) * BK, kend, tid);
    }
    const bf16_t *as = As[cur], *bs = Bs[cur];
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      bf16x8_t af[MI], bfr[NJ];
#pragma unroll
      for (int i = 0; i < MI; ++i) af[i] = *(const bf16x8_t *)(as + arow + i * 32 * LDSP + kk);
#pragma unroll
      for (int j = 0; j < NJ; ++j) bfr[j] = *(const bf16x8_t *)(bs + brow + j * 32 * LDSP + kk);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) {
      ta.store(As[cur ^ 1], tid);
      tb.store(Bs[cur ^ 1], tid);
    }
    __syncthreads();
  }

  // accumulator element r of a 32x32 result: row (r/4)*8 + (lane/32)*4 + r%4, column lane%32
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int col = n0 + wn * (BN / WN) + j * 32 + (lane & 31);
      if (col >= g.N) continue;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * (BM / WM) + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        if (row < g.M) epilogue_store<bf16_t>(g, coff, row, col, acc[i][j][r]);
      }
    }
}

// ---------------------------------------------------------------------------
// fp32 kernel (no reduced-precision matrix path exists for fp32 on gfx950
// other than real fp32): 64x64 tile, 16-wide K slices, 4x4 outputs per thread,
// contraction accumulated in ascending k.
// ---------------------------------------------------------------------------
constexpr int FBM = 64, FBN = 64, FBK = 16;

__global__ __launch_bounds__(256) void gemm_f32_kernel(const GemmArgs g, int ta, int tb) {
  __shared__ float As[FBK][FBM + 4];
  __shared__ float Bs[FBK][FBN + 4];
  const int tid = threadIdx.x;
  const int tile = blockIdx.x;
  const int tm = tile / g.tiles_n, tn = tile % g.tiles_n;
  const int m0 = tm * FBM, n0 = tn * FBN;
  if (g.causal == CAUSAL_SKIP_UPPER && n0 > m0 + FBM - 1) return;
  const int z = blockIdx.y, z1 = z / g.nb2, z2 = z % g.nb2;
  const float *A = (const float *)g.A + z1 * g.sA1 + z2 * g.sA2;
  const float *B = (const float *)g.B + z1 * g.sB1 + z2 * g.sB2;
  const int64_t coff = z1 * g.sC1 + z2 * g.sC2;
  int kbeg = 0, kend = g.K;
  if (g.causal == CAUSAL_K_END) kend = min(g.K, m0 + FBM);
  if (g.causal == CAUSAL_K_BEGIN) kbeg = (m0 / FBK) * FBK;

  const int ty = tid / 16, tx = tid % 16;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int k0 = kbeg; k0 < kend; k0 += FBK) {
    // 64x16 elements per operand, 4 per thread; index so that the contiguous
    // dimension of the source runs along consecutive threads
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int id = tid + i * 256;
      int r, k;
      if (ta) { r = id % FBM; k = id / FBM; } else { k = id % FBK; r = id / FBK; }
      float v = 0.f;
      if (m0 + r < g.M && k0 + k < kend)
        v = ta ? A[(int64_t)(k0 + k) * g.lda + m0 + r] : A[(int64_t)(m0 + r) * g.lda + k0 + k];
      As[k][r] = v;
      if (tb) { r = id % FBN; k = id / FBN; } else { k = id % FBK; r = id / FBK; }
      v = 0.f;
      if (n0 + r < g.N && k0 + k < kend)
        v = tb ? B[(int64_t)(k0 + k) * g.ldb + n0 + r] : B[(int64_t)(n0 + r) * g.ldb + k0 + k];
      Bs[k][r] = v;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < FBK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int row = m0 + ty * 4 + i, col = n0 + tx * 4 + j;
      if (row < g.M && col < g.N) epilogue_store<float>(g, coff, row, col, acc[i][j]);
    }
}

template <int BM, int BN, int WM, int WN>
static hipError_t launch_bf16_cfg(const GemmArgs &a, int ta, int tb, dim3 grid, hipStream_t s) {
  if (ta == 0 && tb == 0) hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, 0, 0>), grid, dim3(256), 0, s, a);
  else if (ta == 0 && tb == 1) hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, 0, 1>), grid, dim3(256), 0, s, a);
  else if (ta == 1 && tb == 1) hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, 1, 1>), grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, 1, 0>), grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

// algorithmic flops of a launch: causal products only count the triangle
static double gemm_flops(const GemmDesc &d) {
  const double nb = (double)d.nb1 * d.nb2;
  if (d.causal == CAUSAL_SKIP_UPPER) return nb * 2.0 * d.K * (0.5 * d.M * (d.M + 1.0));
  if (d.causal == CAUSAL_K_END || d.causal == CAUSAL_K_BEGIN) return nb * 2.0 * d.N * (0.5 * d.M * (d.M + 1.0));
  return nb * 2.0 * d.M * d.N * d.K;
}

static const char *gemm_name(int dtype, int bn, int ta, int tb) {
  static const char *n128[4] = {"gemm_bf16_128x128_nt", "gemm_bf16_128x128_nn", "gemm_bf16_128x128_tt",
                                "gemm_bf16_128x128_tn"};
  static const char *n64[4] = {"gemm_bf16_128x64_nt", "gemm_bf16_128x64_nn", "gemm_bf16_128x64_tt",
                               "gemm_bf16_128x64_tn"};
  if (dtype == DT_F32) return "gemm_f32_64x64";
  return (bn == 128 ? n128 : n64)[ta * 2 + tb];
}

hipError_t launch_gemm(const GemmDesc &d, hipStream_t s) {
  if (d.M <= 0 || d.N <= 0 || d.nb1 * d.nb2 <= 0) return hipSuccess;
  GemmArgs a;
  a.A = d.A; a.B = d.B; a.M = d.M; a.N = d.N; a.K = d.K;
  a.lda = d.lda; a.ldb = d.ldb; a.ldc = d.ldc;
  a.nb2 = d.nb2;
  a.sA1 = d.sA1; a.sA2 = d.sA2; a.sB1 = d.sB1; a.sB2 = d.sB2; a.sC1 = d.sC1; a.sC2 = d.sC2;
  a.alpha = d.alpha; a.bias = d.bias; a.resid = d.resid;
  a.out_f32 = d.out_f32; a.out_act = d.out_act; a.out_act2 = d.out_act2; a.aux = d.aux;
  a.epi = d.epi; a.causal = d.causal;
  const int nbatch = d.nb1 * d.nb2;
  if (d.dtype == DT_F32) {
    a.tiles_m = (d.M + FBM - 1) / FBM;
    a.tiles_n = (d.N + FBN - 1) / FBN;
    dim3 grid(a.tiles_m * a.tiles_n, nbatch);
    ProfScope ps(gemm_name(DT_F32, 0, 0, 0), s, gemm_flops(d), 0);
    hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, s, a, d.ta, d.tb);
    return hipGetLastError();
  }
  // operand alignment the vector loads rely on
  if ((d.lda & 7) || (d.ldb & 7) || (((uintptr_t)d.A) & 15) || (((uintptr_t)d.B) & 15)) return hipErrorInvalidValue;
  if ((d.sA1 & 7) || (d.sA2 & 7) || (d.sB1 & 7) || (d.sB2 & 7)) return hipErrorInvalidValue;
  // tile choice: 128x128 when the grid still covers the chip, else narrower tiles
  const long t128 = (long)((d.M + 127) / 128) * ((d.N + 127) / 128) * nbatch;
  if (d.N > 64 && t128 >= 256) {
    a.tiles_m = (d.M + 127) / 128; a.tiles_n = (d.N + 127) / 128;
    ProfScope ps(gemm_name(DT_BF16, 128, d.ta, d.tb), s, gemm_flops(d), 0);
    return launch_bf16_cfg<128, 128, 2, 2>(a, d.ta, d.tb, dim3(a.tiles_m * a.tiles_n, nbatch), s);
  }
  a.tiles_m = (d.M + 127) / 128; a.tiles_n = (d.N + 63) / 64;
  ProfScope ps(gemm_name(DT_BF16, 64, d.ta, d.tb), s, gemm_flops(d), 0);
  return launch_bf16_cfg<128, 64, 2, 2>(a, d.ta, d.tb, dim3(a.tiles_m * a.tiles_n, nbatch), s);
}

}  // namespace hydra
