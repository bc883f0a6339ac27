// Memory-bound kernels of the decoder shard: embedding, LayerNorm, causal
// softmax, cross-entropy, Adam, casts and column reductions.  One wavefront
// (64 lanes) owns one row wherever a row reduction is needed; reductions over
// rows (bias / gain gradients) are done in two passes with a fixed summation
// order so that results do not depend on scheduling.
#include <cmath>
#include <cstdlib>

#include "kernels.h"

namespace hydra {

__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
__device__ __forceinline__ bf16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
template <typename T> __device__ __forceinline__ float ldv(const T *p, int64_t i);
template <> __device__ __forceinline__ float ldv<float>(const float *p, int64_t i) { return p[i]; }
template <> __device__ __forceinline__ float ldv<bf16_t>(const bf16_t *p, int64_t i) { return bf2f(p[i]); }
template <typename T> __device__ __forceinline__ void stv(T *p, int64_t i, float v);
template <> __device__ __forceinline__ void stv<float>(float *p, int64_t i, float v) { p[i] = v; }
template <> __device__ __forceinline__ void stv<bf16_t>(bf16_t *p, int64_t i, float v) { p[i] = f2bf(v); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ------------------------------------------------------------------ embedding
__global__ void embed_fwd_kernel(const int32_t *__restrict__ tok, const float *__restrict__ wte,
                                 const float *__restrict__ wpe, float *__restrict__ x0, int M, int T, int d) {
  const int m = blockIdx.x;
  const int64_t id = tok[m];
  const int t = m % T;
  for (int c = threadIdx.x * 4; c < d; c += blockDim.x * 4) {
    const float4 a = *(const float4 *)(wte + id * d + c);
    const float4 b = *(const float4 *)(wpe + (int64_t)t * d + c);
    float4 o;
    o.x = a.x + b.x; o.y = a.y + b.y; o.z = a.z + b.z; o.w = a.w + b.w;
    *(float4 *)(x0 + (int64_t)m * d + c) = o;
  }
}

// One block per position m.  The block that holds the first occurrence of a
// token id marks all later occurrences in a bitmap, then sums their rows in
// ascending m and writes the token's gradient row once (adding to what the row
// holds when acc is set); other blocks leave.  Without acc dwte was zeroed before.
constexpr int EMB_MAXW = 1024;  // bitmap words: up to 32768 positions
__global__ __launch_bounds__(256) void embed_bwd_wte_kernel(const int32_t *__restrict__ tok,
                                                            const float *__restrict__ dx0, float *__restrict__ dwte,
                                                            int M, int d, int acc_prev) {
  const int m = blockIdx.x;
  const int id = tok[m];
  __shared__ int earlier;
  __shared__ uint32_t bits[EMB_MAXW];
  if (threadIdx.x == 0) earlier = 0;
  const int nw = (M + 31) / 32;
  for (int w = threadIdx.x; w < nw; w += blockDim.x) bits[w] = 0u;
  __syncthreads();
  int found = 0;
  for (int j = threadIdx.x; j < m; j += blockDim.x) found |= (tok[j] == id);
  if (found) earlier = 1;
  __syncthreads();
  if (earlier) return;
  for (int j = m + 1 + threadIdx.x; j < M; j += blockDim.x)
    if (tok[j] == id) atomicOr(&bits[j >> 5], 1u << (j & 31));
  __syncthreads();
  for (int c = threadIdx.x; c < d; c += blockDim.x) {
    float acc = dx0[(int64_t)m * d + c];
    for (int w = m >> 5; w < nw; ++w) {
      uint32_t b = bits[w];
      while (b) {
        const int j = (w << 5) + __ffs(b) - 1;
        b &= b - 1;
        acc += dx0[(int64_t)j * d + c];
      }
    }
    if (acc_prev) acc = dwte[(int64_t)id * d + c] + acc;
    dwte[(int64_t)id * d + c] = acc;
  }
}

__global__ void embed_bwd_wpe_kernel(const float *__restrict__ dx0, float *__restrict__ dwpe, int B, int T, int d,
                                     int acc_prev) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // over T*d
  if (i >= (int64_t)T * d) return;
  float acc = 0.f;
  for (int b = 0; b < B; ++b) acc += dx0[(int64_t)b * T * d + i];
  dwpe[i] = acc_prev ? dwpe[i] + acc : acc;
}

__global__ void fill_u32_kernel(uint32_t *p, uint32_t v, int64_t n) {
  int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x * 4;
  for (; i < n; i += stride) {
    if (i + 4 <= n && ((((uintptr_t)p) & 15) == 0)) {
      *(uint4 *)(p + i) = make_uint4(v, v, v, v);
    } else {
      for (int64_t j = i; j < n && j < i + 4; ++j) p[j] = v;
    }
  }
}

hipError_t launch_fill_u32(uint32_t *p, uint32_t value, int64_t n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  ProfScope ps("fill_u32", s, 0, 4.0 * n);
  // one workgroup per 1024 elements, however many that makes: on arrays far larger than the caches a capped grid that
  // strides through them streamed a fifth slower (measured on the Adam update: 4.6 against 5.5 TB/s at 4e8 elements)
  int64_t blocks = (n / 4 + 255) / 256;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p, value, n);
  return hipGetLastError();
}

hipError_t launch_embed_fwd(const int32_t *tok, const float *wte, const float *wpe, float *x0, int M, int T, int d,
                            hipStream_t s) {
  ProfScope ps("embed_fwd", s, 0, 12.0 * M * d);
  hipLaunchKernelGGL(embed_fwd_kernel, dim3(M), dim3(128), 0, s, tok, wte, wpe, x0, M, T, d);
  return hipGetLastError();
}

hipError_t launch_embed_bwd(const int32_t *tok, const float *dx0, float *dwte, float *dwpe, int B, int T, int d, int V,
                            int acc_wte, int acc_wpe, hipStream_t s) {
  if (B * T > EMB_MAXW * 32) return hipErrorInvalidValue;
  if (!acc_wte) {
    hipError_t e = launch_fill_u32((uint32_t *)dwte, 0u, (int64_t)V * d, s);
    if (e != hipSuccess) return e;
  }
  ProfScope ps("embed_bwd", s, 0, 8.0 * B * T * d + 4.0 * T * d);
  hipLaunchKernelGGL(embed_bwd_wte_kernel, dim3(B * T), dim3(256), 0, s, tok, dx0, dwte, B * T, d, acc_wte);
  const int64_t n = (int64_t)T * d;
  hipLaunchKernelGGL(embed_bwd_wpe_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, dx0, dwpe, B, T, d, acc_wpe);
  return hipGetLastError();
}

// ------------------------------------------------------------------ LayerNorm
// One wavefront per row, four rows per block.  Mean, then centred variance
// (two passes, as in the definition), then the affine output.  Rows of up to
// 64 * 4 * LN_R = 2048 elements are read once and kept in registers; wider rows
// are re-read (they hit the cache).
constexpr int LN_R = 8;  // float4 per lane kept in registers

__device__ __forceinline__ void st4(float *p, float a, float b, float c, float e) {
  *(float4 *)p = make_float4(a, b, c, e);
}
__device__ __forceinline__ void st4(bf16_t *p, float a, float b, float c, float e) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf2_t;
  typedef __attribute__((ext_vector_type(2))) float f2_t;
  union { bf2_t h[2]; uint2 u; } x;
  const f2_t lo = {a, b}, hi = {c, e};
  x.h[0] = __builtin_convertvector(lo, bf2_t);  // round to nearest even, one instruction on gfx950
  x.h[1] = __builtin_convertvector(hi, bf2_t);
  *(uint2 *)p = x.u;
}

template <typename OutT, bool CACHED>
__global__ __launch_bounds__(256) void layernorm_fwd_kernel(const float *__restrict__ x, const float *__restrict__ gamma,
                                                            const float *__restrict__ beta, OutT *__restrict__ y,
                                                            float *__restrict__ mean, float *__restrict__ rstd, int M,
                                                            int d) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= M) return;
  const float *xr = x + (int64_t)row * d;
  float4 v[LN_R];
  float s = 0.f;
  if (CACHED) {
#pragma unroll
    for (int i = 0; i < LN_R; ++i) {
      const int c = lane * 4 + i * 256;
      v[i] = c < d ? *(const float4 *)(xr + c) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int i = 0; i < LN_R; ++i) s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
  } else {
    for (int c = lane * 4; c < d; c += 256) {
      const float4 w = *(const float4 *)(xr + c);
      s += (w.x + w.y) + (w.z + w.w);
    }
  }
  const float mu = wave_sum(s) / (float)d;
  float q = 0.f;
  if (CACHED) {
#pragma unroll
    for (int i = 0; i < LN_R; ++i)
      if (lane * 4 + i * 256 < d) {
        const float a = v[i].x - mu, b = v[i].y - mu, e = v[i].z - mu, f = v[i].w - mu;
        q += (a * a + b * b) + (e * e + f * f);
      }
  } else {
    for (int c = lane * 4; c < d; c += 256) {
      const float4 w = *(const float4 *)(xr + c);
      const float a = w.x - mu, b = w.y - mu, e = w.z - mu, f = w.w - mu;
      q += (a * a + b * b) + (e * e + f * f);
    }
  }
  const float rs = 1.0f / sqrtf(wave_sum(q) / (float)d + 1e-5f);
  if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
  OutT *yr = y + (int64_t)row * d;
  auto emit = [&](int c, const float4 w) {
    const float4 gm = *(const float4 *)(gamma + c);
    const float4 bt = *(const float4 *)(beta + c);
    st4(yr + c, (w.x - mu) * rs * gm.x + bt.x, (w.y - mu) * rs * gm.y + bt.y, (w.z - mu) * rs * gm.z + bt.z,
        (w.w - mu) * rs * gm.w + bt.w);
  };
  if (CACHED) {
#pragma unroll
    for (int i = 0; i < LN_R; ++i)
      if (lane * 4 + i * 256 < d) emit(lane * 4 + i * 256, v[i]);
  } else {
    for (int c = lane * 4; c < d; c += 256) emit(c, *(const float4 *)(xr + c));
  }
}

hipError_t launch_layernorm_fwd(int dtype, const float *x, const float *gamma, const float *beta, void *y, float *mean,
                                float *rstd, int M, int d, hipStream_t s) {
  dim3 grid((M + 3) / 4), block(256);
  ProfScope ps("layernorm_fwd", s, 0, (double)M * d * (4.0 + dt_size(dtype)) + 8.0 * M);
  const bool cached = d <= 256 * LN_R;
  if (dtype == DT_BF16) {
    if (cached)
      hipLaunchKernelGGL((layernorm_fwd_kernel<bf16_t, true>), grid, block, 0, s, x, gamma, beta, (bf16_t *)y, mean, rstd,
                         M, d);
    else
      hipLaunchKernelGGL((layernorm_fwd_kernel<bf16_t, false>), grid, block, 0, s, x, gamma, beta, (bf16_t *)y, mean,
                         rstd, M, d);
  } else {
    if (cached)
      hipLaunchKernelGGL((layernorm_fwd_kernel<float, true>), grid, block, 0, s, x, gamma, beta, (float *)y, mean, rstd, M,
                         d);
    else
      hipLaunchKernelGGL((layernorm_fwd_kernel<float, false>), grid, block, 0, s, x, gamma, beta, (float *)y, mean, rstd,
                         M, d);
  }
  return hipGetLastError();
}

// dx = rstd * (dxhat - mean(dxhat) - xhat * mean(dxhat * xhat)) [+ dres], dxhat = dy * gamma
// One wavefront per row; rows of up to 2048 elements stay in registers between the two phases.
template <bool CACHED>
__global__ __launch_bounds__(256) void layernorm_bwd_dx_kernel(const float *__restrict__ dy, const float *__restrict__ x,
                                                               const float *__restrict__ mean,
                                                               const float *__restrict__ rstd,
                                                               const float *__restrict__ gamma,
                                                               const float *__restrict__ dres, float *__restrict__ dx,
                                                               bf16_t *__restrict__ dx_bf16, int M, int d) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= M) return;
  const float *xr = x + (int64_t)row * d, *dyr = dy + (int64_t)row * d;
  const float mu = mean[row], rs = rstd[row];
  float4 xh[LN_R], h[LN_R];  // normalised input and dy * gamma
  float s1 = 0.f, s2 = 0.f;
  auto phase1 = [&](int c, float4 &xo, float4 &ho) {
    const float4 v = *(const float4 *)(xr + c);
    const float4 g = *(const float4 *)(dyr + c);
    const float4 gm = *(const float4 *)(gamma + c);
    xo = make_float4((v.x - mu) * rs, (v.y - mu) * rs, (v.z - mu) * rs, (v.w - mu) * rs);
    ho = make_float4(g.x * gm.x, g.y * gm.y, g.z * gm.z, g.w * gm.w);
    s1 += (ho.x + ho.y) + (ho.z + ho.w);
    s2 += (ho.x * xo.x + ho.y * xo.y) + (ho.z * xo.z + ho.w * xo.w);
  };
  if (CACHED) {
#pragma unroll
    for (int i = 0; i < LN_R; ++i)
      if (lane * 4 + i * 256 < d) phase1(lane * 4 + i * 256, xh[i], h[i]);
  } else {
    for (int c = lane * 4; c < d; c += 256) {
      float4 a, b;
      phase1(c, a, b);
    }
  }
  const float m1 = wave_sum(s1) / (float)d, m2 = wave_sum(s2) / (float)d;
  auto phase2 = [&](int c, const float4 &xo, const float4 &ho) {
    float4 o;
    o.x = rs * (ho.x - m1 - xo.x * m2);
    o.y = rs * (ho.y - m1 - xo.y * m2);
    o.z = rs * (ho.z - m1 - xo.z * m2);
    o.w = rs * (ho.w - m1 - xo.w * m2);
    if (dres) {
      const float4 r = *(const float4 *)(dres + (int64_t)row * d + c);
      o.x += r.x; o.y += r.y; o.z += r.z; o.w += r.w;
    }
    *(float4 *)(dx + (int64_t)row * d + c) = o;
    if (dx_bf16) {  // operand-dtype copy for the products that consume this gradient
      uint2 p;
      p.x = (uint32_t)f2bf(o.x) | ((uint32_t)f2bf(o.y) << 16);
      p.y = (uint32_t)f2bf(o.z) | ((uint32_t)f2bf(o.w) << 16);
      *(uint2 *)(dx_bf16 + (int64_t)row * d + c) = p;
    }
  };
  if (CACHED) {
#pragma unroll
    for (int i = 0; i < LN_R; ++i)
      if (lane * 4 + i * 256 < d) phase2(lane * 4 + i * 256, xh[i], h[i]);
  } else {
    for (int c = lane * 4; c < d; c += 256) {
      const float4 v = *(const float4 *)(xr + c);
      const float4 g = *(const float4 *)(dyr + c);
      const float4 gm = *(const float4 *)(gamma + c);
      phase2(c, make_float4((v.x - mu) * rs, (v.y - mu) * rs, (v.z - mu) * rs, (v.w - mu) * rs),
             make_float4(g.x * gm.x, g.y * gm.y, g.z * gm.z, g.w * gm.w));
    }
  }
}

hipError_t launch_layernorm_bwd_dx(const float *dy, const float *x, const float *mean, const float *rstd,
                                   const float *gamma, const float *dres, float *dx, void *dx_bf16v, int M, int d,
                                   hipStream_t s) {
  bf16_t *dx_bf16 = (bf16_t *)dx_bf16v;
  ProfScope ps("layernorm_bwd_dx", s, 0, (double)M * d * ((dres ? 16.0 : 12.0) + (dx_bf16 ? 2.0 : 0.0)));
  if (d <= 256 * LN_R)
    hipLaunchKernelGGL(layernorm_bwd_dx_kernel<true>, dim3((M + 3) / 4), dim3(256), 0, s, dy, x, mean, rstd, gamma, dres,
                       dx, dx_bf16, M, d);
  else
    hipLaunchKernelGGL(layernorm_bwd_dx_kernel<false>, dim3((M + 3) / 4), dim3(256), 0, s, dy, x, mean, rstd, gamma,
                       dres, dx, dx_bf16, M, d);
  return hipGetLastError();
}

// ------------------------------------------------------- column reductions
// pass 1: block (64 columns x 4 row lanes) sums a chunk of CH rows; pass 2 adds
// the chunk partials in ascending chunk order.
constexpr int CH = 128;
int colsum_chunks(int M) { return (M + CH - 1) / CH; }

template <typename T, int MODE>  // MODE 0: plain column sum; 1: LayerNorm dgamma/dbeta
__global__ __launch_bounds__(256) void colsum_pass1_kernel(const T *__restrict__ in, int64_t ld,
                                                           const float *__restrict__ x, const float *__restrict__ mean,
                                                           const float *__restrict__ rstd, float *__restrict__ part,
                                                           int M, int N) {
  __shared__ double sh[2][4][64];
  const int cx = threadIdx.x & 63, ry = threadIdx.x >> 6;
  const int col = blockIdx.x * 64 + cx;
  const int r0 = blockIdx.y * CH, r1 = min(M, r0 + CH);
  double a = 0.0, b = 0.0;  // fp64 adds are free in a memory-bound reduction
  if (col < N) {
    // eight rows' loads are issued before the first is used: the loop is latency-bound otherwise
    constexpr int U = 8;
    for (int rb = r0 + ry; rb < r1; rb += 4 * U) {
      float v[U], xh[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int r = rb + 4 * u;
        v[u] = 0.f;
        xh[u] = 0.f;
        if (r < r1) {
          v[u] = ldv<T>(in, (int64_t)r * ld + col);
          if (MODE == 1) xh[u] = (x[(int64_t)r * ld + col] - mean[r]) * rstd[r];
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {  // ascending rows, as before
        if (MODE == 1) {
          a += (double)(v[u] * xh[u]);
          b += v[u];
        } else {
          a += v[u];
        }
      }
    }
  }
  sh[0][ry][cx] = a;
  sh[1][ry][cx] = b;
  __syncthreads();
  if (ry == 0 && col < N) {
    const int nch = gridDim.y;
    part[(int64_t)blockIdx.y * N + col] = (float)((sh[0][0][cx] + sh[0][1][cx]) + (sh[0][2][cx] + sh[0][3][cx]));
    if (MODE == 1)
      part[(int64_t)(nch + blockIdx.y) * N + col] =
          (float)((sh[1][0][cx] + sh[1][1][cx]) + (sh[1][2][cx] + sh[1][3][cx]));
  }
}

__global__ void colsum_pass2_kernel(const float *__restrict__ part, float *__restrict__ out0, float *__restrict__ out1,
                                    int nch, int N, int acc) {
  const int col = blockIdx.x * blockDim.x + threadIdx.x;
  if (col >= N) return;
  double a = acc ? (double)out0[col] : 0.0;
  for (int c = 0; c < nch; ++c) a += (double)part[(int64_t)c * N + col];
  out0[col] = (float)a;
  if (out1) {
    double b = acc ? (double)out1[col] : 0.0;
    for (int c = 0; c < nch; ++c) b += (double)part[(int64_t)(nch + c) * N + col];
    out1[col] = (float)b;
  }
}

hipError_t launch_colsum(int in_dtype, const void *in, int64_t ld, float *out, float *scratch, int M, int N, int acc,
                         hipStream_t s) {
  const int nch = colsum_chunks(M);
  dim3 grid((N + 63) / 64, nch);
  ProfScope ps("colsum", s, 0, (double)M * N * dt_size(in_dtype));
  if (in_dtype == DT_BF16)
    hipLaunchKernelGGL((colsum_pass1_kernel<bf16_t, 0>), grid, dim3(256), 0, s, (const bf16_t *)in, ld, nullptr,
                       nullptr, nullptr, scratch, M, N);
  else
    hipLaunchKernelGGL((colsum_pass1_kernel<float, 0>), grid, dim3(256), 0, s, (const float *)in, ld, nullptr, nullptr,
                       nullptr, scratch, M, N);
  hipLaunchKernelGGL(colsum_pass2_kernel, dim3((N + 255) / 256), dim3(256), 0, s, scratch, out, nullptr, nch, N, acc);
  return hipGetLastError();
}

hipError_t launch_layernorm_bwd_params(const float *dy, const float *x, const float *mean, const float *rstd,
                                       float *dgamma, float *dbeta, float *scratch, int M, int d, int acc,
                                       hipStream_t s) {
  const int nch = colsum_chunks(M);
  dim3 grid((d + 63) / 64, nch);
  ProfScope ps("layernorm_bwd_params", s, 0, 8.0 * M * d);
  hipLaunchKernelGGL((colsum_pass1_kernel<float, 1>), grid, dim3(256), 0, s, dy, (int64_t)d, x, mean, rstd, scratch, M,
                     d);
  hipLaunchKernelGGL(colsum_pass2_kernel, dim3((d + 255) / 256), dim3(256), 0, s, scratch, dgamma, dbeta, nch, d, acc);
  return hipGetLastError();
}

// ------------------------------------------- fused backward of a LayerNorm
// One pass over the rows gives everything a LayerNorm's backward produces: dx
// (fp32, optionally a bf16 copy) and, per block of LNB_ROWS rows, the partial
// column sums of dy * xhat (-> dgamma), of dy (-> dbeta) and of dx (-> the bias
// gradient of the linear layer whose output gradient dx is).  A wavefront walks
// LNB_ROWS / 4 rows with its column partials in registers; the four
// wavefronts of a block are added in a fixed order through LDS.  The partials
// [gridDim.x][3][d] are summed by colsum_finish_kernel.  NR = float4 per lane
// that cover a row (d <= 256 * NR).
constexpr int LNB_ROWS = 8;
int layernorm_bwd_fused_blocks(int M) { return (M + LNB_ROWS - 1) / LNB_ROWS; }
bool layernorm_bwd_fused_supported(int d) { return d % 4 == 0 && d <= 256 * LN_R; }

template <int NR>
__global__ __launch_bounds__(256) void layernorm_bwd_fused_kernel(const float *__restrict__ dy, const float *__restrict__ x,
                                                                  const float *__restrict__ mean,
                                                                  const float *__restrict__ rstd,
                                                                  const float *__restrict__ gamma,
                                                                  const float *__restrict__ dres, float *__restrict__ dx,
                                                                  bf16_t *__restrict__ dx_bf16, float *__restrict__ part,
                                                                  int M, int d) {
  __shared__ float red[3][NR * 256];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float4 gm[NR], ag[NR], ab[NR], ax[NR];
#pragma unroll
  for (int i = 0; i < NR; ++i) {
    const int c = lane * 4 + i * 256;
    gm[i] = c < d ? *(const float4 *)(gamma + c) : make_float4(0.f, 0.f, 0.f, 0.f);
    ag[i] = ab[i] = ax[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  constexpr int RPW = LNB_ROWS / 4;
#pragma unroll 1
  for (int rr = 0; rr < RPW; ++rr) {
    const int row = blockIdx.x * LNB_ROWS + rr * 4 + wave;  // ascending rows within a wavefront
    if (row >= M) break;
    const float *xr = x + (int64_t)row * d, *dyr = dy + (int64_t)row * d;
    const float mu = mean[row], rs = rstd[row];
    float4 xh[NR], g[NR], h[NR];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < NR; ++i) {
      const int c = lane * 4 + i * 256;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      g[i] = v;
      if (c < d) {
        v = *(const float4 *)(xr + c);
        g[i] = *(const float4 *)(dyr + c);
      }
      xh[i] = c < d ? make_float4((v.x - mu) * rs, (v.y - mu) * rs, (v.z - mu) * rs, (v.w - mu) * rs) : v;
      h[i] = make_float4(g[i].x * gm[i].x, g[i].y * gm[i].y, g[i].z * gm[i].z, g[i].w * gm[i].w);
      s1 += (h[i].x + h[i].y) + (h[i].z + h[i].w);
      s2 += (h[i].x * xh[i].x + h[i].y * xh[i].y) + (h[i].z * xh[i].z + h[i].w * xh[i].w);
    }
    const float m1 = wave_sum(s1) / (float)d, m2 = wave_sum(s2) / (float)d;
#pragma unroll
    for (int i = 0; i < NR; ++i) {
      const int c = lane * 4 + i * 256;
      if (c < d) {
        float4 o;
        o.x = rs * (h[i].x - m1 - xh[i].x * m2);
        o.y = rs * (h[i].y - m1 - xh[i].y * m2);
        o.z = rs * (h[i].z - m1 - xh[i].z * m2);
        o.w = rs * (h[i].w - m1 - xh[i].w * m2);
        if (dres) {
          const float4 r = *(const float4 *)(dres + (int64_t)row * d + c);
          o.x += r.x; o.y += r.y; o.z += r.z; o.w += r.w;
        }
        *(float4 *)(dx + (int64_t)row * d + c) = o;
        if (dx_bf16) {
          uint2 p;
          p.x = (uint32_t)f2bf(o.x) | ((uint32_t)f2bf(o.y) << 16);
          p.y = (uint32_t)f2bf(o.z) | ((uint32_t)f2bf(o.w) << 16);
          *(uint2 *)(dx_bf16 + (int64_t)row * d + c) = p;
        }
        ag[i].x += g[i].x * xh[i].x; ag[i].y += g[i].y * xh[i].y; ag[i].z += g[i].z * xh[i].z; ag[i].w += g[i].w * xh[i].w;
        ab[i].x += g[i].x; ab[i].y += g[i].y; ab[i].z += g[i].z; ab[i].w += g[i].w;
        ax[i].x += o.x; ax[i].y += o.y; ax[i].z += o.z; ax[i].w += o.w;
      }
    }
  }
  // wavefronts 1..3 add to what wavefront 0 holds, one after the other (fixed order)
  float *out = part + (int64_t)blockIdx.x * 3 * d;
  for (int w = 1; w < 4; ++w) {
    if (wave == w) {
#pragma unroll
      for (int i = 0; i < NR; ++i) {
        *(float4 *)&red[0][lane * 4 + i * 256] = ag[i];
        *(float4 *)&red[1][lane * 4 + i * 256] = ab[i];
        *(float4 *)&red[2][lane * 4 + i * 256] = ax[i];
      }
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int i = 0; i < NR; ++i) {
        const float4 a = *(const float4 *)&red[0][lane * 4 + i * 256], b = *(const float4 *)&red[1][lane * 4 + i * 256],
                     c4 = *(const float4 *)&red[2][lane * 4 + i * 256];
        ag[i].x += a.x; ag[i].y += a.y; ag[i].z += a.z; ag[i].w += a.w;
        ab[i].x += b.x; ab[i].y += b.y; ab[i].z += b.z; ab[i].w += b.w;
        ax[i].x += c4.x; ax[i].y += c4.y; ax[i].z += c4.z; ax[i].w += c4.w;
      }
    }
    __syncthreads();
  }
  if (wave == 0) {
#pragma unroll
    for (int i = 0; i < NR; ++i) {
      const int c = lane * 4 + i * 256;
      if (c < d) {
        *(float4 *)(out + c) = ag[i];
        *(float4 *)(out + d + c) = ab[i];
        *(float4 *)(out + 2 * d + c) = ax[i];
      }
    }
  }
}

hipError_t launch_layernorm_bwd_fused(const float *dy, const float *x, const float *mean, const float *rstd,
                                      const float *gamma, const float *dres, float *dx, void *dx_bf16, float *part, int M,
                                      int d, hipStream_t s) {
  if (!layernorm_bwd_fused_supported(d)) return hipErrorInvalidValue;
  const int nr = (d + 255) / 256;
  dim3 grid(layernorm_bwd_fused_blocks(M)), block(256);
  ProfScope ps("layernorm_bwd", s, 0, (double)M * d * ((dres ? 16.0 : 12.0) + (dx_bf16 ? 2.0 : 0.0)) + 12.0 * grid.x * d);
#define HYDRA_LNB(NR_)                                                                                                  \
  hipLaunchKernelGGL(layernorm_bwd_fused_kernel<NR_>, grid, block, 0, s, dy, x, mean, rstd, gamma, dres, dx,             \
                     (bf16_t *)dx_bf16, part, M, d)
  if (nr <= 1) HYDRA_LNB(1);
  else if (nr <= 2) HYDRA_LNB(2);
  else if (nr <= 3) HYDRA_LNB(3);
  else if (nr <= 4) HYDRA_LNB(4);
  else if (nr <= 6) HYDRA_LNB(6);
  else HYDRA_LNB(8);
#undef HYDRA_LNB
  return hipGetLastError();
}

// The third part of layernorm_bwd_fused_kernel's partial sums (column sums of dx over blocks of LNB_ROWS rows) for
// a gradient that was not produced by that kernel (the one a shard receives at its upper boundary), added in the
// same order - rows w and w + 4 per wavefront w, then the wavefronts in ascending order - so that the sum does not
// depend on where the shard boundaries lie.
__global__ __launch_bounds__(256) void colsum_rows8_kernel(const float *__restrict__ in, float *__restrict__ part, int M,
                                                           int d) {
  static_assert(LNB_ROWS == 8, "summation order below is written out for 8 rows");
  const int r0 = blockIdx.x * LNB_ROWS;
  float *out = part + (int64_t)blockIdx.x * 3 * d + 2 * d;
  for (int c = threadIdx.x * 4; c < d; c += 1024) {
    float4 w[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {  // wavefront k of the fused kernel: rows r0 + k, r0 + k + 4
      float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int rr = 0; rr < 2; ++rr) {
        const int row = r0 + rr * 4 + k;
        if (row < M) {
          const float4 v = *(const float4 *)(in + (int64_t)row * d + c);
          a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
        }
      }
      w[k] = a;
    }
    float4 t = w[0];
#pragma unroll
    for (int k = 1; k < 4; ++k) { t.x += w[k].x; t.y += w[k].y; t.z += w[k].z; t.w += w[k].w; }
    *(float4 *)(out + c) = t;
  }
}

hipError_t launch_colsum_rows8(const float *in, float *part, int M, int d, hipStream_t s) {
  if (d % 4) return hipErrorInvalidValue;
  ProfScope ps("colsum", s, 0, 4.0 * M * d);
  hipLaunchKernelGGL(colsum_rows8_kernel, dim3(layernorm_bwd_fused_blocks(M)), dim3(256), 0, s, in, part, M, d);
  return hipGetLastError();
}

// Column sums of two operands of one dtype in one launch (pass 1 of launch_colsum for each): the block's x index
// runs over the 64-column groups of the first operand, then over those of the second.
template <typename T>
__global__ __launch_bounds__(256) void colsum2_pass1_kernel(const T *__restrict__ in0, int N0, float *__restrict__ part0,
                                                            const T *__restrict__ in1, int N1, float *__restrict__ part1,
                                                            int M) {
  __shared__ double sh[4][64];
  const int nb0 = (N0 + 63) / 64;
  const bool second = (int)blockIdx.x >= nb0;
  const T *in = second ? in1 : in0;
  const int N = second ? N1 : N0;
  float *part = second ? part1 : part0;
  const int cx = threadIdx.x & 63, ry = threadIdx.x >> 6;
  const int col = ((int)blockIdx.x - (second ? nb0 : 0)) * 64 + cx;
  const int r0 = blockIdx.y * CH, r1 = min(M, r0 + CH);
  double a = 0.0;
  if (col < N) {
    constexpr int U = 8;
    for (int rb = r0 + ry; rb < r1; rb += 4 * U) {
      float v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int r = rb + 4 * u;
        v[u] = r < r1 ? ldv<T>(in, (int64_t)r * N + col) : 0.f;
      }
#pragma unroll
      for (int u = 0; u < U; ++u) a += v[u];
    }
  }
  sh[ry][cx] = a;
  __syncthreads();
  if (ry == 0 && col < N) part[(int64_t)blockIdx.y * N + col] = (float)((sh[0][cx] + sh[1][cx]) + (sh[2][cx] + sh[3][cx]));
}

// The same with four columns per thread (one 8- or 16-byte load per row) and 16 row lanes: a chunk of CH rows is one
// batch of eight loads per thread.  Needs N0 and N1 multiples of 4 and 16-byte aligned operands; lane r adds rows
// r, r + 16, ... in ascending order, the sixteen lanes are combined in a fixed tree.
template <typename T> struct Vec4Ld;
template <> struct Vec4Ld<float> {
  static __device__ __forceinline__ void ld(const float *p, float (&o)[4]) {
    const float4 v = *(const float4 *)p;
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  }
};
template <> struct Vec4Ld<bf16_t> {
  static __device__ __forceinline__ void ld(const bf16_t *p, float (&o)[4]) {
    const uint2 v = *(const uint2 *)p;
    o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
    o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
  }
};
template <typename T>
__global__ __launch_bounds__(256) void colsum2_pass1_vec_kernel(const T *__restrict__ in0, int N0, float *__restrict__ part0,
                                                                const T *__restrict__ in1, int N1, float *__restrict__ part1,
                                                                int M) {
  __shared__ double sh[16][65];
  const int nb0 = (N0 + 63) / 64;
  const bool second = (int)blockIdx.x >= nb0;
  const T *in = second ? in1 : in0;
  const int N = second ? N1 : N0;
  float *part = second ? part1 : part0;
  const int cx = threadIdx.x & 15, ry = threadIdx.x >> 4;
  const int cb = ((int)blockIdx.x - (second ? nb0 : 0)) * 64;
  const int col = cb + cx * 4;
  const int r0 = blockIdx.y * CH, r1 = min(M, r0 + CH);
  double a[4] = {0.0, 0.0, 0.0, 0.0};
  if (col < N) {
    constexpr int U = 8;
    for (int rb = r0 + ry; rb < r1; rb += 16 * U) {
      float v[U][4];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int r = rb + 16 * u;
        if (r < r1) Vec4Ld<T>::ld(in + (int64_t)r * N + col, v[u]);
        else v[u][0] = v[u][1] = v[u][2] = v[u][3] = 0.f;
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int j = 0; j < 4; ++j) a[j] += v[u][j];
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) sh[ry][cx * 4 + j] = a[j];
  __syncthreads();
  const int c = threadIdx.x;
  if (c < 64 && cb + c < N) {
    double t[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) t[k] = sh[k][c];
#pragma unroll
    for (int w = 1; w < 16; w *= 2)
#pragma unroll
      for (int k = 0; k < 16; k += 2 * w) t[k] += t[k + w];
    part[(int64_t)blockIdx.y * N + cb + c] = (float)t[0];
  }
}

hipError_t launch_colsum2_pass1(int dtype, const void *in0, int N0, float *part0, const void *in1, int N1, float *part1,
                                int M, hipStream_t s) {
  dim3 grid((N0 + 63) / 64 + (N1 + 63) / 64, colsum_chunks(M));
  ProfScope ps("colsum", s, 0, (double)M * (N0 + N1) * dt_size(dtype));
  if (N0 % 4 == 0 && N1 % 4 == 0 && ((((uintptr_t)in0) | ((uintptr_t)in1)) & 15) == 0) {
    if (dtype == DT_BF16)
      hipLaunchKernelGGL(colsum2_pass1_vec_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t *)in0, N0, part0,
                         (const bf16_t *)in1, N1, part1, M);
    else
      hipLaunchKernelGGL(colsum2_pass1_vec_kernel<float>, grid, dim3(256), 0, s, (const float *)in0, N0, part0,
                         (const float *)in1, N1, part1, M);
    return hipGetLastError();
  }
  if (dtype == DT_BF16)
    hipLaunchKernelGGL(colsum2_pass1_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t *)in0, N0, part0,
                       (const bf16_t *)in1, N1, part1, M);
  else
    hipLaunchKernelGGL(colsum2_pass1_kernel<float>, grid, dim3(256), 0, s, (const float *)in0, N0, part0,
                       (const float *)in1, N1, part1, M);
  return hipGetLastError();
}

// Last pass of several column sums in one launch: segment i adds its nch partial rows (stride elements apart) into
// out[0..N) (added to what out holds when acc is set).  A block takes 32 columns of one segment with 32 row lanes of
// 8 threads, four columns each (one 16-byte load per row where the segment allows it, else four 4-byte loads): lane r
// adds rows r, r + 32, ... in ascending order in double, eight loads in flight at a time (256 partial rows, the
// usual count, are one batch); the 32 lanes are combined in a fixed tree.
constexpr int FIN_COLS = 32, FIN_LANES = 32;
__global__ __launch_bounds__(256) void colsum_finish_kernel(const ColsumFinish a) {
  __shared__ double sh[FIN_LANES][FIN_COLS + 1];
  const int cx = threadIdx.x & 7, ry = threadIdx.x >> 3;
  int i = 0;
#pragma unroll 1
  while (i + 1 < a.nseg && (int)blockIdx.x * FIN_COLS >= a.seg[i + 1].col0) ++i;  // uniform over the block
  const ColsumSeg &g = a.seg[i];
  const int cb = blockIdx.x * FIN_COLS - g.col0;  // first column of the block within its segment
  const int c = cb + cx * 4;
  const bool vec = (g.N % 4 == 0) && (g.stride % 4 == 0) && ((((uintptr_t)g.part) & 15) == 0);
  double v[4] = {0.0, 0.0, 0.0, 0.0};
  if (c < g.N) {
    constexpr int U = 8;
    for (int k0 = ry; k0 < g.nch; k0 += FIN_LANES * U) {
      float w[U][4];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int k = k0 + u * FIN_LANES;
        const float *p = g.part + (int64_t)k * g.stride + c;
        if (k >= g.nch) {
          w[u][0] = w[u][1] = w[u][2] = w[u][3] = 0.f;
        } else if (vec) {
          const float4 q = *(const float4 *)p;
          w[u][0] = q.x; w[u][1] = q.y; w[u][2] = q.z; w[u][3] = q.w;
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j) w[u][j] = c + j < g.N ? p[j] : 0.f;
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] += (double)w[u][j];
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) sh[ry][cx * 4 + j] = v[j];
  __syncthreads();
  const int cc = threadIdx.x;
  if (cc < FIN_COLS && cb + cc < g.N) {
    double t[FIN_LANES];
#pragma unroll
    for (int k = 0; k < FIN_LANES; ++k) t[k] = sh[k][cc];
#pragma unroll
    for (int w = 1; w < FIN_LANES; w *= 2)
#pragma unroll
      for (int k = 0; k < FIN_LANES; k += 2 * w) t[k] += t[k + w];
    g.out[cb + cc] = (float)(a.acc ? (double)g.out[cb + cc] + t[0] : t[0]);
  }
}

hipError_t launch_colsum_finish(ColsumFinish &a, hipStream_t s) {
  if (a.nseg <= 0) return hipSuccess;
  if (a.nseg > COLSUM_MAX_SEGS) return hipErrorInvalidValue;
  // segments start at multiples of the block's column count so that a block never straddles two of them
  int col = 0;
  double bytes = 0;
  for (int i = 0; i < a.nseg; ++i) {
    a.seg[i].col0 = col;
    col += (a.seg[i].N + FIN_COLS - 1) / FIN_COLS * FIN_COLS;
    bytes += 4.0 * a.seg[i].N * a.seg[i].nch;
  }
  ProfScope ps("colsum_finish", s, 0, bytes);
  hipLaunchKernelGGL(colsum_finish_kernel, dim3(col / FIN_COLS), dim3(256), 0, s, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------ softmax
// One wavefront per row i of one [T,T] score matrix; only j <= i is read.
// Entries i < j < min(T, roundup(i+1, 256)) are written as exact zeros so that
// tile-granular GEMMs over the lower triangle read zeros beyond the diagonal.
__device__ __forceinline__ int causal_zero_end(int i, int T) { return min(T, ((i + 256) / 256) * 256); }

template <typename OutT>
__global__ __launch_bounds__(256) void softmax_causal_fwd_kernel(const float *__restrict__ S, OutT *__restrict__ P,
                                                                 int64_t rows, int T) {
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const int i = (int)(row % T);
  const float *sr = S + row * T;
  OutT *pr = P + row * T;
  float mx = -INFINITY;
  for (int j = lane; j <= i; j += 64) mx = fmaxf(mx, sr[j]);
  mx = wave_max(mx);
  float sum = 0.f;
  for (int j = lane; j <= i; j += 64) sum += expf(sr[j] - mx);
  sum = wave_sum(sum);
  const float inv = 1.0f / sum;
  const int zend = causal_zero_end(i, T);
  for (int j = lane; j < zend; j += 64) stv<OutT>(pr, j, j <= i ? expf(sr[j] - mx) * inv : 0.f);
}

template <typename ActT>
__global__ __launch_bounds__(256) void softmax_causal_bwd_kernel(const ActT *__restrict__ P, const float *__restrict__ dP,
                                                                 ActT *__restrict__ dS, int64_t rows, int T) {
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const int i = (int)(row % T);
  const ActT *pr = P + row * T;
  const float *dpr = dP + row * T;
  float dot = 0.f;
  for (int j = lane; j <= i; j += 64) dot += ldv<ActT>(pr, j) * dpr[j];
  dot = wave_sum(dot);
  const int zend = causal_zero_end(i, T);
  for (int j = lane; j < zend; j += 64) stv<ActT>(dS + row * T, j, j <= i ? ldv<ActT>(pr, j) * (dpr[j] - dot) : 0.f);
}

hipError_t launch_softmax_causal_fwd(int dtype, const float *S, void *P, int n_mat, int T, hipStream_t s) {
  const int64_t rows = (int64_t)n_mat * T;
  ProfScope ps("softmax_causal_fwd", s, 0, (double)n_mat * (0.5 * T * (T + 1.0)) * (4.0 + dt_size(dtype)));
  dim3 grid((unsigned)((rows + 3) / 4));
  if (dtype == DT_BF16)
    hipLaunchKernelGGL(softmax_causal_fwd_kernel<bf16_t>, grid, dim3(256), 0, s, S, (bf16_t *)P, rows, T);
  else
    hipLaunchKernelGGL(softmax_causal_fwd_kernel<float>, grid, dim3(256), 0, s, S, (float *)P, rows, T);
  return hipGetLastError();
}

hipError_t launch_softmax_causal_bwd(int dtype, const void *P, const float *dP, void *dS, int n_mat, int T,
                                     hipStream_t s) {
  const int64_t rows = (int64_t)n_mat * T;
  ProfScope ps("softmax_causal_bwd", s, 0, (double)n_mat * (0.5 * T * (T + 1.0)) * (4.0 + 2.0 * dt_size(dtype)));
  dim3 grid((unsigned)((rows + 3) / 4));
  if (dtype == DT_BF16)
    hipLaunchKernelGGL(softmax_causal_bwd_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t *)P, dP, (bf16_t *)dS,
                       rows, T);
  else
    hipLaunchKernelGGL(softmax_causal_bwd_kernel<float>, grid, dim3(256), 0, s, (const float *)P, dP, (float *)dS, rows,
                       T);
  return hipGetLastError();
}

// ------------------------------------------------------------ cross-entropy
// One block per row: running (max, sum) per thread in one pass, combined over
// the block, then dlogits = (softmax - onehot) * inv_n in a second pass.  Rows
// whose target is negative contribute no loss and a zero gradient.  Columns
// V..ld-1 of dlogits are written as zeros.
template <typename OutT>
__global__ __launch_bounds__(256) void cross_entropy_kernel(const float *__restrict__ logits,
                                                            const int32_t *__restrict__ targets,
                                                            float *__restrict__ row_loss, OutT *__restrict__ dlogits,
                                                            int V, int64_t ld, float inv_n) {
  __shared__ float shm[4], shs[4];
  const int row = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float *lr = logits + (int64_t)row * ld;
  OutT *dr = dlogits + (int64_t)row * ld;
  const int tgt = targets[row];
  if (tgt < 0 || tgt >= V) {  // ignored position (an id outside the vocabulary is treated the same way)
    for (int c = tid; c < ld; c += 256) stv<OutT>(dr, c, 0.f);
    if (tid == 0) row_loss[row] = 0.f;
    return;
  }
  float mx = -INFINITY, sum = 0.f;
  for (int c = tid; c < V; c += 256) {
    const float v = lr[c];
    if (v > mx) { sum = sum * expf(mx - v) + 1.f; mx = v; } else { sum += expf(v - mx); }
  }
  const float wmx = wave_max(mx);
  sum = wave_sum(mx == -INFINITY ? 0.f : sum * expf(mx - wmx));
  if (lane == 0) { shm[wave] = wmx; shs[wave] = sum; }
  __syncthreads();
  const float bmx = fmaxf(fmaxf(shm[0], shm[1]), fmaxf(shm[2], shm[3]));
  float bsum = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w)
    if (shm[w] != -INFINITY) bsum += shs[w] * expf(shm[w] - bmx);
  const float inv = 1.0f / bsum;
  if (tid == 0) row_loss[row] = (logf(bsum) + bmx) - lr[tgt];
  for (int c = tid; c < ld; c += 256) {
    float g = 0.f;
    if (c < V) g = (expf(lr[c] - bmx) * inv - (c == tgt ? 1.f : 0.f)) * inv_n;
    stv<OutT>(dr, c, g);
  }
}

// The same with the row held in registers between the passes (one block of 1024 threads per row, NV float4 per
// thread): the logits are read once instead of twice.  Needs ld % 4 == 0, ld <= 4096 * NV and aligned pointers.
template <typename OutT, int NV>
__global__ __launch_bounds__(1024) void cross_entropy_row_kernel(const float *__restrict__ logits,
                                                                 const int32_t *__restrict__ targets,
                                                                 float *__restrict__ row_loss, OutT *__restrict__ dlogits,
                                                                 int V, int64_t ld, float inv_n) {
  __shared__ float sh[16];
  const int row = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float *lr = logits + (int64_t)row * ld;
  OutT *dr = dlogits + (int64_t)row * ld;
  const int tgt = targets[row];
  const int n4 = (int)(ld / 4);
  if (tgt < 0 || tgt >= V) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int q = i * 1024 + tid;
      if (q < n4) st4(dr + 4 * q, 0.f, 0.f, 0.f, 0.f);
    }
    if (tid == 0) row_loss[row] = 0.f;
    return;
  }
  float4 v[NV];
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int q = i * 1024 + tid, c = 4 * q;
    float4 w = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
    if (q < n4) {
      w = *(const float4 *)(lr + c);
      if (c + 3 >= V) {  // the pad columns V..ld-1 take no part
        if (c + 0 >= V) w.x = -INFINITY;
        if (c + 1 >= V) w.y = -INFINITY;
        if (c + 2 >= V) w.z = -INFINITY;
        w.w = -INFINITY;
      }
    }
    v[i] = w;
    mx = fmaxf(fmaxf(mx, fmaxf(w.x, w.y)), fmaxf(w.z, w.w));
  }
  mx = wave_max(mx);
  if (lane == 0) sh[wave] = mx;
  __syncthreads();
  float bmx = sh[0];
#pragma unroll
  for (int w = 1; w < 16; ++w) bmx = fmaxf(bmx, sh[w]);
  __syncthreads();
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {  // exp(-inf) = 0 for pad columns and unused slots
    v[i] = make_float4(expf(v[i].x - bmx), expf(v[i].y - bmx), expf(v[i].z - bmx), expf(v[i].w - bmx));
    sum += (v[i].x + v[i].y) + (v[i].z + v[i].w);
  }
  sum = wave_sum(sum);
  if (lane == 0) sh[wave] = sum;
  __syncthreads();
  float bsum = 0.f;
#pragma unroll
  for (int w = 0; w < 16; ++w) bsum += sh[w];  // fixed order
  const float inv = 1.0f / bsum;
  if (tid == 0) row_loss[row] = (logf(bsum) + bmx) - lr[tgt];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int q = i * 1024 + tid, c = 4 * q;
    if (q < n4) {
      float4 g = make_float4(v[i].x * inv, v[i].y * inv, v[i].z * inv, v[i].w * inv);
      if (tgt >= c && tgt < c + 4) {
        if (tgt == c) g.x -= 1.f;
        else if (tgt == c + 1) g.y -= 1.f;
        else if (tgt == c + 2) g.z -= 1.f;
        else g.w -= 1.f;
      }
      st4(dr + c, g.x * inv_n, g.y * inv_n, g.z * inv_n, g.w * inv_n);
    }
  }
}

template <typename OutT>
static bool launch_ce_row(const float *logits, const int32_t *targets, float *row_loss, OutT *dlogits, int M, int V,
                          int64_t ld, float inv_n, hipStream_t s) {
  if ((ld & 3) || ld > 4096 * 16 || (((uintptr_t)logits) & 15) || (((uintptr_t)dlogits) & 15)) return false;
  const int nv = (int)((ld / 4 + 1023) / 1024);
#define HYDRA_CE(NV_)                                                                                          \
  hipLaunchKernelGGL((cross_entropy_row_kernel<OutT, NV_>), dim3(M), dim3(1024), 0, s, logits, targets, row_loss, \
                     dlogits, V, ld, inv_n)
  if (nv <= 1) HYDRA_CE(1);
  else if (nv <= 2) HYDRA_CE(2);
  else if (nv <= 4) HYDRA_CE(4);
  else if (nv <= 8) HYDRA_CE(8);
  else if (nv <= 13) HYDRA_CE(13);
  else HYDRA_CE(16);
#undef HYDRA_CE
  return true;
}

hipError_t launch_cross_entropy(int dtype, const float *logits, const int32_t *targets, float *row_loss, void *dlogits,
                                int M, int V, int64_t ld, float inv_n, hipStream_t s) {
  ProfScope ps("cross_entropy", s, 0, (double)M * V * (4.0 + dt_size(dtype)));
  if (M <= 0) return hipSuccess;
  const bool done = dtype == DT_BF16 ? launch_ce_row(logits, targets, row_loss, (bf16_t *)dlogits, M, V, ld, inv_n, s)
                                     : launch_ce_row(logits, targets, row_loss, (float *)dlogits, M, V, ld, inv_n, s);
  if (done) return hipGetLastError();
  if (dtype == DT_BF16)
    hipLaunchKernelGGL(cross_entropy_kernel<bf16_t>, dim3(M), dim3(256), 0, s, logits, targets, row_loss,
                       (bf16_t *)dlogits, V, ld, inv_n);
  else
    hipLaunchKernelGGL(cross_entropy_kernel<float>, dim3(M), dim3(256), 0, s, logits, targets, row_loss,
                       (float *)dlogits, V, ld, inv_n);
  return hipGetLastError();
}

// single block; thread t sums rows t, t+256, ... in double, then a fixed tree
__global__ __launch_bounds__(256) void loss_reduce_kernel(const float *__restrict__ row_loss, float *__restrict__ loss,
                                                          int M, float inv_n) {
  __shared__ double sh[256];
  double a = 0.0;
  for (int i = threadIdx.x; i < M; i += 256) a += (double)row_loss[i];
  sh[threadIdx.x] = a;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) loss[0] = (float)(sh[0] * (double)inv_n);
}

hipError_t launch_loss_reduce(const float *row_loss, float *loss, int M, float inv_n, hipStream_t s) {
  hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(256), 0, s, row_loss, loss, M, inv_n);
  return hipGetLastError();
}

// ------------------------------------------------------------------ Adam
// m <- b1 m + (1-b1) g ; v <- b2 v + (1-b2) g^2 ; w <- w - lr (m/c1) / (sqrt(v/c2) + eps)
// 16 B read and 12 B (+2 B bf16 copy) written per parameter.
__global__ __launch_bounds__(256) void adam_kernel(float *__restrict__ w, float *__restrict__ m, float *__restrict__ v,
                                                   const float *__restrict__ g, bf16_t *__restrict__ shadow, int64_t n,
                                                   float lr, float b1, float b2, float ob1, float ob2, float eps,
                                                   float c1, float c2) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x * 4;
  for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4; i < n; i += stride) {
    if (i + 4 <= n) {
      float4 W = *(float4 *)(w + i), Mm = *(float4 *)(m + i), Vv = *(float4 *)(v + i);
      const float4 G = *(const float4 *)(g + i);
      float *pw = (float *)&W, *pm = (float *)&Mm, *pv = (float *)&Vv;
      const float *pg = (const float *)&G;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        pm[k] = b1 * pm[k] + ob1 * pg[k];
        pv[k] = b2 * pv[k] + ob2 * (pg[k] * pg[k]);
        pw[k] = pw[k] - lr * (pm[k] / c1) / (sqrtf(pv[k] / c2) + eps);
      }
      *(float4 *)(w + i) = W;
      *(float4 *)(m + i) = Mm;
      *(float4 *)(v + i) = Vv;
      if (shadow) {
        uint2 o;
        o.x = (uint32_t)f2bf(pw[0]) | ((uint32_t)f2bf(pw[1]) << 16);
        o.y = (uint32_t)f2bf(pw[2]) | ((uint32_t)f2bf(pw[3]) << 16);
        *(uint2 *)(shadow + i) = o;
      }
    } else {
      for (int64_t j = i; j < n; ++j) {
        const float gg = g[j];
        const float mm = b1 * m[j] + ob1 * gg;
        const float vv = b2 * v[j] + ob2 * (gg * gg);
        const float ww = w[j] - lr * (mm / c1) / (sqrtf(vv / c2) + eps);
        m[j] = mm; v[j] = vv; w[j] = ww;
        if (shadow) shadow[j] = f2bf(ww);
      }
    }
  }
}

hipError_t launch_adam(float *w, float *m, float *v, const float *g, bf16_t *shadow, int64_t n, double lr, double beta1,
                       double beta2, double eps, int64_t t, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  const float corr1 = (float)(1.0 - pow(beta1, (double)t)), corr2 = (float)(1.0 - pow(beta2, (double)t));
  ProfScope ps("adam", s, 0, (double)n * (shadow ? 30.0 : 28.0));
  int64_t blocks = (n / 4 + 255) / 256;  // uncapped, see launch_fill_u32
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(adam_kernel, dim3((unsigned)blocks), dim3(256), 0, s, w, m, v, g, shadow, n, (float)lr, (float)beta1,
                     (float)beta2, (float)(1.0 - beta1), (float)(1.0 - beta2), (float)eps, corr1, corr2);
  return hipGetLastError();
}

// ------------------------------------------------------------ link copy
// Streams a device buffer into page-locked host memory (mapped into the device
// address space) with plain 16-byte vector stores.  A small grid suffices: the
// host link, not the CUs, bounds it (16 workgroups already reach its rate), and
// the more workgroups copy the slower all compute kernels run meanwhile; how
// many a write-back gets is decided in copy_to_host_blocks.
__global__ __launch_bounds__(256) void copy_to_host_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src,
                                                           int64_t n16, uint8_t *dst_tail, const uint8_t *src_tail,
                                                           int tail) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  // non-temporal stores: the data is never read back on the device, and keeping it out of the L2's way measured
  // 1-3 % more throughput of the whole spilled step than plain stores (two-model GPT-2-small workload with 1, 4 and
  // 8 micro-batches per visit, alternating runs on one machine)
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
    const uint4 v = src[i];
    __builtin_nontemporal_store(v.x, &dst[i].x);
    __builtin_nontemporal_store(v.y, &dst[i].y);
    __builtin_nontemporal_store(v.z, &dst[i].z);
    __builtin_nontemporal_store(v.w, &dst[i].w);
  }
  if (blockIdx.x == 0 && threadIdx.x < tail) dst_tail[threadIdx.x] = src_tail[threadIdx.x];
}

// Workgroups of a write-back copy.  The more workgroups copy, the slower every compute kernel on the device runs
// meanwhile, wherever it runs (measured; presumably stores to host memory wait in the L2 channels' queues, in front
// of everybody else's requests, until the link has taken them; the same write-back through SDMA slows nothing, but
// reaches only 15-30 GB/s next to the promotes), and the more of the link the write-back takes from the promote
// that runs beside it (48 workgroups: 50 GB/s out, 38 in; 12: 46 out, 45 in - together more than before).
//  - Few tokens per visit, large shards (more than 192 MB per state array): the promote of the next shard and the
//    write-back of the last one run side by side for their whole length and carry the same bytes, so they should
//    take equally long: 12 workgroups (four GPT-2-medium models 625 against 660 ms per step with 48, four GPT-2-XL
//    models 2266 against 2390, two 6 B models 4317 against 4599; 8 and 4 workgroups starve the write-back: 4690,
//    5198 ms).
//  - Few tokens per visit, small shards: 16 (two-model GPT-2-small workload, 8 / 12 / 16 / 24 / 48 / 96 workgroups:
//    112 / 97.3 / 96.3 / 97.2 / 99.3 / 101.8 ms per step.  While promotes were still enqueued behind stream waits,
//    48 was best here - the chain promote -> task -> write-back -> promote into the same buffer wanted the buffer
//    free early; with the waits on the host that no longer pays.)
//  - The more tokens a visit works on, the more the compute kernels matter and the fewer workgroups a write-back gets
//    (GPT-2-small workload, tokens per visit 2048 x 4 / 6 / 8 / 12: best at 16 / 12 / 8 / 8 workgroups, up to a fifth
//    faster than with 32 throughout).
int copy_to_host_blocks(int64_t tokens_per_visit, size_t array_bytes) {
  if (tokens_per_visit < 6144) return array_bytes > ((size_t)192 << 20) ? 12 : 16;
  if (tokens_per_visit < 12288) return 16;
  if (tokens_per_visit < 16384) return 12;
  return 8;
}

hipError_t launch_copy_to_host(void *dst_mapped, const void *src, size_t bytes, int64_t tokens_per_visit, int blocks,
                               size_t array_bytes, hipStream_t s) {
  return launch_copy_link(dst_mapped, src, bytes, blocks > 0 ? blocks : copy_to_host_blocks(tokens_per_visit, array_bytes), s);
}

hipError_t launch_copy_link(void *dst_mapped, const void *src, size_t bytes, int max_blocks, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  if ((((uintptr_t)dst_mapped) | ((uintptr_t)src)) & 15) return hipErrorInvalidValue;
  const int64_t n16 = (int64_t)(bytes / 16);
  const int tail = (int)(bytes % 16);
  int64_t blocks = (n16 + 255) / 256;
  if (blocks > max_blocks) blocks = max_blocks;
  if (blocks < 1) blocks = 1;
  ProfScope ps("copy_to_host", s, 0, (double)bytes);
  hipLaunchKernelGGL(copy_to_host_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (uint4 *)dst_mapped, (const uint4 *)src,
                     n16, (uint8_t *)dst_mapped + n16 * 16, (const uint8_t *)src + n16 * 16, tail);
  return hipGetLastError();
}

// An empty kernel: a point in a stream that is certainly ordered after every wait enqueued before it (used by the
// overlap trace, whose interval must not start while its stream still waits for another stream's event).
__global__ void stream_marker_kernel() {}
hipError_t launch_stream_marker(hipStream_t s) {
  hipLaunchKernelGGL(stream_marker_kernel, dim3(1), dim3(64), 0, s);
  return hipGetLastError();
}

// ------------------------------------------------------------------ casts
__global__ __launch_bounds__(256) void cast_bf16_kernel(const float *__restrict__ in, bf16_t *__restrict__ out,
                                                        int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x * 4;
  for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4; i < n; i += stride) {
    if (i + 4 <= n) {
      const float4 a = *(const float4 *)(in + i);
      uint2 o;
      o.x = (uint32_t)f2bf(a.x) | ((uint32_t)f2bf(a.y) << 16);
      o.y = (uint32_t)f2bf(a.z) | ((uint32_t)f2bf(a.w) << 16);
      *(uint2 *)(out + i) = o;
    } else {
      for (int64_t j = i; j < n; ++j) out[j] = f2bf(in[j]);
    }
  }
}

hipError_t launch_cast_bf16(const float *in, bf16_t *out, int64_t n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  ProfScope ps("cast_bf16", s, 0, 6.0 * n);
  int64_t blocks = (n / 4 + 255) / 256;  // uncapped, see launch_fill_u32
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(cast_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, s, in, out, n);
  return hipGetLastError();
}

// 64x64 tile through LDS: coalesced reads along C, coalesced writes along R
__global__ __launch_bounds__(256) void cast_transpose_bf16_kernel(const float *__restrict__ in, bf16_t *__restrict__ out,
                                                                  int R, int C) {
  __shared__ float t[64][65];
  const int c0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int r = ty; r < 64; r += 4)
    t[r][tx] = (r0 + r < R && c0 + tx < C) ? in[(int64_t)(r0 + r) * C + c0 + tx] : 0.f;
  __syncthreads();
  for (int c = ty; c < 64; c += 4)
    if (c0 + c < C && r0 + tx < R) out[(int64_t)(c0 + c) * R + r0 + tx] = f2bf(t[tx][c]);
}

hipError_t launch_cast_transpose_bf16(const float *in, bf16_t *out, int R, int C, hipStream_t s) {
  ProfScope ps("cast_transpose_bf16", s, 0, 6.0 * R * C);
  hipLaunchKernelGGL(cast_transpose_bf16_kernel, dim3((C + 63) / 64, (R + 63) / 64), dim3(256), 0, s, in, out, R, C);
  return hipGetLastError();
}

// four consecutive elements as floats
__device__ __forceinline__ float4 ld4(const float *p) { return *(const float4 *)p; }
__device__ __forceinline__ float4 ld4(const bf16_t *p) {
  const uint2 u = *(const uint2 *)p;
  return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u), __uint_as_float(u.y << 16),
                     __uint_as_float(u.y & 0xffff0000u));
}

// 64x64 tiles through LDS; 16 lanes cover a row of the tile with four elements each, on the way in (along the
// source's columns) and on the way out (along its rows).  VEC: every matrix has R, C multiples of 4 and an offset
// that keeps the vector accesses aligned; otherwise element by element.
template <typename SrcT, bool VEC>
__global__ __launch_bounds__(256) void transpose_group_kernel(const SrcT *__restrict__ src, bf16_t *__restrict__ dst,
                                                              const TransposeGroup g) {
  __shared__ float t[64][65];
  int i = 0;
#pragma unroll 1
  while (i + 1 < g.n && (int)blockIdx.x >= g.tile0[i + 1]) ++i;  // uniform over the block
  const int R = g.R[i], C = g.C[i];
  const int tile = blockIdx.x - g.tile0[i], tc = (C + 63) / 64;
  const int c0 = (tile % tc) * 64, r0 = (tile / tc) * 64;
  const SrcT *in = src + g.off[i];
  bf16_t *out = dst + g.off[i];
  if (VEC) {
    const int q = (threadIdx.x & 15) * 4, p = threadIdx.x >> 4;  // 4 elements at q of line p, p + 16, ...
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int r = p + 16 * k;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (r0 + r < R && c0 + q < C) v = ld4(in + (int64_t)(r0 + r) * C + c0 + q);
      t[r][q] = v.x; t[r][q + 1] = v.y; t[r][q + 2] = v.z; t[r][q + 3] = v.w;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int c = p + 16 * k;
      if (c0 + c < C && r0 + q < R) {
        uint2 o;
        o.x = (uint32_t)f2bf(t[q][c]) | ((uint32_t)f2bf(t[q + 1][c]) << 16);
        o.y = (uint32_t)f2bf(t[q + 2][c]) | ((uint32_t)f2bf(t[q + 3][c]) << 16);
        *(uint2 *)(out + (int64_t)(c0 + c) * R + r0 + q) = o;
      }
    }
    return;
  }
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int r = ty; r < 64; r += 4)
    t[r][tx] = (r0 + r < R && c0 + tx < C) ? ldv<SrcT>(in, (int64_t)(r0 + r) * C + c0 + tx) : 0.f;
  __syncthreads();
  for (int c = ty; c < 64; c += 4)
    if (c0 + c < C && r0 + tx < R) out[(int64_t)(c0 + c) * R + r0 + tx] = f2bf(t[tx][c]);
}

hipError_t launch_transpose_group(int src_dtype, const void *src, bf16_t *dst, TransposeGroup &g, hipStream_t s) {
  if (g.n <= 0) return hipSuccess;
  if (g.n > TRANSPOSE_MAX) return hipErrorInvalidValue;
  int tiles = 0;
  double elems = 0;
  for (int i = 0; i < g.n; ++i) {
    g.tile0[i] = tiles;
    tiles += ((g.R[i] + 63) / 64) * ((g.C[i] + 63) / 64);
    elems += (double)g.R[i] * g.C[i];
  }
  g.tile0[g.n] = tiles;
  bool vec = ((((uintptr_t)src) & 15) == 0) && ((((uintptr_t)dst) & 7) == 0);
  for (int i = 0; i < g.n; ++i) vec = vec && g.R[i] % 4 == 0 && g.C[i] % 4 == 0 && g.off[i] % 4 == 0;
  ProfScope ps("transpose_weights", s, 0, elems * (dt_size(src_dtype) + 2.0));
  if (src_dtype == DT_BF16) {
    if (vec) hipLaunchKernelGGL((transpose_group_kernel<bf16_t, true>), dim3(tiles), dim3(256), 0, s, (const bf16_t *)src, dst, g);
    else hipLaunchKernelGGL((transpose_group_kernel<bf16_t, false>), dim3(tiles), dim3(256), 0, s, (const bf16_t *)src, dst, g);
  } else {
    if (vec) hipLaunchKernelGGL((transpose_group_kernel<float, true>), dim3(tiles), dim3(256), 0, s, (const float *)src, dst, g);
    else hipLaunchKernelGGL((transpose_group_kernel<float, false>), dim3(tiles), dim3(256), 0, s, (const float *)src, dst, g);
  }
  return hipGetLastError();
}

template <typename OutT>
__global__ void cast_act_kernel(const float *__restrict__ in, int64_t ld_in, OutT *__restrict__ out, int64_t ld_out, int R,
                                int C) {
  const int r = blockIdx.y;
  for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < C; c += gridDim.x * blockDim.x)
    stv<OutT>(out, (int64_t)r * ld_out + c, in[(int64_t)r * ld_in + c]);
}

hipError_t launch_cast_act(int dtype, const float *in, int64_t ld_in, void *out, int64_t ld_out, int R, int C,
                           hipStream_t s) {
  dim3 grid(min(64, (C + 255) / 256), R);
  ProfScope ps("cast_act", s, 0, (double)R * C * (4.0 + dt_size(dtype)));
  if (dtype == DT_BF16)
    hipLaunchKernelGGL(cast_act_kernel<bf16_t>, grid, dim3(256), 0, s, in, ld_in, (bf16_t *)out, ld_out, R, C);
  else
    hipLaunchKernelGGL(cast_act_kernel<float>, grid, dim3(256), 0, s, in, ld_in, (float *)out, ld_out, R, C);
  return hipGetLastError();
}

}  // namespace hydra
