// Single-kernel entry points of the C ABI, used by parity tests and by the
// roofline measurements.  All pointers are device pointers.
#include <mutex>

#include "hydra_internal.h"

using namespace hydra;

// ---------------------------------------------------------------------------
// Scratch memory of hydra_op_layernorm_bwd_static, the one entry point that
// must not allocate: a fixed array in every GPU's copy of the code object
// instead of a caller-supplied workspace.  In host code `scratch` is only a
// handle for the symbol; the array's device address - a different one on every
// GPU - comes from hipGetSymbolAddress with that GPU current and is what the
// kernels are given.
// ---------------------------------------------------------------------------
constexpr size_t STATIC_SCRATCH_FLOATS = (size_t)2 << 20;  // 8 MiB on every GPU the library runs on
static __device__ __align__(256) float scratch[STATIC_SCRATCH_FLOATS];

constexpr int STATIC_SCRATCH_MAX_DEVICES = 64;
static float *g_scratch_ptr[STATIC_SCRATCH_MAX_DEVICES];  // per GPU: device address of its copy of `scratch`
static std::mutex g_scratch_mu;

namespace hydra {

// Device address of the current GPU's scratch array; resolved once per GPU (hydra_init does it for the GPU its
// context is created on, the entry point itself on its first call on any other).
hydra_status static_scratch(float **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hipfail(nullptr, e, "hipGetDevice");
  if (dev < 0 || dev >= STATIC_SCRATCH_MAX_DEVICES) return fail(nullptr, HYDRA_E_INVAL, "device index out of range");
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return hipfail(nullptr, e, "hipGetSymbolAddress(scratch)");
    g_scratch_ptr[dev] = (float *)p;
  }
  *out = g_scratch_ptr[dev];
  return HYDRA_OK;
}

}  // namespace hydra

static hydra_status ret(hipError_t e, const char *what) {
  if (e == hipSuccess) return HYDRA_OK;
  return hipfail(nullptr, e, what);
}

extern "C" {

hydra_status hydra_op_gemm(int32_t dtype, int32_t ta, int32_t tb, int32_t M, int32_t N, int32_t K, float alpha,
                           const void *A, int64_t lda, const void *B, int64_t ldb, const float *bias,
                           const float *resid, float *out_f32, void *out_act, int64_t ldc, void *stream) {
  if ((dtype != 0 && dtype != 1) || M < 0 || N < 0 || K < 0 || !A || !B || (!out_f32 && !out_act))
    return fail(nullptr, HYDRA_E_INVAL, "bad GEMM argument");
  // a leading dimension shorter than a stored row would make the kernel read or write outside the operands
  if (lda < (ta ? M : K) || ldb < (tb ? N : K) || ldc < N)
    return fail(nullptr, HYDRA_E_INVAL, "GEMM leading dimension shorter than a stored row");
  GemmDesc g;
  g.dtype = dtype; g.ta = ta != 0; g.tb = tb != 0; g.M = M; g.N = N; g.K = K; g.alpha = alpha;
  g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.ldc = ldc;
  g.bias = bias; g.resid = resid; g.out_f32 = out_f32; g.out_act = out_act;
  return ret(launch_gemm(g, (hipStream_t)stream), "gemm");
}

hydra_status hydra_op_adam(float *w, float *m, float *v, const float *g, void *shadow_bf16, int64_t n, double lr,
                           double beta1, double beta2, double eps, int64_t t, void *stream) {
  if (!w || !m || !v || !g || n < 0 || t < 1) return fail(nullptr, HYDRA_E_INVAL, "bad Adam argument");
  return ret(launch_adam(w, m, v, g, (bf16_t *)shadow_bf16, n, lr, beta1, beta2, eps, t, (hipStream_t)stream), "adam");
}

hydra_status hydra_op_layernorm_fwd(int32_t dtype, const float *x, const float *gamma, const float *beta, void *y,
                                    float *mean, float *rstd, int32_t M, int32_t d, void *stream) {
  if ((dtype != 0 && dtype != 1) || !x || !gamma || !beta || !y || !mean || !rstd || M < 0 || d <= 0 || (d & 7))
    return fail(nullptr, HYDRA_E_INVAL, "bad LayerNorm argument");
  return ret(launch_layernorm_fwd(dtype, x, gamma, beta, y, mean, rstd, M, d, (hipStream_t)stream), "layernorm");
}

hydra_status hydra_op_layernorm_bwd(const float *dy, const float *x, const float *mean, const float *rstd,
                                    const float *gamma, const float *dres, float *dx, void *dx_bf16, float *dgamma,
                                    float *dbeta, float *dx_colsum, float *scratch, int32_t M, int32_t d, void *stream) {
  if (!dy || !x || !mean || !rstd || !gamma || !dx || !dgamma || !dbeta || !scratch || M < 0 || d <= 0 ||
      !layernorm_bwd_fused_supported(d))
    return fail(nullptr, HYDRA_E_INVAL, "bad LayerNorm backward argument (d % 4 == 0, d <= 2048)");
  if (M == 0) return HYDRA_OK;
  hipStream_t st = (hipStream_t)stream;
  hipError_t e = launch_layernorm_bwd_fused(dy, x, mean, rstd, gamma, dres, dx, dx_bf16, scratch, M, d, st);
  if (e != hipSuccess) return ret(e, "layernorm_bwd");
  ColsumFinish fin;
  const int nb = layernorm_bwd_fused_blocks(M);
  fin.add(scratch, 3 * (int64_t)d, nb, d, dgamma);
  fin.add(scratch + d, 3 * (int64_t)d, nb, d, dbeta);
  if (dx_colsum) fin.add(scratch + 2 * d, 3 * (int64_t)d, nb, d, dx_colsum);
  return ret(launch_colsum_finish(fin, st), "layernorm_bwd (column sums)");
}

hydra_status hydra_op_layernorm_bwd_static(const float *dy, const float *x, const float *mean, const float *rstd,
                                           const float *gamma, const float *dres, float *dx, void *dx_bf16,
                                           float *dgamma, float *dbeta, float *dx_colsum, int32_t M, int32_t d,
                                           void *stream) {
  if (!dy || !x || !mean || !rstd || !gamma || !dx || !dgamma || !dbeta || M < 0 || d <= 0 ||
      !layernorm_bwd_fused_supported(d))
    return fail(nullptr, HYDRA_E_INVAL, "bad LayerNorm backward argument (d % 4 == 0, d <= 2048)");
  const int nb = layernorm_bwd_fused_blocks(M);
  if ((size_t)3 * (size_t)d * (size_t)nb > STATIC_SCRATCH_FLOATS)
    return fail(nullptr, HYDRA_E_INVAL, "3 * d * ceil(M / 8) exceeds the 2 Mi floats of the static scratch array");
  if (M == 0) return HYDRA_OK;
  float *part = nullptr;  // this GPU's array: every partial sum read below is written first by this same call
  hydra_status st = static_scratch(&part);
  if (st) return st;
  hipStream_t hs = (hipStream_t)stream;
  ProfSuppress quiet;  // event brackets of a timing context would create events: nothing here may allocate
  hipError_t e = launch_layernorm_bwd_fused(dy, x, mean, rstd, gamma, dres, dx, dx_bf16, part, M, d, hs);
  if (e != hipSuccess) return ret(e, "layernorm_bwd");
  ColsumFinish fin;
  fin.add(part, 3 * (int64_t)d, nb, d, dgamma);
  fin.add(part + d, 3 * (int64_t)d, nb, d, dbeta);
  if (dx_colsum) fin.add(part + 2 * d, 3 * (int64_t)d, nb, d, dx_colsum);
  return ret(launch_colsum_finish(fin, hs), "layernorm_bwd (column sums)");
}

hydra_status hydra_op_softmax_causal(int32_t dtype, const float *S, void *P, int32_t n_mat, int32_t T, void *stream) {
  if ((dtype != 0 && dtype != 1) || !S || !P || n_mat < 0 || T <= 0) return fail(nullptr, HYDRA_E_INVAL, "bad softmax argument");
  return ret(launch_softmax_causal_fwd(dtype, S, P, n_mat, T, (hipStream_t)stream), "softmax");
}

hydra_status hydra_op_cross_entropy(int32_t dtype, const float *logits, const int32_t *targets, float *row_loss,
                                    void *dlogits, int32_t M, int32_t V, int64_t ld, float inv_n, void *stream) {
  if ((dtype != 0 && dtype != 1) || !logits || !targets || !row_loss || !dlogits || M < 0 || V <= 0 || ld < V)
    return fail(nullptr, HYDRA_E_INVAL, "bad cross-entropy argument");
  return ret(launch_cross_entropy(dtype, logits, targets, row_loss, dlogits, M, V, ld, inv_n, (hipStream_t)stream),
             "cross_entropy");
}

hydra_status hydra_host_round_bf16(uint16_t *dst, const float *src, int64_t n) {
  if (!dst || !src || n < 0) return fail(nullptr, HYDRA_E_INVAL, "bad argument");
  host_round_bf16(dst, src, (size_t)n);
  return HYDRA_OK;
}

hydra_status hydra_op_attention_fwd(const void *qkv, void *o, float *lse, int32_t B, int32_t H, int32_t T, int32_t dh,
                                    void *stream) {
  if (!qkv || !o || !lse || B <= 0 || H <= 0 || T <= 0 || (T & 7) || !attention_fused_supported(DT_BF16, dh))
    return fail(nullptr, HYDRA_E_INVAL, "bad attention argument (bf16 only, head width 64 or 128, T % 8 == 0)");
  return ret(launch_attention_fwd(qkv, o, lse, B, H, T, dh, (hipStream_t)stream), "attention_fwd");
}

hydra_status hydra_op_attention_bwd(const void *qkv, const void *o, const void *d_o, const float *lse, float *dsum,
                                    void *dqkv, int32_t B, int32_t H, int32_t T, int32_t dh, void *stream) {
  if (!qkv || !o || !d_o || !lse || !dsum || !dqkv || B <= 0 || H <= 0 || T <= 0 || (T & 7) ||
      !attention_fused_supported(DT_BF16, dh))
    return fail(nullptr, HYDRA_E_INVAL, "bad attention argument (bf16 only, head width 64 or 128, T % 8 == 0)");
  return ret(launch_attention_bwd(qkv, o, d_o, lse, dsum, dqkv, B, H, T, dh, (hipStream_t)stream), "attention_bwd");
}

}  // extern "C"
