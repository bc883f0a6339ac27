// Launchers of the gfx950 kernels.  Host-callable, all pointers are device
// pointers unless stated; every launcher only enqueues on the given stream.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hydra {

typedef uint16_t bf16_t;  // raw bfloat16 storage

enum { DT_F32 = 0, DT_BF16 = 1 };
enum { EPI_NONE = 0, EPI_GELU = 1, EPI_DGELU = 2 };
// causal structure of a batched [T,T] attention operand / result
enum {
  CAUSAL_NONE = 0,
  CAUSAL_SKIP_UPPER = 1,  // result is [T,T]: tiles entirely above the diagonal are not computed
  CAUSAL_K_END = 2,       // A is lower-triangular [i,j]: contraction stops at the row tile's end
  CAUSAL_K_BEGIN = 3      // A^T is used (A stored [i,j], rows of the result are j): contraction starts at the row tile
};

static inline size_t dt_size(int dt) { return dt == DT_BF16 ? 2 : 4; }

// Brackets one kernel launch with two events when per-kernel timing is active
// (no-op otherwise).  flops / bytes: algorithmic work of the launch.
struct ProfScope {
  ProfScope(const char *name, hipStream_t s, double flops, double bytes);
  ~ProfScope();
  hipStream_t stream_;
  long idx_;
};

// While one of these lives on a thread, ProfScope records nothing on that thread.
struct ProfSuppress {
  ProfSuppress();
  ~ProfSuppress();
};

struct GemmDesc {
  int dtype = DT_BF16;
  int ta = 0, tb = 0;  // ta: A stored [K,M]; tb: B stored [K,N] (else [N,K])
  int M = 0, N = 0, K = 0;
  float alpha = 1.f;
  const void *A = nullptr;
  int64_t lda = 0;
  const void *B = nullptr;
  int64_t ldb = 0;
  int64_t ldc = 0;
  int nb1 = 1, nb2 = 1;  // batch = nb1*nb2, matrix (i1,i2) at offset i1*s?1 + i2*s?2 elements
  int64_t sA1 = 0, sA2 = 0, sB1 = 0, sB2 = 0, sC1 = 0, sC2 = 0;
  const float *bias = nullptr;   // [N]
  const float *resid = nullptr;  // fp32, same shape/ld/batching as C
  float *out_f32 = nullptr;
  void *out_act = nullptr;   // operand-dtype output
  int epi = EPI_NONE;
  void *out_act2 = nullptr;  // EPI_GELU: gelu(value); out_act then holds the pre-activation
  const void *aux = nullptr; // EPI_DGELU: pre-activation u (operand dtype, ld = ldc)
  int causal = CAUSAL_NONE;
};

hipError_t launch_gemm(const GemmDesc &g, hipStream_t s);
// n products in one launch where they allow it (bf16, both operands stored with the contraction index strided, no
// batching, contraction of at least 1536): the weight-gradient products of a block; otherwise one launch each
hipError_t launch_gemm_group(const GemmDesc *g, int n, hipStream_t s);

// x0[m,:] = wte[tok[m],:] + wpe[m % T,:]
hipError_t launch_embed_fwd(const int32_t *tok, const float *wte, const float *wpe, float *x0, int M, int T, int d,
                            hipStream_t s);
// dwte = 0 then rows of present tokens accumulate dx0 in ascending m; dwpe[t] = sum_b dx0[b*T+t]
// acc_wte / acc_wpe != 0: add to the gradient already held (a later micro-batch of the same minibatch; for wte
// also the tied LM head's part)
hipError_t launch_embed_bwd(const int32_t *tok, const float *dx0, float *dwte, float *dwpe, int B, int T, int d, int V,
                            int acc_wte, int acc_wpe,
                            hipStream_t s);

hipError_t launch_layernorm_fwd(int dtype, const float *x, const float *gamma, const float *beta, void *y, float *mean,
                                float *rstd, int M, int d, hipStream_t s);
// dx = dres + LN'(dy) (dres may be null); dy is fp32; dx_bf16 (may be null): bf16 copy of dx, same shape
hipError_t launch_layernorm_bwd_dx(const float *dy, const float *x, const float *mean, const float *rstd,
                                   const float *gamma, const float *dres, float *dx, void *dx_bf16, int M, int d,
                                   hipStream_t s);
// dgamma[n] = sum_m dy*xhat, dbeta[n] = sum_m dy ; scratch: fp32 [2 * colsum_chunks(M) * d]; acc != 0 adds to the outputs
hipError_t launch_layernorm_bwd_params(const float *dy, const float *x, const float *mean, const float *rstd,
                                       float *dgamma, float *dbeta, float *scratch, int M, int d, int acc, hipStream_t s);
int colsum_chunks(int M);
// Backward of a LayerNorm in one pass: dx = dres + LN'(dy) (dres may be null), its bf16 copy (dx_bf16 may be null)
// and per-block partial column sums part[blocks][3][d] of dy*xhat, dy and dx, blocks = layernorm_bwd_fused_blocks(M);
// the sums are finished by launch_colsum_finish.  Rows of up to 2048 elements (layernorm_bwd_fused_supported).
bool layernorm_bwd_fused_supported(int d);
int layernorm_bwd_fused_blocks(int M);
hipError_t launch_layernorm_bwd_fused(const float *dy, const float *x, const float *mean, const float *rstd,
                                      const float *gamma, const float *dres, float *dx, void *dx_bf16, float *part, int M,
                                      int d, hipStream_t s);
// part[blocks][3][d]: third part = column sums of in [M,d] over the same row blocks, added in the same order as
// launch_layernorm_bwd_fused adds its dx (bit-identical to it for the same values)
hipError_t launch_colsum_rows8(const float *in, float *part, int M, int d, hipStream_t s);
// pass 1 of the column sums of two [M,N0] / [M,N1] operands of one dtype (leading dimension = N): partials
// part0 [colsum_chunks(M)][N0], part1 [colsum_chunks(M)][N1]
hipError_t launch_colsum2_pass1(int dtype, const void *in0, int N0, float *part0, const void *in1, int N1, float *part1,
                                int M, hipStream_t s);
// Several column sums finished by one launch: out[c] (+)= sum over k < nch of part[k * stride + c], c < N.
constexpr int COLSUM_MAX_SEGS = 10;
struct ColsumSeg {
  const float *part;
  float *out;
  int64_t stride;
  int nch, N, col0;  // col0 is filled in by the launcher
};
struct ColsumFinish {
  ColsumSeg seg[COLSUM_MAX_SEGS];
  int nseg = 0, acc = 0;
  void add(const float *part, int64_t stride, int nch, int N, float *out) {
    if (nseg < COLSUM_MAX_SEGS) seg[nseg] = ColsumSeg{part, out, stride, nch, N, 0};
    ++nseg;
  }
};
hipError_t launch_colsum_finish(ColsumFinish &a, hipStream_t s);
// out[n] (+)= sum_m in[m,n]; in has operand dtype (or fp32 when in_dtype == DT_F32); scratch fp32 [colsum_chunks(M)*N]
hipError_t launch_colsum(int in_dtype, const void *in, int64_t ld, float *out, float *scratch, int M, int N, int acc,
                         hipStream_t s);

// Fused causal attention (bf16 operands, head width 64 or 128).  qkv [B*T, 3d] (q | k | v, head h at columns
// h*dh of each part), o [B*T, d], lse [B*H*T] = log-sum-exp of every score row.  Backward: d_o [B*T, d] -> dqkv
// [B*T, 3d]; dsum [B*H*T] is scratch (row sums of dO * O).
bool attention_fused_supported(int dtype, int dh);
hipError_t launch_attention_fwd(const void *qkv, void *o, float *lse, int B, int H, int T, int dh, hipStream_t s);
hipError_t launch_attention_bwd(const void *qkv, const void *o, const void *d_o, const float *lse, float *dsum,
                                void *dqkv, int B, int H, int T, int dh, hipStream_t s);

// P[z,i,j] = softmax_j<=i S[z,i,j]; zero for i < j < min(T, roundup(i+1,256)); nothing written beyond
hipError_t launch_softmax_causal_fwd(int dtype, const float *S, void *P, int n_mat, int T, hipStream_t s);
// dS = P * (dP - rowsum(dP*P)), same zero-fill rule; dP fp32
hipError_t launch_softmax_causal_bwd(int dtype, const void *P, const float *dP, void *dS, int n_mat, int T,
                                     hipStream_t s);

hipError_t launch_cross_entropy(int dtype, const float *logits, const int32_t *targets, float *row_loss, void *dlogits,
                                int M, int V, int64_t ld, float inv_n, hipStream_t s);
// loss[0] = (sum_m row_loss[m]) * inv_n, summed in double in a fixed order
hipError_t launch_loss_reduce(const float *row_loss, float *loss, int M, float inv_n, hipStream_t s);

// hyper-parameters in double; the kernel receives beta, 1-beta and 1-beta^t each rounded once to fp32
hipError_t launch_adam(float *w, float *m, float *v, const float *g, bf16_t *shadow, int64_t n, double lr, double beta1,
                       double beta2, double eps, int64_t t, hipStream_t s);

hipError_t launch_cast_bf16(const float *in, bf16_t *out, int64_t n, hipStream_t s);
// out[c, r] = bf16(in[r, c]) ; in is [R, C] row-major, out is [C, R]
hipError_t launch_cast_transpose_bf16(const float *in, bf16_t *out, int R, int C, hipStream_t s);
// Several matrices of one flat array transposed by one launch: matrix i is [R[i], C[i]] row-major at element offset
// off[i] of src (fp32 or bf16) and is written as bf16 [C[i], R[i]] at the same offset of dst.
constexpr int TRANSPOSE_MAX = 64;
struct TransposeGroup {
  int n = 0;
  int64_t off[TRANSPOSE_MAX];
  int R[TRANSPOSE_MAX], C[TRANSPOSE_MAX];
  int tile0[TRANSPOSE_MAX + 1];  // filled in by the launcher: first 64x64 tile of every matrix
  bool add(int64_t o, int r, int c) {
    if (n >= TRANSPOSE_MAX) return false;
    off[n] = o; R[n] = r; C[n] = c;
    ++n;
    return true;
  }
};
hipError_t launch_transpose_group(int src_dtype, const void *src, bf16_t *dst, TransposeGroup &g, hipStream_t s);
// fp32 [R,C] (ld_in) -> operand dtype [R,C] (ld_out)
hipError_t launch_cast_act(int dtype, const float *in, int64_t ld_in, void *out, int64_t ld_out, int R, int C,
                           hipStream_t s);
hipError_t launch_stream_marker(hipStream_t s);  // empty kernel
hipError_t launch_fill_u32(uint32_t *p, uint32_t value, int64_t n, hipStream_t s);
// device -> page-locked host memory through its device-side mapping (both 16-byte aligned); blocks workgroups, or
// (blocks <= 0) as many as copy_to_host_blocks gives for the tokens a shard visit works on and the size of the state
// array the copy is (a piece of)
hipError_t launch_copy_to_host(void *dst_mapped, const void *src, size_t bytes, int64_t tokens_per_visit, int blocks,
                               size_t array_bytes, hipStream_t s);
int copy_to_host_blocks(int64_t tokens_per_visit, size_t array_bytes);
// the same kernel in either direction (one side is the device-side mapping of page-locked host memory), grid capped
hipError_t launch_copy_link(void *dst, const void *src, size_t bytes, int max_blocks, hipStream_t s);

}  // namespace hydra
