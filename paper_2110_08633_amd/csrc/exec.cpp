// Shard executor: the kernel sequence of a forward visit, a backward visit
// (recompute from the boundary checkpoint, then back-propagate; paper Section
// 2.3) and the Adam step of one shard, all enqueued on the compute stream.
#include <algorithm>
#include <cmath>

#include "hydra_internal.h"

namespace hydra {

static inline uint64_t up256(uint64_t x) { return (x + 255) / 256 * 256; }

namespace {

// Bump allocator over the shared workspace; one task at a time uses it.
struct Bump {
  char *base;
  uint64_t cap, used = 0;
  bool ok = true;
  template <typename T> T *take(uint64_t count, uint64_t elem = sizeof(T)) {
    const uint64_t bytes = up256(count * elem);
    if (used + bytes > cap) {
      ok = false;
      return nullptr;
    }
    T *p = (T *)(base + used);
    used += bytes;
    return p;
  }
};

struct LayerActs {  // what the backward visit keeps of one block's forward
  float *x1, *mean1, *rstd1, *mean2, *rstd2;
  void *a, *qkv, *P, *o, *c, *u, *g;
  float *lse;  // fused attention: log-sum-exp per score row instead of the probabilities P
};

// fused attention kernels serve the bf16 path at head widths 64 and 128; everything else runs the products and
// the softmax as separate kernels with the T x T matrices in the workspace
inline bool fused_attn(const ModelShape &s, int dt) { return attention_fused_supported(dt, s.dh); }

hipError_t launch_colsum_finish_one(const float *part, int64_t stride, int nch, int N, float *out, int acc,
                                    hipStream_t st) {
  ColsumFinish f;
  f.acc = acc;
  f.add(part, stride, nch, N, out);
  return launch_colsum_finish(f, st);
}

struct BlockW {  // pointers into a shard buffer for one block
  const float *ln1_g, *ln1_b, *b_qkv, *b_o, *ln2_g, *ln2_b, *b_fc, *b_proj;
  const void *w_qkv, *w_o, *w_fc, *w_proj;  // operand dtype (bf16 working copy, or the fp32 master itself), [in, out]
  const void *t_qkv, *t_o, *t_fc, *t_proj;  // bf16 path: the same matrices transposed, [out, in]; null in the fp32 path
  float *G;                                  // gradient base of the block
};

uint64_t layer_act_bytes(const ModelShape &s, int dt) {
  const uint64_t e = dt_size(dt), M = s.M, d = s.d, F = s.F;
  const uint64_t P = fused_attn(s, dt) ? (uint64_t)s.B * s.H * s.T * 4 : (uint64_t)s.B * s.H * s.T * s.T * e;
  return up256(M * d * 4) + 4 * up256(M * 4) + 3 * up256(M * d * e) + up256(M * 3 * d * e) + up256(P) +
         2 * up256(M * F * e);
}

LayerActs take_layer(Bump &b, const ModelShape &s, int dt) {
  const uint64_t e = dt_size(dt), M = s.M, d = s.d, F = s.F;
  LayerActs A;
  A.x1 = b.take<float>(M * d);
  A.mean1 = b.take<float>(M); A.rstd1 = b.take<float>(M);
  A.mean2 = b.take<float>(M); A.rstd2 = b.take<float>(M);
  A.a = b.take<char>(M * d * e);
  A.qkv = b.take<char>(M * 3 * d * e);
  if (fused_attn(s, dt)) {
    A.P = nullptr;
    A.lse = b.take<float>((uint64_t)s.B * s.H * s.T);
  } else {
    A.P = b.take<char>((uint64_t)s.B * s.H * s.T * s.T * e);
    A.lse = nullptr;
  }
  A.o = b.take<char>(M * d * e);
  A.c = b.take<char>(M * d * e);
  A.u = b.take<char>(M * F * e);
  A.g = b.take<char>(M * F * e);
  return A;
}

BlockW block_ptrs(const ModelShape &s, const Slot *sl, int dt, int j) {
  const BlockOffsets &o = s.bo;
  const int64_t base = (int64_t)j * o.size;
  const float *w = sl->w + base;
  BlockW B;
  B.ln1_g = w + o.ln1_g; B.ln1_b = w + o.ln1_b; B.b_qkv = w + o.b_qkv; B.b_o = w + o.b_o;
  B.ln2_g = w + o.ln2_g; B.ln2_b = w + o.ln2_b; B.b_fc = w + o.b_fc; B.b_proj = w + o.b_proj;
  if (dt == DT_BF16) {
    const bf16_t *h = sl->wb + base, *t = sl->wbt + base;
    B.w_qkv = h + o.w_qkv; B.w_o = h + o.w_o; B.w_fc = h + o.w_fc; B.w_proj = h + o.w_proj;
    B.t_qkv = t + o.w_qkv; B.t_o = t + o.w_o; B.t_fc = t + o.w_fc; B.t_proj = t + o.w_proj;
  } else {
    B.w_qkv = w + o.w_qkv; B.w_o = w + o.w_o; B.w_fc = w + o.w_fc; B.w_proj = w + o.w_proj;
    B.t_qkv = B.t_o = B.t_fc = B.t_proj = nullptr;
  }
  B.G = sl->g + base;
  return B;
}

inline const void *off_act(const void *p, int64_t elems, int dt) { return (const char *)p + elems * (int64_t)dt_size(dt); }
inline void *off_act(void *p, int64_t elems, int dt) { return (char *)p + elems * (int64_t)dt_size(dt); }

// y = x*W + b : X [M,K] operand dtype, W [K,N]; Wt (may be null) is the same matrix stored [N,K]: both operands then
// have the contraction index contiguous, which is the layout the direct-to-LDS kernel with its large tiles serves
hipError_t linear(int dt, int M, int N, int K, const void *X, const void *W, const void *Wt, const float *bias,
                  const float *resid, float *out_f32, void *out_act, int epi, void *out_act2, hipStream_t st) {
  GemmDesc g;
  g.dtype = dt; g.ta = 0; g.M = M; g.N = N; g.K = K;
  g.A = X; g.lda = K; g.ldc = N;
  if (Wt) { g.tb = 0; g.B = Wt; g.ldb = K; }
  else { g.tb = 1; g.B = W; g.ldb = N; }
  g.bias = bias; g.resid = resid; g.out_f32 = out_f32; g.out_act = out_act; g.epi = epi; g.out_act2 = out_act2;
  return launch_gemm(g, st);
}
// dx = dy*W^T : dY [M,N], W [K,N] -> [M,K]
hipError_t linear_dx(int dt, int M, int N, int K, const void *dY, const void *W, float *out_f32, void *out_act, int epi,
                     const void *aux, hipStream_t st) {
  GemmDesc g;
  g.dtype = dt; g.ta = 0; g.tb = 0; g.M = M; g.N = K; g.K = N;
  g.A = dY; g.lda = N; g.B = W; g.ldb = N; g.ldc = K;
  g.out_f32 = out_f32; g.out_act = out_act; g.epi = epi; g.aux = aux;
  return launch_gemm(g, st);
}
// dW (+)= x^T*dy : X [M,K] (ldx), dY [M,N] (ldy) -> fp32 [K,N]; acc adds to what dW holds
GemmDesc dw_desc(int dt, int M, int N, int K, const void *X, int64_t ldx, const void *dY, int64_t ldy, float *dW,
                 int acc) {
  GemmDesc g;
  g.dtype = dt; g.ta = 1; g.tb = 1; g.M = K; g.N = N; g.K = M;
  g.A = X; g.lda = ldx; g.B = dY; g.ldb = ldy; g.ldc = N;
  g.out_f32 = dW;
  if (acc) g.resid = dW;  // every element is read and then written by the same thread
  return g;
}
hipError_t linear_dw(int dt, int M, int N, int K, const void *X, int64_t ldx, const void *dY, int64_t ldy, float *dW,
                     int acc, hipStream_t st) {
  return launch_gemm(dw_desc(dt, M, N, K, X, ldx, dY, ldy, dW, acc), st);
}

#define CK(call)                                \
  do {                                          \
    hipError_t e__ = (call);                    \
    if (e__ != hipSuccess) return e__;          \
  } while (0)

// batched attention GEMM over (sample, head)
GemmDesc attn_desc(const ModelShape &s, int dt) {
  GemmDesc g;
  g.dtype = dt;
  g.nb1 = s.B; g.nb2 = s.H;
  return g;
}

// attention of one block as separate kernels (fp32 path, and head widths the fused kernels do not serve): scores
// into Sbuf (fp32, [B,H,T,T], lower triangle), softmax into A.P, P V into A.o
hipError_t attention_unfused_fwd(const ModelShape &s, int dt, const LayerActs &A, float *Sbuf, hipStream_t st) {
  const int d = s.d, T = s.T, dh = s.dh;
  const int64_t TT = (int64_t)T * T;
  {  // scores = q k^T / sqrt(dh), lower triangle
    GemmDesc g = attn_desc(s, dt);
    g.ta = 0; g.tb = 0; g.M = T; g.N = T; g.K = dh; g.alpha = 1.0f / sqrtf((float)dh);
    g.A = A.qkv; g.lda = 3 * d; g.sA1 = (int64_t)T * 3 * d; g.sA2 = dh;
    g.B = off_act(A.qkv, d, dt); g.ldb = 3 * d; g.sB1 = (int64_t)T * 3 * d; g.sB2 = dh;
    g.out_f32 = Sbuf; g.ldc = T; g.sC1 = s.H * TT; g.sC2 = TT;
    g.causal = CAUSAL_SKIP_UPPER;
    CK(launch_gemm(g, st));
  }
  CK(launch_softmax_causal_fwd(dt, Sbuf, A.P, s.B * s.H, T, st));
  {  // o = p v, heads merged
    GemmDesc g = attn_desc(s, dt);
    g.ta = 0; g.tb = 1; g.M = T; g.N = dh; g.K = T;
    g.A = A.P; g.lda = T; g.sA1 = s.H * TT; g.sA2 = TT;
    g.B = off_act(A.qkv, 2 * d, dt); g.ldb = 3 * d; g.sB1 = (int64_t)T * 3 * d; g.sB2 = dh;
    g.out_act = A.o; g.ldc = d; g.sC1 = (int64_t)T * d; g.sC2 = dh;
    g.causal = CAUSAL_K_END;
    CK(launch_gemm(g, st));
  }
  return hipSuccess;
}

hipError_t block_forward(const ModelShape &s, int dt, const BlockW &W, const float *x_in, float *x_out,
                         const LayerActs &A, float *Sbuf, hipStream_t st) {
  const int M = (int)s.M, d = s.d, F = s.F, T = s.T, dh = s.dh;
  CK(launch_layernorm_fwd(dt, x_in, W.ln1_g, W.ln1_b, A.a, A.mean1, A.rstd1, M, d, st));
  CK(linear(dt, M, 3 * d, d, A.a, W.w_qkv, W.t_qkv, W.b_qkv, nullptr, nullptr, A.qkv, EPI_NONE, nullptr, st));
  if (fused_attn(s, dt)) CK(launch_attention_fwd(A.qkv, A.o, A.lse, s.B, s.H, T, dh, st));
  else CK(attention_unfused_fwd(s, dt, A, Sbuf, st));
  CK(linear(dt, M, d, d, A.o, W.w_o, W.t_o, W.b_o, x_in, A.x1, nullptr, EPI_NONE, nullptr, st));
  CK(launch_layernorm_fwd(dt, A.x1, W.ln2_g, W.ln2_b, A.c, A.mean2, A.rstd2, M, d, st));
  CK(linear(dt, M, F, d, A.c, W.w_fc, W.t_fc, W.b_fc, nullptr, nullptr, A.u, EPI_GELU, A.g, st));
  CK(linear(dt, M, d, F, A.g, W.w_proj, W.t_proj, W.b_proj, A.x1, x_out, nullptr, EPI_NONE, nullptr, st));
  return hipSuccess;
}

struct BwdScratch {  // shared by the layers of a visit
  float *dP;    // [B,H,T,T] fp32 (also the score buffer of the recomputation)
  void *dS;     // [B,H,T,T] operand dtype
  void *d_o;    // [M,d]
  float *red;   // column-reduction partials
  float *dsum;  // fused attention: row sums of dO * O
};

// Activation gradients of one block, each written once per micro-batch, and the partial column sums behind the
// block's bias and LayerNorm gradients.  A set per block: the weight-gradient work of a block may then be placed
// anywhere after its operands exist (the sums of a block are finished by one launch at its end).
struct LayerGrads {
  float *gin;    // [M,d] fp32: gradient arriving from the block above (blocks below the shard's last one)
  void *dact2;   // [M,d] operand-dtype copy of the gradient at the block's output
  void *dact1;   // [M,d] operand-dtype copy of dx1
  void *du;      // [M,F]
  void *dqkv;    // [M,3d]
  float *dc;     // [M,d] fp32
  float *da;     // [M,d] fp32
  float *dx1;    // [M,d] fp32: gradient of the residual stream between attention and MLP
  float *part1;  // [blocks][3][d]: partial sums of the first LayerNorm's backward (dgamma, dbeta, sum of dx)
  float *part2;  // the same for the second LayerNorm
  float *pdu;    // [chunks][F] partial column sums of du
  float *pdqkv;  // [chunks][3d] partial column sums of dqkv
};

// fp32 -> operand dtype view of an [M,d] gradient (no copy in the fp32 path)
hipError_t act_view(int dt, const float *src, void *scratch, int M, int d, const void **out, hipStream_t st) {
  if (dt == DT_F32) {
    *out = src;
    return hipSuccess;
  }
  *out = scratch;
  return launch_cast_act(dt, src, d, scratch, d, M, d, st);
}

// backward of attention_unfused_fwd: d_o (Z.d_o) -> dq | dk | dv (dqkv) through dP, the softmax backward and
// three more batched products
hipError_t attention_unfused_bwd(const ModelShape &s, int dt, const LayerActs &A, const BwdScratch &Z, void *dqkv,
                                 hipStream_t st) {
  const int d = s.d, T = s.T, dh = s.dh;
  const int64_t TT = (int64_t)T * T;
  const float scale = 1.0f / sqrtf((float)dh);
  const void *q = A.qkv, *k = off_act((const void *)A.qkv, d, dt), *v = off_act((const void *)A.qkv, 2 * d, dt);
  const int64_t sQ1 = (int64_t)T * 3 * d;
  {  // dP = dO V^T
    GemmDesc g = attn_desc(s, dt);
    g.ta = 0; g.tb = 0; g.M = T; g.N = T; g.K = dh;
    g.A = Z.d_o; g.lda = d; g.sA1 = (int64_t)T * d; g.sA2 = dh;
    g.B = v; g.ldb = 3 * d; g.sB1 = sQ1; g.sB2 = dh;
    g.out_f32 = Z.dP; g.ldc = T; g.sC1 = s.H * TT; g.sC2 = TT;
    g.causal = CAUSAL_SKIP_UPPER;
    CK(launch_gemm(g, st));
  }
  {  // dV = P^T dO
    GemmDesc g = attn_desc(s, dt);
    g.ta = 1; g.tb = 1; g.M = T; g.N = dh; g.K = T;
    g.A = A.P; g.lda = T; g.sA1 = s.H * TT; g.sA2 = TT;
    g.B = Z.d_o; g.ldb = d; g.sB1 = (int64_t)T * d; g.sB2 = dh;
    g.out_act = off_act(dqkv, 2 * d, dt); g.ldc = 3 * d; g.sC1 = sQ1; g.sC2 = dh;
    g.causal = CAUSAL_K_BEGIN;
    CK(launch_gemm(g, st));
  }
  CK(launch_softmax_causal_bwd(dt, A.P, Z.dP, Z.dS, s.B * s.H, T, st));
  {  // dQ = dS K / sqrt(dh)
    GemmDesc g = attn_desc(s, dt);
    g.ta = 0; g.tb = 1; g.M = T; g.N = dh; g.K = T; g.alpha = scale;
    g.A = Z.dS; g.lda = T; g.sA1 = s.H * TT; g.sA2 = TT;
    g.B = k; g.ldb = 3 * d; g.sB1 = sQ1; g.sB2 = dh;
    g.out_act = dqkv; g.ldc = 3 * d; g.sC1 = sQ1; g.sC2 = dh;
    g.causal = CAUSAL_K_END;
    CK(launch_gemm(g, st));
  }
  {  // dK = dS^T Q / sqrt(dh)
    GemmDesc g = attn_desc(s, dt);
    g.ta = 1; g.tb = 1; g.M = T; g.N = dh; g.K = T; g.alpha = scale;
    g.A = Z.dS; g.lda = T; g.sA1 = s.H * TT; g.sA2 = TT;
    g.B = q; g.ldb = 3 * d; g.sB1 = sQ1; g.sB2 = dh;
    g.out_act = off_act(dqkv, d, dt); g.ldc = 3 * d; g.sC1 = sQ1; g.sC2 = dh;
    g.causal = CAUSAL_K_BEGIN;
    CK(launch_gemm(g, st));
  }
  return hipSuccess;
}

// dx2 / dx2a: gradient at the block's output in fp32 and in the operand dtype (the same pointer in the fp32 path).
// dx2_part: partial sums [blocks][3][d] of the LayerNorm backward that produced dx2 (its third part sums dx2 over
// the rows = the gradient of b_proj), or null when dx2 came from elsewhere.
// dx_out / dx_out_act: gradient at the block's input; the operand-dtype copy is written only when dx_out_act is set.
// The gradients of the biases and of the LayerNorm parameters are column sums over the tokens; where the row fits
// the fused LayerNorm backward, its partial sums and those of one two-operand pass over du and dqkv are finished
// by a single launch at the end of the block (2 launches instead of 12).
hipError_t block_backward(const ModelShape &s, int dt, const BlockW &W, const float *x_in, const LayerActs &A,
                          const float *dx2, const void *dx2a, const float *dx2_part, float *dx_out, void *dx_out_act,
                          const BwdScratch &Z, const LayerGrads &L, int acc, hipStream_t st) {
  const int M = (int)s.M, d = s.d, F = s.F, T = s.T, dh = s.dh;
  const BlockOffsets &o = s.bo;
  const bool bf = dt == DT_BF16;
  const bool fl = layernorm_bwd_fused_supported(d);
  const int nb = layernorm_bwd_fused_blocks(M), nch = colsum_chunks(M);
  ColsumFinish fin;
  fin.acc = acc;
  // MLP down projection
  if (fl) {
    if (!dx2_part) {  // the gradient came in over the shard boundary: sum it the way the LayerNorm backward would have
      CK(launch_colsum_rows8(dx2, L.part2, M, d, st));  // (part2 is rewritten by this block's second LayerNorm later)
      CK(launch_colsum_finish_one(L.part2 + 2 * d, 3 * (int64_t)d, nb, d, W.G + o.b_proj, acc, st));
    } else {
      fin.add(dx2_part + 2 * d, 3 * (int64_t)d, nb, d, W.G + o.b_proj);
    }
  } else {
    CK(launch_colsum(DT_F32, dx2, d, W.G + o.b_proj, Z.red, M, d, acc, st));
  }
  CK(linear_dx(dt, M, d, F, dx2a, W.w_proj, nullptr, L.du, EPI_DGELU, A.u, st));  // du = (dx2 Wp^T) * gelu'(u)
  // MLP up projection
  CK(linear_dx(dt, M, F, d, L.du, W.w_fc, L.dc, nullptr, EPI_NONE, nullptr, st));
  if (fl) {
    CK(launch_layernorm_bwd_fused(L.dc, A.x1, A.mean2, A.rstd2, W.ln2_g, dx2, L.dx1, bf ? L.dact1 : nullptr, L.part2, M, d, st));
    fin.add(L.part2, 3 * (int64_t)d, nb, d, W.G + o.ln2_g);
    fin.add(L.part2 + d, 3 * (int64_t)d, nb, d, W.G + o.ln2_b);
    fin.add(L.part2 + 2 * d, 3 * (int64_t)d, nb, d, W.G + o.b_o);
  } else {
    CK(launch_layernorm_bwd_params(L.dc, A.x1, A.mean2, A.rstd2, W.G + o.ln2_g, W.G + o.ln2_b, Z.red, M, d, acc, st));
    CK(launch_layernorm_bwd_dx(L.dc, A.x1, A.mean2, A.rstd2, W.ln2_g, dx2, L.dx1, bf ? L.dact1 : nullptr, M, d, st));
    CK(launch_colsum(DT_F32, L.dx1, d, W.G + o.b_o, Z.red, M, d, acc, st));
  }
  // attention output projection
  const void *dx1a = bf ? (const void *)L.dact1 : (const void *)L.dx1;
  CK(linear_dx(dt, M, d, d, dx1a, W.w_o, nullptr, Z.d_o, EPI_NONE, nullptr, st));
  // attention core
  if (fused_attn(s, dt)) CK(launch_attention_bwd(A.qkv, A.o, Z.d_o, A.lse, Z.dsum, L.dqkv, s.B, s.H, T, dh, st));
  else CK(attention_unfused_bwd(s, dt, A, Z, L.dqkv, st));
  // QKV projection
  CK(linear_dx(dt, M, 3 * d, d, L.dqkv, W.w_qkv, L.da, nullptr, EPI_NONE, nullptr, st));
  if (fl) {
    CK(launch_layernorm_bwd_fused(L.da, x_in, A.mean1, A.rstd1, W.ln1_g, L.dx1, dx_out, bf ? dx_out_act : nullptr, L.part1, M, d, st));
    fin.add(L.part1, 3 * (int64_t)d, nb, d, W.G + o.ln1_g);
    fin.add(L.part1 + d, 3 * (int64_t)d, nb, d, W.G + o.ln1_b);
    // bias gradients of the two wide linears: one pass over du and dqkv, then every sum of the block in one launch
    CK(launch_colsum2_pass1(dt, L.du, F, L.pdu, L.dqkv, 3 * d, L.pdqkv, M, st));
    fin.add(L.pdu, F, nch, F, W.G + o.b_fc);
    fin.add(L.pdqkv, 3 * (int64_t)d, nch, 3 * d, W.G + o.b_qkv);
    CK(launch_colsum_finish(fin, st));
  } else {
    CK(launch_layernorm_bwd_params(L.da, x_in, A.mean1, A.rstd1, W.G + o.ln1_g, W.G + o.ln1_b, Z.red, M, d, acc, st));
    CK(launch_layernorm_bwd_dx(L.da, x_in, A.mean1, A.rstd1, W.ln1_g, L.dx1, dx_out, bf ? dx_out_act : nullptr, M, d, st));
    CK(launch_colsum(dt, L.du, F, W.G + o.b_fc, Z.red, M, F, acc, st));
    CK(launch_colsum(dt, L.dqkv, 3 * d, W.G + o.b_qkv, Z.red, M, 3 * d, acc, st));
  }
  // The four weight-gradient products of the block, in one launch where the kernel allows it: each alone leaves
  // most of the chip idle (72-288 tiles, a contraction over all tokens), and nothing waits for them before Adam.
  const GemmDesc dw[4] = {dw_desc(dt, M, d, F, A.g, F, dx2a, d, W.G + o.w_proj, acc),
                          dw_desc(dt, M, F, d, A.c, d, L.du, F, W.G + o.w_fc, acc),
                          dw_desc(dt, M, d, d, A.o, d, dx1a, d, W.G + o.w_o, acc),
                          dw_desc(dt, M, 3 * d, d, A.a, d, L.dqkv, 3 * d, W.G + o.w_qkv, acc)};
  CK(launch_gemm_group(dw, 4, st));
  return hipSuccess;
}

uint64_t red_elems(const ModelShape &s) {
  const uint64_t widest = (uint64_t)(3 * s.d > s.F ? 3 * s.d : s.F);
  return 2 * (uint64_t)colsum_chunks((int)s.M) * widest;
}

uint64_t bwd_scratch_bytes(const ModelShape &s, int dt) {
  const uint64_t e = dt_size(dt), M = s.M, d = s.d;
  const bool fused = fused_attn(s, dt);
  const uint64_t PP = fused ? (uint64_t)s.B * s.H * s.T : (uint64_t)s.B * s.H * s.T * s.T;
  return up256(PP * 4) + up256(PP * e) + up256(M * d * e) + up256(red_elems(s) * 4);
}

BwdScratch take_bwd(Bump &b, const ModelShape &s, int dt) {
  const uint64_t e = dt_size(dt), M = s.M, d = s.d;
  const bool fused = fused_attn(s, dt);
  const uint64_t PP = fused ? (uint64_t)s.B * s.H * s.T : (uint64_t)s.B * s.H * s.T * s.T;
  BwdScratch Z;
  Z.dP = b.take<float>(PP);   // fused: serves as dsum
  Z.dS = b.take<char>(PP * e);
  Z.dsum = Z.dP;
  Z.d_o = b.take<char>(M * d * e);
  Z.red = b.take<float>(red_elems(s));
  return Z;
}

uint64_t layer_grad_bytes(const ModelShape &s, int dt) {
  const uint64_t e = dt_size(dt), M = s.M, d = s.d, F = s.F;
  const uint64_t nb = layernorm_bwd_fused_blocks((int)s.M), nch = colsum_chunks((int)s.M);
  return 4 * up256(M * d * 4) + 2 * up256(M * d * e) + up256(M * F * e) + up256(M * 3 * d * e) +
         2 * up256(nb * 3 * d * 4) + up256(nch * F * 4) + up256(nch * 3 * d * 4);
}

LayerGrads take_layer_grads(Bump &b, const ModelShape &s, int dt) {
  const uint64_t e = dt_size(dt), M = s.M, d = s.d, F = s.F;
  LayerGrads L;
  L.gin = b.take<float>(M * d);
  L.dc = b.take<float>(M * d);
  L.da = b.take<float>(M * d);
  L.dx1 = b.take<float>(M * d);
  L.dact2 = b.take<char>(M * d * e);
  L.dact1 = b.take<char>(M * d * e);
  L.du = b.take<char>(M * F * e);
  L.dqkv = b.take<char>(M * 3 * d * e);
  const uint64_t nb = layernorm_bwd_fused_blocks((int)s.M), nch = colsum_chunks((int)s.M);
  L.part1 = b.take<float>(nb * 3 * d);
  L.part2 = b.take<float>(nb * 3 * d);
  L.pdu = b.take<float>(nch * F);
  L.pdqkv = b.take<float>(nch * 3 * d);
  return L;
}

uint64_t head_bytes(const ModelShape &s, int dt) {
  const uint64_t e = dt_size(dt), M = s.M, d = s.d;
  return up256(M * s.Vpad * 4) + up256(M * d * e) + 2 * up256(M * 4) + up256(M * d * 4) + up256(red_elems(s) * 4);
}

// Runs the kernel sequence of a block-shard visit.  With HYDRA_FLAG_GRAPHS the second visit of a (model, shard,
// phase, shard buffer) combination is captured from the stream as a HIP graph and every later one replays it: the
// sequence is dozens of launches whose arguments depend on nothing else, and issuing them one by one costs the host
// more time than the device needs to run them.  phase: 0 forward, 1 / 2 backward by boundary-gradient parity.
template <typename F>
hydra_status run_visit(hydra_ctx *ctx, Model *mm, Slot *sl, int shard, int phase, hipStream_t st, F &&enqueue) {
  const bool use = (ctx->init.flags & HYDRA_FLAG_GRAPHS) && !(ctx->init.flags & HYDRA_FLAG_TIMING);
  if (!use) {
    HYDRA_HIP(ctx, enqueue());
    return HYDRA_OK;
  }
  const uint64_t model_i = (uint64_t)(std::find(ctx->models.begin(), ctx->models.end(), mm) - ctx->models.begin());
  const uint64_t slot_i = (uint64_t)(sl - ctx->slots.data());
  const uint64_t key = (model_i << 40) | ((uint64_t)shard << 24) | ((uint64_t)phase << 16) | slot_i;
  hydra_ctx::GraphEntry &e = ctx->graphs[key];
  if (e.exec) {
    HYDRA_HIP(ctx, hipGraphLaunch(e.exec, st));
    ctx->graph_launches++;
    return HYDRA_OK;
  }
  if (e.failed || e.seen == 0) {  // first visit: plain launches (one-time set-up of the kernels happens here)
    e.seen++;
    HYDRA_HIP(ctx, enqueue());
    return HYDRA_OK;
  }
  hipGraph_t graph = nullptr;
  // no other thread of the library calls into the HIP runtime while the visit is being captured (hydra_ctx::hip_gate)
  std::unique_lock<std::mutex> gate(ctx->hip_gate, std::defer_lock);
  if (ctx->gate_on) gate.lock();
  hipError_t err = hipStreamBeginCapture(st, hipStreamCaptureModeRelaxed);
  if (err == hipSuccess) {
    const hipError_t launch_err = enqueue();
    err = hipStreamEndCapture(st, &graph);
    if (err == hipSuccess) err = launch_err;
  }
  if (err == hipSuccess) err = hipGraphInstantiate(&e.exec, graph, nullptr, nullptr, 0);
  if (gate.owns_lock()) gate.unlock();
  if (graph) (void)hipGraphDestroy(graph);
  if (err != hipSuccess) {  // capture is an optimisation: fall back to plain launches for this combination
    (void)hipGetLastError();
    e.exec = nullptr;
    e.failed = true;
    HYDRA_HIP(ctx, enqueue());
    return HYDRA_OK;
  }
  HYDRA_HIP(ctx, hipGraphLaunch(e.exec, st));
  ctx->graph_launches++;
  return HYDRA_OK;
}

}  // namespace

uint64_t workspace_need(const ModelShape &s, int dtype) {
  const uint64_t act = up256((uint64_t)s.M * s.d * 4);
  // backward visit: k kept layers + k inter-layer activations + k sets of activation gradients + shared scratch
  const uint64_t bwd = (uint64_t)s.k * (layer_act_bytes(s, dtype) + act + layer_grad_bytes(s, dtype)) +
                       bwd_scratch_bytes(s, dtype);
  const uint64_t head = head_bytes(s, dtype);
  return (bwd > head ? bwd : head) + 4096;
}

// Make the bf16 working copies of a shard current.  Block shards keep two: the shard as stored (wb: operand of the
// dx products, dy W^T) and every matrix transposed (wbt: operand of the forward products, so that they too have both
// operands contraction-contiguous).  A forward visit needs only wbt, taken straight from the fp32 master; a backward
// visit needs both (wbt for the recomputation) and transposes the bf16 copy, which Adam keeps current while the
// shard stays resident.
static hipError_t ensure_working_copy(hydra_ctx *ctx, Model *mm, Slot *sl, int shard, bool backward) {
  if (mm->dtype != DT_BF16) return hipSuccess;
  const ModelShape &s = mm->sh;
  hipStream_t st = ctx->lanes[mm->lane].stream;
  if (shard >= 1 && shard <= s.S) {
    if (backward && !sl->wb_valid) {
      CK(launch_cast_bf16(sl->w, sl->wb, s.shard_off[shard + 1] - s.shard_off[shard], st));
      sl->wb_valid = true;
    }
    if (!sl->wbt_valid) {
      const BlockOffsets &o = s.bo;
      const bool from_bf16 = sl->wb_valid;
      TransposeGroup g;
      for (int j = 0; j < s.k; ++j) {
        const int64_t base = (int64_t)j * o.size;
        const bool ok = g.add(base + o.w_qkv, s.d, 3 * s.d) && g.add(base + o.w_o, s.d, s.d) &&
                        g.add(base + o.w_fc, s.d, s.F) && g.add(base + o.w_proj, s.F, s.d);
        if (!ok || g.n + 4 > TRANSPOSE_MAX || j == s.k - 1) {
          if (!ok) return hipErrorInvalidValue;
          CK(launch_transpose_group(from_bf16 ? DT_BF16 : DT_F32, from_bf16 ? (const void *)sl->wb : (const void *)sl->w,
                                    sl->wbt, g, st));
          g = TransposeGroup();
        }
      }
      sl->wbt_valid = true;
    }
  } else if (shard == s.S + 1 && !sl->wb_valid) {
    // LM head kept transposed [V,d] so that the odd vocabulary size never is a leading dimension; a tied head's
    // copy of wte already is [V,d]
    if (s.tie) CK(launch_cast_bf16(sl->w + 2 * s.d, sl->wb + 2 * s.d, (int64_t)s.V * s.d, st));
    else CK(launch_cast_transpose_bf16(sl->w + 2 * s.d, sl->wb + 2 * s.d, s.d, s.V, st));
    sl->wb_valid = true;
  }
  return hipSuccess;
}

hydra_status exec_forward(hydra_ctx *ctx, Model *mm, Slot *sl, int shard) {
  const ModelShape &s = mm->sh;
  const int dt = mm->dtype;
  hipStream_t st = ctx->lanes[mm->lane].stream;
  const int M = (int)s.M, d = s.d;
  const int64_t act = (int64_t)M * d;  // elements of one micro-batch's boundary activation
  HYDRA_HIP(ctx, ensure_working_copy(ctx, mm, sl, shard, false));
  hydra_ctx::Lane &ln = ctx->lanes[mm->lane];
  Bump b{ln.ws, ctx->ws_bytes};
  if (shard == 0) {
    // one launch over every micro-batch: a row's position is its index modulo T
    HYDRA_HIP(ctx, launch_embed_fwd(mm->tok, sl->w, sl->w + (int64_t)s.V * d, mm->ckpt[0], (int)s.Mt, s.T, d, st));
    return HYDRA_OK;
  }
  if (shard <= s.S) {
    ln.logits_owner = -1;  // the shared workspace is about to be overwritten
    LayerActs A = take_layer(b, s, dt);
    float *Sbuf = fused_attn(s, dt) ? nullptr : b.take<float>((uint64_t)s.B * s.H * s.T * s.T);
    float *pp[2] = {b.take<float>((uint64_t)M * d), b.take<float>((uint64_t)M * d)};
    if (!b.ok) return fail(ctx, HYDRA_E_NOMEM, "workspace too small (forward)");
    // nothing but kernel launches with arguments that depend only on (model, shard, shard buffer): graphable
    auto enqueue = [&]() -> hipError_t {
      for (int u = 0; u < s.nm; ++u) {  // micro-batches share the workspace, one after the other
        const float *x = mm->ckpt[shard - 1] + u * act;
        for (int j = 0; j < s.k; ++j) {
          float *y = (j == s.k - 1) ? mm->ckpt[shard] + u * act : pp[j & 1];
          CK(block_forward(s, dt, block_ptrs(s, sl, dt, j), x, y, A, Sbuf, st));
          x = y;
        }
      }
      return hipSuccess;
    };
    return run_visit(ctx, mm, sl, shard, 0, st, enqueue);
  }
  // HEAD: final LayerNorm, logits, loss and d(loss)/d(logits)
  float *logits = b.take<float>((uint64_t)M * s.Vpad);
  void *z = b.take<char>((uint64_t)M * d * dt_size(dt));
  float *mean = b.take<float>(M), *rstd = b.take<float>(M);
  if (!b.ok) return fail(ctx, HYDRA_E_NOMEM, "workspace too small (head)");
  const float inv_n = 1.0f / (float)mm->n_valid;  // valid targets of the whole minibatch
  for (int u = 0; u < s.nm; ++u) {
    HYDRA_HIP(ctx, launch_layernorm_fwd(dt, mm->ckpt[s.S] + u * act, sl->w, sl->w + d, z, mean, rstd, M, d, st));
    GemmDesc g;
    g.dtype = dt; g.M = M; g.N = s.V; g.K = d; g.A = z; g.lda = d; g.ta = 0;
    if (dt == DT_BF16) { g.tb = 0; g.B = sl->wb + 2 * d; g.ldb = d; }
    else if (s.tie) { g.tb = 0; g.B = sl->w + 2 * d; g.ldb = d; }  // wte [V,d]: logits = z wte^T
    else { g.tb = 1; g.B = sl->w + 2 * d; g.ldb = s.V; }
    g.out_f32 = logits; g.ldc = s.Vpad;
    HYDRA_HIP(ctx, launch_gemm(g, st));
    HYDRA_HIP(ctx, launch_cross_entropy(dt, logits, mm->tgt + (int64_t)u * M, mm->row_loss + (int64_t)u * M,
                                        off_act(mm->dlogits, (int64_t)u * M * s.Vpad, dt), M, s.V, s.Vpad, inv_n, st));
  }
  HYDRA_HIP(ctx, launch_loss_reduce(mm->row_loss, mm->loss, (int)s.Mt, inv_n, st));
  ln.logits = logits;
  ln.logits_owner = (int)(std::find(ctx->models.begin(), ctx->models.end(), mm) - ctx->models.begin());
  for (Model *o : ctx->models)
    if (o != mm) o->logits_valid = false;
  return HYDRA_OK;
}

hydra_status exec_backward(hydra_ctx *ctx, Model *mm, Slot *sl, int shard) {
  const ModelShape &s = mm->sh;
  const int dt = mm->dtype;
  hipStream_t st = ctx->lanes[mm->lane].stream;
  const int M = (int)s.M, d = s.d;
  const int64_t act = (int64_t)M * d;
  HYDRA_HIP(ctx, ensure_working_copy(ctx, mm, sl, shard, true));
  hydra_ctx::Lane &ln = ctx->lanes[mm->lane];
  Bump b{ln.ws, ctx->ws_bytes};
  if (shard == s.S + 1) {
    // the logits of the forward visit were turned into dlogits there; only the
    // normalised input z is recomputed
    if (ln.logits_owner >= 0 && ctx->models[ln.logits_owner] == mm)
      b.take<float>((uint64_t)M * s.Vpad);  // leave this model's logits readable
    else
      ln.logits_owner = -1;
    void *z = b.take<char>((uint64_t)M * d * dt_size(dt));
    float *mean = b.take<float>(M), *rstd = b.take<float>(M);
    float *dz = b.take<float>((uint64_t)M * d);
    float *red = b.take<float>(red_elems(s));
    if (!b.ok) return fail(ctx, HYDRA_E_NOMEM, "workspace too small (head backward)");
    mm->dcur = 0;
    for (int u = 0; u < s.nm; ++u) {  // gradients of the shard's tensors add up over micro-batches
      const float *x = mm->ckpt[s.S] + u * act;
      const void *dl = off_act((const void *)mm->dlogits, (int64_t)u * M * s.Vpad, dt);
      HYDRA_HIP(ctx, launch_layernorm_fwd(dt, x, sl->w, sl->w + d, z, mean, rstd, M, d, st));
      if (s.tie) {  // the head's part of the wte gradient, [V,d] = dlogits^T z, kept for the EMBED backward visit
        GemmDesc w;
        w.dtype = dt; w.ta = 1; w.tb = 1; w.M = s.V; w.N = d; w.K = M;
        w.A = dl; w.lda = s.Vpad; w.B = z; w.ldb = d; w.ldc = d;
        w.out_f32 = mm->tied_g;
        if (u > 0) w.resid = mm->tied_g;
        HYDRA_HIP(ctx, launch_gemm(w, st));
      } else {
        HYDRA_HIP(ctx, linear_dw(dt, M, s.V, d, z, d, dl, s.Vpad, sl->g + 2 * d, u > 0, st));
      }
      GemmDesc g;
      g.dtype = dt; g.M = M; g.N = d; g.K = s.V; g.A = dl; g.lda = s.Vpad; g.ta = 0;
      if (dt == DT_BF16) { g.tb = 1; g.B = sl->wb + 2 * d; g.ldb = d; }
      else if (s.tie) { g.tb = 1; g.B = sl->w + 2 * d; g.ldb = d; }
      else { g.tb = 0; g.B = sl->w + 2 * d; g.ldb = s.V; }
      g.out_f32 = dz; g.ldc = d;
      HYDRA_HIP(ctx, launch_gemm(g, st));
      HYDRA_HIP(ctx, launch_layernorm_bwd_params(dz, x, mean, rstd, sl->g, sl->g + d, red, M, d, u > 0, st));
      HYDRA_HIP(ctx, launch_layernorm_bwd_dx(dz, x, mean, rstd, sl->w, nullptr, mm->dbound[0] + u * act, nullptr, M, d, st));
    }
    return HYDRA_OK;
  }
  if (shard >= 1) {
    ln.logits_owner = -1;  // the shared workspace is about to be overwritten
    std::vector<LayerActs> acts(s.k);
    std::vector<float *> xs(s.k + 1);
    for (int j = 0; j < s.k; ++j) acts[j] = take_layer(b, s, dt);
    for (int j = 1; j <= s.k; ++j) xs[j] = b.take<float>((uint64_t)M * d);
    BwdScratch Z = take_bwd(b, s, dt);
    std::vector<LayerGrads> grads(s.k);
    for (int j = 0; j < s.k; ++j) grads[j] = take_layer_grads(b, s, dt);
    if (!b.ok) return fail(ctx, HYDRA_E_NOMEM, "workspace too small (backward)");
    const int dcur = mm->dcur;
    auto enqueue = [&]() -> hipError_t {
      for (int u = 0; u < s.nm; ++u) {  // recompute and back-propagate one micro-batch at a time
        xs[0] = mm->ckpt[shard - 1] + u * act;
        for (int j = 0; j < s.k; ++j)
          CK(block_forward(s, dt, block_ptrs(s, sl, dt, j), xs[j], xs[j + 1], acts[j], Z.dP, st));
        const float *dx = mm->dbound[dcur] + u * act;
        const void *dxa;  // its operand-dtype copy: cast here for the shard's last block, written by the
        CK(act_view(dt, dx, grads[s.k - 1].dact2, M, d, &dxa, st));  // LayerNorm backward of the block above otherwise
        const float *dx_part = nullptr;
        for (int j = s.k - 1; j >= 0; --j) {
          float *out = (j == 0) ? mm->dbound[dcur ^ 1] + u * act : grads[j - 1].gin;
          void *out_act = (j == 0) ? nullptr : grads[j - 1].dact2;
          CK(block_backward(s, dt, block_ptrs(s, sl, dt, j), xs[j], acts[j], dx, dxa, dx_part, out, out_act, Z, grads[j],
                            u > 0, st));
          dx = out;
          dxa = dt == DT_BF16 ? (const void *)out_act : (const void *)out;
          dx_part = grads[j].part1;
        }
      }
      return hipSuccess;
    };
    const hydra_status rs = run_visit(ctx, mm, sl, shard, 1 + dcur, st, enqueue);
    if (rs == HYDRA_OK) mm->dcur ^= 1;
    return rs;
  }
  // EMBED
  if (s.tie)  // start from the LM head's part of the wte gradient
    HYDRA_HIP(ctx, hipMemcpyAsync(sl->g, mm->tied_g, (size_t)s.V * d * 4, hipMemcpyDeviceToDevice, st));
  for (int u = 0; u < s.nm; ++u)
    HYDRA_HIP(ctx, launch_embed_bwd(mm->tok + (int64_t)u * M, mm->dbound[mm->dcur] + u * act, sl->g,
                                    sl->g + (int64_t)s.V * d, s.B, s.T, d, s.V, u > 0 || s.tie, u > 0, st));
  return HYDRA_OK;
}

hydra_status exec_adam(hydra_ctx *ctx, Model *mm, Slot *sl, int shard) {
  const ModelShape &s = mm->sh;
  const hydra_model_desc &h = mm->desc;
  const int64_t n = s.shard_off[shard + 1] - s.shard_off[shard];
  // block shards keep their bf16 working copy current for the next visit
  bf16_t *shadow = (mm->dtype == DT_BF16 && shard >= 1 && shard <= s.S) ? sl->wb : nullptr;
  HYDRA_HIP(ctx, launch_adam(sl->w, sl->m, sl->v, sl->g, shadow, n, h.lr, h.beta1, h.beta2, h.eps, mm->t,
                             ctx->lanes[mm->lane].stream));
  sl->wb_valid = shadow != nullptr;
  sl->wbt_valid = false;  // re-made from the bf16 copy at the shard's next visit
  return HYDRA_OK;
}

}  // namespace hydra
