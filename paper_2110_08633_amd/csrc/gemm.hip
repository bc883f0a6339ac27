// GEMM kernels for gfx950: bf16 MFMA (LDS-tiled, fp32 accumulate) and a plain
// fp32 kernel, both with the same fused epilogues (bias, residual, GELU,
// GELU', scale) and the same causal short-cuts for attention operands.
//
// The linear layers of a block (y = x*W + b), their input gradients
// (dx = dy*W^T) and weight gradients (dW = x^T*dy) and the batched attention
// products are all instances of C = alpha * op(A) * op(B) with a row-major C.
#include <cstdlib>
#include <type_traits>

#include "kernels.h"
#include "tile_ops.h"

namespace hydra {

struct GemmArgs {
  const void *A, *B;
  int M, N, K;
  int64_t lda, ldb, ldc;
  int nb2;
  int64_t sA1, sA2, sB1, sB2, sC1, sC2;
  const float *bias, *resid;
  float *out_f32;
  void *out_act, *out_act2;
  const void *aux;
  int epi, causal;
  int tiles_m, tiles_n;
  float alpha;  // kept among the 32-bit fields: next to a pointer the compiler fused both into one 16-byte load and
  int grp;      // parked it in scratch memory, and a kernel that uses scratch pays microseconds per launch
                // grp: tile rows per group of the tile numbering (see xcd_group_rows)
};

// Tiles are numbered so that the run of tiles an XCD works on (consecutive workgroup ids go round-robin to the 8
// XCDs, each with its own L2) is a block of grp tile rows by a few tile columns: every XCD then fetches grp row
// panels of A and those few column panels of B once.  grp minimises the operand rows + columns such a block
// spans; a fixed 8 made the XCDs of an N = 768 product fetch 60 MB for 17 MB of operands, 4 rows give 44 MB.
// What shares an L2 in time is the set of tiles in flight on the XCD (32 CUs x blocks per CU), not its whole run:
// a launch of several rounds is sized for that set, walked column by column so that the row panels stay (the
// 4096 x 16384 x 1024 weight gradient: 16 rows per group 588, 8 rows 605 TFLOP/s; 16384 x 4096: 527 -> 604).
static int xcd_group_rows(int tiles_m, int tiles_n, int bm, int bn, int inflight_per_xcd = 64) {
  long per = ((long)tiles_m * tiles_n + 7) / 8;  // tiles per XCD
  if (per > inflight_per_xcd) per = inflight_per_xcd;
  int best = 1;
  long best_cost = -1;
  for (int g = 1; g <= 16 && g <= tiles_m; ++g) {
    const long cols = (per + g - 1) / g;
    const long cost = (long)g * bm + (cols < tiles_n ? cols : tiles_n) * bn;
    if (best_cost < 0 || cost <= best_cost) { best = g; best_cost = cost; }
  }
  return best;
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
// BM x BN tile of C.  K is consumed in slices of BK = 64:
//   global -> registers : 16-byte loads, issued three slices ahead
//   registers -> LDS    : one slice ahead, two LDS buffers, one barrier per slice
//   LDS -> MFMA operands: ds_read_b128 for operands whose contraction index is
//                         contiguous in memory, ds_read_tr16_b64 (transposing
//                         read) for operands stored with it strided, so both
//                         kinds sit in LDS exactly as they sit in memory
// LDS tiles carry no padding; their 16-byte chunks are XOR-swizzled so that the
// operand reads of 16 neighbouring lanes fall into distinct banks.
// The MFMA is issued with the B fragment as first operand, which leaves every
// lane with runs of 4 consecutive columns of one row of C: the epilogue then
// stores 16-byte (fp32) or 8-byte (bf16) vectors.
// ---------------------------------------------------------------------------
// 4 consecutive columns of one row of C
template <typename ActT>
__device__ __forceinline__ void epilogue_store4(const GemmArgs &g, int64_t coff, int row, int col, const f32x4_t acc,
                                                bool vec) {
  if (!vec || col + 3 >= g.N) {
#pragma unroll 1
    for (int e = 0; e < 4; ++e) {
      // chosen by comparison, not by address: an indexed local array would live in scratch memory, and a kernel
      // that uses scratch pays several microseconds per launch for its set-up
      const float x = e == 0 ? acc[0] : e == 1 ? acc[1] : e == 2 ? acc[2] : acc[3];
      if (col + e < g.N) epilogue_store<ActT>(g, coff, row, col + e, x);
    }
    return;
  }
  float v[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) v[e] = acc[e] * g.alpha;
  if (g.bias) {
    const f32x4_t b = *(const f32x4_t *)(g.bias + col);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] += b[e];
  }
  const int64_t idx = coff + (int64_t)row * g.ldc + col;
  if (g.epi == EPI_GELU) {
    u32x2_t u, h;
    u.x = (uint32_t)f2bf(v[0]) | ((uint32_t)f2bf(v[1]) << 16);
    u.y = (uint32_t)f2bf(v[2]) | ((uint32_t)f2bf(v[3]) << 16);
    h.x = (uint32_t)f2bf(gelu_f(v[0])) | ((uint32_t)f2bf(gelu_f(v[1])) << 16);
    h.y = (uint32_t)f2bf(gelu_f(v[2])) | ((uint32_t)f2bf(gelu_f(v[3])) << 16);
    *(u32x2_t *)((bf16_t *)g.out_act + idx) = u;
    *(u32x2_t *)((bf16_t *)g.out_act2 + idx) = h;
    return;
  }
  if (g.epi == EPI_DGELU) {
    const u32x2_t a = *(const u32x2_t *)((const bf16_t *)g.aux + idx);
    v[0] *= dgelu_f(__uint_as_float(a.x << 16));
    v[1] *= dgelu_f(__uint_as_float(a.x & 0xffff0000u));
    v[2] *= dgelu_f(__uint_as_float(a.y << 16));
    v[3] *= dgelu_f(__uint_as_float(a.y & 0xffff0000u));
  }
  if (g.resid) {
    const f32x4_t r = *(const f32x4_t *)(g.resid + idx);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] += r[e];
  }
  if (g.out_f32) {
    f32x4_t o = {v[0], v[1], v[2], v[3]};
    *(f32x4_t *)(g.out_f32 + idx) = o;
  }
  if (g.out_act) {
    u32x2_t o;
    o.x = (uint32_t)f2bf(v[0]) | ((uint32_t)f2bf(v[1]) << 16);
    o.y = (uint32_t)f2bf(v[2]) | ((uint32_t)f2bf(v[3]) << 16);
    *(u32x2_t *)((bf16_t *)g.out_act + idx) = o;
  }
}

// tanh(x) = 1 - 2 / (exp(2x) + 1): exact limits at both infinities; the absolute error of about 1e-7 near zero
// is far below what a bf16 result keeps
__device__ __forceinline__ float tanh_fast(float x) {
  return 1.f - 2.f * __builtin_amdgcn_rcpf(__expf(2.f * x) + 1.f);
}
__device__ __forceinline__ float gelu_fast(float u) {
  const float c = 0.7978845608028654f;
  return 0.5f * u * (1.f + tanh_fast(c * (u + 0.044715f * u * u * u)));
}
__device__ __forceinline__ float dgelu_fast(float u) {
  const float c = 0.7978845608028654f;
  const float t = tanh_fast(c * (u + 0.044715f * u * u * u));
  const float dt = (1.f - t * t) * c * (1.f + 3.f * 0.044715f * u * u);
  return 0.5f * (1.f + t) + 0.5f * u * dt;
}

// Row-wise write-out of a wavefront's staged [32][WTN] fp32 patch (LDS, pitch WTN + 4) to rows row0.. and columns
// col0.. of C.  LPR lanes cover a row with 4 columns each, so one instruction stores whole row segments.  With one
// wavefront per SIMD nothing hides latency here, so the work is batched: the epilogue kind is a template
// parameter, addresses advance by addition, and the rows are handled four instructions' worth at a time - all LDS
// reads and all global loads (residual, GELU pre-activation) of a batch are issued before the first is used, and
// all its stores follow together (a load issued after a store has to wait until that store has completed).
// bf16 packing is the hardware conversion.  Needs: 16-byte aligned fp32 pointers, 8-byte aligned bf16 pointers,
// ldc % 4 == 0, col0 + WTN <= N, row0 + 32 <= M.
template <int WTN, int EPI>
__device__ __forceinline__ void store_patch_rows(const GemmArgs &g, int64_t coff, const float *patch, int row0,
                                                 int col0, int lane) {
  constexpr int SP = WTN + 4, LPR = WTN / 4, RPI = 64 / LPR, NIT = 32 / RPI, U = NIT < 4 ? NIT : 4;
  const int c = (lane % LPR) * 4, r0 = lane / LPR;
  const int col = col0 + c;
  f32x4_t b4 = {0.f, 0.f, 0.f, 0.f};
  if (g.bias) b4 = *(const f32x4_t *)(g.bias + col);
  const float alpha = g.alpha;
  int64_t idx = coff + (int64_t)(row0 + r0) * g.ldc + col;
  const int64_t step = (int64_t)RPI * g.ldc;
  const float *pp = patch + r0 * SP + c;
  const bool has_resid = g.resid != nullptr, has_f32 = g.out_f32 != nullptr, has_act = g.out_act != nullptr;
#pragma unroll 1
  for (int p0 = 0; p0 < NIT; p0 += U, idx += U * step, pp += U * RPI * SP) {
    f32x4_t v[U], r[U];
    u32x2_t a[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = *(const f32x4_t *)(pp + u * RPI * SP);
    if (EPI == EPI_DGELU) {
#pragma unroll
      for (int u = 0; u < U; ++u) a[u] = *(const u32x2_t *)((const bf16_t *)g.aux + idx + u * step);
    }
    if (EPI != EPI_GELU && has_resid) {
#pragma unroll
      for (int u = 0; u < U; ++u) r[u] = *(const f32x4_t *)(g.resid + idx + u * step);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = v[u] * alpha + b4;
    if (EPI == EPI_GELU) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        u32x2_t o, h;
        o.x = pack_bf16(v[u][0], v[u][1]);
        o.y = pack_bf16(v[u][2], v[u][3]);
        h.x = pack_bf16(gelu_fast(v[u][0]), gelu_fast(v[u][1]));
        h.y = pack_bf16(gelu_fast(v[u][2]), gelu_fast(v[u][3]));
        *(u32x2_t *)((bf16_t *)g.out_act + idx + u * step) = o;
        *(u32x2_t *)((bf16_t *)g.out_act2 + idx + u * step) = h;
      }
      continue;
    }
    if (EPI == EPI_DGELU) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        v[u][0] *= dgelu_fast(__uint_as_float(a[u].x << 16));
        v[u][1] *= dgelu_fast(__uint_as_float(a[u].x & 0xffff0000u));
        v[u][2] *= dgelu_fast(__uint_as_float(a[u].y << 16));
        v[u][3] *= dgelu_fast(__uint_as_float(a[u].y & 0xffff0000u));
      }
    }
    if (has_resid) {
#pragma unroll
      for (int u = 0; u < U; ++u) v[u] += r[u];
    }
    if (has_f32) {
#pragma unroll
      for (int u = 0; u < U; ++u) *(f32x4_t *)(g.out_f32 + idx + u * step) = v[u];
    }
    if (has_act) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        u32x2_t o;
        o.x = pack_bf16(v[u][0], v[u][1]);
        o.y = pack_bf16(v[u][2], v[u][3]);
        *(u32x2_t *)((bf16_t *)g.out_act + idx + u * step) = o;
      }
    }
  }
}

template <int WTN>
__device__ __forceinline__ void store_patch(const GemmArgs &g, int64_t coff, const float *patch, int row0, int col0,
                                            int lane, bool vec) {
  if (vec && col0 + WTN <= g.N && row0 + 32 <= g.M) {  // uniform over the wavefront
    if (g.epi == EPI_GELU) store_patch_rows<WTN, EPI_GELU>(g, coff, patch, row0, col0, lane);
    else if (g.epi == EPI_DGELU) store_patch_rows<WTN, EPI_DGELU>(g, coff, patch, row0, col0, lane);
    else store_patch_rows<WTN, EPI_NONE>(g, coff, patch, row0, col0, lane);
    return;
  }
  // ragged edge or unaligned operands: element-wise, one copy of the code
  constexpr int SP = WTN + 4, LPR = WTN / 4, RPI = 64 / LPR;
#pragma unroll 1
  for (int p = 0; p < 32 / RPI; ++p) {
    const int r = p * RPI + lane / LPR, c = (lane % LPR) * 4;
    const f32x4_t v4 = *(const f32x4_t *)(patch + r * SP + c);
    const int row = row0 + r, col = col0 + c;
    if (row < g.M && col < g.N) epilogue_store4<bf16_t>(g, coff, row, col, v4, vec);
  }
}


// One tile of one product: g describes the product, bid is the workgroup's index among the nt workgroups that
// work on it, z its batch index.
template <int BM, int BN, int WM, int WN, int TA, int TB, int D>
__device__ __forceinline__ void gemm_bf16_tile(const GemmArgs &g, const int bid, const int nt, const int z) {
  static_assert(D >= 2 && D % 2 == 0, "slices in flight");
  constexpr int WTM = BM / WM, WTN = BN / WN;
  constexpr int MI = WTM / 32, NJ = WTN / 32;
  // one LDS block: two buffers per operand during the K loop, per-wavefront staging of C in the epilogue
  __shared__ __attribute__((aligned(16))) bf16_t lds_all[2 * (BM + BN) * BK];
  bf16_t *const As[2] = {lds_all, lds_all + BM * BK};
  bf16_t *const Bs[2] = {lds_all + 2 * BM * BK, lds_all + 2 * BM * BK + BN * BK};

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  // consecutive workgroup ids are dealt round-robin to the 8 XCDs; renumber so that each XCD (own L2)
  // works on a contiguous run of tiles, which share operand rows
  const int xcd = bid & 7, per = nt >> 3, rem = nt & 7;
  const int tile = xcd * per + min(xcd, rem) + (bid >> 3);
  // ... and within the run, groups of up to g.grp tile rows are walked column by column: the tiles an XCD works on
  // at any time then share a few row panels of A and a few column panels of B instead of one A panel and all of B
  const int gsz = g.grp * g.tiles_n;
  const int grp = tile / gsz, in_grp = tile - grp * gsz;
  const int rows_in_grp = min(g.grp, g.tiles_m - grp * g.grp);
  const int tm = grp * g.grp + in_grp % rows_in_grp, tn = in_grp / rows_in_grp;
  const int m0 = tm * BM, n0 = tn * BN;
  if (g.causal == CAUSAL_SKIP_UPPER && n0 > m0 + BM - 1) return;
  const int z1 = z / g.nb2, z2 = z % g.nb2;
  const bf16_t *A = (const bf16_t *)g.A + z1 * g.sA1 + z2 * g.sA2;
  const bf16_t *B = (const bf16_t *)g.B + z1 * g.sB1 + z2 * g.sB2;
  const int64_t coff = z1 * g.sC1 + z2 * g.sC2;

  int kbeg = 0, kend = g.K;
  if (g.causal == CAUSAL_K_END) kend = min(g.K, m0 + BM);
  if (g.causal == CAUSAL_K_BEGIN) kbeg = m0;
  const int nk = (kend - kbeg + BK - 1) / BK;

  Mover<BM, TA> ma;
  Mover<BN, TB> mb;
  ma.init(A, g.lda, m0, g.M, kbeg, tid);
  mb.init(B, g.ldb, n0, g.N, kbeg, tid);
  u32x4_t ra[D][Mover<BM, TA>::N], rb[D][Mover<BN, TB>::N];

  int ao[MI][BK / 16][2], bo[NJ][BK / 16][2];
#pragma unroll
  for (int kk = 0; kk < BK / 16; ++kk) {
#pragma unroll
    for (int i = 0; i < MI; ++i) fragment_offsets<BM, TA>(wm * WTM + i * 32, kk, lane, ao[i][kk][0], ao[i][kk][1]);
#pragma unroll
    for (int j = 0; j < NJ; ++j) fragment_offsets<BN, TB>(wn * WTN + j * 32, kk, lane, bo[j][kk][0], bo[j][kk][1]);
  }

  f32x16_t acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int klen = kend - kbeg;
#pragma unroll
  for (int p = 0; p < D; ++p) {
    ma.load_tail(ra[p], p, klen - p * BK);
    mb.load_tail(rb[p], p, klen - p * BK);
  }
  ma.store(ra[0], As[0]);
  mb.store(rb[0], Bs[0]);
  __syncthreads();

  // All operand fragments of a slice are requested from LDS before the first MFMA: with one wavefront per SIMD
  // nothing else hides the LDS latency, and LDS returns data in order, so the MFMAs start as the first arrive.
  auto compute = [&](const bf16_t *as, const bf16_t *bs) {
    bf16x8_t af[BK / 16][MI], bfr[BK / 16][NJ];
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
#pragma unroll
      for (int i = 0; i < MI; ++i) af[kk][i] = fragment<TA>(as, ao[i][kk][0], ao[i][kk][1]);
#pragma unroll
      for (int j = 0; j < NJ; ++j) bfr[kk][j] = fragment<TB>(bs, bo[j][kk][0], bo[j][kk][1]);
    }
    __builtin_amdgcn_sched_barrier(0);  // keep the scheduler from sinking the reads between the MFMAs
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk)
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[kk][j], af[kk][i], acc[i][j], 0, 0, 0);
  };

  // Step for slice u = t + j: request slice u + D into the register set that slice u left, move slice u + 1 from
  // registers to the other LDS buffer, multiply slice u out of LDS buffer u & 1.  D slices are in flight.  Both
  // loops are free of conditions around the MFMAs, so the accumulators never move; the drain loop zero-fills
  // slices past the end of the contraction range (at most D - 1 all-zero slices are multiplied).
  int t = 0;
  if (nk <= 1) {  // a single slice (the head-width contractions of attention): nothing to pipeline
    compute(As[0], Bs[0]);
    t = nk;
    __syncthreads();  // the epilogue reuses the operand buffers: every wavefront must be done reading them
  }
  for (; t + 2 * D + 1 <= nk; t += D) {
#pragma unroll
    for (int j = 0; j < D; ++j) {
      ma.load_full(ra[j], t + j + D);
      mb.load_full(rb[j], t + j + D);
      ma.store(ra[(j + 1) % D], As[(j + 1) & 1]);
      mb.store(rb[(j + 1) % D], Bs[(j + 1) & 1]);
      compute(As[j & 1], Bs[j & 1]);
      __syncthreads();
    }
  }
  for (; t < nk; t += D) {
#pragma unroll
    for (int j = 0; j < D; ++j) {
      ma.load_tail(ra[j], t + j + D, klen - (t + j + D) * BK);
      mb.load_tail(rb[j], t + j + D, klen - (t + j + D) * BK);
      ma.store(ra[(j + 1) % D], As[(j + 1) & 1]);
      mb.store(rb[(j + 1) % D], Bs[(j + 1) & 1]);
      compute(As[j & 1], Bs[j & 1]);
      __syncthreads();
    }
  }
  // Epilogue through LDS.  Lane L of a 32x32 result (B fragment first) holds row L%32 and columns
  // (r/4)*8 + (L/32)*4 + r%4: storing that directly would touch 32 different rows per instruction.  Each
  // wavefront instead parks 32 rows of its sub-tile in a private LDS patch [32][WTN + 4] (fp32) and reads it
  // back row-wise, so every store instruction covers whole row segments of C.
  const bool vec = ((g.ldc & 3) == 0) && ((coff & 3) == 0) &&
                   ((((uintptr_t)g.out_f32 | (uintptr_t)g.resid | (uintptr_t)g.bias) & 15) == 0) &&
                   ((((uintptr_t)g.out_act | (uintptr_t)g.out_act2 | (uintptr_t)g.aux) & 7) == 0);
  constexpr int SP = WTN + 4;                 // patch pitch in floats
  static_assert(4 * 32 * SP * 4 <= 2 * (BM + BN) * BK * 2, "staging patches must fit the operand buffers");
  float *const patch = (float *)lds_all + wave * 32 * SP;
  // every wavefront has passed the last barrier of the K loop, so nobody reads the operand buffers any more
#pragma unroll
  for (int i = 0; i < MI; ++i) {
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        f32x4_t v = {acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]};
        *(f32x4_t *)(patch + (lane & 31) * SP + j * 32 + q * 8 + (lane >> 5) * 4) = v;
      }
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the patch is written (LDS serves a wavefront in order)
    __builtin_amdgcn_wave_barrier();
    store_patch<WTN>(g, coff, patch, m0 + wm * WTM + i * 32, n0 + wn * WTN, lane, vec);
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_wave_barrier();
  }
}

template <int BM, int BN, int WM, int WN, int TA, int TB, int D>
__global__ __launch_bounds__(256, 2) void gemm_bf16_kernel(const GemmArgs g) {
  gemm_bf16_tile<BM, BN, WM, WN, TA, TB, D>(g, blockIdx.x, gridDim.x, blockIdx.y);
}

// Several products of one layout in one launch (the weight-gradient products of a block: each alone has 72-288
// tiles for the 512 tile slots of the chip and a long contraction, together they fill it): workgroups
// tile0[i] .. tile0[i+1]-1 work on product i.
constexpr int GEMM_GROUP_MAX = 4;
struct GemmGroup {
  GemmArgs p[GEMM_GROUP_MAX];
  int tile0[GEMM_GROUP_MAX + 1];
  int n;
};

template <int BM, int BN, int WM, int WN, int TA, int TB, int D>
__global__ __launch_bounds__(256, 2) void gemm_bf16_group_kernel(const GemmGroup gg) {
  int i = 0;
#pragma unroll 1
  while (i + 1 < gg.n && (int)blockIdx.x >= gg.tile0[i + 1]) ++i;  // uniform over the workgroup
  gemm_bf16_tile<BM, BN, WM, WN, TA, TB, D>(gg.p[i], blockIdx.x - gg.tile0[i], gg.tile0[i + 1] - gg.tile0[i], 0);
}

// ---------------------------------------------------------------------------
// bf16 MFMA kernel for plain products (one matrix, no causal short-cut, K a
// multiple of the slice width) with large tiles.
//
// Two per-CU rates bound a bf16 GEMM on this chip besides the MFMA rate (about
// 4096 flop per clock and CU): the vector-memory path delivers about 60 bytes
// per clock (measured; 43 for rows of only 64 bytes), so a tile needs
// 2*BM*BN/(BM+BN) >= 64 flop per operand byte just to keep up (128x128 tiles
// sit exactly on that line, 256x256 tiles need half of it), and LDS serves
// every byte once on its way in and once per wavefront that multiplies it.
// Hence
//   - a group of 2 x WGN wavefronts covers the tile, a wavefront owns
//     (BM/2) x (BN/WGN) results (up to 128x128, accumulators in up to 256
//     registers); KW such groups may share a tile, group kg multiplying
//     contraction steps kg*KS .. kg*KS+KS-1 of every slice into accumulators
//     of its own, which are summed through LDS before the write-out: more
//     wavefronts to hide latency behind, at unchanged LDS traffic;
//   - operand slices go from global memory straight into LDS (16 bytes per
//     lane; lane l of a wavefront fills LDS base + 16*l), so nothing is staged
//     in registers and no LDS store is issued; the XOR swizzle of the tiles is
//     applied on the global side (which 16 bytes a lane fetches);
//   - S LDS stages of BKT contraction steps each.  The loads of a slice are
//     spread one by one between groups of MFMAs (issued in a burst they stall
//     the wavefront for as long as the memory path needs to take them);
//   - the only barrier of a slice sits before its last contraction step: by
//     then every wavefront has read that slice completely, so its stage is
//     handed to the loads of slice t + S, and the first fragments of slice
//     t + 1 are read while the last MFMAs of slice t run;
//   - fragments for step kk + 1 are read one by one between the MFMAs of step
//     kk (one wavefront per SIMD: the overlap has to come from inside it).
// Tiles of C are numbered so that each XCD (own L2) works through groups of up
// to 8 tile rows column by column: the operand panels of a group stay in L2.
// ---------------------------------------------------------------------------
template <int BKT> __device__ __forceinline__ int kc_swz_t(int row) {
  return BKT == 64 ? ((row >> 1) & 7) : ((row >> 2) & 3);
}

template <int R, int RCL, int BKT, int NW>
struct DirectMover {
  static constexpr int CPRT = BKT / 8;             // 16-byte chunks per row of a contraction-contiguous tile
  static constexpr int N = R * CPRT / (64 * NW);   // chunks per thread and slice (NW wavefronts share the work)
  static_assert(N * 64 * NW == R * CPRT, "the slice divides evenly over the wavefronts");
  static constexpr int CPK = R / 8;
  const bf16_t *base;
  int64_t kstep;
  uint32_t off[N];
  __device__ __forceinline__ void init(const bf16_t *mat, int64_t ld, int row0, int rows, int tid) {
    const int lane = tid & 63, wave = tid >> 6;
    if (!RCL) {
      base = mat + (int64_t)row0 * ld;
      kstep = BKT;
    } else {
      base = mat + row0;
      kstep = (int64_t)BKT * ld;
    }
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int p = (i * NW + wave) * 64 + lane;  // LDS chunk this lane fills
      if (!RCL) {
        int row = p / CPRT;
        const int kc = (p % CPRT) ^ kc_swz_t<BKT>(row);
        if (row0 + row >= rows) row = 0;
        off[i] = (uint32_t)(row * ld + kc * 8);
      } else {
        const int k = p / CPK;
        int c = (p % CPK) ^ rc_swz<R>(k);
        if (row0 + c * 8 >= rows) c = 0;
        off[i] = (uint32_t)(k * ld + c * 8);
      }
    }
  }
  // chunk i of slice t into the operand's tile at lds
  __device__ __forceinline__ void issue(int i, int t, bf16_t *lds, int wave) const {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(base + t * kstep + off[i]),
                                     (__attribute__((address_space(3))) void *)(lds + (i * NW + wave) * 64 * 8), 16, 0, 0);
  }
};

// LDS addresses of a wavefront's operand fragments: NF groups of 32 rows from row rb0 on, contraction steps
// kbase .. kbase + KSW - 1 of a slice.  Only NF or KSW per-lane offsets are kept; the other index enters as a
// compile-time constant.
template <int R, int RCL, int NF, int BKT, int KSW>
struct FragAddr {
  static constexpr int CPRT = BKT / 8;
  static constexpr int CPK = R / 8;
  static constexpr int NO = RCL ? NF : KSW;
  int o[NO];
  __device__ __forceinline__ void init(int rb0, int lane, int kbase) {
    if (!RCL) {
      const int row = rb0 + (lane & 31), s = kc_swz_t<BKT>(row), hi = lane >> 5;
#pragma unroll
      for (int kk = 0; kk < KSW; ++kk) o[kk] = (row * CPRT + (((kbase + kk) * 2 + hi) ^ s)) * 8;
    } else {
      const int G = lane >> 4, sl = lane & 15;
      const int k0 = (G >> 1) * 8 + (sl >> 2);
      const int m0 = rb0 + 16 * (G & 1) + 4 * (sl & 3);
#pragma unroll
      for (int f = 0; f < NF; ++f) {
        const int m = m0 + f * 32;
        o[f] = (k0 * CPK + ((m >> 3) ^ rc_swz<R>(k0))) * 8 + ((m >> 2) & 1) * 4 + kbase * 16 * CPK * 8;
      }
    }
  }
  __device__ __forceinline__ bf16x8_t get(const bf16_t *lds, int f, int kk) const {
    if (!RCL) return fragment<0>(lds, o[kk] + f * 32 * CPRT * 8, 0);
    const int b = o[f] + kk * 16 * CPK * 8;  // 16 further contraction steps leave the swizzle unchanged
    return fragment<1>(lds, b, b + 4 * CPK * 8);
  }
};

template <int n> __device__ __forceinline__ void wait_loads_le() {
  // vmcnt (outstanding vector-memory loads) is split over bits 3:0 and 15:14; lgkmcnt(0): this wavefront's LDS
  // reads have returned; expcnt is left alone
  static_assert(n >= 0 && n <= 63, "vmcnt range");
  __builtin_amdgcn_s_waitcnt((n & 15) | ((n >> 4) << 14) | 0x0070);
}

template <int BM, int BN, int TA, int TB, int BKT, int S, int OCC, int KW, int WGN>
__global__ __launch_bounds__(128 * WGN * KW, OCC * KW * WGN / 2) void gemm_bf16_big_kernel(const GemmArgs g) {
  constexpr int WTM = BM / 2, WTN = BN / WGN;
  constexpr int MI = WTM / 32, NJ = WTN / 32;
  constexpr int WPG = 2 * WGN;                   // wavefronts of a group: 2 x WGN over the tile
  constexpr int NW = WPG * KW;                   // KW groups; group kg takes steps kg*KS.. of a slice
  constexpr int KS = BKT / 16 / KW;              // contraction steps of one MFMA per slice and wavefront
  constexpr int STAGE = (BM + BN) * BKT;         // elements per stage
  constexpr int NLA = DirectMover<BM, TA, BKT, NW>::N, NLB = DirectMover<BN, TB, BKT, NW>::N, NL = NLA + NLB;
  constexpr int G = KS * MI;                     // groups of NJ MFMAs per slice
  constexpr int QB = (KS - 1) * MI;              // the barrier sits before this group
  static_assert(KS % 2 == 0 && KS * KW * 16 == BKT && NL <= G && S >= 2, "pipeline shape");
  static_assert(KW == 1 || MI % KW == 0, "the groups share the write-out by rows of fragments");
  extern __shared__ __attribute__((aligned(16))) bf16_t lds_dyn[];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kg = wave / WPG, wig = wave % WPG, wm = wig / WGN, wn = wig % WGN;
  const int nt = gridDim.x, bid = blockIdx.x;
  const int xcd = bid & 7, per = nt >> 3, rem = nt & 7;
  const int tile = xcd * per + min(xcd, rem) + (bid >> 3);
  // groups of up to g.grp tile rows, walked column by column
  const int gsz = g.grp * g.tiles_n;
  const int grp = tile / gsz, in_grp = tile - grp * gsz;
  const int rows_in_grp = min(g.grp, g.tiles_m - grp * g.grp);
  const int tm = grp * g.grp + in_grp % rows_in_grp, tn = in_grp / rows_in_grp;
  const int m0 = tm * BM, n0 = tn * BN;
  const int nk = g.K / BKT;

  DirectMover<BM, TA, BKT, NW> ma;
  DirectMover<BN, TB, BKT, NW> mb;
  ma.init((const bf16_t *)g.A, g.lda, m0, g.M, tid);
  mb.init((const bf16_t *)g.B, g.ldb, n0, g.N, tid);
  FragAddr<BM, TA, MI, BKT, KS> fa;
  FragAddr<BN, TB, NJ, BKT, KS> fb;
  fa.init(wm * WTM, lane, kg * KS);
  fb.init(wn * WTN, lane, kg * KS);

  // load l (0..NL-1: first A's chunks, then B's) of slice sl into stage sg
  auto issue = [&](int l, int sl, int sg) {
    bf16_t *base = lds_dyn + sg * STAGE;
    if (l < NLA) ma.issue(l, sl, base, wave);
    else mb.issue(l - NLA, sl, base + BM * BKT, wave);
  };

  f32x16_t acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // prologue: slices 0 .. S-2 completely and the head of slice S-1 (what the steady state issues after a barrier)
  constexpr int HEAD = (G - QB) < NL ? (G - QB) : NL;
#pragma unroll
  for (int p = 0; p < S - 1; ++p)
    if (p < nk) {
#pragma unroll
      for (int l = 0; l < NL; ++l) issue(l, p, p);
    }
  if (S - 1 < nk) {
#pragma unroll
    for (int l = 0; l < HEAD; ++l) issue(l, S - 1, S - 1);
  }
  if (nk >= S) wait_loads_le<(S - 2) * NL + HEAD>();
  else wait_loads_le<0>();
  __builtin_amdgcn_s_barrier();
  bf16x8_t af[2][MI], bfr[2][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i) af[0][i] = fa.get(lds_dyn, i, 0);
#pragma unroll
  for (int j = 0; j < NJ; ++j) bfr[0][j] = fb.get(lds_dyn + BM * BKT, j, 0);

  // One slice.  GUARD = false: steady state (slices t + S - 1 and t + S exist, so every load is issued and the
  // number of loads in flight at the barrier is known); GUARD = true: the last S slices.
  auto slice = [&](int t, int st, auto guard) {
    constexpr bool GUARD = decltype(guard)::value;
    const bf16_t *as = lds_dyn + st * STAGE, *bs = as + BM * BKT;
    const int st_prev = (st == 0) ? S - 1 : st - 1;   // stage of slice t + S - 1
    const int st_next = (st + 1 == S) ? 0 : st + 1;   // stage of slice t + 1
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      // fragments of the next step: step kk + 1 of this slice, or step 0 of slice t + 1 once everybody is through
      // with slice t.  Their MI + NJ reads go out one by one between this step's MI * NJ MFMAs, in the order the
      // next step needs them and from the first MFMA on, so that the last has returned when the step ends (a
      // wavefront that issues them in a burst stands still until LDS has taken them all, and with one wavefront
      // per SIMD the matrix pipe stands still with it).
      const bool more = (kk + 1 < KS) || !GUARD || (t + 1 < nk);
      const bf16_t *na = as, *nb = bs;
      if (kk + 1 == KS && more) {
        // slice t + 1 must have landed (S - 2 younger slices may stay in flight) and this wavefront's reads of
        // slice t must be complete before anybody overwrites its stage
        if (!GUARD) wait_loads_le<(S - 2) * NL>();
        else wait_loads_le<0>();
        __builtin_amdgcn_s_barrier();
        na = lds_dyn + st_next * STAGE;
        nb = na + BM * BKT;
      }
      constexpr int NR = MI + NJ, NS = MI * NJ;
      const int nkk = (kk + 1 < KS) ? kk + 1 : 0, nbuf = (kk + 1) & 1;
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < MI; ++i) {
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[kk & 1][j], af[kk & 1][i], acc[i][j], 0, 0, 0);
          if (more) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int r = 0; r < NR; ++r)
              if ((NS >= NR ? r : r * NS / NR) == i * NJ + j) {  // read r: a0, b0 .. b(NJ-1), a1 .. a(MI-1)
                if (r == 0) af[nbuf][0] = fa.get(na, 0, nkk);
                else if (r <= NJ) bfr[nbuf][r - 1] = fb.get(nb, r - 1, nkk);
                else af[nbuf][r - NJ] = fa.get(na, r - NJ, nkk);
              }
            __builtin_amdgcn_sched_barrier(0);
          }
          if (j == NJ - 1) {
            __builtin_amdgcn_sched_barrier(0);
            const int q = kk * MI + i;
            if (q >= QB) {  // after the barrier: the head of slice t + S goes into the stage slice t just left
              if (q - QB < NL && (!GUARD || t + S < nk)) issue(q - QB, t + S, st);
            } else {        // before it: the rest of slice t + S - 1
              if (q + (G - QB) < NL && (!GUARD || t + S - 1 < nk)) issue(q + (G - QB), t + S - 1, st_prev);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
    }
  };

  int t = 0, st = 0;
  for (; t + S < nk; ++t) {
    slice(t, st, std::false_type{});
    if (++st == S) st = 0;
  }
  for (; t < nk; ++t) {
    slice(t, st, std::true_type{});
    if (++st == S) st = 0;
  }
  wait_loads_le<0>();
  __builtin_amdgcn_s_barrier();  // the epilogue reuses the stages

  const bool vec = ((g.ldc & 3) == 0) &&
                   ((((uintptr_t)g.out_f32 | (uintptr_t)g.resid | (uintptr_t)g.bias) & 15) == 0) &&
                   ((((uintptr_t)g.out_act | (uintptr_t)g.out_act2 | (uintptr_t)g.aux) & 7) == 0);
  constexpr int SP = WTN + 4;
  static_assert(NW * 32 * SP * 4 <= S * STAGE * 2, "staging patches must fit the stages");
  if constexpr (KW > 1) {
    // Each group holds a partial sum of the whole tile.  Group kg writes out the fragment rows i with i % KW == kg:
    // it hands its other rows to their owner through LDS (lane-contiguous 16-byte pieces, one area per position in
    // the 2 x 2 arrangement and owner) and adds what it receives (two terms: the order cannot matter).
    static_assert(KW <= 2, "one partner per fragment row");
    constexpr int XA = (MI / KW) * NJ * 4 * 64;  // 16-byte pieces per area
    static_assert(WPG * KW * XA * 16 <= S * STAGE * 2, "exchange areas must fit the stages");
    f32x4_t *const xch = (f32x4_t *)lds_dyn + wig * KW * XA + lane;
#pragma unroll
    for (int i = 0; i < MI; ++i)
      if (i % KW != kg) {
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            f32x4_t v = {acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]};
            xch[(i % KW) * XA + (((i / KW) * NJ + j) * 4 + q) * 64] = v;
          }
      }
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int i = 0; i < MI; ++i)
      if (i % KW == kg) {
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const f32x4_t v = xch[(i % KW) * XA + (((i / KW) * NJ + j) * 4 + q) * 64];
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][q * 4 + r] += v[r];
          }
      }
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_s_barrier();  // the staging patches overlap the exchange area
  }
  float *const patch = (float *)lds_dyn + wave * 32 * SP;
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    if (KW > 1 && i % KW != kg) continue;
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        f32x4_t v = {acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]};
        *(f32x4_t *)(patch + (lane & 31) * SP + j * 32 + q * 8 + (lane >> 5) * 4) = v;
      }
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_wave_barrier();
    store_patch<WTN>(g, 0, patch, m0 + wm * WTM + i * 32, n0 + wn * WTN, lane, vec);
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_wave_barrier();
  }
}

template <int BM, int BN, int BKT, int S, int OCC, int KW = 1, int WGN = 2>
static hipError_t launch_bf16_big(const GemmArgs &a, int ta, int tb, int ntiles, hipStream_t s) {
  constexpr size_t lds = (size_t)S * (BM + BN) * BKT * 2;
  static_assert(lds <= 160 * 1024, "LDS per CU");
#define HYDRA_BIG(TA_, TB_)                                                                                   \
  do {                                                                                                         \
    auto kern = gemm_bf16_big_kernel<BM, BN, TA_, TB_, BKT, S, OCC, KW, WGN>;                                          \
    static hipError_t attr = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                                 (int)lds);                                                    \
    if (attr != hipSuccess) return attr;                                                                       \
    hipLaunchKernelGGL(kern, dim3(ntiles), dim3(128 * WGN * KW), lds, s, a);                                         \
  } while (0)
  if (ta == 0 && tb == 0) HYDRA_BIG(0, 0);
  else if (ta == 0 && tb == 1) HYDRA_BIG(0, 1);
  else if (ta == 1 && tb == 1) HYDRA_BIG(1, 1);
  else HYDRA_BIG(1, 0);
#undef HYDRA_BIG
  return hipGetLastError();
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


template <int BM, int BN, int WM, int WN, int D>
static hipError_t launch_bf16_cfg(const GemmArgs &a, int ta, int tb, dim3 grid, hipStream_t s) {
  if (ta == 0 && tb == 0) hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, 0, 0, D>), grid, dim3(256), 0, s, a);
  else if (ta == 0 && tb == 1) hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, 0, 1, D>), grid, dim3(256), 0, s, a);
  else if (ta == 1 && tb == 1) hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, 1, 1, D>), grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, 1, 0, D>), grid, dim3(256), 0, s, a);
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
  static const char *n64[4] = {"gemm_bf16_x64_nt", "gemm_bf16_x64_nn", "gemm_bf16_x64_tt", "gemm_bf16_x64_tn"};
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
  a.grp = 8;
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
  // tile choice: 128x128 only for problems of many waves of tiles (the LM head); at a few thousand tokens per
  // visit the block GEMMs have 100-400 tiles and the narrower tile measured faster on every one of them
  const long t128 = (long)((d.M + 127) / 128) * ((d.N + 127) / 128) * nbatch;
  const long t256 = (long)((d.M + 255) / 256) * ((d.N + 255) / 256);
  int tile = (d.N > 64 && t128 >= 2048) ? 1 : 2;
  // plain products whose operands both have the contraction index contiguous go to the direct-to-LDS kernel:
  // 256x256 tiles once they fill three quarters of the CUs, else 128x64 tiles.  Operands stored the other way
  // round need two half-rate transposing LDS reads per fragment, which takes the advantage away (measured).
  // (128x64 tiles: three LDS stages and two blocks per CU; with more than 512 tiles, two stages and three blocks per
  // CU, which takes such a product through in one round of tiles - measured 15.3 against 16.5 us at 2048x2304x768 -
  // while with fewer tiles the shallower pipeline only costs: 30.6 against 18.9 us at 2048x768x3072)
  // Between the two: a round of 256x128 tiles worked on by eight wavefronts (two groups that split every slice's
  // contraction steps) once there are 200 of them (measured 22.8 against 26.1 us at 2048x4096x1024, 26.5 against
  // 33.5 us at 1024x6400x1600), and one round of 128x128 tiles for long contractions (39.9 against 44.3 us at
  // 1024x4096x4096, 131 against 156 us at 1024x4096x16384).
  if (d.ta == 0 && d.tb == 0) {
    const long t256x128 = (long)((d.M + 255) / 256) * ((d.N + 127) / 128);
    if (t256 >= 192) tile = 4;
    else if (t256x128 >= 200) tile = 16;
    else if (t128 >= 192 && t128 <= 256 && d.K >= 2048) tile = 11;
    else tile = (long)((d.M + 127) / 128) * ((d.N + 63) / 64) > 512 ? 12 : 10;
  }
  // too few 128x64 tiles to occupy half the CUs (the d x d weight gradient): 64x64 tiles measured a third faster
  else if (tile == 2 && (long)((d.M + 127) / 128) * ((d.N + 63) / 64) * nbatch < 128 && d.M > 64) tile = 3;
  // slices in flight: a deeper pipeline pays once the contraction is long enough to amortise filling it
  int D = (d.causal == CAUSAL_NONE && d.K >= 24 * BK) ? 4 : 2;
#define HYDRA_LAUNCH(BM_, BN_, DD_)                                                                      \
  do {                                                                                                    \
    a.tiles_m = (d.M + BM_ - 1) / BM_;                                                                    \
    a.tiles_n = (d.N + BN_ - 1) / BN_;                                                                    \
    a.grp = xcd_group_rows(a.tiles_m, a.tiles_n, BM_, BN_);                                               \
    ProfScope ps(gemm_name(DT_BF16, BN_, d.ta, d.tb), s, gemm_flops(d), 0);                              \
    return launch_bf16_cfg<BM_, BN_, 2, 2, DD_>(a, d.ta, d.tb, dim3(a.tiles_m * a.tiles_n, nbatch), s); \
  } while (0)
  const bool plain = d.causal == CAUSAL_NONE && nbatch == 1 && d.K % BK == 0 && d.K >= 2 * BK;
#define HYDRA_LAUNCH_BIG(BM_, BN_, BK_, S_, OCC_, NAME_)                                       \
  do {                                                                                          \
    a.tiles_m = (d.M + BM_ - 1) / BM_;                                                          \
    a.tiles_n = (d.N + BN_ - 1) / BN_;                                                          \
    a.grp = xcd_group_rows(a.tiles_m, a.tiles_n, BM_, BN_, 32 * OCC_);                          \
    static const char *names[4] = {NAME_ "_nt", NAME_ "_nn", NAME_ "_tt", NAME_ "_tn"};         \
    ProfScope ps(names[d.ta * 2 + d.tb], s, gemm_flops(d), 0);                                  \
    return launch_bf16_big<BM_, BN_, BK_, S_, OCC_>(a, d.ta, d.tb, a.tiles_m * a.tiles_n, s);   \
  } while (0)
#define HYDRA_LAUNCH_BIGW(BM_, BN_, BK_, S_, OCC_, KW_, WGN_, NAME_)                                      \
  do {                                                                                          \
    a.tiles_m = (d.M + BM_ - 1) / BM_;                                                          \
    a.tiles_n = (d.N + BN_ - 1) / BN_;                                                          \
    a.grp = xcd_group_rows(a.tiles_m, a.tiles_n, BM_, BN_, 32 * OCC_);                          \
    static const char *names[4] = {NAME_ "_nt", NAME_ "_nn", NAME_ "_tt", NAME_ "_tn"};         \
    ProfScope ps(names[d.ta * 2 + d.tb], s, gemm_flops(d), 0);                                  \
    return launch_bf16_big<BM_, BN_, BK_, S_, OCC_, KW_, WGN_>(a, d.ta, d.tb, a.tiles_m * a.tiles_n, s); \
  } while (0)
  if (plain && tile == 4) HYDRA_LAUNCH_BIG(256, 256, 32, 4, 1, "gemm_bf16_256x256");
  if (plain && tile == 10) HYDRA_LAUNCH_BIG(128, 64, 64, 3, 2, "gemm_bf16_d128x64k64");
  if (plain && tile == 11) HYDRA_LAUNCH_BIG(128, 128, 64, 3, 1, "gemm_bf16_d128x128k64");
  if (plain && tile == 12) HYDRA_LAUNCH_BIG(128, 64, 64, 2, 3, "gemm_bf16_d128x64k64s2");
  if (plain && tile == 16) HYDRA_LAUNCH_BIGW(256, 128, 64, 3, 1, 2, 2, "gemm_bf16_w8_256x128k64");
#undef HYDRA_LAUNCH_BIG
#undef HYDRA_LAUNCH_BIGW
  if (tile >= 4) tile = 2;
  if (tile == 1) {
    HYDRA_LAUNCH(128, 128, 2);
  }
  if (tile == 3) {
    if (D == 4) HYDRA_LAUNCH(64, 64, 4);
    HYDRA_LAUNCH(64, 64, 2);
  }
  if (D == 4) HYDRA_LAUNCH(128, 64, 4);
  HYDRA_LAUNCH(128, 64, 2);
#undef HYDRA_LAUNCH
}

static void fill_args(GemmArgs &a, const GemmDesc &d) {
  a.A = d.A; a.B = d.B; a.M = d.M; a.N = d.N; a.K = d.K;
  a.lda = d.lda; a.ldb = d.ldb; a.ldc = d.ldc;
  a.nb2 = d.nb2;
  a.sA1 = d.sA1; a.sA2 = d.sA2; a.sB1 = d.sB1; a.sB2 = d.sB2; a.sC1 = d.sC1; a.sC2 = d.sC2;
  a.alpha = d.alpha; a.bias = d.bias; a.resid = d.resid;
  a.out_f32 = d.out_f32; a.out_act = d.out_act; a.out_act2 = d.out_act2; a.aux = d.aux;
  a.epi = d.epi; a.causal = d.causal;
  a.grp = 8;
}

hipError_t launch_gemm_group(const GemmDesc *d, int n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  bool groupable = n <= GEMM_GROUP_MAX && d[0].dtype == DT_BF16;
  for (int i = 0; i < n && groupable; ++i) {
    const GemmDesc &x = d[i];
    // (a product with more than a round of 128x64 tiles fills the chip by itself and may want another tile)
    groupable = x.dtype == DT_BF16 && x.ta == 1 && x.tb == 1 && x.causal == CAUSAL_NONE && x.nb1 * x.nb2 == 1 &&
                x.M > 0 && x.N > 0 && x.K >= 24 * BK && !(x.lda & 7) && !(x.ldb & 7) && !(((uintptr_t)x.A) & 15) &&
                !(((uintptr_t)x.B) & 15) && (long)((x.M + 127) / 128) * ((x.N + 63) / 64) <= 512;
  }
  if (!groupable) {  // other layouts, dtypes or short contractions: one launch each
    for (int i = 0; i < n; ++i) {
      hipError_t e = launch_gemm(d[i], s);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  GemmGroup gg;
  gg.n = n;
  int tiles = 0;
  double flops = 0;
  for (int i = 0; i < n; ++i) {
    GemmArgs &a = gg.p[i];
    fill_args(a, d[i]);
    a.tiles_m = (d[i].M + 127) / 128;
    a.tiles_n = (d[i].N + 63) / 64;
    a.grp = xcd_group_rows(a.tiles_m, a.tiles_n, 128, 64);
    gg.tile0[i] = tiles;
    tiles += a.tiles_m * a.tiles_n;
    flops += gemm_flops(d[i]);
  }
  for (int i = n; i <= GEMM_GROUP_MAX; ++i) gg.tile0[i] = tiles;
  ProfScope ps("gemm_bf16_x64_tn_group", s, flops, 0);
  hipLaunchKernelGGL((gemm_bf16_group_kernel<128, 64, 2, 2, 1, 1, 4>), dim3(tiles), dim3(256), 0, s, gg);
  return hipGetLastError();
}

}  // namespace hydra
