// Canonical flat parameter layout of a model and its division into shards
// ("rewriting a full model into shards", paper Section 1; cut points are given
// by layers_per_shard rather than found by the pilot pass of Section 2.2).
#include <cstdio>
#include <cstring>

#include "hydra_internal.h"

namespace hydra {

static thread_local std::string g_err = "";
void set_global_error(const std::string &msg) { g_err = msg; }
const char *global_error() { return g_err.c_str(); }

hydra_status build_shape(const hydra_model_desc *d, ModelShape *s, std::string *err) {
  auto bad = [&](const char *m) {
    if (err) *err = m;
    return (hydra_status)HYDRA_E_INVAL;
  };
  if (!d || !s) return bad("null model description");
  if (d->n_layer <= 0 || d->d_model <= 0 || d->n_head <= 0 || d->d_ff <= 0 || d->vocab <= 0 || d->seq <= 0 ||
      d->batch <= 0 || d->layers_per_shard <= 0)
    return bad("model dimensions must be positive");
  if (d->n_layer % d->layers_per_shard) return bad("layers_per_shard must divide n_layer");
  if (d->d_model % d->n_head) return bad("n_head must divide d_model");
  if (d->d_model % 8 || d->d_ff % 8 || d->seq % 8) return bad("d_model, d_ff and seq must be multiples of 8");
  if ((d->d_model / d->n_head) % 8) return bad("head width d_model/n_head must be a multiple of 8");
  if (d->dtype != 0 && d->dtype != 1) return bad("dtype must be 0 (fp32) or 1 (bf16)");
  if ((int64_t)d->batch * d->seq > 32768) return bad("batch*seq above 32768 tokens is not supported");
  if (d->n_micro < 0 || d->n_micro > 4096) return bad("n_micro must be in 0..4096");
  if (d->tie_embeddings != 0 && d->tie_embeddings != 1) return bad("tie_embeddings must be 0 or 1");
  s->L = d->n_layer; s->d = d->d_model; s->H = d->n_head; s->F = d->d_ff; s->V = d->vocab;
  s->T = d->seq; s->B = d->batch; s->k = d->layers_per_shard; s->S = s->L / s->k; s->dh = s->d / s->H;
  s->M = (int64_t)s->B * s->T;
  s->nm = d->n_micro > 0 ? d->n_micro : 1;
  s->Mt = s->M * s->nm;
  s->Vpad = ((int64_t)s->V + 63) / 64 * 64;
  const int64_t dd = s->d, F = s->F;
  BlockOffsets &b = s->bo;
  int64_t o = 0;
  b.ln1_g = o; o += dd;
  b.ln1_b = o; o += dd;
  b.w_qkv = o; o += dd * 3 * dd;
  b.b_qkv = o; o += 3 * dd;
  b.w_o = o; o += dd * dd;
  b.b_o = o; o += dd;
  b.ln2_g = o; o += dd;
  b.ln2_b = o; o += dd;
  b.w_fc = o; o += dd * F;
  b.b_fc = o; o += F;
  b.w_proj = o; o += F * dd;
  b.b_proj = o; o += dd;
  b.size = o;
  s->shard_off.assign(s->S + 3, 0);
  int64_t off = 0;
  s->shard_off[0] = 0;
  off += (int64_t)s->V * dd + (int64_t)s->T * dd;
  for (int i = 1; i <= s->S; ++i) {
    s->shard_off[i] = off;
    off += b.size * s->k;
  }
  s->shard_off[s->S + 1] = off;
  s->tie = d->tie_embeddings != 0;
  off += 2 * dd + (s->tie ? 0 : dd * (int64_t)s->V);
  s->shard_off[s->S + 2] = off;
  s->n_params = off;
  // a tied HEAD shard owns 2d parameters but its buffer also holds a copy of wte
  s->max_shard = 2 * dd + dd * (int64_t)s->V;
  for (int i = 0; i < s->S + 2; ++i) {
    const int64_t c = s->shard_off[i + 1] - s->shard_off[i];
    if (c > s->max_shard) s->max_shard = c;
  }
  return HYDRA_OK;
}

void list_tensors(const ModelShape &s, std::vector<TensorInfo> *out) {
  out->clear();
  const int64_t d = s.d;
  out->push_back({"wte", 0, s.V, d, 0});
  out->push_back({"wpe", (int64_t)s.V * d, s.T, d, 0});
  for (int l = 0; l < s.L; ++l) {
    const int shard = 1 + l / s.k;
    const int64_t base = s.shard_off[shard] + (int64_t)(l % s.k) * s.bo.size;
    char p[16];
    snprintf(p, sizeof p, "h%d.", l);
    const std::string P = p;
    out->push_back({P + "ln1_g", base + s.bo.ln1_g, d, 1, shard});
    out->push_back({P + "ln1_b", base + s.bo.ln1_b, d, 1, shard});
    out->push_back({P + "w_qkv", base + s.bo.w_qkv, d, 3 * d, shard});
    out->push_back({P + "b_qkv", base + s.bo.b_qkv, 3 * d, 1, shard});
    out->push_back({P + "w_o", base + s.bo.w_o, d, d, shard});
    out->push_back({P + "b_o", base + s.bo.b_o, d, 1, shard});
    out->push_back({P + "ln2_g", base + s.bo.ln2_g, d, 1, shard});
    out->push_back({P + "ln2_b", base + s.bo.ln2_b, d, 1, shard});
    out->push_back({P + "w_fc", base + s.bo.w_fc, d, s.F, shard});
    out->push_back({P + "b_fc", base + s.bo.b_fc, s.F, 1, shard});
    out->push_back({P + "w_proj", base + s.bo.w_proj, s.F, d, shard});
    out->push_back({P + "b_proj", base + s.bo.b_proj, d, 1, shard});
  }
  const int64_t h = s.shard_off[s.S + 1];
  out->push_back({"lnf_g", h, d, 1, s.S + 1});
  out->push_back({"lnf_b", h + d, d, 1, s.S + 1});
  if (!s.tie) out->push_back({"w_lm", h + 2 * d, d, s.V, s.S + 1});
}

}  // namespace hydra

using namespace hydra;

extern "C" {

hydra_status hydra_model_layout(const hydra_model_desc *desc, hydra_layout *out) {
  ModelShape s;
  std::string err;
  if (!out) {
    set_global_error("null output");
    return HYDRA_E_INVAL;
  }
  hydra_status st = build_shape(desc, &s, &err);
  if (st != HYDRA_OK) {
    set_global_error(err);
    return st;
  }
  out->n_params = s.n_params;
  out->params_per_block = s.bo.size;
  out->n_block_shards = s.S;
  out->n_shards = s.S + 2;
  out->n_tensors = 2 + 12 * s.L + (s.tie ? 2 : 3);
  out->reserved = 0;
  return HYDRA_OK;
}

hydra_status hydra_model_tensor(const hydra_model_desc *desc, int32_t index, char name[32], int64_t *offset,
                                int64_t *rows, int64_t *cols, int32_t *shard) {
  ModelShape s;
  std::string err;
  hydra_status st = build_shape(desc, &s, &err);
  if (st != HYDRA_OK) {
    set_global_error(err);
    return st;
  }
  std::vector<TensorInfo> ts;
  list_tensors(s, &ts);
  if (index < 0 || index >= (int32_t)ts.size()) {
    set_global_error("tensor index out of range");
    return HYDRA_E_INVAL;
  }
  const TensorInfo &t = ts[index];
  if (name) {
    strncpy(name, t.name.c_str(), 31);
    name[31] = 0;
  }
  if (offset) *offset = t.off;
  if (rows) *rows = t.rows;
  if (cols) *cols = t.cols;
  if (shard) *shard = t.shard;
  return HYDRA_OK;
}

hydra_status hydra_shard_range(const hydra_model_desc *desc, int32_t shard, int64_t *offset, int64_t *count) {
  ModelShape s;
  std::string err;
  hydra_status st = build_shape(desc, &s, &err);
  if (st != HYDRA_OK) {
    set_global_error(err);
    return st;
  }
  if (shard < 0 || shard >= s.S + 2) {
    set_global_error("shard index out of range");
    return HYDRA_E_INVAL;
  }
  if (offset) *offset = s.shard_off[shard];
  if (count) *count = s.shard_off[shard + 1] - s.shard_off[shard];
  return HYDRA_OK;
}

}  // extern "C"
