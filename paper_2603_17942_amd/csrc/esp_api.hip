// C ABI of the ESP decode step: argument validation, workspace partition, kernel sequencing.
// Every step of the path runs in this library's kernels; nothing here computes on the host.
#include <new>

#include "esp_internal.h"

namespace {

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline size_t elt(int dtype) { return dtype == ESP_F32 ? 4 : 2; }

struct WsLayout {
  size_t h, xn, q, attn_out, act, gemm_out, attn_part, rope_tab, logits, topk_scratch, idx_a, idx_b, idx_c, idx_d, status, total;
  size_t gemm_out_floats, attn_part_floats, logits_rows;
};

esp_status check_model(const esp_model_desc* m) {
  if (!m) return ESP_EINVAL;
  if (m->dtype != ESP_F32 && m->dtype != ESP_BF16) return ESP_EDTYPE;
  if (m->n_layers < 1 || m->d_model < 1 || m->n_q_heads < 1 || m->n_kv_heads < 1 || m->head_dim < 1 ||
      m->d_ff < 1 || m->vocab < 1)
    return ESP_EINVAL;
  if (m->n_q_heads % m->n_kv_heads) return ESP_ESHAPE;
  if (m->head_dim != 64 && m->head_dim != 128) return ESP_ESHAPE;
  if (m->d_model % 4 || m->d_ff % 4) return ESP_ESHAPE;   // float4 paths of the glue kernels
  if (m->dtype == ESP_BF16) {
    // MFMA GEMM: K multiple of 64, N multiple of 32
    if (m->d_model % 64 || m->d_ff % 64 || (m->n_q_heads * m->head_dim) % 64 || m->vocab % 32) return ESP_ESHAPE;
  }
  if (!(m->rope_theta > 0.f) || !(m->rms_eps >= 0.f)) return ESP_EINVAL;
  return ESP_OK;
}

int max_splits_of(const esp_model_desc* m, int M) {
  int nqkv = (m->n_q_heads + 2 * m->n_kv_heads) * m->head_dim;
  int s = 1;
  s = std::max(s, gemm_plan(m->dtype, M, nqkv, m->d_model).splits);
  return s;
}

WsLayout ws_layout(const esp_model_desc* m, int max_batch, int max_rows, int64_t max_kv_len) {
  WsLayout w{};
  const size_t M = (size_t)max_batch * max_rows;
  const size_t e = elt(m->dtype);
  const int d = m->d_model, hq = m->n_q_heads, hkv = m->n_kv_heads, hd = m->head_dim, ff = m->d_ff;
  const int nqkv = (hq + 2 * hkv) * hd;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  w.h = take(M * d * 4);
  w.xn = take(M * (size_t)std::max(d, hq * hd) * e);
  w.q = take(M * (size_t)hq * hd * e);
  w.attn_out = take(M * (size_t)hq * hd * e);
  w.act = take(M * (size_t)ff * e);
  size_t go = 0;
  go = std::max(go, gemm_out_elems(gemm_plan(m->dtype, (int)M, nqkv, d), (int)M, nqkv));
  go = std::max(go, gemm_out_elems(gemm_plan(m->dtype, (int)M, d, hq * hd), (int)M, d));
  go = std::max(go, gemm_out_elems(gemm_plan(m->dtype, (int)M, 2 * ff, d), (int)M, 2 * ff));
  go = std::max(go, gemm_out_elems(gemm_plan(m->dtype, (int)M, d, ff), (int)M, d));
  w.gemm_out_floats = go;
  w.gemm_out = take(go * 4);
  int lb = (int)std::min<int64_t>(max_kv_len, 0x7fffffff);
  AttnPlan ap = attn_plan(max_batch, max_rows, hq, hkv, lb);
  // a call may use fewer rows / shorter bound and hence another split count: size for the worst
  size_t apf = attn_partial_floats(m->dtype, max_batch, max_rows, hq, hkv, hd, std::max(ap.nsplit, 64));
  w.attn_part_floats = apf;
  w.attn_part = take(apf * 4);
  w.rope_tab = take(M * (size_t)hd * 4);
  w.logits_rows = std::max<size_t>(M, (size_t)max_batch * ESP_MAX_MASKS);
  // node-row logits only need max_batch*max_rows rows in debug mode; otherwise nodes <= rows
  w.logits = take(w.logits_rows * (size_t)m->vocab * 4);
  w.topk_scratch = take(softmax_topk_scratch_floats(max_batch * ESP_MAX_MASKS, m->vocab, ESP_MAX_TOPK) * 4);
  w.idx_a = take(std::max<size_t>(M, (size_t)max_batch * ESP_MAX_MASKS) * 4);
  w.idx_b = take(std::max<size_t>(M, (size_t)max_batch * ESP_MAX_MASKS) * 4);
  w.idx_c = take(std::max<size_t>(M, (size_t)max_batch * ESP_MAX_MASKS) * 4);
  w.idx_d = take(std::max<size_t>(M, (size_t)max_batch * ESP_MAX_MASKS) * 4);
  w.status = take(256);
  w.total = off;
  return w;
}

BlockDev to_dev(const esp_block* b) {
  BlockDev d;
  d.batch = b->batch; d.rows_per_seq = b->rows_per_seq; d.k_masks = b->k_masks; d.layout = b->layout;
  d.anc_words = b->anc_words;
  d.n_rows = b->n_rows; d.n_nodes = b->n_nodes; d.tok = b->tok; d.parent = b->parent; d.depth = b->depth;
  d.mask_j = b->mask_j; d.attach = b->attach; d.anc = b->anc;
  return d;
}
KvDev to_dev(const esp_kv* k) {
  KvDev d;
  d.k = k->k; d.v = k->v; d.len = k->len; d.base = k->base; d.seq_cap = k->seq_cap; d.capacity = k->capacity;
  d.len_bound = k->len_bound;
  return d;
}

esp_status check_block(const esp_ctx* c, const esp_block* b) {
  if (!b) return ESP_EINVAL;
  if (!b->n_rows || !b->n_nodes || !b->tok || !b->parent || !b->depth || !b->mask_j || !b->attach || !b->anc)
    return ESP_EINVAL;
  if (b->batch < 1 || b->rows_per_seq < 1 || b->k_masks < 0 || b->k_masks > ESP_MAX_MASKS) return ESP_EINVAL;
  if (b->layout != ESP_LAYOUT_PER_NODE && b->layout != ESP_LAYOUT_ROOT_CHAIN) return ESP_EINVAL;
  if (b->rows_per_seq > ESP_MAX_ROWS_PER_SEQ) return ESP_ECAPACITY;
  if (b->anc_words != (b->rows_per_seq + 63) / 64) return ESP_EINVAL;
  if (c && (b->batch > c->max_batch || b->rows_per_seq > c->max_rows)) return ESP_ECAPACITY;
  return ESP_OK;
}

esp_status check_kv(const esp_ctx* c, const esp_kv* kv, const esp_block* b) {
  if (!kv || !kv->k || !kv->v || !kv->len || !kv->base || !kv->seq_cap) return ESP_EINVAL;
  if (kv->capacity < 64 || kv->capacity % 64) return ESP_EINVAL;
  if (kv->len_bound < 0) return ESP_EINVAL;
  if (c && b && (int64_t)kv->len_bound + b->rows_per_seq > c->max_kv_len) return ESP_ECAPACITY;
  return ESP_OK;
}

#define ESP_HIP(expr)                          \
  do {                                         \
    hipError_t e__ = (expr);                   \
    if (e__ != hipSuccess) return ESP_EDEVICE; \
  } while (0)

int nodes_bound(const esp_block* b) {
  if (b->k_masks == 0) return b->rows_per_seq;
  if (b->layout == ESP_LAYOUT_PER_NODE) return b->rows_per_seq / (b->k_masks + 1);
  return std::max(b->rows_per_seq - b->k_masks, 1);
}

hipEvent_t prof_event(esp_ctx* c) {
  if (!c->prof_pool.empty()) {
    hipEvent_t e = c->prof_pool.back();
    c->prof_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

// Times everything enqueued during its lifetime when the site is enabled; otherwise free.  With
// `attach` (a scope around exactly one bf16 GEMM launch) the two events are handed to that launch and
// carry the kernel's own begin and end; a launch that does not take them leaves the span unrecorded.
struct ProfScope {
  esp_ctx* c = nullptr;
  hipEvent_t stop = nullptr;
  bool attached = false;
  ProfScope(esp_ctx* ctx, int site, bool attach = false) {
    if (!((ctx->prof_mask >> site) & 1u)) return;
    hipEvent_t start = prof_event(ctx);
    stop = prof_event(ctx);
    if (!start || !stop) return;
    c = ctx;
    attached = attach;
    if (attach) g_launch_events = LaunchEvents{start, stop};
    else (void)hipEventRecord(start, c->stream);
    c->prof_open.push_back({site, start, stop});
  }
  ~ProfScope() {
    if (!c) return;
    if (attached) g_launch_events = LaunchEvents{};
    else (void)hipEventRecord(stop, c->stream);
  }
};
#define ESP_CAT2(a, b) a##b
#define ESP_CAT(a, b) ESP_CAT2(a, b)
#define ESP_PROF(site) ProfScope ESP_CAT(prof_scope_, __LINE__)(c, site)
#define ESP_PROF_KERNEL(site, attach) ProfScope ESP_CAT(prof_scope_, __LINE__)(c, site, attach)

// sums split-K partials in split order into C
__global__ void k_reduce_splits(const float* __restrict__ part, int splits, size_t n, float* __restrict__ out) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float v = 0.f;
  for (int s = 0; s < splits; ++s) v += part[(size_t)s * n + i];
  out[i] = v;
}

}  // namespace

extern "C" {

const char* esp_status_str(esp_status s) {
  switch (s) {
    case ESP_OK: return "ok";
    case ESP_EINVAL: return "invalid argument";
    case ESP_ESHAPE: return "unsupported shape";
    case ESP_ECAPACITY: return "capacity exceeded";
    case ESP_EDTYPE: return "unsupported dtype";
    case ESP_EDEVICE: return "HIP call failed";
    case ESP_ESTATE: return "bad state";
  }
  return "unknown";
}

size_t esp_workspace_bytes(const esp_model_desc* m, int32_t max_batch, int32_t max_rows, int64_t max_kv_len) {
  if (check_model(m) != ESP_OK || max_batch < 1 || max_rows < 1 || max_rows > ESP_MAX_ROWS_PER_SEQ ||
      max_kv_len < 1)
    return 0;
  return ws_layout(m, max_batch, max_rows, max_kv_len).total;
}

esp_status esp_create(const esp_model_desc* m, const esp_weights* w, int32_t max_batch, int32_t max_rows,
                      int64_t max_kv_len, void* workspace, size_t workspace_bytes, void* stream, esp_ctx** out) {
  if (!out) return ESP_EINVAL;
  *out = nullptr;
  esp_status st = check_model(m);
  if (st != ESP_OK) return st;
  if (!w || !workspace) return ESP_EINVAL;
  if (max_batch < 1 || max_rows < 1 || max_kv_len < 1) return ESP_EINVAL;
  if (max_rows > ESP_MAX_ROWS_PER_SEQ) return ESP_ECAPACITY;
  if (!w->embed || !w->lm_head || !w->final_norm || !w->wqkv || !w->wo || !w->w_gate_up || !w->w_down ||
      !w->norm_attn || !w->norm_mlp)
    return ESP_EINVAL;
  if (m->qk_norm && (!w->q_norm || !w->k_norm)) return ESP_EINVAL;
  if (gemm_prepare() != hipSuccess || attn_prepare() != hipSuccess) return ESP_EDEVICE;
  if (((uintptr_t)workspace) % 256) return ESP_EINVAL;
  for (int l = 0; l < m->n_layers; ++l) {
    if (!w->wqkv[l] || !w->wo[l] || !w->w_gate_up[l] || !w->w_down[l] || !w->norm_attn[l] || !w->norm_mlp[l])
      return ESP_EINVAL;
    if (m->qk_norm && (!w->q_norm[l] || !w->k_norm[l])) return ESP_EINVAL;
  }
  WsLayout L = ws_layout(m, max_batch, max_rows, max_kv_len);
  if (workspace_bytes < L.total) return ESP_ECAPACITY;
  esp_ctx* c = new (std::nothrow) esp_ctx();
  if (!c) return ESP_ESTATE;
  c->m = *m;
  c->embed = w->embed; c->lm_head = w->lm_head; c->final_norm = w->final_norm;
  for (int l = 0; l < m->n_layers; ++l) {
    c->wqkv.push_back(w->wqkv[l]); c->wo.push_back(w->wo[l]); c->wgu.push_back(w->w_gate_up[l]);
    c->wdown.push_back(w->w_down[l]); c->norm_attn.push_back(w->norm_attn[l]);
    c->norm_mlp.push_back(w->norm_mlp[l]);
    c->q_norm.push_back(m->qk_norm ? w->q_norm[l] : nullptr);
    c->k_norm.push_back(m->qk_norm ? w->k_norm[l] : nullptr);
  }
  c->max_batch = max_batch; c->max_rows = max_rows; c->max_kv_len = max_kv_len;
  c->stream = (hipStream_t)stream;
  c->ws = (char*)workspace; c->ws_bytes = workspace_bytes;
  c->h = (float*)(c->ws + L.h); c->xn = c->ws + L.xn; c->q = c->ws + L.q; c->attn_out = c->ws + L.attn_out;
  c->act = c->ws + L.act; c->gemm_out = (float*)(c->ws + L.gemm_out); c->attn_part = (float*)(c->ws + L.attn_part);
  c->rope_tab = (float*)(c->ws + L.rope_tab); c->logits = (float*)(c->ws + L.logits);
  c->topk_scratch = (float*)(c->ws + L.topk_scratch);
  c->idx_a = (int32_t*)(c->ws + L.idx_a); c->idx_b = (int32_t*)(c->ws + L.idx_b);
  c->idx_c = (int32_t*)(c->ws + L.idx_c); c->idx_d = (int32_t*)(c->ws + L.idx_d);
  c->status = (int32_t*)(c->ws + L.status);
  c->gemm_out_floats = L.gemm_out_floats; c->attn_part_floats = L.attn_part_floats; c->logits_rows = L.logits_rows;
  if (hipMemsetAsync(c->status, 0, 256, c->stream) != hipSuccess) {
    delete c;
    return ESP_EDEVICE;
  }
  *out = c;
  return ESP_OK;
}

esp_status esp_destroy(esp_ctx* ctx) {
  if (!ctx) return ESP_EINVAL;
  for (auto& sp : ctx->prof_open) {
    (void)hipEventDestroy(sp.start);
    (void)hipEventDestroy(sp.stop);
  }
  for (auto e : ctx->prof_pool) (void)hipEventDestroy(e);
  delete ctx;
  return ESP_OK;
}

esp_status esp_profile_enable(esp_ctx* ctx, uint32_t site_mask) {
  if (!ctx) return ESP_EINVAL;
  ctx->prof_mask = site_mask & ((1u << ESP_SITE_COUNT) - 1u);
  return ESP_OK;
}

esp_status esp_profile_read(esp_ctx* ctx, int32_t site, int64_t* launches, double* total_ms) {
  if (!ctx || !launches || !total_ms || site < 0 || site >= ESP_SITE_COUNT) return ESP_EINVAL;
  ESP_HIP(hipStreamSynchronize(ctx->stream));
  for (auto& sp : ctx->prof_open) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, sp.start, sp.stop) == hipSuccess) {
      ctx->prof_ms[sp.site] += ms;
      ctx->prof_n[sp.site] += 1;
    }
    ctx->prof_pool.push_back(sp.start);
    ctx->prof_pool.push_back(sp.stop);
  }
  ctx->prof_open.clear();
  *launches = ctx->prof_n[site];
  *total_ms = ctx->prof_ms[site];
  ctx->prof_n[site] = 0;
  ctx->prof_ms[site] = 0.0;
  return ESP_OK;
}

esp_status esp_last_device_status(esp_ctx* ctx, int32_t* host_out) {
  if (!ctx || !host_out) return ESP_EINVAL;
  int32_t v = 0;
  ESP_HIP(hipMemcpyAsync(&v, ctx->status, 4, hipMemcpyDeviceToHost, ctx->stream));
  ESP_HIP(hipStreamSynchronize(ctx->stream));
  *host_out = v;
  if (v) {
    // clear with a small copy of a zero word (no memset node: callers may capture later calls)
    static const int32_t zero = 0;
    ESP_HIP(hipMemcpyAsync(ctx->status, &zero, 4, hipMemcpyHostToDevice, ctx->stream));
    ESP_HIP(hipStreamSynchronize(ctx->stream));
  }
  return ESP_OK;
}

esp_status esp_set_sampling(esp_ctx* c, int32_t enabled, uint32_t seed) {
  if (!c) return ESP_EINVAL;
  c->sample_on = enabled ? 1 : 0;
  c->sample_seed = seed;
  return ESP_OK;
}

esp_status esp_tree_forward(esp_ctx* c, const esp_block* blk, const void* mask_embed, const esp_kv* kv,
                            void* hidden_out, int32_t* node_argmax, float* logits_dbg) {
  if (!c) return ESP_EINVAL;
  esp_status st = check_block(c, blk);
  if (st != ESP_OK) return st;
  st = check_kv(c, kv, blk);
  if (st != ESP_OK) return st;
  if (!hidden_out || (blk->k_masks > 0 && !mask_embed)) return ESP_EINVAL;
  c->lm_cache_hidden = nullptr;     // whatever logits an earlier forward left behind are stale now
  const esp_model_desc& m = c->m;
  const int dt = m.dtype, d = m.d_model, hq = m.n_q_heads, hkv = m.n_kv_heads, hd = m.head_dim, ff = m.d_ff;
  const int nqkv = (hq + 2 * hkv) * hd;
  const int M = blk->batch * blk->rows_per_seq;
  hipStream_t s = c->stream;
  BlockDev bd = to_dev(blk);
  KvDev kd = to_dev(kv);
  const bool pk = dt == ESP_BF16;   // bf16 matrices arrive in the streaming layout

  const GemmPlan p_qkv = gemm_plan(dt, M, nqkv, d);
  const GemmPlan p_o = gemm_plan(dt, M, d, hq * hd);
  const GemmPlan p_gu = gemm_plan(dt, M, 2 * ff, d);
  const GemmPlan p_dn = gemm_plan(dt, M, d, ff);
  if (gemm_out_elems(p_qkv, M, nqkv) > c->gemm_out_floats || gemm_out_elems(p_o, M, d) > c->gemm_out_floats ||
      gemm_out_elems(p_gu, M, 2 * ff) > c->gemm_out_floats || gemm_out_elems(p_dn, M, d) > c->gemm_out_floats)
    return ESP_ECAPACITY;
  const AttnPlan ap = attn_plan(blk->batch, blk->rows_per_seq, hq, hkv, kv->len_bound);
  if (attn_partial_floats(dt, blk->batch, blk->rows_per_seq, hq, hkv, hd, ap.nsplit) > c->attn_part_floats)
    return ESP_ECAPACITY;
  // the LM-head passes below need an unsplit plan (their epilogues see whole rows): refuse before
  // anything is launched, so that no K/V has been appended when the call fails
  if (logits_dbg || node_argmax) {
    const int Mlm = logits_dbg ? M : blk->batch * nodes_bound(blk);
    if (!logits_dbg && (size_t)Mlm > c->logits_rows) return ESP_ECAPACITY;
    if (gemm_plan(dt, Mlm, m.vocab, d).splits != 1) return ESP_ESHAPE;
  }

  { ESP_PROF(ESP_SITE_GLUE);
  ESP_HIP(launch_embed(s, dt, bd, kd, c->embed, mask_embed, c->h, d, m.vocab, c->rope_tab, hd, m.rope_theta,
                       c->status, c->mask_per_seq ? (size_t)blk->k_masks * d : 0));
  ESP_HIP(launch_residual_norm(s, dt, c->h, nullptr, 0, M, d, c->norm_attn[0], m.rms_eps, c->xn)); }
  for (int l = 0; l < m.n_layers; ++l) {
    { ESP_PROF_KERNEL(ESP_SITE_GEMM_LAYER, dt == ESP_BF16);
      ESP_HIP(launch_gemm(s, dt, c->xn, nullptr, c->wqkv[l], c->gemm_out, M, nqkv, d, p_qkv, pk)); }
    { ESP_PROF(ESP_SITE_GLUE);
      ESP_HIP(launch_qkv_post(s, dt, bd, kd, l, c->gemm_out, p_qkv.splits, M, hq, hkv, hd, m.qk_norm, c->q_norm[l],
                              c->k_norm[l], m.rms_eps, c->rope_tab, c->q)); }
    { ESP_PROF(ESP_SITE_ATTN);
      ESP_HIP(launch_attn(s, dt, bd, kd, l, hq, hkv, hd, c->q, c->attn_part, ap)); }
    { ESP_PROF(ESP_SITE_ATTN_MERGE);
      ESP_HIP(launch_attn_merge(s, dt, bd, kd, hq, hkv, hd, c->attn_part, ap, c->attn_out)); }
    { ESP_PROF_KERNEL(ESP_SITE_GEMM_LAYER, dt == ESP_BF16);
      ESP_HIP(launch_gemm(s, dt, c->attn_out, nullptr, c->wo[l], c->gemm_out, M, d, hq * hd, p_o, pk)); }
    { ESP_PROF(ESP_SITE_GLUE);
      ESP_HIP(launch_residual_norm(s, dt, c->h, c->gemm_out, p_o.splits, M, d, c->norm_mlp[l], m.rms_eps, c->xn)); }
    if (dt == ESP_BF16) {   // gate/up projection with the SwiGLU in its epilogue (interleaved weight rows)
      ESP_PROF_KERNEL(ESP_SITE_GEMM_LAYER, true);
      ESP_HIP(launch_gemm_swiglu(s, c->xn, c->wgu[l], c->act, M, ff, d));
    } else {
      { ESP_PROF(ESP_SITE_GEMM_LAYER);
        ESP_HIP(launch_gemm(s, dt, c->xn, nullptr, c->wgu[l], c->gemm_out, M, 2 * ff, d, p_gu, pk)); }
      { ESP_PROF(ESP_SITE_GLUE);
        ESP_HIP(launch_swiglu(s, dt, c->gemm_out, p_gu.splits, M, ff, c->act)); }
    }
    { ESP_PROF_KERNEL(ESP_SITE_GEMM_LAYER, dt == ESP_BF16);
      ESP_HIP(launch_gemm(s, dt, c->act, nullptr, c->wdown[l], c->gemm_out, M, d, ff, p_dn, pk)); }
    const bool last = l + 1 == m.n_layers;
    { ESP_PROF(ESP_SITE_GLUE);
      ESP_HIP(launch_residual_norm(s, dt, c->h, c->gemm_out, p_dn.splits, M, d,
                                   last ? c->final_norm : c->norm_attn[l + 1], m.rms_eps, last ? hidden_out : c->xn)); }
  }
  // LM head + argmax at the tree rows (Sec. 2 Eq. 3 needs the base model's own next token there)
  if (logits_dbg) {
    const GemmPlan p_lm = gemm_plan(dt, M, m.vocab, d);
    if (p_lm.splits != 1) return ESP_ESHAPE;
    { ESP_PROF(ESP_SITE_LM_HEAD);
      ESP_HIP(launch_gemm(s, dt, hidden_out, nullptr, c->lm_head, logits_dbg, M, m.vocab, d, p_lm, pk)); }
    if (node_argmax) {
      const int nb = nodes_bound(blk);
      ESP_PROF(ESP_SITE_GLUE);
      ESP_HIP(launch_node_rows(s, bd, nb, c->idx_a, c->idx_b, kd.len, c->idx_d));
      ESP_HIP(launch_argmax(s, logits_dbg, (size_t)m.vocab, c->idx_a, blk->batch * nb, m.vocab, node_argmax,
                            c->idx_b, c->sample_on ? c->idx_d : nullptr, c->sample_seed));
    }
  } else if (node_argmax) {
    const int nb = nodes_bound(blk);
    const int Mn = blk->batch * nb;
    if ((size_t)Mn > c->logits_rows) return ESP_ECAPACITY;
    const GemmPlan p_lm = gemm_plan(dt, Mn, m.vocab, d);
    if (p_lm.splits != 1) return ESP_ESHAPE;
    const int32_t* draw_list = c->sample_on ? c->idx_d : nullptr;   // draw positions per node-list entry
    { ESP_PROF(ESP_SITE_GLUE);
      ESP_HIP(launch_node_rows(s, bd, nb, c->idx_a, c->idx_b, kd.len, c->idx_d));
      if (c->sample_on) ESP_HIP(launch_row_positions(s, bd, kd.len, c->idx_c)); }
    if (blk->k_masks > 0 && gemm_argmax_supported(dt, M, m.vocab, d, true) && (size_t)M <= c->logits_rows &&
        gemm_argmax_scratch_floats(M, m.vocab) <= c->gemm_out_floats) {
      // few rows (<= 128): one pass over the LM head for all block rows.  The tree rows get their
      // arg-max from the epilogue; the logits of every row stay in the workspace, where
      // esp_mask_topk on these hidden states finds its mask rows without a second pass over the
      // 2*vocab*d_model bytes of the matrix.
      ESP_PROF(ESP_SITE_LM_HEAD);
      ESP_HIP(launch_gemm_argmax(s, hidden_out, nullptr, c->lm_head, M, m.vocab, d, c->gemm_out, node_argmax,
                                 c->idx_b, 0, c->logits, c->idx_a, Mn, c->sample_on ? c->idx_c : nullptr,
                                 c->sample_seed));
      c->lm_cache_hidden = hidden_out;
      c->lm_cache_rows = M;
    } else if (gemm_argmax_supported(dt, Mn, m.vocab, d, false) &&
        gemm_argmax_scratch_floats(Mn, m.vocab) <= c->logits_rows * (size_t)m.vocab) {
      // arg-max in the GEMM epilogue: the [rows, vocab] logits are never written
      ESP_PROF(ESP_SITE_LM_HEAD);
      ESP_HIP(launch_gemm_argmax(s, hidden_out, c->idx_a, c->lm_head, Mn, m.vocab, d, c->logits, node_argmax,
                                 c->idx_b, 0, nullptr, nullptr, Mn, draw_list, c->sample_seed));
    } else {
      { ESP_PROF(ESP_SITE_LM_HEAD);
        ESP_HIP(launch_gemm(s, dt, hidden_out, c->idx_a, c->lm_head, c->logits, Mn, m.vocab, d, p_lm, pk)); }
      { ESP_PROF(ESP_SITE_GLUE);
        ESP_HIP(launch_argmax(s, c->logits, (size_t)m.vocab, nullptr, Mn, m.vocab, node_argmax, c->idx_b, draw_list,
                              c->sample_seed)); }
    }
  }
  return ESP_OK;
}

esp_status esp_verify_accept(esp_ctx* c, const esp_block* blk, const int32_t* node_argmax, const esp_kv* kv,
                             int32_t* n_emit, int32_t* emit_tok, int32_t* accepted_row, int32_t* star_row) {
  if (!c) return ESP_EINVAL;
  esp_status st = check_block(c, blk);
  if (st != ESP_OK) return st;
  st = check_kv(c, kv, blk);
  if (st != ESP_OK) return st;
  if (!node_argmax || !n_emit || !emit_tok || !accepted_row || !star_row) return ESP_EINVAL;
  ESP_PROF(ESP_SITE_TREE);
  ESP_HIP(launch_verify_accept(c->stream, c->m.dtype, to_dev(blk), to_dev(kv), node_argmax, c->m.n_layers,
                               c->m.n_kv_heads, c->m.head_dim, n_emit, emit_tok, accepted_row, star_row,
                               c->status));
  return ESP_OK;
}

esp_status esp_mask_topk(esp_ctx* c, const esp_block* blk, const int32_t* star_row, const int32_t* n_emit,
                         const void* hidden, int32_t Kp, int32_t* topk_id, float* topk_p, int32_t* n_lists,
                         float* logits_out) {
  if (!c) return ESP_EINVAL;
  esp_status st = check_block(c, blk);
  if (st != ESP_OK) return st;
  if (!star_row || !n_emit || !hidden || !topk_id || !topk_p || !n_lists) return ESP_EINVAL;
  if (Kp < 1 || Kp > ESP_MAX_TOPK || Kp > c->m.vocab || blk->k_masks < 1) return ESP_EINVAL;
  const esp_model_desc& m = c->m;
  const int rows = blk->batch * blk->k_masks;
  hipStream_t s = c->stream;
  BlockDev bd = to_dev(blk);
  { ESP_PROF(ESP_SITE_TREE);
    ESP_HIP(launch_mask_rows(s, bd, star_row, n_emit, c->idx_a, n_lists)); }
  if (!logits_out && c->lm_cache_hidden == hidden && c->lm_cache_rows == blk->batch * blk->rows_per_seq) {
    // the forward that produced `hidden` left the logits of all its rows in the workspace
    ESP_PROF(ESP_SITE_TOPK);
    ESP_HIP(launch_softmax_topk(s, c->logits, rows, m.vocab, Kp, topk_id, topk_p, c->topk_scratch, c->idx_a));
    return ESP_OK;
  }
  c->lm_cache_hidden = nullptr;          // c->logits is about to be overwritten
  const GemmPlan p_lm = gemm_plan(m.dtype, rows, m.vocab, m.d_model);
  if (p_lm.splits != 1) return ESP_ESHAPE;
  float* lg = logits_out ? logits_out : c->logits;
  { ESP_PROF(ESP_SITE_LM_HEAD);
    ESP_HIP(launch_gemm(s, m.dtype, hidden, c->idx_a, c->lm_head, lg, rows, m.vocab, m.d_model, p_lm, m.dtype == ESP_BF16)); }
  { ESP_PROF(ESP_SITE_TOPK);
    ESP_HIP(launch_softmax_topk(s, lg, rows, m.vocab, Kp, topk_id, topk_p, c->topk_scratch)); }
  return ESP_OK;
}

esp_status esp_build_prune_tree(esp_ctx* c, const esp_tree_params* p, const int32_t* topk_id, const float* topk_p,
                                int32_t Kp, const int32_t* n_lists, const int32_t* n_emit, const int32_t* emit_tok,
                                esp_block* next) {
  if (!c || !p) return ESP_EINVAL;
  esp_status st = check_block(c, next);
  if (st != ESP_OK) return st;
  if (!topk_id || !topk_p || !n_lists || !n_emit || !emit_tok) return ESP_EINVAL;
  if (p->B < 1 || p->B > ESP_MAX_TREE_NODES || p->k < 1 || p->k > ESP_MAX_MASKS || p->K < 1 || Kp < 1 ||
      Kp > ESP_MAX_TOPK)
    return ESP_EINVAL;
  if (p->k != next->k_masks || p->layout != next->layout) return ESP_EINVAL;
  int nodes = p->B;
  if (p->static_widths[0] > 0) {
    if (p->expand_width != 1) return ESP_EINVAL;
    nodes = 1;
    for (int i = 0; i < p->k; ++i) {
      if (p->static_widths[i] < 1 || p->static_widths[i] > Kp) return ESP_EINVAL;
      nodes += p->static_widths[i];
    }
    if (nodes > ESP_MAX_TREE_NODES) return ESP_ECAPACITY;
  }
  const int rows = p->layout == ESP_LAYOUT_PER_NODE ? nodes * (p->k + 1) : nodes + p->k;
  if (rows > next->rows_per_seq) return ESP_ECAPACITY;
  // candidates Alg. 1 can create: depth i expands at most min(width, B-i+1) nodes by min(K, B-i, Kp)
  {
    long long total = 1, prev = 1;
    for (int i = 1; i <= p->k; ++i) {
      long long ex = std::min<long long>(prev, std::max(p->B - i + 1, 1));
      if (p->expand_width > 0) ex = std::min<long long>(ex, p->expand_width);
      long long ch = p->static_widths[0] > 0 ? p->static_widths[i - 1] : std::min(std::min(p->K, Kp), std::max(p->B - i, 0));
      prev = ex * ch;
      total += prev;
    }
    if (total > 4096) return ESP_ECAPACITY;
  }
  // a fixed tree's rows are built once per block: later calls with the same parameters on the
  // same block only write its tokens (the kernel still checks, per sequence, that the block
  // holds a tree of that size and that every list is there, and builds in full otherwise)
  bool reuse = false;
  uint64_t sig = 0;
  if (p->static_widths[0] > 0) {
    sig = 0x9E3779B97F4A7C15ull;
    auto mix = [&](uint64_t v) { sig = (sig ^ v) * 0x100000001B3ull; };
    mix((uint64_t)p->k); mix((uint64_t)p->layout); mix((uint64_t)p->prune_parent); mix((uint64_t)p->prune_last);
    mix((uint64_t)Kp); mix((uint64_t)next->batch); mix((uint64_t)next->rows_per_seq);
    for (int i = 0; i < p->k; ++i) mix((uint64_t)p->static_widths[i]);
  }
  esp_ctx::StaticTreeSlot* slot = nullptr;
  for (auto& sl : c->static_trees)
    if (sl.tok == next->tok) slot = &sl;
  if (p->static_widths[0] > 0) {
    reuse = slot && slot->sig == sig;
    if (!slot) {   // take a free slot, else the first one
      slot = &c->static_trees[0];
      for (auto& sl : c->static_trees)
        if (!sl.tok) { slot = &sl; break; }
    }
    slot->tok = next->tok;
    slot->sig = sig;
  } else if (slot) {
    slot->tok = nullptr;      // a dynamic tree overwrites the block's rows
  }
  ESP_PROF(ESP_SITE_TREE);
  ESP_HIP(launch_build_tree(c->stream, *p, next->batch, topk_id, topk_p, Kp, n_lists, n_emit, emit_tok,
                            next->rows_per_seq, next->anc_words, next->n_rows, next->n_nodes, next->tok,
                            next->parent, next->depth, next->mask_j, next->attach, next->anc, c->status, reuse));
  return ESP_OK;
}

esp_status esp_block_from_tree(esp_ctx* c, esp_block* blk) {
  if (!c) return ESP_EINVAL;
  esp_status st = check_block(c, blk);
  if (st != ESP_OK) return st;
  for (auto& sl : c->static_trees)
    if (sl.tok == blk->tok) sl.tok = nullptr;     // the block's rows are rewritten
  ESP_HIP(launch_block_from_tree(c->stream, blk->batch, blk->rows_per_seq, blk->k_masks, blk->layout, blk->anc_words,
                                 blk->n_rows, blk->n_nodes, blk->tok, blk->parent, blk->depth, blk->mask_j,
                                 blk->attach, blk->anc, c->status));
  return ESP_OK;
}

esp_status esp_mask_mean(esp_ctx* c, const int32_t* tokens, int32_t n_tokens, int32_t k, void* mask_embed) {
  if (!c || !tokens || !mask_embed || n_tokens < 1 || k < 1 || k > ESP_MAX_MASKS) return ESP_EINVAL;
  ESP_HIP(launch_mask_mean(c->stream, c->m.dtype, c->embed, tokens, n_tokens, k, c->m.d_model, c->m.vocab,
                           mask_embed));
  return ESP_OK;
}

esp_status esp_mask_last_k(esp_ctx* c, const int32_t* tokens, int32_t n_tokens, int32_t k, void* mask_embed) {
  if (!c || !tokens || !mask_embed || k < 1 || k > ESP_MAX_MASKS || n_tokens < k) return ESP_EINVAL;
  ESP_HIP(launch_mask_last_k(c->stream, c->m.dtype, c->embed, tokens, n_tokens, k, c->m.d_model, c->m.vocab,
                             mask_embed));
  return ESP_OK;
}

esp_status esp_mask_gaussian(esp_ctx* c, const float* z, float shift, int32_t k, void* mask_embed) {
  if (!c || !mask_embed || k < 1 || k > ESP_MAX_MASKS) return ESP_EINVAL;
  // the statistics use the logits buffer as scratch: whatever esp_tree_forward left there for
  // esp_mask_topk is gone
  const size_t room = c->logits_rows * (size_t)c->m.vocab;
  if (room < mask_gaussian_scratch_floats(c->m.d_model)) return ESP_ECAPACITY;
  c->lm_cache_hidden = nullptr;
  c->lm_cache_rows = 0;
  ESP_HIP(launch_mask_gaussian(c->stream, c->m.dtype, c->embed, c->m.vocab, c->m.d_model, z, shift, k, c->logits, room,
                               mask_embed));
  return ESP_OK;
}

esp_status esp_mask_ema(esp_ctx* c, const int32_t* n_emit, const int32_t* emit_tok, float lambda, int32_t k,
                        void* mask_embed) {
  if (!c || !n_emit || !emit_tok || !mask_embed || k < 1 || k > ESP_MAX_MASKS) return ESP_EINVAL;
  ESP_HIP(launch_mask_ema(c->stream, c->m.dtype, c->embed, n_emit, emit_tok, lambda, k, c->m.d_model, c->m.vocab,
                          mask_embed, 1));
  return ESP_OK;
}

esp_status esp_set_mask_batch(esp_ctx* c, int32_t per_sequence) {
  if (!c) return ESP_EINVAL;
  c->mask_per_seq = per_sequence != 0;
  return ESP_OK;
}

esp_status esp_mask_ema_batch(esp_ctx* c, int32_t batch, const int32_t* n_emit, const int32_t* emit_tok, float lambda,
                              int32_t k, void* mask_embed) {
  if (!c || !n_emit || !emit_tok || !mask_embed || k < 1 || k > ESP_MAX_MASKS) return ESP_EINVAL;
  if (batch < 1 || batch > c->max_batch) return ESP_EINVAL;
  ESP_HIP(launch_mask_ema(c->stream, c->m.dtype, c->embed, n_emit, emit_tok, lambda, k, c->m.d_model, c->m.vocab,
                          mask_embed, batch));
  return ESP_OK;
}

static esp_status kv_copy(esp_ctx* c, const esp_kv* kv, int layer, int seq_base, int first_slot, int n_slots,
                          void* k_rows, void* v_rows, int to_cache) {
  if (!c || !kv || !kv->k || !kv->v || !k_rows || !v_rows) return ESP_EINVAL;
  if (layer < 0 || layer >= c->m.n_layers || seq_base < 0 || first_slot < 0 || n_slots < 0) return ESP_EINVAL;
  if (kv->capacity < 64 || kv->capacity % 64) return ESP_EINVAL;
  if ((int64_t)seq_base + first_slot + n_slots > kv->capacity) return ESP_ECAPACITY;
  KvDev kd;
  kd.k = kv->k; kd.v = kv->v; kd.len = kv->len; kd.base = kv->base; kd.seq_cap = kv->seq_cap;
  kd.capacity = kv->capacity; kd.len_bound = kv->len_bound;
  ESP_HIP(launch_kv_copy(c->stream, c->m.dtype, kd, layer, c->m.n_kv_heads, c->m.head_dim, seq_base, first_slot,
                         n_slots, k_rows, v_rows, to_cache));
  return ESP_OK;
}

esp_status esp_kv_store(esp_ctx* c, const esp_kv* kv, int32_t layer, int32_t seq_base, int32_t first_slot,
                        int32_t n_slots, const void* k_rows, const void* v_rows) {
  return kv_copy(c, kv, layer, seq_base, first_slot, n_slots, const_cast<void*>(k_rows), const_cast<void*>(v_rows),
                 1);
}

esp_status esp_kv_load(esp_ctx* c, const esp_kv* kv, int32_t layer, int32_t seq_base, int32_t first_slot,
                       int32_t n_slots, void* k_rows, void* v_rows) {
  return kv_copy(c, kv, layer, seq_base, first_slot, n_slots, k_rows, v_rows, 0);
}

size_t esp_gemm_scratch_bytes(int32_t M, int32_t N, int32_t K) {
  if (M < 1 || N < 1 || K < 1) return 0;
  GemmPlan p = gemm_plan(ESP_BF16, M, N, K);
  return gemm_out_elems(p, M, N) * 4 + 256;
}

esp_status esp_pack_weight(void* stream, const void* src, void* dst, int32_t N, int32_t K) {
  if (!src || !dst || src == dst) return ESP_EINVAL;
  if (N < 32 || K < 64 || N % 32 || K % 64) return ESP_ESHAPE;
  ESP_HIP(launch_pack_weight((hipStream_t)stream, src, dst, N, K));
  return ESP_OK;
}

esp_status esp_gemm(void* stream, int32_t dtype, const void* A, const void* W, int32_t w_packed, float* C, int32_t M,
                    int32_t N, int32_t K, void* partials, size_t partial_bytes) {
  if (!A || !W || !C || M < 1 || N < 1 || K < 1) return ESP_EINVAL;
  if (dtype != ESP_F32 && dtype != ESP_BF16) return ESP_EDTYPE;
  if (dtype == ESP_BF16 && (N % 32 || K % 64)) return ESP_ESHAPE;
  if (w_packed && dtype != ESP_BF16) return ESP_EDTYPE;
  GemmPlan p = gemm_plan(dtype, M, N, K);
  hipStream_t s = (hipStream_t)stream;
  if (p.splits == 1) {
    ESP_HIP(launch_gemm(s, dtype, A, nullptr, W, C, M, N, K, p, w_packed != 0));
    return ESP_OK;
  }
  if (!partials || partial_bytes < gemm_out_elems(p, M, N) * 4) return ESP_ECAPACITY;
  ESP_HIP(launch_gemm(s, dtype, A, nullptr, W, (float*)partials, M, N, K, p, w_packed != 0));
  size_t n = (size_t)M * N;
  hipLaunchKernelGGL(k_reduce_splits, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (const float*)partials,
                     p.splits, n, C);
  ESP_HIP(hipGetLastError());
  return ESP_OK;
}

size_t esp_gemm_argmax_scratch_bytes(int32_t M, int32_t N) {
  if (M < 1 || N < 1) return 0;
  return gemm_argmax_scratch_floats(M, N) * 4;
}

esp_status esp_gemm_argmax(void* stream, const void* A, const void* W, int32_t M, int32_t N, int32_t K, void* scratch,
                           size_t scratch_bytes, int32_t* argmax) {
  if (!A || !W || !argmax || M < 1 || N < 1 || K < 1) return ESP_EINVAL;
  if (N % 32 || K % 64) return ESP_ESHAPE;
  if (!gemm_argmax_supported(ESP_BF16, M, N, K, false)) return ESP_ESHAPE;
  if (!scratch || scratch_bytes < gemm_argmax_scratch_floats(M, N) * 4) return ESP_ECAPACITY;
  ESP_HIP(launch_gemm_argmax((hipStream_t)stream, A, nullptr, W, M, N, K, (float*)scratch, argmax, nullptr, 0, nullptr,
                             nullptr, M, nullptr, 0u));
  return ESP_OK;
}

esp_status esp_attn_tree(esp_ctx* c, const esp_block* blk, const esp_kv* kv, int32_t layer, const void* q,
                         void* out) {
  if (!c || !q || !out) return ESP_EINVAL;
  esp_status st = check_block(c, blk);
  if (st != ESP_OK) return st;
  st = check_kv(c, kv, blk);
  if (st != ESP_OK) return st;
  if (layer < 0 || layer >= c->m.n_layers) return ESP_EINVAL;
  const esp_model_desc& m = c->m;
  const AttnPlan ap = attn_plan(blk->batch, blk->rows_per_seq, m.n_q_heads, m.n_kv_heads, kv->len_bound);
  if (attn_partial_floats(m.dtype, blk->batch, blk->rows_per_seq, m.n_q_heads, m.n_kv_heads, m.head_dim, ap.nsplit) >
      c->attn_part_floats)
    return ESP_ECAPACITY;
  { ESP_PROF(ESP_SITE_ATTN);
    ESP_HIP(launch_attn(c->stream, m.dtype, to_dev(blk), to_dev(kv), layer, m.n_q_heads, m.n_kv_heads, m.head_dim, q,
                        c->attn_part, ap)); }
  { ESP_PROF(ESP_SITE_ATTN_MERGE);
    ESP_HIP(launch_attn_merge(c->stream, m.dtype, to_dev(blk), to_dev(kv), m.n_q_heads, m.n_kv_heads, m.head_dim, c->attn_part, ap,
                              out)); }
  return ESP_OK;
}

size_t esp_softmax_topk_scratch_bytes(int32_t rows, int32_t vocab, int32_t Kp) {
  if (rows < 1 || vocab < 1 || Kp < 1) return 0;
  return softmax_topk_scratch_floats(rows, vocab, Kp) * 4;
}

esp_status esp_softmax_topk(void* stream, const float* logits, int32_t rows, int32_t vocab, int32_t Kp,
                            int32_t* ids, float* probs, void* scratch, size_t scratch_bytes) {
  if (!logits || !ids || !probs || !scratch) return ESP_EINVAL;
  if (rows < 1 || vocab < 1 || Kp < 1 || Kp > ESP_MAX_TOPK || Kp > vocab) return ESP_EINVAL;
  if (scratch_bytes < esp_softmax_topk_scratch_bytes(rows, vocab, Kp)) return ESP_ECAPACITY;
  ESP_HIP(launch_softmax_topk((hipStream_t)stream, logits, rows, vocab, Kp, ids, probs, (float*)scratch));
  return ESP_OK;
}

}  // extern "C"
