// Host side of libvvs: argument validation, buffer planning, tree tables and the C ABI entry
// points.  Everything here runs before any launch, so bad input never reaches a kernel.
#include "vvs_internal.h"

#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <algorithm>
#include <cmath>
#include <vector>

namespace vvs {

static std::string g_last_error;   // for failures that have no context (query / create)

static vvs_status fail(std::string* err, vvs_status st, const std::string& msg) {
  if (err) *err = msg;
  g_last_error = msg;
  return st;
}

GemmPlan plan_gemm(const Ctx* c, int M, int N, int K) {
  GemmPlan p{64, 64, 1};
  if (c->cfg.dtype != VVS_BF16) return p;           // fp32 path: one wave per output column, no split
  // bf16: 64 x 64 output tiles (32 x 64 for up to 32 rows); every workgroup already splits its K range
  // over its 4 waves.  Add grid-level K splits until there is about one workgroup per CU, keeping at
  // least 8 k-steps of 16 per wave.
  p.bm = M <= 32 ? 32 : 64;
  // 128 x 128 tiles with the operands shared through LDS when that still gives most CUs a workgroup:
  // half the operand bytes per MFMA come through a CU's L1
  if (M > 192 && N % 128 == 0 && K % 32 == 0 && ((M + 127) / 128) * (N / 128) >= 160) { p.bm = p.bn = 128; return p; }
  // 64 x 128 tiles when they give one workgroup for (nearly) every CU and no second round: a CU then
  // pulls (64 + 128) K-rows through its L1 instead of 2 x (64 + 64)
  if (p.bm == 64 && N % 128 == 0) {
    const int t128 = ((M + 63) / 64) * (N / 128);
    if (t128 >= 160 && t128 <= 256) { p.bn = 128; return p; }
  }
  // up to 32 rows (weight streaming): 32 x 128 tiles under the same condition - with 64-column tiles such an
  // N gives between one and two workgroups per CU, and the kernel lasts as long as the CUs that got two
  if (p.bm == 32 && N % 128 == 0 && N / 128 >= 160 && N / 128 <= 256) { p.bn = 128; return p; }
  const int tiles = ((M + p.bm - 1) / p.bm) * (N / 64);
  const int kb = K / 16;
  int splits = 1;
  if (tiles < 256) {
    splits = std::min({(256 + tiles - 1) / tiles, 8, std::max(1, kb / 32)});
    const int per = (kb + splits - 1) / splits;
    splits = (kb + per - 1) / per;
  }
  p.splits = splits;
  return p;
}

// The fused layer (5 kernels, no separate normalisation) is taken when a layer's weights are so small (below
// ~48 MB: the B and XL widths, a drafter) that a launch costs more than streaming them: then fewer launches
// win.  Wide layers stream their weights through K-split GEMMs with separate normalisation kernels, which
// also round the norm's output where the definition does: the other placement costs more accuracy the wider
// the layer is (measured without any kernel: 2 x the noise floor of a correct bf16 evaluation at d = 1280,
// 3 x at d = 4096).
bool plan_fused(const Ctx* c, int M) {
  (void)M;
  if (c->cfg.dtype != VVS_BF16 || c->cfg.norm_mode == VVS_NORM_SEPARATE) return false;
  const size_t layer_weight_bytes = c->esz * ((size_t)4 * c->d * c->d + (size_t)3 * c->d * c->F);
  return layer_weight_bytes <= ((size_t)48 << 20);
}

vvs_status plan_sizes(const vvs_config* cfg, Ctx* c, std::string* err) {
  if (!cfg) return fail(err, VVS_EINVAL, "config is NULL");
  const vvs_config& g = *cfg;
  if (g.n_layers < 1 || g.d_model < 4 || g.n_heads < 1 || g.d_ff < 1 || g.vocab < 1 || g.n_prompts < 1 ||
      g.grid_h < 1 || g.grid_w < 1 || g.prefix_len < 1 || g.max_nodes < 0)
    return fail(err, VVS_EINVAL, "config: a dimension is not positive");
  if (g.d_model % g.n_heads) return fail(err, VVS_EINVAL, "config: d_model is not a multiple of n_heads");
  if (g.logit_lo < 0 || g.logit_hi > g.vocab || g.logit_lo >= g.logit_hi)
    return fail(err, VVS_EINVAL, "config: logit slice must satisfy 0 <= lo < hi <= vocab");
  if (g.dtype != VVS_FP32 && g.dtype != VVS_BF16) return fail(err, VVS_EINVAL, "config: unknown dtype");
  if (g.prefix_kind != VVS_PREFIX_CLASS && g.prefix_kind != VVS_PREFIX_DENSE)
    return fail(err, VVS_EINVAL, "config: unknown prefix_kind");
  if (g.prefix_kind == VVS_PREFIX_CLASS && g.n_classes < 1) return fail(err, VVS_EINVAL, "config: n_classes < 1");
  if (g.max_nodes > VVS_MAX_T - 1) return fail(err, VVS_ESIZE, "config: max_nodes exceeds VVS_MAX_T - 1");
  if (g.relax_k < 0 || g.relax_k > 64) return fail(err, VVS_ESIZE, "config: relax_k must be in [0, 64]");
  if (!(g.relax_delta >= 0.f)) return fail(err, VVS_EINVAL, "config: relax_delta < 0");
  if (!(g.rms_eps > 0.f) || !(g.rope_base > 1.f)) return fail(err, VVS_EINVAL, "config: rms_eps / rope_base");
  if (g.feature_slots < 0 || g.feature_slots > VVS_MAX_FEATURE_SLOTS)
    return fail(err, VVS_ESIZE, "config: feature_slots must be in [0, VVS_MAX_FEATURE_SLOTS]");
  if (g.feature_pre_norm != 0 && g.feature_pre_norm != 1) return fail(err, VVS_EINVAL, "config: feature_pre_norm must be 0 or 1");
  if (g.draft_input != 0 && g.draft_input != 1) return fail(err, VVS_EINVAL, "config: draft_input must be 0 or 1");
  if (g.norm_mode != VVS_NORM_AUTO && g.norm_mode != VVS_NORM_SEPARATE) return fail(err, VVS_EINVAL, "config: unknown norm_mode");
  int dh = g.d_model / g.n_heads;
  if (dh % 4) return fail(err, VVS_ESIZE, "config: head size must be a multiple of 4 (2D rotary pairs)");
  if (g.d_model % 8 || g.d_ff % 8) return fail(err, VVS_ESIZE, "config: d_model and d_ff must be multiples of 8");
  if (g.d_model > 16384) return fail(err, VVS_ESIZE, "config: d_model above 16384 is not supported");
  if (dh > 256) return fail(err, VVS_ESIZE, "config: head size above 256 is not supported");
  int veff = g.logit_hi - g.logit_lo;
  if (g.dtype == VVS_BF16) {
    if (g.d_model % 64 || g.d_ff % 64 || veff % 64)
      return fail(err, VVS_ESIZE, "config: bf16 needs d_model, d_ff and the logit slice width to be multiples of 64");
    if (dh != 64 && dh != 128) return fail(err, VVS_ESIZE, "config: bf16 needs head size 64 or 128");
    if (dh == 128 && g.max_nodes > 31) return fail(err, VVS_ESIZE, "config: bf16 with head size 128 supports max_nodes <= 31");
  }
  c->cfg = g;
  c->B = g.n_prompts; c->R = 2 * g.n_prompts; c->d = g.d_model; c->H = g.n_heads; c->dh = dh; c->F = g.d_ff;
  c->L = g.n_layers; c->V = g.vocab; c->lo = g.logit_lo; c->veff = veff; c->P = g.prefix_len;
  c->G = g.grid_h * g.grid_w; c->Tmax = g.max_nodes + 1;
  c->chunk = (dh > 64) ? 32 : 64;
  c->Mmax = (int)align_up((size_t)c->R * std::max(c->Tmax, c->chunk), 32);   // packed operands come in 32-row blocks
  c->Mlog = (int)align_up((size_t)c->R * c->Tmax, 32);
  c->S_cap = (int)align_up((size_t)c->P + c->G + VVS_MAX_T, 32);
  c->rope_pos = std::max(g.grid_h + VVS_MAX_T / g.grid_w + 2, g.grid_w);
  c->esz = g.dtype == VVS_BF16 ? 2 : 4;
  // KV cache: K [L][R][H][S_cap][dh], then V [L][R][H][S_cap/32][dh][32]
  c->kv_head_stride = (size_t)c->S_cap * dh;
  c->kv_row_stride = c->kv_head_stride * c->H;
  c->kv_layer_stride = c->kv_row_stride * c->R;
  c->kv_v_off = c->kv_layer_stride * c->L;
  // GEMM partial-sum buffer: worst case over every M this context can be asked for
  size_t go = 0;
  int d = c->d, F = c->F;
  const int shapes[5][2] = {{3 * d, d}, {d, d}, {2 * F, d}, {d, F}, {d, 2 * d}};   // the last one: a drafter's input map
  for (int M = 1; M <= c->Mmax; ++M)
    for (auto& sh : shapes) {
      if (sh[1] == 2 * d && !g.draft_input) continue;
      GemmPlan p = plan_gemm(c, M, sh[0], sh[1]);
      go = std::max(go, (size_t)p.splits * M * sh[0]);
    }
  c->gemm_out_elems = go;
  // workspace carve-up
  Workspace& w = c->w;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  w.state = take(sizeof(int32_t) * 3 * c->B);
  w.ring_state = take(sizeof(int32_t) * 2 * c->R);        // per row: features held, slot of the oldest (zeroed with the state)
  w.outcome = take(sizeof(int32_t) * c->B * (2 + VVS_MAX_T));
  w.node_result = take(sizeof(int32_t) * c->B * VVS_MAX_T * 2);
  w.tokens = take(sizeof(int32_t) * c->B * VVS_MAX_T);
  w.rope_tab = take(sizeof(float) * 2 * c->rope_pos * (dh / 4));
  w.x = take(sizeof(float) * (size_t)c->Mmax * d);
  w.h = take(c->esz * (size_t)c->Mmax * d);
  w.gemm_out = take(sizeof(float) * go);
  w.q = take(c->esz * (size_t)c->Mmax * d);
  w.attn = take(c->esz * (size_t)c->Mmax * d);
  w.act = take(c->esz * (size_t)c->Mmax * F);
  w.hf = take(c->esz * (size_t)c->Mlog * d);
  w.logits = take(sizeof(float) * (size_t)c->Mlog * veff);
  w.probs = take(sizeof(float) * (size_t)c->B * c->Tmax * veff);
  w.pq_work = take(sizeof(float) * (size_t)c->B * c->Tmax * 2 * veff);
  w.ss = take(sizeof(float) * (size_t)c->Mmax * (((d + 63) / 64 + 3) & ~3));     // per-row, per-64-column sums of squares of the residual
  w.ss2 = take(sizeof(float) * (size_t)c->Mlog * (((d + 63) / 64 + 3) & ~3));
  w.ring = take(c->esz * (size_t)c->R * std::max(g.feature_slots, 1) * d);
  w.din = take(g.draft_input ? c->esz * (size_t)c->Mmax * 2 * d : 0);                // drafter: [embedding ; feature] rows
  w.total = off;
  // packed weights
  PackedLayout& p = c->p;
  off = 0;
  size_t e = c->esz;
  p.embed = take(e * (size_t)c->V * d);
  p.prefix_embed = take(e * (size_t)(g.n_classes + 1) * d);
  p.gf = take(sizeof(float) * d);
  p.wout = take(e * (size_t)veff * d);
  p.layer0 = off;
  size_t base = off;
  p.g1 = take(sizeof(float) * d) - base;
  p.wqkv = take(e * (size_t)3 * d * d) - base;
  p.wo = take(e * (size_t)d * d) - base;
  p.g2 = take(sizeof(float) * d) - base;
  p.wgu = take(e * (size_t)2 * F * d) - base;
  p.wd = take(e * (size_t)d * F) - base;
  p.layer_stride = off - base;
  off = p.layer0 + p.layer_stride * c->L;
  p.fc = take(g.draft_input ? e * (size_t)2 * d * d : 0);
  p.total = off;
  return VVS_OK;
}

// Validates the topology and fills the kernel-side tables.
vvs_status build_tree(int n_nodes, const int32_t* h_parent, const uint8_t* h_mask, TreeDesc* t, std::string* err) {
  if (n_nodes < 0 || n_nodes > VVS_MAX_T - 1) return fail(err, VVS_ESIZE, "tree: n_nodes out of range");
  const int T = n_nodes + 1;
  std::vector<int> par(T, -1);
  if (h_parent) {
    for (int j = 1; j < T; ++j) {
      int p = h_parent[j - 1];
      if (p < 0 || p > j - 1) return fail(err, VVS_EINVAL, "tree: parent of node j must lie in [0, j-1]");
      par[j] = p;
    }
  } else if (h_mask) {
    // the parent is the closest proper ancestor = the largest index among them
    for (int j = 1; j < T; ++j) {
      int p = -1;
      for (int i = 0; i < j; ++i) if (h_mask[(size_t)j * T + i]) p = i;
      if (p < 0) return fail(err, VVS_EINVAL, "tree mask: a node does not see the root");
      par[j] = p;
    }
  } else {
    for (int j = 1; j < T; ++j) par[j] = j - 1;
  }
  memset(t, 0, sizeof(*t));
  t->T = T;
  bool chain = true;
  for (int j = 0; j < VVS_MAX_T; ++j) { t->parent[j] = -1; t->first_child[j] = -1; t->next_sibling[j] = -1; }
  std::vector<int> last_child(T, -1);
  for (int j = 0; j < T; ++j) {
    uint64_t m = 1ull << j;
    if (j) {
      t->parent[j] = (int8_t)par[j];
      t->depth[j] = (int8_t)(t->depth[par[j]] + 1);
      m |= t->anc[par[j]];
      if (par[j] != j - 1) chain = false;
      if (last_child[par[j]] < 0) t->first_child[par[j]] = (int8_t)j;
      else t->next_sibling[last_child[par[j]]] = (int8_t)j;
      last_child[par[j]] = j;
    }
    t->anc[j] = m;
  }
  t->causal = chain ? 1 : 0;
  if (h_mask) {
    for (int i = 0; i < T; ++i)
      for (int j = 0; j < T; ++j) {
        bool want = (t->anc[i] >> j) & 1ull;
        if ((h_mask[(size_t)i * T + j] != 0) != want)
          return fail(err, VVS_EINVAL, "tree mask is not the ancestor-or-self closure of the parent array");
      }
  }
  return VVS_OK;
}

static void causal_tree(int T, TreeDesc* t) {
  memset(t, 0, sizeof(*t));
  t->T = T;
  t->causal = 1;
  for (int j = 0; j < VVS_MAX_T; ++j) { t->parent[j] = (int8_t)(j - 1); t->first_child[j] = -1; t->next_sibling[j] = -1; }
  for (int j = 0; j < T && j < VVS_MAX_T; ++j) {
    t->depth[j] = (int8_t)j;
    t->anc[j] = (j == 63) ? ~0ull : ((1ull << (j + 1)) - 1);
  }
}

static vvs_status hip_fail(Ctx* c, hipError_t e, const char* what) {
  return fail(&c->err, VVS_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

static vvs_status check_launch(Ctx* c, const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(c, e, what);
  return VVS_OK;
}

}  // namespace vvs

using namespace vvs;

extern "C" {

vvs_status vvs_query_sizes(const vvs_config* cfg, size_t* kv_bytes, size_t* workspace_bytes, size_t* packed_weight_bytes) {
  Ctx c{};
  vvs_status st = plan_sizes(cfg, &c, nullptr);
  if (st != VVS_OK) return st;
  if (kv_bytes) *kv_bytes = 2 * c.kv_v_off * c.esz;
  if (workspace_bytes) *workspace_bytes = c.w.total;
  if (packed_weight_bytes) *packed_weight_bytes = c.p.total;
  return VVS_OK;
}

int32_t vvs_plan_is_fused(const vvs_ctx* ctx, int32_t n_tokens) {
  const Ctx* c = (const Ctx*)ctx;
  return c && n_tokens >= 1 && plan_fused(c, c->R * n_tokens) ? 1 : 0;
}

int32_t vvs_num_weight_tensors(const vvs_config* cfg) { return cfg ? 4 + 9 * cfg->n_layers + (cfg->draft_input ? 1 : 0) : 0; }

vvs_status vvs_check_tree(int32_t n_nodes, const int32_t* h_parent, const uint8_t* h_tree_mask, int32_t* h_depth,
                          int32_t* h_parent_out) {
  TreeDesc t;
  vvs_status st = build_tree(n_nodes, h_parent, h_tree_mask, &t, nullptr);
  if (st != VVS_OK) return st;
  for (int j = 0; j <= n_nodes; ++j) {
    if (h_depth) h_depth[j] = t.depth[j];
    if (h_parent_out && j) h_parent_out[j - 1] = t.parent[j];
  }
  return VVS_OK;
}

vvs_status vvs_create(const vvs_config* cfg, void* d_kv, void* d_workspace, void* d_packed_weights, vvs_ctx** out) {
  if (!out) return fail(nullptr, VVS_EINVAL, "create: out is NULL");
  *out = nullptr;
  if (!d_kv || !d_workspace || !d_packed_weights) return fail(nullptr, VVS_EINVAL, "create: NULL device buffer");
  if (((uintptr_t)d_kv | (uintptr_t)d_workspace | (uintptr_t)d_packed_weights) & 255)
    return fail(nullptr, VVS_EINVAL, "create: device buffers must be 256-byte aligned");
  Ctx* c = new Ctx{};
  vvs_status st = plan_sizes(cfg, c, nullptr);
  if (st != VVS_OK) { delete c; return st; }
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) {
    delete c;
    return fail(nullptr, VVS_EHIP, "create: no HIP device (this library has no CPU path)");
  }
  c->kv = (char*)d_kv; c->ws = (char*)d_workspace; c->pw = (char*)d_packed_weights;
  c->nbr = nullptr;
  c->codebook = nullptr;
  c->code_dim = 0;
  // zero the KV cache (padded slots are read, multiplied by zero weights) and the state block
  launch_fill_zero(c->kv, 2 * c->kv_v_off * c->esz, nullptr);
  launch_fill_zero(c->ws, c->w.x, nullptr);
  // rotary table in double -> float: [pos][pair] (cos, sin); theta_i = base^(-2i / (dh/2))
  int np = c->dh / 4;
  std::vector<float> tab((size_t)2 * c->rope_pos * np);
  for (int pos = 0; pos < c->rope_pos; ++pos)
    for (int i = 0; i < np; ++i) {
      double th = pow((double)c->cfg.rope_base, -2.0 * i / (c->dh / 2));
      tab[((size_t)pos * np + i) * 2 + 0] = (float)cos(pos * th);
      tab[((size_t)pos * np + i) * 2 + 1] = (float)sin(pos * th);
    }
  hipError_t e = hipMemcpy(c->ws + c->w.rope_tab, tab.data(), tab.size() * sizeof(float), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) { std::string m = std::string("create: ") + hipGetErrorString(e); delete c; return fail(nullptr, VVS_EHIP, m); }
  *out = reinterpret_cast<vvs_ctx*>(c);
  return VVS_OK;
}

void vvs_destroy(vvs_ctx* ctx) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return;
  for (auto& t : c->timed) { (void)hipEventDestroy(t.t0); (void)hipEventDestroy(t.t1); }
  delete c;
}

vvs_status vvs_timing_enable(vvs_ctx* ctx, int32_t on) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return VVS_EINVAL;
  c->timing = on != 0;
  if (on) c->n_timed = 0;
  return VVS_OK;
}

vvs_status vvs_timing_read(vvs_ctx* ctx, int32_t kernel_class, int32_t* n_launches, float* total_ms) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return VVS_EINVAL;
  if (kernel_class < 0 || kernel_class >= VVS_K_CLASSES || !n_launches || !total_ms)
    return fail(&c->err, VVS_EINVAL, "timing_read: bad argument");
  int n = 0;
  float ms = 0.f;
  for (size_t i = 0; i < c->n_timed; ++i) {
    TimedLaunch& t = c->timed[i];
    if (t.cls != kernel_class) continue;
    hipError_t e = hipEventSynchronize(t.t1);
    float one = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&one, t.t0, t.t1);
    if (e != hipSuccess) return hip_fail(c, e, "timing_read");
    ms += one;
    ++n;
  }
  *n_launches = n;
  *total_ms = ms;
  return VVS_OK;
}

vvs_status vvs_set_state(vvs_ctx* ctx, const int32_t* d_state, vvs_stream s) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return VVS_EINVAL;
  if (!d_state) return fail(&c->err, VVS_EINVAL, "set_state: NULL");
  if (!c->prefilled) return fail(&c->err, VVS_ESTATE, "set_state: call vvs_prefill first");
  launch_set_state(c, d_state, (hipStream_t)s);
  vvs_status rc = check_launch(c, "set_state");
  if (rc == VVS_OK) c->verify_pending = false;
  return rc;
}

const char* vvs_last_error(const vvs_ctx* ctx) {
  if (!ctx) return g_last_error.c_str();
  return reinterpret_cast<const Ctx*>(ctx)->err.c_str();
}

vvs_status vvs_load_weights(vvs_ctx* ctx, const void* const* d_tensors, int32_t n, vvs_stream s) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return VVS_EINVAL;
  if (!d_tensors) return fail(&c->err, VVS_EINVAL, "load_weights: tensor list is NULL");
  if (n != vvs_num_weight_tensors(&c->cfg)) return fail(&c->err, VVS_EINVAL, "load_weights: wrong number of tensors");
  for (int i = 0; i < n; ++i)
    if (!d_tensors[i] && !(i == 1 && c->cfg.prefix_kind == VVS_PREFIX_DENSE))
      return fail(&c->err, VVS_EINVAL, "load_weights: a tensor pointer is NULL");
  launch_pack_weights(c, d_tensors, (hipStream_t)s);
  vvs_status st = check_launch(c, "load_weights");
  if (st == VVS_OK) c->weights_loaded = true;
  return st;
}

vvs_status vvs_set_neighbors(vvs_ctx* ctx, const int32_t* d_nbr) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return VVS_EINVAL;
  if (!d_nbr) return fail(&c->err, VVS_EINVAL, "set_neighbors: table is NULL");
  if (c->cfg.relax_k < 1) return fail(&c->err, VVS_EINVAL, "set_neighbors: context was created with relax_k = 0");
  c->nbr = d_nbr;
  return VVS_OK;
}

vvs_status vvs_prefill(vvs_ctx* ctx, const void* d_prefix_cond, const void* d_prefix_uncond, int32_t n_forced,
                       const int32_t* d_forced_tokens, const float* d_uniform, int32_t* d_first_token, vvs_stream s) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return VVS_EINVAL;
  if (c->cfg.draft_input) return fail(&c->err, VVS_EINVAL, "prefill: this is a drafter context (use vvs_draft)");
  if (!c->weights_loaded) return fail(&c->err, VVS_ESTATE, "prefill: weights not loaded");
  if (!d_prefix_cond || !d_uniform || !d_first_token) return fail(&c->err, VVS_EINVAL, "prefill: NULL argument");
  if (c->cfg.prefix_kind == VVS_PREFIX_DENSE && !d_prefix_uncond)
    return fail(&c->err, VVS_EINVAL, "prefill: dense prefixes need the shared null prefix");
  if (n_forced < 0 || n_forced > c->G - 1) return fail(&c->err, VVS_EINVAL, "prefill: n_forced must be in [0, G-1]");
  if (n_forced > 0 && !d_forced_tokens) return fail(&c->err, VVS_EINVAL, "prefill: forced tokens are NULL");
  hipStream_t st = (hipStream_t)s;
  const int total = c->P + n_forced;
  PosDesc pos{nullptr, nullptr, 0, c->P, c->cfg.grid_w};
  for (int c0 = 0; c0 < total; c0 += c->chunk) {
    int T = std::min(c->chunk, total - c0);
    TreeDesc tree;
    causal_tree(T, &tree);
    pos.kv_base = c0;
    bool last = c0 + T >= total;
    launch_forward(c, tree, pos, T, nullptr, d_prefix_cond, d_prefix_uncond, c0, d_forced_tokens, n_forced, last ? 2 : 0, st);
    if (last) {
      TreeDesc one;
      causal_tree(1, &one);
      launch_accept(c, one, 1, (const float*)(c->ws + c->w.logits), nullptr, nullptr, d_uniform, 1, 0, 0, 0, VVS_STRICT,
                    false, nullptr, nullptr, nullptr, false, st);
      launch_prefill_finish(c, n_forced, d_first_token, st);
      launch_push_prefill_feature(c, T, st);
    }
  }
  vvs_status rc = check_launch(c, "prefill");
  if (rc != VVS_OK) return rc;
  c->prefilled = true;
  c->verify_pending = false;
  c->last_T = 1;
  return VVS_OK;
}

static vvs_status check_verify_args(Ctx* c, const char* who, int32_t n_nodes, const int32_t* d_draft_tokens,
                                    const float* d_draft_probs, const float* d_uniforms, int32_t mode,
                                    int32_t* d_accept_len, int32_t* d_path, int32_t* d_next_token) {
  std::string w(who);
  if (n_nodes < 0) return fail(&c->err, VVS_EINVAL, w + ": n_nodes < 0");
  if (n_nodes > c->cfg.max_nodes) return fail(&c->err, VVS_ESIZE, w + ": n_nodes exceeds max_nodes of the context");
  if (n_nodes > 0 && (!d_draft_tokens || !d_draft_probs)) return fail(&c->err, VVS_EINVAL, w + ": draft tokens / probs are NULL");
  if (!d_uniforms || !d_accept_len || !d_path || !d_next_token) return fail(&c->err, VVS_EINVAL, w + ": NULL argument");
  if (mode != VVS_STRICT && mode != VVS_RELAXED) return fail(&c->err, VVS_EINVAL, w + ": unknown mode");
  if (mode == VVS_RELAXED && c->cfg.relax_k > 0 && !c->nbr)
    return fail(&c->err, VVS_ESTATE, w + ": relaxed mode needs vvs_set_neighbors first");
  return VVS_OK;
}

vvs_status vvs_verify_post(vvs_ctx* ctx, int32_t n_nodes, int32_t n_post, const int32_t* h_parent, const uint8_t* h_tree_mask,
                           const int32_t* d_draft_tokens, const float* d_draft_probs, const float* d_uniforms, int32_t mode,
                           int32_t* d_accept_len, int32_t* d_path, int32_t* d_next_token, vvs_stream s) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return VVS_EINVAL;
  if (!c->prefilled) return fail(&c->err, VVS_ESTATE, "verify: call vvs_prefill first");
  if (c->verify_pending) return fail(&c->err, VVS_ESTATE, "verify: the previous verify was not committed");
  vvs_status rc = check_verify_args(c, "verify", n_nodes, d_draft_tokens, d_draft_probs, d_uniforms, mode, d_accept_len,
                                    d_path, d_next_token);
  if (rc != VVS_OK) return rc;
  if (n_post < 0 || n_post > n_nodes) return fail(&c->err, VVS_EINVAL, "verify: n_post must be in [0, n_nodes]");
  TreeDesc tree;
  rc = build_tree(n_nodes, h_parent, h_tree_mask, &tree, &c->err);
  if (rc != VVS_OK) return rc;
  for (int j = 1; j <= n_nodes; ++j) {
    if (j <= n_post && tree.parent[j] != j - 1)
      return fail(&c->err, VVS_EINVAL, "verify: the post-verified tokens must form a chain below the root");
    if (j > n_post && tree.parent[j] < n_post)
      return fail(&c->err, VVS_EINVAL, "verify: every candidate must descend from the last post-verified token");
  }
  tree.n_forced = n_post;
  hipStream_t st = (hipStream_t)s;
  const int T = n_nodes + 1;
  const int32_t* state = (const int32_t*)(c->ws + c->w.state);
  PosDesc pos{state, state + c->B, 0, c->P, c->cfg.grid_w};
  launch_build_tokens(c, T, d_draft_tokens, st);
  launch_forward(c, tree, pos, T, (const int32_t*)(c->ws + c->w.tokens), nullptr, nullptr, 0, nullptr, 0, 1, st);
  launch_accept(c, tree, T, (const float*)(c->ws + c->w.logits), d_draft_tokens, d_draft_probs, d_uniforms, 2 * T, 2, 0, 1,
                mode, true, d_accept_len, d_path, d_next_token, true, st);
  rc = check_launch(c, "verify");
  if (rc != VVS_OK) return rc;
  c->verify_pending = true;
  c->last_T = T;
  return VVS_OK;
}

vvs_status vvs_verify(vvs_ctx* ctx, int32_t n_nodes, const int32_t* h_parent, const uint8_t* h_tree_mask,
                      const int32_t* d_draft_tokens, const float* d_draft_probs, const float* d_uniforms, int32_t mode,
                      int32_t* d_accept_len, int32_t* d_path, int32_t* d_next_token, vvs_stream s) {
  return vvs_verify_post(ctx, n_nodes, 0, h_parent, h_tree_mask, d_draft_tokens, d_draft_probs, d_uniforms, mode, d_accept_len,
                         d_path, d_next_token, s);
}

vvs_status vvs_accept_from_logits(vvs_ctx* ctx, int32_t n_nodes, const int32_t* h_parent, const uint8_t* h_tree_mask,
                                  const float* d_raw_logits, const int32_t* d_draft_tokens, const float* d_draft_probs,
                                  const float* d_uniforms, int32_t mode, int32_t* d_accept_len, int32_t* d_path,
                                  int32_t* d_next_token, vvs_stream s) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return VVS_EINVAL;
  if (!d_raw_logits) return fail(&c->err, VVS_EINVAL, "accept_from_logits: logits are NULL");
  vvs_status rc = check_verify_args(c, "accept_from_logits", n_nodes, d_draft_tokens, d_draft_probs, d_uniforms, mode,
                                    d_accept_len, d_path, d_next_token);
  if (rc != VVS_OK) return rc;
  TreeDesc tree;
  rc = build_tree(n_nodes, h_parent, h_tree_mask, &tree, &c->err);
  if (rc != VVS_OK) return rc;
  launch_accept(c, tree, n_nodes + 1, d_raw_logits, d_draft_tokens, d_draft_probs, d_uniforms, 2 * (n_nodes + 1), 2, 0, 1,
                mode, false, d_accept_len, d_path, d_next_token, false, (hipStream_t)s);
  return check_launch(c, "accept_from_logits");
}

vvs_status vvs_accept_from_logits_noalloc(vvs_ctx* ctx, int32_t n_nodes, const int32_t* h_parent, const uint8_t* h_tree_mask,
                                          const float* d_raw_logits, const int32_t* d_draft_tokens, const float* d_draft_probs,
                                          const float* d_uniforms, int32_t mode, int32_t* d_accept_len, int32_t* d_path,
                                          int32_t* d_next_token, vvs_stream s) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return VVS_EINVAL;
  if (!d_raw_logits) return fail(&c->err, VVS_EINVAL, "accept_from_logits_noalloc: logits are NULL");
  vvs_status rc = check_verify_args(c, "accept_from_logits_noalloc", n_nodes, d_draft_tokens, d_draft_probs, d_uniforms, mode,
                                    d_accept_len, d_path, d_next_token);
  if (rc != VVS_OK) return rc;
  TreeDesc tree;
  rc = build_tree(n_nodes, h_parent, h_tree_mask, &tree, &c->err);
  if (rc != VVS_OK) return rc;
  std::string msg;
  rc = launch_accept_noalloc(c, tree, n_nodes + 1, d_raw_logits, d_draft_tokens, d_draft_probs, d_uniforms, mode, d_accept_len, d_path,
                             d_next_token, (hipStream_t)s, &msg);
  if (rc != VVS_OK) return fail(&c->err, rc, msg);
  return check_launch(c, "accept_from_logits_noalloc");
}

vvs_status vvs_kv_commit(vvs_ctx* ctx, vvs_stream s) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return VVS_EINVAL;
  if (!c->verify_pending) return fail(&c->err, VVS_ESTATE, "kv_commit: no verify to commit");
  launch_commit(c, (hipStream_t)s);
  vvs_status rc = check_launch(c, "kv_commit");
  if (rc != VVS_OK) return rc;
  c->verify_pending = false;
  return VVS_OK;
}

vvs_status vvs_select_unverified(int32_t n_nodes, const int32_t* h_parent, const uint8_t* h_tree_mask, float u, int32_t* h_nodes,
                                 int32_t* n_kept) {
  if (!h_nodes || !n_kept) return VVS_EINVAL;
  if (!(u >= 0.f && u < 1.f)) return VVS_EINVAL;
  TreeDesc t;
  vvs_status st = build_tree(n_nodes, h_parent, h_tree_mask, &t, nullptr);
  if (st != VVS_OK) return st;
  *n_kept = 0;
  // candidate paths = one per leaf, in leaf order; their lengths are the leaves' depths
  std::vector<int> leaves;
  long total = 0;
  for (int j = 1; j <= n_nodes; ++j)
    if (t.first_child[j] < 0) { leaves.push_back(j); total += t.depth[j]; }
  if (leaves.empty()) return VVS_OK;
  const int n_paths = (int)leaves.size();
  const int sel = std::min((int)std::floor((double)u * n_paths), n_paths - 1);
  const int mean_floor = (int)(total / n_paths);                     // floor of the mean path length (Eq. 1)
  const int len = t.depth[leaves[sel]], keep = std::min(len, mean_floor);
  int node = leaves[sel];
  for (int k = len - 1; k >= 0; --k) {                               // walk up; position k of the path is the ancestor at depth k + 1
    if (k < keep) h_nodes[k] = node;
    node = t.parent[node];
  }
  *n_kept = keep;
  return VVS_OK;
}

int32_t vvs_skip_uniform(int32_t step_index, int32_t interval) {
  return interval >= 2 && step_index >= 0 && (step_index + 1) % interval == 0;
}

int32_t vvs_skip_dynamic(float similarity, float threshold, int32_t last_step_verified) {
  return last_step_verified != 0 && similarity >= threshold;
}

vvs_status vvs_set_codebook(vvs_ctx* ctx, const float* d_embed, int32_t dim) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return VVS_EINVAL;
  if (!d_embed) return fail(&c->err, VVS_EINVAL, "set_codebook: table is NULL");
  if (dim < 1 || dim > 64) return fail(&c->err, VVS_ESIZE, "set_codebook: dim must be in [1, 64]");
  c->codebook = d_embed;
  c->code_dim = dim;
  return VVS_OK;
}

vvs_status vvs_path_similarity(vvs_ctx* ctx, int32_t n_nodes, const int32_t* h_parent, const uint8_t* h_tree_mask,
                               const int32_t* d_draft_tokens, float alpha, int32_t stride, float* d_similarity, vvs_stream s) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return VVS_EINVAL;
  if (!c->codebook) return fail(&c->err, VVS_ESTATE, "path_similarity: call vvs_set_codebook first");
  if (!d_similarity || (n_nodes > 0 && !d_draft_tokens)) return fail(&c->err, VVS_EINVAL, "path_similarity: NULL argument");
  if (stride < 1) return fail(&c->err, VVS_EINVAL, "path_similarity: stride < 1");
  if (!(alpha > 0.f)) return fail(&c->err, VVS_EINVAL, "path_similarity: alpha must be positive");
  if (n_nodes > c->cfg.max_nodes) return fail(&c->err, VVS_ESIZE, "path_similarity: n_nodes exceeds max_nodes of the context");
  TreeDesc tree;
  vvs_status rc = build_tree(n_nodes, h_parent, h_tree_mask, &tree, &c->err);
  if (rc != VVS_OK) return rc;
  launch_path_similarity(c, tree, n_nodes, d_draft_tokens, alpha, stride, d_similarity, (hipStream_t)s);
  return check_launch(c, "path_similarity");
}

vvs_status vvs_read_features(vvs_ctx* ctx, float* d_features, int32_t* d_count, vvs_stream s) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return VVS_EINVAL;
  if (!d_features || !d_count) return fail(&c->err, VVS_EINVAL, "read_features: NULL");
  if (c->cfg.feature_slots < 1) return fail(&c->err, VVS_ESTATE, "read_features: the context was created with feature_slots = 0");
  if (!c->prefilled) return fail(&c->err, VVS_ESTATE, "read_features: call vvs_prefill first");
  launch_read_features(c, d_features, d_count, (hipStream_t)s);
  return check_launch(c, "read_features");
}

vvs_status vvs_draft(vvs_ctx* drafter, vvs_ctx* target, int32_t n_nodes, const int32_t* h_parent, const uint8_t* h_tree_mask,
                     int32_t n_ctx, const int32_t* d_recent_tokens, int32_t n_unverified, const int32_t* d_given_tokens,
                     int32_t* d_draft_tokens, float* d_draft_probs, vvs_stream s) {
  Ctx* dr = reinterpret_cast<Ctx*>(drafter);
  Ctx* tg = reinterpret_cast<Ctx*>(target);
  if (!dr) return VVS_EINVAL;
  if (!tg) return fail(&dr->err, VVS_EINVAL, "draft: target context is NULL");
  if (!dr->cfg.draft_input) return fail(&dr->err, VVS_EINVAL, "draft: the first context was not created with draft_input = 1");
  if (tg->cfg.draft_input) return fail(&dr->err, VVS_EINVAL, "draft: the target is a drafter context");
  if (!dr->weights_loaded) return fail(&dr->err, VVS_ESTATE, "draft: drafter weights not loaded");
  if (!tg->prefilled) return fail(&dr->err, VVS_ESTATE, "draft: call vvs_prefill on the target first");
  const vvs_config &a = dr->cfg, &b = tg->cfg;
  if (a.d_model != b.d_model || a.dtype != b.dtype || a.n_prompts != b.n_prompts || a.vocab != b.vocab || a.logit_lo != b.logit_lo ||
      a.logit_hi != b.logit_hi || a.grid_h != b.grid_h || a.grid_w != b.grid_w)
    return fail(&dr->err, VVS_EINVAL, "draft: drafter and target differ in d_model, dtype, prompts, vocabulary slice or grid");
  if (a.feature_pre_norm != b.feature_pre_norm)
    return fail(&dr->err, VVS_EINVAL, "draft: drafter and target keep different kinds of feature (feature_pre_norm)");
  if (n_nodes < 1) return fail(&dr->err, VVS_EINVAL, "draft: n_nodes < 1");
  if (n_ctx < 1 || n_ctx > b.feature_slots) return fail(&dr->err, VVS_EINVAL, "draft: n_ctx must be in [1, feature_slots of the target]");
  if (n_unverified < 0 || n_unverified > VVS_MAX_FEATURE_SLOTS) return fail(&dr->err, VVS_EINVAL, "draft: n_unverified out of range");
  if (!d_recent_tokens || !d_draft_tokens || !d_draft_probs) return fail(&dr->err, VVS_EINVAL, "draft: NULL argument");
  TreeDesc shape;
  vvs_status rc = build_tree(n_nodes, h_parent, h_tree_mask, &shape, &dr->err);
  if (rc != VVS_OK) return rc;
  // block tokens of the drafter's forwards: the n_ctx pairs (the last is the root), then the nodes that
  // have children, ordered by depth and then id, so that a level only appends tokens
  const int T = n_nodes + 1, k = n_ctx;
  std::vector<int> order;
  int last_level = 0;
  for (int j = 1; j < T; ++j)
    if (shape.first_child[j] >= 0) { order.push_back(j); last_level = std::max(last_level, (int)shape.depth[j]); }
  std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return shape.depth[x] < shape.depth[y]; });
  if (k + (int)order.size() > dr->Tmax)
    return fail(&dr->err, VVS_ESIZE, "draft: n_ctx + expanded nodes exceeds max_nodes + 1 of the drafter context");
  std::vector<int> slot(T, -1);
  slot[0] = k - 1;
  for (size_t i = 0; i < order.size(); ++i) slot[order[i]] = k + (int)i;
  hipStream_t st = (hipStream_t)s;
  launch_draft_state(dr, tg, k, n_unverified, st);
  launch_draft_zero_leaves(dr, shape, d_draft_probs, st);
  const int32_t* state = (const int32_t*)(dr->ws + dr->w.state);
  PosDesc pos{state, state + dr->B, 0, dr->P, dr->cfg.grid_w};
  DraftLevel lv;
  memset(&lv, 0, sizeof(lv));
  lv.k = k;
  lv.n_nodes = n_nodes;
  int n_in = 0;
  for (int level = 0; level <= last_level; ++level) {
    while (n_in < (int)order.size() && shape.depth[order[n_in]] <= level) ++n_in;
    lv.Tq = k + n_in;
    std::vector<int32_t> bp(lv.Tq > 1 ? lv.Tq - 1 : 1);
    for (int t = 1; t < lv.Tq; ++t) {
      if (t < k) { bp[t - 1] = t - 1; continue; }
      const int j = order[t - k];
      lv.node[t] = (int8_t)j;
      lv.parent_slot[t] = (int8_t)slot[shape.parent[j]];
      bp[t - 1] = slot[shape.parent[j]];
    }
    TreeDesc blk;
    rc = build_tree(lv.Tq - 1, bp.data(), nullptr, &blk, &dr->err);
    if (rc != VVS_OK) return rc;
    lv.n_sel = 0;
    for (int j = 0; j < T; ++j)
      if (shape.first_child[j] >= 0 && shape.depth[j] == level) {
        lv.sel_node[lv.n_sel] = (int8_t)j;
        lv.sel_slot[lv.n_sel] = (int8_t)slot[j];
        ++lv.n_sel;
      }
    launch_draft_input(dr, tg, lv, d_recent_tokens, d_draft_tokens, st);
    launch_forward(dr, blk, pos, lv.Tq, nullptr, nullptr, nullptr, 0, nullptr, 0, 1, st, true);
    launch_draft_select(dr, lv, shape, d_given_tokens, d_draft_tokens, d_draft_probs, st);
    lv.Tq_prev = lv.Tq;
  }
  rc = check_launch(dr, "draft");
  if (rc != VVS_OK) return rc;
  dr->last_T = lv.Tq;
  return VVS_OK;
}

vvs_status vvs_read_state(vvs_ctx* ctx, int32_t* d_state, vvs_stream s) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return VVS_EINVAL;
  if (!d_state) return fail(&c->err, VVS_EINVAL, "read_state: NULL");
  launch_read_state(c, d_state, (hipStream_t)s);
  return check_launch(c, "read_state");
}

vvs_status vvs_debug_logits(vvs_ctx* ctx, float* d_raw, float* d_mixed, float* d_probs, vvs_stream s) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return VVS_EINVAL;
  if (c->last_T < 1) return fail(&c->err, VVS_ESTATE, "debug_logits: nothing has run yet");
  launch_debug_logits(c, d_raw, d_mixed, d_probs, (hipStream_t)s);
  return check_launch(c, "debug_logits");
}

vvs_status vvs_debug_kv(vvs_ctx* ctx, int32_t layer, int32_t row, int32_t n_slots, float* d_k, float* d_v, vvs_stream s) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return VVS_EINVAL;
  if (layer < 0 || layer >= c->L || row < 0 || row >= c->R || n_slots < 0 || n_slots > c->S_cap || !d_k || !d_v)
    return fail(&c->err, VVS_EINVAL, "debug_kv: argument out of range");
  launch_debug_kv(c, layer, row, n_slots, d_k, d_v, (hipStream_t)s);
  return check_launch(c, "debug_kv");
}

vvs_status vvs_debug_copy(vvs_ctx* ctx, void* d_dst, const void* d_src, size_t bytes, vvs_stream s) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return VVS_EINVAL;
  if (!d_dst || !d_src || (bytes & 15) || (((uintptr_t)d_dst | (uintptr_t)d_src) & 15))
    return fail(&c->err, VVS_EINVAL, "debug_copy: pointers and size must be multiples of 16");
  launch_copy_bytes(d_dst, d_src, bytes, (hipStream_t)s);
  return check_launch(c, "debug_copy");
}

vvs_status vvs_debug_fill_probe(vvs_ctx* ctx, const void* d_src, size_t region_bytes, size_t wg_stride_bytes, int32_t reps, int32_t mode,
                                int32_t n_workgroups, int32_t waves, uint32_t* d_sink, vvs_stream s) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return VVS_EINVAL;
  if (!d_src || !d_sink || ((uintptr_t)d_src & 15) || region_bytes < 8192 || (region_bytes & 8191) || region_bytes > ((size_t)1 << 30) ||
      (wg_stride_bytes & 15) || wg_stride_bytes > ((size_t)1 << 30))
    return fail(&c->err, VVS_EINVAL, "debug_fill_probe: the region must be 16-byte aligned and a multiple of 8192 bytes, region and stride at most 1 GiB");
  if (reps < 1 || reps > (1 << 20) || (mode != 0 && mode != 1) || n_workgroups < 1 || n_workgroups > 65536 || waves < 1 || waves > 16)
    return fail(&c->err, VVS_EINVAL, "debug_fill_probe: reps, mode, workgroups or waves out of range");
  launch_fill_probe(d_src, region_bytes, wg_stride_bytes, reps, mode, n_workgroups, waves, d_sink, (hipStream_t)s);
  return check_launch(c, "debug_fill_probe");
}

size_t vvs_debug_gemm_scratch_bytes(const vvs_ctx* ctx, int32_t m, int32_t n, int32_t k) {
  const Ctx* c = reinterpret_cast<const Ctx*>(ctx);
  if (!c || m < 1 || n < 1 || k < 1) return 0;
  GemmPlan p = plan_gemm(c, m, n, k);
  return align_up((size_t)n * k * c->esz, 256) + align_up(align_up((size_t)m, 32) * k * c->esz, 256) +
         align_up((size_t)p.splits * m * n * sizeof(float), 256);
}

vvs_status vvs_debug_gemm(vvs_ctx* ctx, int32_t m, int32_t n, int32_t k, const void* d_a, const void* d_w, void* d_scratch,
                          float* d_c, vvs_stream s) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return VVS_EINVAL;
  if (m < 1 || n < 1 || k < 1 || !d_a || !d_w || !d_scratch || !d_c) return fail(&c->err, VVS_EINVAL, "debug_gemm: bad argument");
  if (c->cfg.dtype == VVS_BF16 && (n % 64 || k % 64)) return fail(&c->err, VVS_ESIZE, "debug_gemm: bf16 needs n, k multiples of 64");
  launch_debug_gemm(c, m, n, k, d_a, d_w, d_scratch, d_c, (hipStream_t)s);
  return check_launch(c, "debug_gemm");
}

}  // extern "C"
