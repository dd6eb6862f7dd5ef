// Host-only exerciser of the library's planner and argument checks, built with AddressSanitizer and
// UndefinedBehaviorSanitizer by tests/test_host_sanitized.py.  The HIP runtime and every kernel launcher
// are replaced by host stand-ins (a "device" buffer is ordinary memory of exactly the size vvs_query_sizes
// asked for; fills and copies really touch it), so that the complete call sequences - create, load, prefill,
// verify with and without unverified tokens, commit, draft, path similarity, inspection - run their host
// side under the sanitizers without a GPU, on random valid and invalid inputs.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <random>
#include <vector>
#include "vvs_internal.h"

// ---- HIP runtime stand-ins (only what the host file uses)
extern "C" {
hipError_t hipGetDeviceCount(int* n) { *n = 1; return hipSuccess; }
hipError_t hipMemcpy(void* dst, const void* src, size_t n, hipMemcpyKind) { memcpy(dst, src, n); return hipSuccess; }
hipError_t hipDeviceSynchronize() { return hipSuccess; }
hipError_t hipGetLastError() { return hipSuccess; }
const char* hipGetErrorString(hipError_t) { return "stub"; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipEventElapsedTime(float* ms, hipEvent_t, hipEvent_t) { *ms = 0.f; return hipSuccess; }
hipError_t hipEventCreate(hipEvent_t* e) { *e = nullptr; return hipSuccess; }
hipError_t hipEventDestroy(hipEvent_t) { return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
}

// ---- launcher stand-ins: no arithmetic; the ones that have a size touch their buffers
namespace vvs {
static long g_launches = 0;
void launch_fill_zero(void* p, size_t bytes, hipStream_t) { memset(p, 0, bytes); ++g_launches; }
void launch_copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t) { memmove(dst, src, bytes); ++g_launches; }
void launch_fill_probe(const void*, size_t, size_t, int, int, int, int, uint32_t*, hipStream_t) { ++g_launches; }
void launch_pack_weights(Ctx*, const void* const*, hipStream_t) { ++g_launches; }
void launch_forward(Ctx* c, const TreeDesc& tree, const PosDesc&, int T, const int32_t*, const void*, const void*, int, const int32_t*, int,
                    int, hipStream_t, bool from_din) {
  if (T < 1 || T > c->Tmax && T > c->chunk) abort();            // a forward never exceeds what the workspace was sized for
  if (tree.T != T) abort();
  for (int t = 0; t < T; ++t)
    if (!((tree.anc[t] >> t) & 1ull) || (t && tree.parent[t] >= t)) abort();
  memset(c->ws + c->w.x, 0, sizeof(float) * (size_t)c->R * T * c->d);
  if (from_din) memset(c->ws + c->w.din, 0, c->esz * (size_t)c->R * T * 2 * c->d);
  ++g_launches;
}
void launch_build_tokens(Ctx* c, int T, const int32_t*, hipStream_t) { memset(c->ws + c->w.tokens, 0, sizeof(int32_t) * c->B * T); ++g_launches; }
void launch_accept(Ctx*, const TreeDesc&, int, const float*, const int32_t*, const float*, const float*, int, int, int, int, int, bool, int32_t*,
                   int32_t*, int32_t*, bool, hipStream_t) { ++g_launches; }
vvs_status launch_accept_noalloc(Ctx*, const TreeDesc&, int, const float*, const int32_t*, const float*, const float*, int, int32_t*, int32_t*,
                                 int32_t*, hipStream_t, std::string*) { ++g_launches; return VVS_OK; }
void launch_prefill_finish(Ctx*, int, int32_t*, hipStream_t) { ++g_launches; }
void launch_commit(Ctx*, hipStream_t) { ++g_launches; }
void launch_push_prefill_feature(Ctx*, int, hipStream_t) { ++g_launches; }
void launch_read_features(Ctx*, float*, int32_t*, hipStream_t) { ++g_launches; }
void launch_path_similarity(Ctx*, const TreeDesc&, int, const int32_t*, float, int, float*, hipStream_t) { ++g_launches; }
void launch_read_state(Ctx*, int32_t*, hipStream_t) { ++g_launches; }
void launch_set_state(Ctx*, const int32_t*, hipStream_t) { ++g_launches; }
void launch_debug_logits(Ctx*, float*, float*, float*, hipStream_t) { ++g_launches; }
void launch_debug_kv(Ctx*, int, int, int, float*, float*, hipStream_t) { ++g_launches; }
void launch_debug_gemm(Ctx*, int, int, int, const void*, const void*, void*, float*, hipStream_t) { ++g_launches; }
void launch_draft_state(Ctx*, const Ctx*, int, int, hipStream_t) { ++g_launches; }
void launch_draft_zero_leaves(Ctx*, const TreeDesc&, float*, hipStream_t) { ++g_launches; }
void launch_draft_input(Ctx* dr, const Ctx*, const DraftLevel& lv, const int32_t*, const int32_t*, hipStream_t) {
  if (lv.Tq < lv.k || lv.Tq > dr->Tmax) abort();
  for (int t = lv.k; t < lv.Tq; ++t)
    if (lv.node[t] < 1 || lv.node[t] > lv.n_nodes || lv.parent_slot[t] < lv.k - 1 || lv.parent_slot[t] >= t || lv.parent_slot[t] >= lv.Tq_prev) abort();
  ++g_launches;
}
void launch_draft_select(Ctx*, const DraftLevel& lv, const TreeDesc& shape, const int32_t*, int32_t*, float*, hipStream_t) {
  for (int i = 0; i < lv.n_sel; ++i)
    if (lv.sel_slot[i] < lv.k - 1 || lv.sel_slot[i] >= lv.Tq || shape.first_child[lv.sel_node[i]] < 0) abort();
  ++g_launches;
}
}  // namespace vvs

static std::mt19937 rng(12345);
static int ri(int lo, int hi) { return lo + (int)(rng() % (unsigned)(hi - lo + 1)); }

static vvs_config base_config(bool bf16, bool drafter) {
  vvs_config c;
  memset(&c, 0, sizeof(c));
  c.n_layers = drafter ? 1 : 2; c.d_model = bf16 ? 256 : 64; c.n_heads = 4; c.d_ff = bf16 ? 512 : 96; c.vocab = 512;
  c.logit_lo = bf16 ? 64 : 0; c.logit_hi = bf16 ? 64 + 256 : 512; c.grid_h = 6; c.grid_w = 5; c.prefix_len = 3;
  c.prefix_kind = VVS_PREFIX_CLASS; c.n_classes = 10; c.n_prompts = 3; c.max_nodes = 40; c.dtype = bf16 ? VVS_BF16 : VVS_FP32;
  c.cfg_scale = 3.f; c.rms_eps = 1e-5f; c.rope_base = 10000.f; c.relax_k = 0; c.relax_delta = 0.f;
  c.feature_slots = drafter ? 0 : 5; c.feature_pre_norm = 0; c.draft_input = drafter ? 1 : 0;
  return c;
}

struct Dev {   // the three "device" buffers of a context, exactly as large as asked for
  std::vector<char> kv, ws, pw;
  char *akv, *aws, *apw;
  void alloc(const vvs_config& c) {
    size_t a, b, d;
    if (vvs_query_sizes(&c, &a, &b, &d) != VVS_OK) { printf("query_sizes failed: %s\n", vvs_last_error(nullptr)); exit(1); }
    kv.resize(a + 256); ws.resize(b + 256); pw.resize(d + 256);
    akv = (char*)(((uintptr_t)kv.data() + 255) & ~(uintptr_t)255);
    aws = (char*)(((uintptr_t)ws.data() + 255) & ~(uintptr_t)255);
    apw = (char*)(((uintptr_t)pw.data() + 255) & ~(uintptr_t)255);
    // shrink to the exact size so that a write past the end is caught: copies with no slack behind the aligned start
    kv.resize((akv - kv.data()) + a); ws.resize((aws - ws.data()) + b); pw.resize((apw - pw.data()) + d);
    akv = (char*)(((uintptr_t)kv.data() + 255) & ~(uintptr_t)255);
    aws = (char*)(((uintptr_t)ws.data() + 255) & ~(uintptr_t)255);
    apw = (char*)(((uintptr_t)pw.data() + 255) & ~(uintptr_t)255);
  }
};

static void random_tree(int n, std::vector<int32_t>& parent, bool valid) {
  parent.resize(n > 0 ? n : 1);
  for (int j = 1; j <= n; ++j) parent[j - 1] = valid ? ri(0, j - 1) : ri(-2, j + 2);
}

int main() {
  // 1. topology checks and the verification-free step on random input, valid and not
  for (int it = 0; it < 4000; ++it) {
    const int n = ri(-2, 70);
    std::vector<int32_t> parent;
    const bool valid = it % 3 != 0;
    random_tree(n, parent, valid);
    int32_t depth[VVS_MAX_T + 8], pout[VVS_MAX_T + 8], nodes[VVS_MAX_T], kept = -1;
    vvs_status st = vvs_check_tree(n, n > 0 ? parent.data() : nullptr, nullptr, depth, pout);
    if (valid && n >= 0 && n <= VVS_MAX_T - 1 && st != VVS_OK) { printf("valid tree refused (n %d)\n", n); return 1; }
    if ((n < 0 || n > VVS_MAX_T - 1) && st == VVS_OK) { printf("n %d accepted\n", n); return 1; }
    if (st == VVS_OK && n > 0) {
      const int T = n + 1;
      std::vector<uint8_t> mask((size_t)T * T, 0);
      for (int i = 0; i < T; ++i) { int j = i; for (;;) { mask[(size_t)i * T + j] = 1; if (!j) break; j = pout[j - 1]; } }
      if (vvs_check_tree(n, nullptr, mask.data(), depth, pout) != VVS_OK) { printf("own mask refused\n"); return 1; }
      if (vvs_check_tree(n, parent.data(), mask.data(), nullptr, nullptr) != VVS_OK) { printf("parent + mask refused\n"); return 1; }
      mask[(size_t)ri(1, n) * T] = 0;                         // a node that no longer sees the root
      if (vvs_check_tree(n, nullptr, mask.data(), nullptr, nullptr) == VVS_OK) { printf("broken mask accepted\n"); return 1; }
      const float u = it % 7 == 0 ? 1.0f : (float)(rng() % 1000) / 1000.f;
      st = vvs_select_unverified(n, parent.data(), nullptr, u, nodes, &kept);
      if (u >= 1.0f) {                                        // the uniform must lie in [0, 1)
        if (st != VVS_EINVAL) { printf("select_unverified accepted u = 1\n"); return 1; }
        continue;
      }
      if (st != VVS_OK || kept < 1 || kept > n) { printf("select_unverified: status %d kept %d\n", st, kept); return 1; }
      for (int i = 0; i < kept; ++i)
        if (nodes[i] < 1 || nodes[i] > n || (i ? pout[nodes[i] - 1] != nodes[i - 1] : pout[nodes[i] - 1] != 0)) { printf("kept path is not a path\n"); return 1; }
    }
    (void)vvs_skip_uniform(ri(-3, 50), ri(-2, 6));
    (void)vvs_skip_dynamic((float)ri(-5, 15) / 10.f, 0.7f, ri(0, 1));
  }
  // 2. size queries on random configurations never crash and refuse what they cannot serve
  for (int it = 0; it < 2000; ++it) {
    vvs_config c = base_config(it & 1, it & 2);
    switch (ri(0, 10)) {
      case 0: c.d_model = ri(-8, 300); break;
      case 1: c.n_heads = ri(-1, 9); break;
      case 2: c.max_nodes = ri(-2, 80); break;
      case 3: c.logit_hi = ri(-5, 600); break;
      case 4: c.feature_slots = ri(-2, 12); break;
      case 5: c.dtype = ri(-1, 3); break;
      case 6: c.n_prompts = ri(-1, 5); break;
      case 7: c.draft_input = ri(-1, 2); break;
      case 8: c.relax_k = ri(-1, 70); break;
      case 9: c.norm_mode = ri(-1, 2); break;
      default: break;
    }
    size_t a = 0, b = 0, d = 0;
    vvs_status st = vvs_query_sizes(&c, &a, &b, &d);
    if (st == VVS_OK && (a == 0 || b == 0 || d == 0)) { printf("empty buffer sizes accepted\n"); return 1; }
  }
  // 3. the call sequences, launchers replaced: target + drafter, fp32 and bf16 planning
  for (int bf16 = 0; bf16 < 2; ++bf16) {
    vvs_config tc = base_config(bf16, false), dc = base_config(bf16, true);
    Dev td, dd;
    td.alloc(tc); dd.alloc(dc);
    vvs_ctx *tg = nullptr, *dr = nullptr;
    if (vvs_create(&tc, td.akv, td.aws, td.apw, &tg) != VVS_OK || vvs_create(&dc, dd.akv, dd.aws, dd.apw, &dr) != VVS_OK) {
      printf("create failed: %s\n", vvs_last_error(nullptr)); return 1;
    }
    std::vector<const void*> wt(vvs_num_weight_tensors(&tc), (const void*)td.apw), wd(vvs_num_weight_tensors(&dc), (const void*)dd.apw);
    int32_t dummy_i[4096]; float dummy_f[64];
    memset(dummy_i, 0, sizeof(dummy_i));
    void* fake = dummy_i;    // pointers handed to launchers are never dereferenced by the stand-ins
    if (vvs_verify(tg, 0, nullptr, nullptr, nullptr, nullptr, dummy_f, VVS_STRICT, dummy_i, dummy_i, dummy_i, nullptr) != VVS_ESTATE) { printf("verify before prefill\n"); return 1; }
    if (vvs_load_weights(tg, wt.data(), (int)wt.size(), nullptr) != VVS_OK || vvs_load_weights(dr, wd.data(), (int)wd.size(), nullptr) != VVS_OK) { printf("load\n"); return 1; }
    if (vvs_load_weights(dr, wd.data(), (int)wd.size() - 1, nullptr) == VVS_OK) { printf("short weight list accepted\n"); return 1; }
    if (vvs_draft(dr, tg, 3, nullptr, nullptr, 1, dummy_i, 0, nullptr, dummy_i, dummy_f, nullptr) != VVS_ESTATE) { printf("draft before prefill\n"); return 1; }
    if (vvs_prefill(tg, fake, nullptr, 7, dummy_i, dummy_f, dummy_i, nullptr) != VVS_OK) { printf("prefill: %s\n", vvs_last_error(tg)); return 1; }
    if (vvs_prefill(dr, fake, nullptr, 0, nullptr, dummy_f, dummy_i, nullptr) == VVS_OK) { printf("prefill on a drafter accepted\n"); return 1; }
    int ok_verify = 0, ok_draft = 0;
    for (int it = 0; it < 1500; ++it) {
      const int n = ri(0, 45);
      std::vector<int32_t> parent;
      random_tree(n, parent, it % 5 != 0);
      int n_post = it % 4 == 0 ? ri(0, 6) : 0;
      if (n_post && n >= n_post) {                              // hang the tree below a chain of unverified tokens
        for (int j = 1; j <= n; ++j) parent[j - 1] = j <= n_post ? j - 1 : std::max(parent[j - 1], (int32_t)n_post);
      }
      vvs_status st = vvs_verify_post(tg, n, n_post, n ? parent.data() : nullptr, nullptr, dummy_i, dummy_f, dummy_f, VVS_STRICT, dummy_i, dummy_i, dummy_i, nullptr);
      if (st == VVS_OK) {
        ++ok_verify;
        if (vvs_verify(tg, 0, nullptr, nullptr, nullptr, nullptr, dummy_f, VVS_STRICT, dummy_i, dummy_i, dummy_i, nullptr) != VVS_ESTATE) { printf("second verify without commit\n"); return 1; }
        if (vvs_kv_commit(tg, nullptr) != VVS_OK) { printf("commit\n"); return 1; }
        if (vvs_kv_commit(tg, nullptr) != VVS_ESTATE) { printf("double commit accepted\n"); return 1; }
      } else if (n > tc.max_nodes && st != VVS_ESIZE) { printf("oversized verify: status %d\n", st); return 1; }
      const int k = ri(0, 6), nu = ri(-1, 9);
      st = vvs_draft(dr, tg, n, n ? parent.data() : nullptr, nullptr, k, dummy_i, nu, it & 1 ? dummy_i : nullptr, dummy_i, dummy_f, nullptr);
      if (st == VVS_OK) ++ok_draft;
      (void)vvs_path_similarity(tg, n, n ? parent.data() : nullptr, nullptr, dummy_i, 0.8f, ri(0, 3), dummy_f, nullptr);
    }
    if (ok_verify < 200 || ok_draft < 50) { printf("too few valid calls: %d verify, %d draft\n", ok_verify, ok_draft); return 1; }
    (void)vvs_read_features(tg, dummy_f, dummy_i, nullptr);
    (void)vvs_debug_logits(tg, nullptr, nullptr, nullptr, nullptr);
    (void)vvs_debug_logits(dr, nullptr, nullptr, nullptr, nullptr);
    vvs_destroy(tg);
    vvs_destroy(dr);
    printf("dtype %d: %d verify calls and %d drafting calls passed the host checks\n", bf16, ok_verify, ok_draft);
  }
  printf("host fuzz ok, %ld launches reached the stand-ins\n", vvs::g_launches);
  return 0;
}
