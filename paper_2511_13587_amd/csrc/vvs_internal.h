// Internal declarations shared by the host planner and the HIP kernels of libvvs.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <string>
#include <vector>
#include "vvs.h"

namespace vvs {

typedef uint16_t bf16_t;   // raw bf16 bits

// Tree topology of one verify call, handed to kernels by value (no device allocation, no copy).
struct TreeDesc {
  int32_t T;                       // query tokens per row (root + N)
  int32_t causal;                  // 1: chain / prefill chunk (token i sees tokens 0..i of the block)
  int32_t n_forced;                // nodes 1..n_forced are accepted without a test (post verification)
  int8_t parent[VVS_MAX_T];        // parent[0] = -1
  int8_t depth[VVS_MAX_T];
  int8_t first_child[VVS_MAX_T];   // -1 = leaf
  int8_t next_sibling[VVS_MAX_T];  // -1 = last child
  uint64_t anc[VVS_MAX_T];         // bit j set iff block token j is visible to token i
};

// How the positions of the T block tokens of row r are found.
struct PosDesc {
  const int32_t* kv_len;      // device [B] (verify) or nullptr (prefill: kv_base for every row)
  const int32_t* n_emitted;   // device [B] (verify) or nullptr
  int32_t kv_base;            // prefill: first slot of this chunk
  int32_t prefix_len;
  int32_t grid_w;
};

struct GemmPlan { int bm, bn, splits; };

// Byte offsets into the caller's workspace.
struct Workspace {
  size_t state, outcome, node_result, tokens, rope_tab, x, h, gemm_out, q, attn, act, hf, logits, probs,
      pq_work, ss, ss2, ring, ring_state, din, total;
};

struct PackedLayout {
  size_t embed, prefix_embed, gf, wout;
  size_t layer0, layer_stride;           // per layer block
  size_t g1, wqkv, wo, g2, wgu, wd;      // offsets inside a layer block
  size_t fc;                             // drafter contexts: the input map [2d -> d]
  size_t total;
};

struct TimedLaunch { int cls; hipEvent_t t0, t1; };

struct Ctx {
  vvs_config cfg;
  int B, R, d, H, dh, F, L, V, lo, veff, P, G, Tmax, chunk, Mmax, Mlog, S_cap, rope_pos;
  size_t esz;                            // bytes per model element
  char* kv; char* ws; char* pw;
  size_t kv_layer_stride, kv_row_stride, kv_head_stride, kv_v_off;  // in elements; V half starts at kv_v_off
  Workspace w;
  PackedLayout p;
  size_t gemm_out_elems;
  const int32_t* nbr;
  const float* codebook; int code_dim;   // latent codebook of the path-similarity kernel (by reference)
  bool weights_loaded, prefilled, verify_pending;
  int last_T;                            // T of the last verify / prefill (for debug export)
  std::string err;
  bool timing;                           // bracket launches with events
  std::vector<TimedLaunch> timed;        // recorded launches (events are reused across enables)
  size_t n_timed;
};

// Brackets the launches made during its lifetime with two events when timing is enabled.
struct Timed {
  Ctx* c; hipStream_t s; TimedLaunch* t;
  Timed(Ctx* ctx, int cls, hipStream_t st) : c(ctx), s(st), t(nullptr) {
    if (!c->timing) return;
    if (c->n_timed == c->timed.size()) {
      TimedLaunch n{cls, nullptr, nullptr};
      if (hipEventCreate(&n.t0) != hipSuccess || hipEventCreate(&n.t1) != hipSuccess) return;
      c->timed.push_back(n);
    }
    t = &c->timed[c->n_timed++];
    t->cls = cls;
    (void)hipEventRecord(t->t0, s);
  }
  ~Timed() { if (t) (void)hipEventRecord(t->t1, s); }
};

// ---- host planner (vvs_host.cpp)
vvs_status plan_sizes(const vvs_config* cfg, Ctx* c, std::string* err);
GemmPlan plan_gemm(const Ctx* c, int M, int N, int K);
bool plan_fused(const Ctx* c, int M);   // true: the fused 5-kernel layer runs for M GEMM rows
vvs_status build_tree(int n_nodes, const int32_t* h_parent, const uint8_t* h_mask, TreeDesc* out, std::string* err);

// ---- launchers (kernels_*.hip); all asynchronous on the stream
void launch_fill_zero(void* p, size_t bytes, hipStream_t s);
void launch_copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t s);
void launch_pack_weights(Ctx* c, const void* const* tensors, hipStream_t s);
void launch_forward(Ctx* c, const TreeDesc& tree, const PosDesc& pos, int T, const int32_t* d_tokens_bt,
                    const void* d_prefix_cond, const void* d_prefix_uncond, int chunk_start,
                    const int32_t* d_forced, int n_forced, int logits_mode /*0 none, 1 every token, 2 last token of each row*/,
                    hipStream_t s, bool from_din = false /*drafter: inputs = fc applied to the rows of workspace din*/);
void launch_build_tokens(Ctx* c, int T, const int32_t* d_draft, hipStream_t s);
void launch_accept(Ctx* c, const TreeDesc& tree, int T, const float* d_logits, const int32_t* d_draft_tokens,
                   const float* d_q, const float* d_u, int u_stride_b, int u_stride_j, int u_off_acc, int u_off_term,
                   int mode, bool use_state, int32_t* d_accept_len, int32_t* d_path, int32_t* d_next,
                   bool keep_outcome, hipStream_t s);
vvs_status launch_accept_noalloc(Ctx* c, const TreeDesc& tree, int T, const float* d_logits, const int32_t* d_draft_tokens,
                                 const float* d_q, const float* d_u, int mode, int32_t* d_accept_len, int32_t* d_path, int32_t* d_next,
                                 hipStream_t s, std::string* err);
void launch_prefill_finish(Ctx* c, int n_forced, int32_t* d_first, hipStream_t s);
void launch_commit(Ctx* c, hipStream_t s);
void launch_push_prefill_feature(Ctx* c, int T_last_chunk, hipStream_t s);
void launch_read_features(Ctx* c, float* d_features, int32_t* d_count, hipStream_t s);
void launch_path_similarity(Ctx* c, const TreeDesc& tree, int n_nodes, const int32_t* d_draft_tokens, float alpha, int stride,
                            float* d_similarity, hipStream_t s);

// One level of a drafting call: which block token is which node of the candidate tree.
struct DraftLevel {
  int32_t k;                        // context pairs (block tokens 0 .. k-1)
  int32_t Tq, Tq_prev;              // block tokens per row of this level's forward and of the previous one
  int32_t n_nodes;                  // N of the candidate tree
  int8_t node[VVS_MAX_T];           // block token t >= k: its node id
  int8_t parent_slot[VVS_MAX_T];    // block token t >= k: block index of the node's parent
  int32_t n_sel;                    // nodes expanded at this level
  int8_t sel_node[VVS_MAX_T], sel_slot[VVS_MAX_T];
};
void launch_draft_state(Ctx* dr, const Ctx* tg, int k, int n_unverified, hipStream_t s);
void launch_draft_zero_leaves(Ctx* dr, const TreeDesc& shape, float* d_probs, hipStream_t s);
void launch_draft_input(Ctx* dr, const Ctx* tg, const DraftLevel& lv, const int32_t* d_recent, const int32_t* d_draft_tokens,
                        hipStream_t s);
void launch_draft_select(Ctx* dr, const DraftLevel& lv, const TreeDesc& shape, const int32_t* d_given_tokens, int32_t* d_draft_tokens,
                         float* d_probs, hipStream_t s);
void launch_read_state(Ctx* c, int32_t* d_state, hipStream_t s);
void launch_set_state(Ctx* c, const int32_t* d_state, hipStream_t s);
void launch_debug_logits(Ctx* c, float* raw, float* mixed, float* probs, hipStream_t s);
void launch_debug_kv(Ctx* c, int layer, int row, int n_slots, float* dk, float* dv, hipStream_t s);
void launch_fill_probe(const void* src, size_t region_bytes, size_t wg_stride_bytes, int reps, int mode, int n_workgroups, int waves,
                       uint32_t* sink, hipStream_t s);
void launch_debug_gemm(Ctx* c, int m, int n, int k, const void* a, const void* w, void* scratch, float* out, hipStream_t s);

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace vvs
