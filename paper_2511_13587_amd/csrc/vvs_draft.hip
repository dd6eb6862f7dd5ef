// Draft side (Algorithm 2: "C_t <- M_D(f_t, a)"; Section 3, "Stale Feature Reusability"): the kernels
// around the drafter's forwards.  A drafting call runs the drafter level by level; every level is one
// forward of the ordinary kind (ancestor-masked block, the drafter context's own small KV region, cached
// length 0) over the n_ctx (feature, token) pairs and every node expanded so far.  These kernels build the
// forward's input rows and turn its logits into the distributions and tokens of the next level.
#include "vvs_device.h"

namespace vvs {

// Per prompt: cached length 0 and the number of emitted tokens that puts block token t at image index
// first + depth(t), first = max(0, root - (k - 1)), root = emitted tokens of the target - 1 + n_unverified.
__global__ void k_draft_state(int32_t* __restrict__ state, const int32_t* __restrict__ target_state, int B, int k, int n_unverified) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const int root = target_state[B + b] - 1 + n_unverified;
  state[b] = 0;
  state[B + b] = max(0, root - (k - 1)) + 1;
  state[2 * B + b] = -1;
}

void launch_draft_state(Ctx* dr, const Ctx* tg, int k, int n_unverified, hipStream_t s) {
  hipLaunchKernelGGL(k_draft_state, dim3((dr->B + 63) / 64), dim3(64), 0, s, (int32_t*)(dr->ws + dr->w.state),
                     (const int32_t*)(tg->ws + tg->w.state), dr->B, k, n_unverified);
}

struct LeafList { int32_t n; int8_t node[VVS_MAX_T]; };

__global__ void k_draft_zero_rows(float* __restrict__ probs, LeafList leaves, int T, int V) {
  float* row = probs + ((size_t)blockIdx.x * T + leaves.node[blockIdx.y]) * V;
  for (int i = threadIdx.x; i < V; i += blockDim.x) row[i] = 0.f;
}

void launch_draft_zero_leaves(Ctx* dr, const TreeDesc& shape, float* d_probs, hipStream_t s) {
  LeafList leaves;
  leaves.n = 0;
  for (int j = 0; j < shape.T; ++j)
    if (shape.first_child[j] < 0) leaves.node[leaves.n++] = (int8_t)j;
  if (!leaves.n) return;
  hipLaunchKernelGGL(k_draft_zero_rows, dim3(dr->B, leaves.n), dim3(256), 0, s, d_probs, leaves, shape.T, dr->veff);
}

// One workgroup per block token m = r * Tq + t: writes the row [embedding of the token ; feature] of the
// input map's operand (row-major fp32, or the packed bf16 operand order).
//   t <  k: token = recent[b][t]; feature = the (k - t)-th newest entry of the target's ring of row r
//           (zeros when the ring holds fewer entries);
//   t >= k: token = the node's drafted token; feature = what the previous level's forward left for the
//           node's parent in the residual stream x: rmsnorm(x) * gf, or x itself (pre_norm), in the model's
//           storage precision - the same kind of vector the target caches.
template <typename T>
__global__ __launch_bounds__(256) void k_draft_input(T* __restrict__ din, const T* __restrict__ embed, const T* __restrict__ ring,
                                                     const int32_t* __restrict__ ring_state, const float* __restrict__ x,
                                                     const float* __restrict__ gf, const int32_t* __restrict__ recent,
                                                     const int32_t* __restrict__ draft_tokens, DraftLevel lv, int R, int d, int V,
                                                     int slots, int pre_norm, float eps) {
  __shared__ float red[16];
  const int m = blockIdx.x, r = m / lv.Tq, t = m % lv.Tq, b = r >> 1;
  int tok;
  const T* feat = nullptr;
  const float* xr = nullptr;
  if (t < lv.k) {
    tok = recent[b * lv.k + t];
    const int held = ring_state[r], oldest = ring_state[R + r], e = held - lv.k + t;
    if (e >= 0) feat = ring + ((size_t)r * slots + (oldest + e) % slots) * d;
  } else {
    tok = draft_tokens[b * lv.n_nodes + lv.node[t] - 1];
    xr = x + ((size_t)r * lv.Tq_prev + lv.parent_slot[t]) * d;
  }
  tok = min(max(tok, 0), V - 1);
  const T* emb = embed + (size_t)tok * d;
  float scale = 1.f;
  if (xr && !pre_norm) {
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += blockDim.x) ss += xr[i] * xr[i];
    ss = block_sum(ss, red);
    scale = 1.0f / sqrtf(ss / (float)d + eps);
  }
  for (int k0 = threadIdx.x * 8; k0 < d; k0 += blockDim.x * 8) {
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = ld(emb + k0 + i);
    store8(din, m, k0, 2 * d, v);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (xr) v[i] = pre_norm ? xr[k0 + i] : xr[k0 + i] * scale * gf[k0 + i];
      else v[i] = feat ? ld(feat + k0 + i) : 0.f;
    }
    store8(din, m, d + k0, 2 * d, v);
  }
}

void launch_draft_input(Ctx* dr, const Ctx* tg, const DraftLevel& lv, const int32_t* d_recent, const int32_t* d_draft_tokens,
                        hipStream_t s) {
  Timed timed(dr, VVS_K_ELEMENTWISE, s);
  const int M = dr->R * lv.Tq;
  const float* x = (const float*)(dr->ws + dr->w.x);
  const float* gf = (const float*)(dr->pw + dr->p.gf);
  const int32_t* ring_state = (const int32_t*)(tg->ws + tg->w.ring_state);
  if (dr->cfg.dtype == VVS_BF16)
    hipLaunchKernelGGL(k_draft_input<bf16_t>, dim3(M), dim3(256), 0, s, (bf16_t*)(dr->ws + dr->w.din), (const bf16_t*)(dr->pw + dr->p.embed),
                       (const bf16_t*)(tg->ws + tg->w.ring), ring_state, x, gf, d_recent, d_draft_tokens, lv, dr->R, dr->d, dr->V,
                       tg->cfg.feature_slots, dr->cfg.feature_pre_norm, dr->cfg.rms_eps);
  else
    hipLaunchKernelGGL(k_draft_input<float>, dim3(M), dim3(256), 0, s, (float*)(dr->ws + dr->w.din), (const float*)(dr->pw + dr->p.embed),
                       (const float*)(tg->ws + tg->w.ring), ring_state, x, gf, d_recent, d_draft_tokens, lv, dr->R, dr->d, dr->V,
                       tg->cfg.feature_slots, dr->cfg.feature_pre_norm, dr->cfg.rms_eps);
}

// One workgroup per (prompt, node expanded at this level): mixes the node's conditional and unconditional
// logit rows, writes the softmax as the distribution of the node's children, and gives the c-th child the
// id with the c-th largest mixed logit (ties to the lower id) - or the caller's token.
struct Best { float v; int i; };
__device__ __forceinline__ Best better(Best a, Best b) { return (b.v > a.v || (b.v == a.v && b.i < a.i)) ? b : a; }

__global__ __launch_bounds__(1024) void k_draft_select(const float* __restrict__ logits, DraftLevel lv, TreeDesc shape,
                                                       const int32_t* __restrict__ given, int32_t* __restrict__ draft_tokens,
                                                       float* __restrict__ probs, int V, int lo, float cfg_scale) {
  __shared__ float red[16];
  __shared__ float s_bv[16];
  __shared__ int s_bi[16];
  __shared__ int s_taken[VVS_MAX_T];
  const int b = blockIdx.x, j = lv.sel_node[blockIdx.y], t = lv.sel_slot[blockIdx.y];
  const float* lc = logits + ((size_t)(2 * b) * lv.Tq + t) * V;
  const float* lu = logits + ((size_t)(2 * b + 1) * lv.Tq + t) * V;
  float* out = probs + ((size_t)b * shape.T + j) * V;
  float mx = -INFINITY;
  for (int i = threadIdx.x; i < V; i += blockDim.x) mx = fmaxf(mx, lu[i] + cfg_scale * (lc[i] - lu[i]));
  mx = block_max(mx, red);
  float sum = 0.f;
  for (int i = threadIdx.x; i < V; i += blockDim.x) sum += expf(lu[i] + cfg_scale * (lc[i] - lu[i]) - mx);
  sum = block_sum(sum, red);
  const float inv = 1.0f / sum;
  for (int i = threadIdx.x; i < V; i += blockDim.x) out[i] = expf(lu[i] + cfg_scale * (lc[i] - lu[i]) - mx) * inv;
  int n_taken = 0;
  for (int c = shape.first_child[j]; c >= 0; c = shape.next_sibling[c]) {
    if (given) {
      if (threadIdx.x == 0) draft_tokens[b * lv.n_nodes + c - 1] = given[b * lv.n_nodes + c - 1];
      continue;
    }
    Best best{-INFINITY, 0x7fffffff};
    for (int i = threadIdx.x; i < V; i += blockDim.x) {
      bool free_id = true;
      for (int q = 0; q < n_taken; ++q) free_id = free_id && s_taken[q] != i;
      if (free_id) best = better(best, Best{lu[i] + cfg_scale * (lc[i] - lu[i]), i});
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) best = better(best, Best{__shfl_xor(best.v, o, 64), __shfl_xor(best.i, o, 64)});
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { s_bv[threadIdx.x >> 6] = best.v; s_bi[threadIdx.x >> 6] = best.i; }
    __syncthreads();
    if (threadIdx.x == 0) {
      Best w{s_bv[0], s_bi[0]};
      for (int q = 1; q < (int)(blockDim.x >> 6); ++q) w = better(w, Best{s_bv[q], s_bi[q]});
      s_taken[n_taken] = w.i;
      draft_tokens[b * lv.n_nodes + c - 1] = lo + w.i;
    }
    ++n_taken;
    __syncthreads();
  }
}

// The same for slices of at most 16 * 1024 ids: a thread keeps its 16 mixed logits in registers, so the
// rows are read once and a taken id is simply removed from its owner's registers.
__global__ __launch_bounds__(1024) void k_draft_select_regs(const float* __restrict__ logits, DraftLevel lv, TreeDesc shape,
                                                            const int32_t* __restrict__ given, int32_t* __restrict__ draft_tokens,
                                                            float* __restrict__ probs, int V, int lo, float cfg_scale) {
  constexpr int NR = 16;
  __shared__ float red[16];
  __shared__ float s_bv[16];
  __shared__ int s_bi[16];
  __shared__ int s_win;
  const int b = blockIdx.x, j = lv.sel_node[blockIdx.y], t = lv.sel_slot[blockIdx.y];
  const float* lc = logits + ((size_t)(2 * b) * lv.Tq + t) * V;
  const float* lu = logits + ((size_t)(2 * b + 1) * lv.Tq + t) * V;
  float* out = probs + ((size_t)b * shape.T + j) * V;
  float mixed[NR];
  float mx = -INFINITY;
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    const int i = threadIdx.x + r * 1024;
    mixed[r] = -INFINITY;
    if (i < V) mixed[r] = lu[i] + cfg_scale * (lc[i] - lu[i]);
    mx = fmaxf(mx, mixed[r]);
  }
  mx = block_max(mx, red);
  float e[NR];
  float sum = 0.f;
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    e[r] = threadIdx.x + r * 1024 < V ? expf(mixed[r] - mx) : 0.f;
    sum += e[r];
  }
  sum = block_sum(sum, red);
  const float inv = 1.0f / sum;
#pragma unroll
  for (int r = 0; r < NR; ++r)
    if (threadIdx.x + r * 1024 < V) out[threadIdx.x + r * 1024] = e[r] * inv;
  for (int c = shape.first_child[j]; c >= 0; c = shape.next_sibling[c]) {
    if (given) {
      if (threadIdx.x == 0) draft_tokens[b * lv.n_nodes + c - 1] = given[b * lv.n_nodes + c - 1];
      continue;
    }
    Best best{-INFINITY, 0x7fffffff};
#pragma unroll
    for (int r = 0; r < NR; ++r)                       // ascending ids: a later equal value does not replace an earlier one
      if (mixed[r] > best.v) best = Best{mixed[r], (int)threadIdx.x + r * 1024};
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) best = better(best, Best{__shfl_xor(best.v, o, 64), __shfl_xor(best.i, o, 64)});
    if ((threadIdx.x & 63) == 0) { s_bv[threadIdx.x >> 6] = best.v; s_bi[threadIdx.x >> 6] = best.i; }
    __syncthreads();
    if (threadIdx.x == 0) {
      Best w{s_bv[0], s_bi[0]};
      for (int q = 1; q < 16; ++q) w = better(w, Best{s_bv[q], s_bi[q]});
      s_win = w.i;
      draft_tokens[b * lv.n_nodes + c - 1] = lo + w.i;
    }
    __syncthreads();
    const int win = s_win;
#pragma unroll
    for (int r = 0; r < NR; ++r)
      if (threadIdx.x + r * 1024 == win) mixed[r] = -INFINITY;
    __syncthreads();                                   // s_win and the per-wave slots are rewritten by the next child
  }
}

void launch_draft_select(Ctx* dr, const DraftLevel& lv, const TreeDesc& shape, const int32_t* d_given_tokens, int32_t* d_draft_tokens,
                         float* d_probs, hipStream_t s) {
  if (!lv.n_sel) return;
  Timed timed(dr, VVS_K_ACCEPT, s);
  if (dr->veff <= 16 * 1024)
    hipLaunchKernelGGL(k_draft_select_regs, dim3(dr->B, lv.n_sel), dim3(1024), 0, s, (const float*)(dr->ws + dr->w.logits), lv, shape,
                       d_given_tokens, d_draft_tokens, d_probs, dr->veff, dr->lo, dr->cfg.cfg_scale);
  else
    hipLaunchKernelGGL(k_draft_select, dim3(dr->B, lv.n_sel), dim3(1024), 0, s, (const float*)(dr->ws + dr->w.logits), lv, shape,
                       d_given_tokens, d_draft_tokens, d_probs, dr->veff, dr->lo, dr->cfg.cfg_scale);
}

}  // namespace vvs
